"""MI355X-native hot path of communication-free vertex-cut GNN training (arxiv 2308.03209).

`paper_2308_03209_amd.inputs` draws the seeded synthetic workloads; the HIP library and
its ctypes binding live in `paper_2308_03209_amd.binding` (imported lazily so that the
input generators can be used without the compiled library).
"""
__all__ = ["inputs"]
