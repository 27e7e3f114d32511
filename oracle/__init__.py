"""CPU oracle for the per-partition training step of communication-free vertex-cut GNN
training (arxiv 2308.03209).

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 numpy code written from the paper; it shares
no code with the HIP library and must never be imported by the product path
(`paper_2308_03209_amd/`).  Only `tests/`, `__graft_entry__.smoke()` and the `cpu_baseline`
leg of `bench.py` may use it.

Modules
-------
counter_rng : Philox-4x32-10 counter-based generator (Salmon et al., SC'11) and the draws
              the method takes from it (edge -> partition, DropEdge-K masks, mask pick, dropout).
partition   : random vertex cut (Section 3 "Vertex Cut Partitioning"; proof of Theorem 2),
              per-partition CSR, duplicated-node map, degrees, Degree-Aware Reweighting
              weights (Section 4.3, Algorithm 1 line 4), replication factor (Eq. 1).
dropedge    : DropEdge-K masks and the masked partition graph (Section 4.4, Algorithm 1 lines 5-9).
layers      : GraphSAGE-mean layer as printed in Section 3, and the GCN layer, forward and backward.
loss        : reweighted loss of Eq. 3 with softmax cross-entropy.
step        : parameter update (Algorithm 1 line 11) and Adam (Appendix B).
epoch       : one training iteration on one or several partitions (Algorithm 1 lines 6-12,
              gradients summed over partitions as in Eq. 2).

Every function here is pinned by `tests/test_oracle_*.py` against closed forms, brute force
on tiny graphs, published known-answer vectors or finite differences.  The one claim that
is NOT pinned is Theorem 3's "the reweighted sum of partition gradients recovers the
full-graph gradient": the paper states it only approximately (parity unpinned); two exact
special cases of it are tested instead.
"""
