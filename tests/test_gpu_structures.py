"""GPU parity: partition arrays on the device, DropEdge-K mask bits and compacted graphs - bit-exact."""
import numpy as np
import pytest

from oracle import dropedge as o_dropedge
from oracle import partition as o_partition
from paper_2308_03209_amd import inputs

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03209_amd import binding
    assert binding.device_count() >= 1
    return binding


class _RawDevice:
    """Exposes a raw device pointer to torch through the CUDA array interface."""

    def __init__(self, ptr, count, typestr):
        self.__cuda_array_interface__ = {"shape": (count,), "typestr": typestr, "data": (ptr, False), "version": 2}


def device_to_numpy(ptr, count, dtype):
    import torch
    typestr = {torch.int64: "<i8", torch.int32: "<i4", torch.float32: "<f4"}[dtype]
    if count == 0:
        return torch.empty(0, dtype=dtype).numpy()
    return torch.as_tensor(_RawDevice(ptr, count, typestr), device="cuda").cpu().numpy()


@pytest.mark.parametrize("cfg,scale,p,part", [(0, 1.0, 4, 2), (2, 0.01, 8, 0)])
def test_partition_device_arrays_bit_exact(B, cfg, scale, p, part):
    import torch
    wl = inputs.WORKLOADS[cfg].scaled(scale) if scale != 1.0 else inputs.WORKLOADS[cfg]
    src, dst = inputs.workload_graph(wl)
    print(f"[case] partition cfg{cfg} x{scale} p={p} part={part} edges={len(src)}", flush=True)
    P = B.build_partition(wl.n_nodes, src, dst, p, part, inputs.SEED_CUT)
    O = o_partition.build_partition(wl.n_nodes, src, dst, p, part, inputs.SEED_CUT)
    for which, name, dt in [(B.ARR_ROWPTR, "rowptr", torch.int64), (B.ARR_COL, "col", torch.int32),
                            (B.ARR_DEG_LOCAL, "deg_local", torch.int32),
                            (B.ARR_DAR_WEIGHT, "dar_weight", torch.float32),
                            (B.ARR_LOCAL2GLOBAL, "local2global", torch.int64)]:
        ptr, n = P.device_array(which)
        got = device_to_numpy(ptr, n, dt)
        assert np.array_equal(got.view(np.uint8), O[name].view(np.uint8)), name
        assert np.array_equal(P.host_array(which).view(np.uint8), O[name].view(np.uint8)), name


@pytest.mark.parametrize("which,K,p_drop", [("cfg0", 3, 0.5), ("cfg2s", 4, 0.5), ("cfg0", 2, 0.0), ("cfg0", 3, 0.9)])
def test_dropedge_masks_bit_exact(B, which, K, p_drop):
    # cfg0 partition: n_edges is not a multiple of 64 (ragged last word); scaled cfg2; extremes of p_drop
    wl = inputs.WORKLOADS[0] if which == "cfg0" else inputs.WORKLOADS[2].scaled(0.01)
    src, dst = inputs.workload_graph(wl)
    p = 4 if which == "cfg0" else 8
    K = int(K)
    print(f"[case] masks wl={wl.name} K={K} p_drop={p_drop}", flush=True)
    P = B.build_partition(wl.n_nodes, src, dst, p, 1, inputs.SEED_CUT)
    O = o_partition.build_partition(wl.n_nodes, src, dst, p, 1, inputs.SEED_CUT)
    M = B.dropedge_k(P, K, p_drop, inputs.SEED_MASKS)
    assert M.count == K
    keep = o_dropedge.masks(O["n_edges"], K, p_drop, inputs.SEED_MASKS)
    for k in range(K):
        bits = M.host_bits(k)
        assert np.array_equal(bits, o_dropedge.pack_bits(keep[k])), f"mask {k} bits"
        rowptr, col = M.host_graph(k)
        r_ref, c_ref, _ = o_dropedge.masked_graph(O, keep[k])
        assert np.array_equal(rowptr, r_ref) and np.array_equal(col, c_ref), f"mask {k} graph"
    if p_drop == 0.0:
        rowptr, col = M.host_graph(0)
        assert np.array_equal(rowptr, O["rowptr"]) and np.array_equal(col, O["col"])


def test_dropedge_rejects_bad_arguments(B):
    P = B.build_partition(5, np.array([0, 1]), np.array([1, 2]), 1, 0, 1)
    for K, p in [(0, 0.5), (2, 1.0), (2, -0.1)]:
        with pytest.raises(B.CofreeError) as e:
            B.dropedge_k(P, K, p, 1)
        assert e.value.code == B.EINVAL


def test_empty_partition_on_device(B):
    P = B.build_partition(5, np.array([], np.int64), np.array([], np.int64), 2, 0, 1)
    assert P.num_nodes == 0
    M = B.dropedge_k(P, 2, 0.5, 1)
    assert M.host_bits(0).size == 0
