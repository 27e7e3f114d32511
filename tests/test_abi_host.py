"""CPU-side tests of the C-ABI library: exported symbols and the host-only partition builder
(bit-exact against the oracle).  No GPU compute is called here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import dropedge as o_dropedge
from oracle import partition as o_partition
from paper_2308_03209_amd import inputs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2308_03209_amd import binding
    return binding


def test_library_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "cofree.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(cofree_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations found"
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(raw, name), f"{name} declared in cofree.h but not exported"
    assert declared == set(B.EXPORTS)


def test_layer_descriptor_layout_matches_the_library(B):
    assert B.lib.cofree_layer_desc_size() == ctypes.sizeof(B.LayerDesc) == 56


def test_device_count_never_faults(B):
    assert B.device_count() >= -1


ARRAYS = ["local2global", "rowptr", "col", "eid", "deg_local", "deg_global", "dar_weight", "edge_lo", "edge_hi"]


def compare_partition(B, P, O):
    assert P.num_nodes == O["n_nodes"] and P.num_edges == O["n_edges"] and P.num_nnz == O["nnz"]
    ids = [B.ARR_LOCAL2GLOBAL, B.ARR_ROWPTR, B.ARR_COL, B.ARR_EID, B.ARR_DEG_LOCAL, B.ARR_DEG_GLOBAL,
           B.ARR_DAR_WEIGHT, B.ARR_EDGE_LO, B.ARR_EDGE_HI]
    for which, name in zip(ids, ARRAYS):
        got = P.host_array(which)
        assert got.dtype == O[name].dtype, name
        assert np.array_equal(got.view(np.uint8), O[name].view(np.uint8)), name   # bit-exact


@pytest.mark.parametrize("p", [1, 4])
def test_host_partition_bit_exact_cfg0(B, p):
    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    for i in range(p):
        P = B.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT, flags=B.HOST_ONLY)
        O = o_partition.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        compare_partition(B, P, O)


def test_host_partition_bit_exact_midsize_threaded_path(B):
    # large enough to take the multi-threaded hashing / bucketed sort path of the builder
    wl = inputs.WORKLOADS[2].scaled(0.02)
    src, dst = inputs.workload_graph(wl)
    assert len(src) > (1 << 18)
    P = B.build_partition(wl.n_nodes, src, dst, 8, 3, inputs.SEED_CUT, flags=B.HOST_ONLY)
    O = o_partition.build_partition(wl.n_nodes, src, dst, 8, 3, inputs.SEED_CUT)
    compare_partition(B, P, O)


def test_host_partition_explicit_assignment_and_dedup(B):
    n = 50
    src, dst = inputs.small_random_graph(n, 120, 4)
    assign = np.random.default_rng(0).integers(0, 3, len(src)).astype(np.int32)
    for i in range(3):
        P = B.build_partition(n, src, dst, 3, i, 0, assignment=assign, flags=B.HOST_ONLY)
        O = o_partition.build_partition(n, src, dst, 3, i, 0, assignment=assign)
        compare_partition(B, P, O)
    s2, d2 = np.r_[src, dst[:10]], np.r_[dst, src[:10]]          # ten edges repeated, reversed
    with pytest.raises(B.CofreeError) as e:
        B.build_partition(n, s2, d2, 2, 0, 1, flags=B.HOST_ONLY)
    assert e.value.code == B.EINVAL
    P = B.build_partition(n, s2, d2, 2, 0, 1, flags=B.HOST_ONLY | B.DEDUP)
    O = o_partition.build_partition(n, s2, d2, 2, 0, 1, dedup=True)
    compare_partition(B, P, O)


def test_host_partition_rejects_bad_input(B):
    ok = dict(flags=B.HOST_ONLY)
    for args in [
        (5, [0, 1], [1, 1], 2, 0, 1),      # self loop
        (5, [0, 1], [1, 5], 2, 0, 1),      # id out of range
        (5, [0, -1], [1, 2], 2, 0, 1),     # negative id
        (5, [0], [1], 0, 0, 1),            # n_parts
        (5, [0], [1], 2, 2, 1),            # part_id
        (0, [], [], 1, 0, 1),              # n_nodes
    ]:
        with pytest.raises(B.CofreeError) as e:
            B.build_partition(args[0], np.array(args[1], np.int64), np.array(args[2], np.int64), *args[3:], **ok)
        assert e.value.code == B.EINVAL
        assert B.last_error()
    with pytest.raises(B.CofreeError):
        B.build_partition(5, np.array([0]), np.array([1]), 2, 0, 1, assignment=np.array([2], np.int32), **ok)
    # an empty partition is valid
    P = B.build_partition(5, np.array([], np.int64), np.array([], np.int64), 2, 0, 1, **ok)
    assert P.num_nodes == 0 and P.num_nnz == 0


def test_host_only_partition_refuses_device_work(B):
    P = B.build_partition(5, np.array([0, 1]), np.array([1, 2]), 1, 0, 1, flags=B.HOST_ONLY)
    with pytest.raises(B.CofreeError) as e:
        P.device_array(B.ARR_COL)
    assert e.value.code == B.ESTATE
    out = ctypes.c_void_p()
    rc = B.lib.cofree_dropedge_k(P.handle, 2, 0.5, 1, 0, None, ctypes.byref(out))
    assert rc == B.ESTATE


def test_mask_pick_matches_oracle(B):
    for K in (1, 4, 10):
        for t in list(range(50)) + [2 ** 33 + 5]:
            assert B.dropedge_pick(7, t, K) == o_dropedge.pick(7, t, K)
    with pytest.raises(B.CofreeError):
        B.dropedge_pick(7, 0, 0)


def test_workspace_sizes_are_sane(B):
    d = B.layer_desc(B.SAGE_MEAN, 602, 256, 256)
    assert B.layer_workspace_bytes(d, 1000, False) >= 256
    need = B.layer_workspace_bytes(d, 1000, True)
    assert need >= 2 * 1000 * 256 * 4
    d2 = B.layer_desc(B.GCN, 64, 0, 16)
    assert B.layer_workspace_bytes(d2, 1000, False) >= 1000 * 16 * 4
    assert B.loss_workspace_bytes() > 0


def test_host_partition_degree_aware_cut_and_replication_counts(B):
    """The degree-aware hash cut and RF(v_j), bit-exact against the oracle (small and threaded sizes,
    more than 64 partitions included)."""
    cases = [(inputs.WORKLOADS[0], 4), (inputs.WORKLOADS[0], 70), (inputs.WORKLOADS[2].scaled(0.02), 8)]
    for wl, p in cases:
        src, dst = inputs.workload_graph(wl)
        for method, flag in (("random", 0), ("dbh", B.CUT_DBH)):
            Os = [o_partition.build_partition(wl.n_nodes, src, dst, p, i, 11, method=method) for i in range(p)]
            rf = o_partition.node_replication(wl.n_nodes, Os)
            for i in sorted({0, p // 2, p - 1}):
                P = B.build_partition(wl.n_nodes, src, dst, p, i, 11, flags=B.HOST_ONLY | B.WITH_RF | flag)
                compare_partition(B, P, Os[i])
                got = P.host_array(B.ARR_RF)
                assert got.dtype == np.int32
                assert np.array_equal(got, rf[Os[i]["local2global"]])


def test_replication_counts_with_explicit_assignment_and_flag_errors(B):
    n = 50
    src, dst = inputs.small_random_graph(n, 120, 4)
    assign = np.random.default_rng(1).integers(0, 3, len(src)).astype(np.int32)
    Os = [o_partition.build_partition(n, src, dst, 3, i, 0, assignment=assign) for i in range(3)]
    rf = o_partition.node_replication(n, Os)
    P = B.build_partition(n, src, dst, 3, 1, 0, assignment=assign, flags=B.HOST_ONLY | B.WITH_RF)
    assert np.array_equal(P.host_array(B.ARR_RF), rf[Os[1]["local2global"]])
    # not requested -> not there
    Q = B.build_partition(n, src, dst, 3, 1, 0, flags=B.HOST_ONLY)
    with pytest.raises(B.CofreeError) as e:
        Q.host_array(B.ARR_RF)
    assert e.value.code == B.ESTATE
    # the degree-aware cut decides the assignment itself
    with pytest.raises(B.CofreeError) as e:
        B.build_partition(n, src, dst, 3, 1, 0, assignment=assign, flags=B.HOST_ONLY | B.CUT_DBH)
    assert e.value.code == B.EINVAL
    # duplicates + explicit assignment + RF: which copy counts would be ambiguous
    s2, d2 = np.r_[src, dst[:5]], np.r_[dst, src[:5]]
    a2 = np.r_[assign, (assign[:5] + 1) % 3].astype(np.int32)
    with pytest.raises(B.CofreeError) as e:
        B.build_partition(n, s2, d2, 3, 0, 0, assignment=a2, flags=B.HOST_ONLY | B.WITH_RF | B.DEDUP)
    assert e.value.code == B.EINVAL
