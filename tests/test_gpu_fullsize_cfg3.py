"""cfg3 at full size (110M nodes, 796M undirected edges, 16-way cut, one partition of 28M nodes), in the launch
configuration bench.py times: the graph is streamed block by block into the piece-wise builder.

The oracle cannot build this partition whole, so it builds what the sampled outputs depend on.  The stream is read
twice: the first pass keeps the edges incident to a set S of sampled nodes (600 uniformly drawn ones, of which
about a quarter have an edge in partition 0, and the four heaviest nodes of the recipe); from them the oracle's edge
assignment gives S's neighbours in partition 0; the
second pass (the one that also feeds the library's builder) keeps every edge incident to S or to those neighbours.
`oracle.partition.build_partition` on that edge list - with the full node count, so every edge hashes as it does in
the full graph - yields a partition in which the rows of S, and the degrees of S's neighbours, are those of the full
partition.  Structures are compared by global id; aggregation, a GCN layer and the loss are the oracle's functions
evaluated on that partition, compared on the rows of S (the heavy nodes' rows of a few thousand neighbours:
structures and the plain mean).
Matrices at this size have more than 2^32 elements, which none of the smaller tests reach."""
import numpy as np
import pytest

from oracle import dropedge as o_dropedge
from oracle import layers as o_layers
from oracle import loss as o_loss
from oracle import partition as o_partition
from paper_2308_03209_amd import inputs
from util import TOL_BF16, assert_close, progress

pytestmark = pytest.mark.gpu

N_SAMPLED = 600
WORKERS = 12


def from_bf16(t):
    return t.float().cpu().numpy().astype(np.float64)


def incident(src, dst, flag):
    keep = flag[src] | flag[dst]
    return src[keep], dst[keep]


@pytest.fixture(scope="module")
def cfg3():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03209_amd import binding as B
    wl = inputs.WORKLOADS[3]
    stream = inputs.workload_stream(wl)
    rng = np.random.default_rng(2024)
    heavy = stream.perm()[:4].astype(np.int64)        # ranks 0-3 of the recipe: the nodes of largest expected degree
    S = np.unique(np.r_[rng.integers(0, wl.n_nodes, N_SAMPLED), heavy]).astype(np.int64)
    flag_s = np.zeros(wl.n_nodes, dtype=bool)
    flag_s[S] = True

    # pass 1: edges incident to S
    es, ed = [], []
    for k, (src, dst) in enumerate(stream.blocks(workers=WORKERS)):
        a, b = incident(src, dst, flag_s)
        es.append(a)
        ed.append(b)
        if k % 8 == 7:
            progress(f"cfg3 full size: pass 1, block {k + 1} of {stream.n_blocks}")
    es, ed = np.concatenate(es), np.concatenate(ed)
    lo, hi = o_partition.canonical_edges(wl.n_nodes, es, ed)
    mine = o_partition.assign_edges(lo, hi, wl.n_parts, inputs.SEED_CUT) == 0
    small = S[~np.isin(S, heavy)]
    flag_t = np.zeros(wl.n_nodes, dtype=bool)         # S and the neighbours of its small members
    flag_t[S] = True
    in_small = np.isin(lo[mine], small) | np.isin(hi[mine], small)
    flag_t[lo[mine][in_small]] = True
    flag_t[hi[mine][in_small]] = True
    progress(f"cfg3 full size: {len(S)} sampled nodes, {len(es)} incident edges, {int(flag_t.sum())} nodes in the second set")

    # pass 2: the library's builder, and every edge incident to the second set
    bld = B.PartitionBuilder(wl.n_nodes, wl.n_parts, 0, inputs.SEED_CUT, 0)
    ts, td = [], []
    for k, (src, dst) in enumerate(stream.blocks(workers=WORKERS)):
        bld.add_edges(src, dst)
        a, b = incident(src, dst, flag_t)
        ts.append(a)
        td.append(b)
        if k % 8 == 7:
            progress(f"cfg3 full size: pass 2, block {k + 1} of {stream.n_blocks}")
    P = bld.finish()
    progress(f"cfg3 full size: library partition {P.num_nodes} nodes, {P.num_nnz} directed edges")
    ts, td = np.concatenate(ts), np.concatenate(td)
    O = o_partition.build_partition(wl.n_nodes, ts, td, wl.n_parts, 0, inputs.SEED_CUT)
    progress(f"cfg3 full size: oracle partition of the sampled neighbourhood {O['n_nodes']} nodes, {O['nnz']} directed edges")

    l2g = P.host_array(B.ARR_LOCAL2GLOBAL)
    # rows of the library's partition that hold the oracle partition's nodes, and the sampled rows in both numberings
    lib_of_o = np.searchsorted(l2g, O["local2global"])
    assert np.array_equal(l2g[lib_of_o], O["local2global"]), "a node of the sampled neighbourhood is missing"
    present = S[np.isin(S, O["local2global"])]
    o_rows = np.searchsorted(O["local2global"], present)
    lib_rows = np.searchsorted(l2g, present)
    is_small = ~np.isin(present, heavy)
    o_small, lib_small = o_rows[is_small], lib_rows[is_small]
    return dict(B=B, torch=torch, wl=wl, P=P, O=O, S=S, heavy=heavy, l2g=l2g, lib_of_o=lib_of_o, present=present,
                o_rows=o_rows, lib_rows=lib_rows, o_small=o_small, lib_small=lib_small)


def test_cfg3_sampled_structures_bit_exact_at_full_size(cfg3):
    B, P, O, l2g = cfg3["B"], cfg3["P"], cfg3["O"], cfg3["l2g"]
    assert P.num_nodes == len(l2g) and np.all(np.diff(l2g) > 0)
    absent = cfg3["S"][~np.isin(cfg3["S"], O["local2global"])]
    pos = np.minimum(np.searchsorted(l2g, absent), len(l2g) - 1)
    assert not np.any(l2g[pos] == absent), "a node without an edge in the partition was duplicated into it"
    assert len(cfg3["present"]) > N_SAMPLED // 8 and np.all(np.isin(cfg3["heavy"], cfg3["present"]))
    rowptr, col = P.host_array(B.ARR_ROWPTR), P.host_array(B.ARR_COL)
    deg_l, deg_g = P.host_array(B.ARR_DEG_LOCAL), P.host_array(B.ARR_DEG_GLOBAL)
    dar = P.host_array(B.ARR_DAR_WEIGHT)
    longest = 0
    for o, i in zip(cfg3["o_rows"], cfg3["lib_rows"]):
        want = O["local2global"][O["col"][O["rowptr"][o]:O["rowptr"][o + 1]]]
        got = l2g[col[rowptr[i]:rowptr[i + 1]]]
        assert np.array_equal(got, want), f"neighbours of node {l2g[i]}"
        assert deg_l[i] == O["deg_local"][o] == len(want) and deg_g[i] == O["deg_global"][o]
        assert dar[i] == O["dar_weight"][o] and dar.dtype == O["dar_weight"].dtype
        longest = max(longest, len(want))
    progress(f"cfg3 full size: longest sampled row {longest}, longest row of the partition {int(deg_l.max())}")
    assert longest >= 1024, "the heaviest nodes are meant to have rows far longer than a wavefront's batch of ids"
    # neighbours of the small sampled nodes: their degrees are complete in the oracle's partition as well
    nbr = np.unique(np.concatenate([O["col"][O["rowptr"][o]:O["rowptr"][o + 1]] for o in cfg3["o_small"]]))
    assert np.array_equal(deg_l[cfg3["lib_of_o"][nbr]], O["deg_local"][nbr])
    assert np.array_equal(deg_g[cfg3["lib_of_o"][nbr]], O["deg_global"][nbr])


@pytest.mark.parametrize("width", [128, 256])
def test_cfg3_aggregation_sampled_rows_at_full_size(cfg3, width):
    """bf16 aggregation over all 28M rows (7.2e9 elements at 256 columns); the sampled rows against the oracle's
    functions on the sampled neighbourhood: all three modes on the small nodes, the plain mean on the heavy nodes' rows as well."""
    B, P, O, torch = cfg3["B"], cfg3["P"], cfg3["O"], cfg3["torch"]
    n = P.num_nodes
    gen = torch.Generator(device="cuda").manual_seed(width)
    X = torch.randn((n, width), device="cuda", generator=gen, dtype=torch.float32).to(torch.bfloat16)
    Y = torch.empty_like(X)
    g = o_dropedge.full_graph(O)
    Xo = from_bf16(X[torch.from_numpy(cfg3["lib_of_o"]).cuda()])
    for mode, ref_fn, rows_o, rows_lib in [
            (B.AGG_MEAN, o_layers.mean_aggregate, cfg3["o_rows"], cfg3["lib_rows"]),
            (B.AGG_MEAN_T, o_layers.mean_aggregate_bwd, cfg3["o_small"], cfg3["lib_small"]),
            (B.AGG_GCN, o_layers.gcn_aggregate, cfg3["o_small"], cfg3["lib_small"])]:
        progress(f"cfg3 full size: aggregate width {width} mode {mode}")
        Y.fill_(float("nan"))
        B.aggregate(P, None, 0, mode, X, Y, width, B.BF16)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(Y[-1]).all()) and bool(torch.isfinite(Y[n // 2]).all())
        got = from_bf16(Y[torch.from_numpy(rows_lib).cuda()])
        assert_close(got, ref_fn(g, Xo)[rows_o], 5e-3, f"aggregate width {width} mode {mode}")
    del X, Y
    torch.cuda.empty_cache()


def test_cfg3_gcn_layer_sampled_rows_at_full_size(cfg3):
    """The first layer of cfg3's model shape (GCN, 128 -> 256, ReLU, bf16) over the whole partition; sampled rows
    against the oracle's layer on the sampled neighbourhood."""
    B, P, O, torch = cfg3["B"], cfg3["P"], cfg3["O"], cfg3["torch"]
    n, d_in, d_out = P.num_nodes, 128, 256
    gen = torch.Generator(device="cuda").manual_seed(17)
    H = torch.randn((n, d_in), device="cuda", generator=gen).to(torch.bfloat16)
    W = (torch.randn((d_out, d_in), device="cuda", generator=gen) * 0.1).contiguous()
    b = (torch.randn((d_out,), device="cuda", generator=gen) * 0.1).contiguous()
    desc = B.layer_desc(B.GCN, d_in, 0, d_out, act=1, dtype=B.BF16)
    out = torch.full((n, d_out), float("nan"), device="cuda", dtype=torch.bfloat16)
    saved = {"A": torch.empty((n, d_in), device="cuda", dtype=torch.bfloat16)}
    ws = torch.empty(max(B.layer_workspace_bytes(desc, n, False), 256), dtype=torch.uint8, device="cuda")
    progress("cfg3 full size: GCN layer 128 -> 256")
    B.layer_fwd(P, None, 0, desc, H, {"W": W, "bW": b}, out, saved, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out[-1]).all())
    prm = {"W": W.cpu().numpy().astype(np.float64), "bW": b.cpu().numpy().astype(np.float64)}
    Ho = from_bf16(H[torch.from_numpy(cfg3["lib_of_o"]).cuda()])
    ref, _ = o_layers.gcn_fwd(o_dropedge.full_graph(O), Ho, prm, relu=True)
    got = from_bf16(out[torch.from_numpy(cfg3["lib_small"]).cuda()])
    assert_close(got, ref[cfg3["o_small"]], TOL_BF16, "GCN layer 128 -> 256, sampled rows")
    del H, out, saved, ws
    torch.cuda.empty_cache()


def test_cfg3_loss_at_full_size(cfg3):
    """Weighted softmax loss over 28M x 172 bf16 logits (4.8e9 elements).  The training mask selects the first and
    last 150k nodes, a run in the middle and one node in 200 elsewhere: the loss and the selected nodes' gradients
    against the oracle on exactly those nodes, the gradient of every other node zero."""
    B, P, torch = cfg3["B"], cfg3["P"], cfg3["torch"]
    n, C, c = P.num_nodes, 172, 1.0 / 110_000_000
    gen = torch.Generator(device="cuda").manual_seed(5)
    z = (3.0 * torch.randn((n, C), device="cuda", generator=gen)).to(torch.bfloat16)
    y = torch.randint(0, C, (n,), device="cuda", generator=gen, dtype=torch.int32)
    w = torch.rand((n,), device="cuda", generator=gen, dtype=torch.float32)
    mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
    mask[:150_000] = 1
    mask[n - 150_000:] = 1
    mask[n // 2:n // 2 + 150_000] = 1
    mask[torch.arange(7, n, 200, device="cuda")] = 1
    dz = torch.full((n, C), float("nan"), device="cuda", dtype=torch.bfloat16)
    loss = torch.zeros(1, device="cuda")
    ws = torch.empty(B.loss_workspace_bytes(), dtype=torch.uint8, device="cuda")
    progress("cfg3 full size: loss")
    B.loss_weighted(P, B.W_CUSTOM, w, z, y, mask, C, c, loss, dz, ws, B.BF16)
    torch.cuda.synchronize()
    sel = torch.nonzero(mask).flatten()
    L_ref, g_ref = o_loss.weighted_softmax_ce(from_bf16(z[sel]), y[sel].cpu().numpy(), w[sel].cpu().numpy().astype(np.float64), c)
    assert abs(loss.item() - L_ref) <= 1e-4 * abs(L_ref)
    assert_close(from_bf16(dz[sel]), g_ref, 5e-3, "dlogits of the selected nodes")
    # everything else: exactly zero (checked in pieces to keep temporaries small)
    off = mask == 0
    for a in range(0, n, 4_000_000):
        piece = dz[a:a + 4_000_000][off[a:a + 4_000_000]]
        assert bool((piece == 0).all()), f"non-zero gradient of an unselected node in rows {a}.."
