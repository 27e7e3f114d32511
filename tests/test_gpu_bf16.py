"""GPU parity of the bfloat16-storage path (features / activations in bf16, float32 accumulation and
parameters) against the float64 oracle evaluated on the bf16-rounded inputs; tolerance 2e-2."""
import numpy as np
import pytest

from oracle import dropedge as o_dropedge
from oracle import epoch as o_epoch
from oracle import layers as o_layers
from oracle import loss as o_loss
from oracle import partition as o_partition
from paper_2308_03209_amd import inputs
from gate_slack import sampled_flip_slack
from util import TOL_BF16, assert_close, to_f64_model

BF16_UNIT = 2.0 ** -9 / np.sqrt(3.0)   # rms relative error of rounding to 8 significant bits (uniform in +-2^-9)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import model as M
    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    P = B.build_partition(wl.n_nodes, src, dst, 4, 0, inputs.SEED_CUT)
    O = o_partition.build_partition(wl.n_nodes, src, dst, 4, 0, inputs.SEED_CUT)
    Mk = B.dropedge_k(P, 2, 0.5, inputs.SEED_MASKS)
    keep = o_dropedge.masks(O["n_edges"], 2, 0.5, inputs.SEED_MASKS)
    return dict(B=B, M=M, torch=torch, P=P, O=O, masks=Mk, keep=keep)


def to_bf16(torch, x):
    """float32 numpy -> (bf16 cuda tensor, the exactly representable values as float64 numpy)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.cuda(), t.float().numpy().astype(np.float64)


def from_bf16(t):
    return t.float().cpu().numpy().astype(np.float64)


# A ReLU gate is a decision taken on a floating point value.  An evaluation from bf16-rounded operands
# (relative precision 2^-9) takes the other branch on a fraction of a percent of the elements whose
# float64 pre-activation is close to zero; the forward value is unaffected (ReLU is continuous) but the
# gradient through such an element is not, and a few dozen flipped gates move a weight gradient by
# several percent.  Both outcomes are valid, so gradients are compared with the gates held equal: the
# backward pass on the GPU runs on the forward state (messages, means, layer outputs) the ORACLE computed,
# rounded to bf16.  Forward parity is checked separately on the GPU's own forward pass.


def oracle_layer_states(kind, om, graph, X64, q, seed, epoch):
    """Layer by layer forward with the oracle: list of (layer output, saved dict)."""
    n_layers = len(om["layers"])
    H, states = X64, []
    for l, prm in enumerate(om["layers"]):
        last = l == n_layers - 1
        drop = None if (last or q <= 0.0) else (q, seed, epoch, l)
        if kind == "sage":
            H, sv = o_layers.sage_fwd(graph, H, prm, drop)
        elif kind == "sage_conv":
            H, sv = o_layers.sage_conv_fwd(graph, H, prm, relu=not last, drop=drop)
        else:
            H, sv = o_layers.gcn_fwd(graph, H, prm, relu=not last, drop=drop)
        states.append((H, sv))
    return states


def force_forward_state(run, kind, states, torch):
    """Overwrite the runner's forward buffers with the oracle's forward state (rounded to the storage type)."""
    for l, (out, sv) in enumerate(states):
        run.H[l + 1].copy_(torch.from_numpy(out).to(run.H[l + 1].dtype))
        if kind == "sage":
            run.saved[l]["Z"].copy_(torch.from_numpy(sv["Z"]).to(run.saved[l]["Z"].dtype))
            run.saved[l]["A"].copy_(torch.from_numpy(sv["A"]).to(run.saved[l]["A"].dtype))
        elif "A" in run.saved[l]:
            agg = sv["M"] if kind == "sage_conv" else sv["AH"]
            run.saved[l]["A"].copy_(torch.from_numpy(agg).to(run.saved[l]["A"].dtype))


@pytest.mark.parametrize("width", [1, 7, 8, 47, 64, 100, 128, 172, 256, 264, 512, 1032])
@pytest.mark.parametrize("launch", ["0", "1", "8"])
def test_aggregate_bf16(G, width, launch, monkeypatch):
    B, torch, P, O = G["B"], G["torch"], G["P"], G["O"]
    print(f"[case] bf16 aggregate width={width} launch={launch}", flush=True)
    monkeypatch.setenv("COFREE_AGG_SLICES", launch)
    g = o_dropedge.masked_graph(O, G["keep"][1])
    n = O["n_nodes"]
    Xd, X64 = to_bf16(torch, np.random.default_rng(width).standard_normal((n, width)))
    Yd = torch.full((n, width), float("nan"), device="cuda", dtype=torch.bfloat16)
    for mode, ref_fn in [(B.AGG_MEAN, o_layers.mean_aggregate), (B.AGG_MEAN_T, o_layers.mean_aggregate_bwd),
                         (B.AGG_GCN, o_layers.gcn_aggregate)]:
        Yd.fill_(float("nan"))
        B.aggregate(P, G["masks"], 1, mode, Xd, Yd, width, B.BF16)
        torch.cuda.synchronize()
        # one rounding of the float32 sum to bf16: 2^-9 relative per element
        assert_close(from_bf16(Yd), ref_fn(g, X64), 5e-3, f"bf16 mode {mode} width {width}")


def rne_bf16_bits(x64):
    """float64 values (exactly representable in float32) -> bf16 bit patterns, round-to-nearest-even."""
    u = np.asarray(x64, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


@pytest.mark.parametrize("width", [8, 27])
def test_bf16_store_rounds_to_nearest_even(G, width):
    """On a cycle every mean is (x_a + x_b) / 2, exact in float32 for bf16 inputs of similar magnitude and
    a rounding tie in about half of the cases: the stored bf16 must be the RNE rounding, bit for bit."""
    B, torch = G["B"], G["torch"]
    n = 1000
    src = np.arange(n, dtype=np.int64)
    dst = (src + 1) % n
    P = B.build_partition(n, src, dst, 1, 0, 5)
    O = o_partition.build_partition(n, src, dst, 1, 0, 5)
    assert O["n_nodes"] == n and np.all(O["deg_local"] == 2)
    rng = np.random.default_rng(width)
    X = rng.uniform(1.0, 4.0, (n, width)) * rng.choice([-1.0, 1.0], (n, width))
    Xd, X64 = to_bf16(torch, X)
    Yd = torch.full((n, width), float("nan"), device="cuda", dtype=torch.bfloat16)
    B.aggregate(P, None, -1, B.AGG_MEAN, Xd, Yd, width, B.BF16)
    torch.cuda.synchronize()
    exact = o_layers.mean_aggregate(o_dropedge.full_graph(O), X64)      # float64, exact here
    assert np.array_equal(exact.astype(np.float32).astype(np.float64), exact)
    got = Yd.view(torch.int16).cpu().numpy().view(np.uint16)
    want = rne_bf16_bits(exact)
    ties = np.count_nonzero((exact.astype(np.float32).view(np.uint32) & 0xFFFF) == 0x8000)
    assert ties > 100, "the test is meant to contain rounding ties"
    assert np.array_equal(got, want)


@pytest.mark.parametrize("C", [1, 2, 7, 8, 9, 41, 47, 64, 65, 128, 129, 172, 256, 257, 300, 512, 513])
def test_loss_bf16(G, C):
    B, torch, P, O = G["B"], G["torch"], G["P"], G["O"]
    n = O["n_nodes"]
    rng = np.random.default_rng(C)
    zd, z64 = to_bf16(torch, 3 * rng.standard_normal((n, C)))
    y = rng.integers(0, C, n).astype(np.int32)
    dz = torch.empty_like(zd)
    loss = torch.zeros(1, device="cuda")
    ws = torch.empty(B.loss_workspace_bytes(), dtype=torch.uint8, device="cuda")
    B.loss_weighted(P, B.W_DAR, None, zd, torch.from_numpy(y).cuda(), None, C, 0.37, loss, dz, ws, B.BF16)
    torch.cuda.synchronize()
    L_ref, g_ref = o_loss.weighted_softmax_ce(z64, y, O["dar_weight"], 0.37)
    assert abs(loss.item() - L_ref) <= 1e-4 * abs(L_ref)        # float32 arithmetic on exact inputs
    assert_close(from_bf16(dz), g_ref, 5e-3, "bf16 dlogits")


@pytest.mark.parametrize("kind", ["sage", "gcn", "sage_conv"])
@pytest.mark.parametrize("dims", [(64, 16, 8), (20, 24, 40), (33, 7, 33), (100, 256, 256), (129, 5, 257), (128, 128, 136)])
def test_single_layer_bf16(G, kind, dims):
    check_single_layer_bf16(G, kind, dims)


@pytest.mark.parametrize("kind", ["sage", "gcn", "sage_conv"])
@pytest.mark.parametrize("dims", [(100, 256, 256), (129, 5, 257), (128, 128, 136), (300, 264, 520)])
def test_single_layer_bf16_large_tile(G, kind, dims, monkeypatch):
    """The same check with every product of more than 128 output columns sent through the 256x256 block tile
    (chosen by itself only for matrices of 131072 rows and more): ragged in rows, columns and k, two column
    tiles at 520."""
    monkeypatch.setenv("COFREE_BF16_TILE", "256")
    check_single_layer_bf16(G, kind, dims)


def check_single_layer_bf16(G, kind, dims):
    """One layer forward + backward in bf16 storage, with dropout and a DropEdge mask."""
    B, torch, P, O, masks = G["B"], G["torch"], G["P"], G["O"], G["masks"]
    d_in, d_msg, d_out = dims
    print(f"[case] bf16 layer kind={kind} dims={dims}", flush=True)
    g = o_dropedge.masked_graph(O, G["keep"][0])
    n = O["n_nodes"]
    rng = np.random.default_rng(d_in)
    q = 0.25
    prm = inputs.model_params(kind, [dims], seed=d_in, random_bias=True)[0]
    Hd, H64 = to_bf16(torch, rng.standard_normal((n, d_in)))
    dOd, dO64 = to_bf16(torch, rng.standard_normal((n, d_out)))
    code = {"sage": B.SAGE_MEAN, "gcn": B.GCN, "sage_conv": B.SAGE_CONV}[kind]
    desc = B.layer_desc(code, d_in, d_msg, d_out, act=1, dropout_q=q, layer_id=1, seed=5, epoch=2, dtype=B.BF16)
    prm_d = {k: torch.from_numpy(v).cuda() for k, v in prm.items()}
    grads_d = {k: torch.full_like(v, float("nan")) for k, v in prm_d.items()}
    bf = dict(device="cuda", dtype=torch.bfloat16)
    out_d = torch.empty((n, d_out), **bf)
    dH_d = torch.empty((n, d_in), **bf)
    saved = {"Z": torch.empty((n, max(d_msg, 1)), **bf), "A": torch.empty((n, max(d_msg, d_in)), **bf)}
    ws = torch.empty(max(B.layer_workspace_bytes(desc, n, False), B.layer_workspace_bytes(desc, n, True)),
                     dtype=torch.uint8, device="cuda")
    B.layer_fwd(P, masks, 0, desc, Hd, prm_d, out_d, saved, ws)
    torch.cuda.synchronize()
    p64 = {k: v.astype(np.float64) for k, v in prm.items()}
    drop = (q, 5, 2, 1)
    if kind == "sage":
        ref_out, sv = o_layers.sage_fwd(g, H64, p64, drop)
        ref_dH, ref_g = o_layers.sage_bwd(g, p64, sv, dO64)
    elif kind == "sage_conv":
        ref_out, sv = o_layers.sage_conv_fwd(g, H64, p64, True, drop)
        ref_dH, ref_g = o_layers.sage_conv_bwd(g, p64, sv, dO64)
    else:
        ref_out, sv = o_layers.gcn_fwd(g, H64, p64, True, drop)
        ref_dH, ref_g = o_layers.gcn_bwd(g, p64, sv, dO64)
    assert_close(from_bf16(out_d), ref_out, TOL_BF16, "H_out")
    if kind == "sage":
        assert_close(from_bf16(saved["Z"][:, :d_msg].contiguous()) if saved["Z"].shape[1] != d_msg else from_bf16(saved["Z"]),
                     sv["Z"], TOL_BF16, "Z")
    # backward with the gates held equal: forward state from the oracle
    bf16 = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).cuda()
    out_f = bf16(ref_out)
    if kind == "sage":
        saved_f = {"Z": bf16(sv["Z"]), "A": bf16(sv["A"])}
    elif kind == "sage_conv":
        saved_f = {"Z": saved["Z"], "A": bf16(sv["M"])}
    else:
        saved_f = {"Z": saved["Z"], "A": bf16(sv["AH"])}
    B.layer_bwd(P, masks, 0, desc, Hd, out_f, prm_d, saved_f, dOd, dH_d, grads_d, False, ws)
    torch.cuda.synchronize()
    assert_close(from_bf16(dH_d), ref_dH, TOL_BF16, "dH_in")
    for name in ref_g:
        assert_close(grads_d[name].cpu().numpy(), ref_g[name], TOL_BF16, f"d{name}")
    if kind == "sage":
        return
    # the neighbouring layers' ReLU backward carried by this call (grad_flags)
    flagged = B.layer_desc(code, d_in, d_msg, d_out, act=1, dropout_q=q, layer_id=1, seed=5, epoch=2, dtype=B.BF16,
                           grad_flags=B.GRAD_IN_GATED | B.GRAD_OUT_GATED, dropout_q_below=0.2)
    dO_gated, dOg64 = to_bf16(torch, dO64 * (ref_out > 0) / (1.0 - q))
    dH_d.fill_(float("nan"))
    B.layer_bwd(P, masks, 0, flagged, Hd, out_f, prm_d, saved_f, dO_gated, dH_d, grads_d, False, ws)
    torch.cuda.synchronize()
    assert_close(from_bf16(dH_d), ref_dH * (H64 > 0) * 1.25, TOL_BF16, "gated dH_in")
    for name in ref_g:
        assert_close(grads_d[name].cpu().numpy(), ref_g[name], TOL_BF16, f"d{name} from a gated dH_out")


def run_bf16_iteration(G, wl, kind, dims, p, part, K, q, epoch):
    B, M, torch = G["B"], G["M"], G["torch"]
    print(f"[case] bf16 iteration {wl.name} kind={kind} dims={dims} K={K} q={q}", flush=True)
    src, dst = inputs.workload_graph(wl)
    P = B.build_partition(wl.n_nodes, src, dst, p, part, inputs.SEED_CUT)
    O = o_partition.build_partition(wl.n_nodes, src, dst, p, part, inputs.SEED_CUT)
    masks, graph = None, o_dropedge.full_graph(O)
    ids = O["local2global"]
    Xd, X64 = to_bf16(torch, inputs.node_features(ids, dims[0][0]))
    y = inputs.node_labels(ids, dims[-1][2])
    layers = inputs.model_params(kind, dims, random_bias=True)
    model = M.Model(kind, dims)
    model.load(layers)
    if K:
        masks = B.dropedge_k(P, K, 0.5, inputs.SEED_MASKS)
    run = M.PartitionRunner(P, model, masks, dropout_q=q, dropout_seed=inputs.SEED_DROPOUT, dtype="bf16")
    c = 1.0 / wl.n_nodes
    yd = torch.from_numpy(y).cuda()
    k = run.iteration(Xd, yd, epoch, mask_seed=inputs.SEED_MASKS, scale_c=c)
    torch.cuda.synchronize()
    if K:
        keep = o_dropedge.masks(O["n_edges"], K, 0.5, inputs.SEED_MASKS)
        assert k == o_dropedge.pick(inputs.SEED_MASKS, epoch, K)
        graph = o_dropedge.masked_graph(O, keep[k])
    om = to_f64_model(kind, layers)
    states = oracle_layer_states(kind, om, graph, X64, q, inputs.SEED_DROPOUT, epoch)
    logits_ref = states[-1][0]
    L_ref, dlogits_ref = o_loss.weighted_softmax_ce(logits_ref, y, O["dar_weight"], c)
    G_ref = o_epoch.backward(om, graph, [sv for _, sv in states], dlogits_ref)
    # 1. the GPU's own forward pass and loss
    for l, (out, _) in enumerate(states):
        assert_close(from_bf16(run.H[l + 1]), out, TOL_BF16, f"layer {l} output")
    assert abs(run.loss.item() - L_ref) <= TOL_BF16 * abs(L_ref), (run.loss.item(), L_ref)
    # 2. end to end gradients of that pass.  Its gates are decided on pre-activations computed from operands
    #    rounded to bf16, so a fraction of a percent of them differ from the oracle's, legitimately.  The slack
    #    that allows is derived on the oracle's side: every gate flips with the probability its pre-activation
    #    and the rounding noise of its operands give it, flip patterns are drawn, and the oracle's backward
    #    pass is repeated with them (gate_slack.sampled_flip_slack).  Bar: 2e-2 plus twice the largest
    #    deviation seen over the draws, in the Frobenius norm, per gradient tensor.
    saved_ref = [sv for _, sv in states]
    slack, n_flips = sampled_flip_slack(om, graph, saved_ref, dlogits_ref, o_epoch.backward, BF16_UNIT)
    print(f"[case] expected gate flips under bf16 operand rounding: {n_flips:.0f}", flush=True)
    for l, (got, ref) in enumerate(zip(model.grads, G_ref)):
        for name in ref:
            nrm = np.linalg.norm(ref[name])
            e = np.linalg.norm(got[name].cpu().numpy() - ref[name])
            bar = TOL_BF16 * nrm + 2.0 * slack[l][name]
            print(f"[case] end-to-end layer {l} d{name}: Frobenius rel err {e / nrm:.3e}, bar {bar / nrm:.3e} "
                  f"(gate slack {slack[l][name] / nrm:.3e})", flush=True)
            assert e <= bar, f"end-to-end layer {l} d{name}: Frobenius rel err {e / nrm:.3e} > {bar / nrm:.3e}"
    # 3. backward with the gates held equal (forward state from the oracle): the stated tolerance
    force_forward_state(run, kind, states, torch)
    run.loss_backward(yd, B.W_DAR, c, k, epoch, False)
    torch.cuda.synchronize()
    for l, (got, ref) in enumerate(zip(model.grads, G_ref)):
        for name in ref:
            assert_close(got[name].cpu().numpy(), ref[name], TOL_BF16, f"layer {l} d{name}")


def test_cfg0_bf16_gcn_iteration(G):
    wl = inputs.WORKLOADS[0]
    run_bf16_iteration(G, wl, "gcn", wl.layer_dims(), 4, 0, K=0, q=0.0, epoch=0)


def test_cfg2_shape_scaled_sage3_bf16_dropedge(G):
    """cfg2's model (100 -> 256 -> 256 -> 47, d_msg 256, 3 layers, DropEdge-K K=4 p=0.5) on a 1/500 scale graph."""
    wl = inputs.WORKLOADS[2].scaled(0.002)
    run_bf16_iteration(G, wl, "sage", wl.layer_dims(), 8, 0, K=4, q=0.0, epoch=3)


def test_cfg2_shape_scaled_sage3_bf16_large_tile(G, monkeypatch):
    """The same iteration with the 256x256 block tile forced for the 256-column products."""
    monkeypatch.setenv("COFREE_BF16_TILE", "256")
    wl = inputs.WORKLOADS[2].scaled(0.002)
    run_bf16_iteration(G, wl, "sage", wl.layer_dims(), 8, 0, K=4, q=0.0, epoch=3)


def test_paper_depth_conventional_sage_bf16(G):
    """The experiments' ogbn-products model (3 layers, hidden 128; Appendix B) with conventional GraphSAGE-mean
    layers, on a 1/500 scale cfg2 graph."""
    wl = inputs.WORKLOADS[2].scaled(0.002)
    run_bf16_iteration(G, wl, "sage_conv", [(100, 0, 128), (128, 0, 128), (128, 0, 47)], 8, 0, K=4, q=0.3, epoch=4)


def test_cfg3_shape_scaled_gcn3_bf16(G):
    """cfg3's model (128 -> 256 -> 256 -> 172) on a tiny graph of the same recipe."""
    wl = inputs.WORKLOADS[3].scaled(0.00005)
    run_bf16_iteration(G, wl, "gcn", wl.layer_dims(), 16, 0, K=0, q=0.2, epoch=1)


def test_cfg2_at_one_twentieth_scale_sage3_bf16_dropedge(G):
    """cfg2's model and DropEdge-K setting on a 1/20 node-count copy of its graph (120k nodes, partition 0 of
    about 94k): the size at which the 256-column products are still on the 128x128 tile but every launch spans
    hundreds of workgroups.  Forward at 2e-2, gradients of the unforced pass at 2e-2 plus the sampled gate
    slack, gradients with the oracle's gates at 2e-2."""
    wl = inputs.WORKLOADS[2].scaled(0.05)
    run_bf16_iteration(G, wl, "sage", wl.layer_dims(), 8, 0, K=4, q=0.0, epoch=3)


def test_cfg3_at_one_hundredth_scale_through_the_streamed_builder(G):
    """cfg3's model (GCN-3, 128 -> 256 -> 256 -> 172, bf16) on a 1/100 node-count copy of its graph (1.1M nodes,
    8M undirected edges), built the way the full-size run builds it: the block-wise generator feeds the
    library's piece-wise partition builder.  Structures bit for bit against the oracle's piece-wise twin, then
    one iteration: forward at 2e-2 and the gradients with the oracle's gates at 2e-2."""
    from util import progress
    B, M, torch = G["B"], G["M"], G["torch"]
    wl = inputs.WORKLOADS[3].scaled(0.01)
    stream = inputs.workload_stream(wl, block_pairs=1 << 21)
    assert stream.n_blocks >= 3
    blocks = list(stream.blocks(workers=4))
    bld = B.PartitionBuilder(wl.n_nodes, wl.n_parts, 0, inputs.SEED_CUT)
    for s_, d_ in blocks:
        bld.add_edges(s_, d_)
    P = bld.finish()
    progress("cfg3 x0.01: oracle piece-wise build")
    O = o_partition.build_partition_chunked(wl.n_nodes, blocks, wl.n_parts, 0, inputs.SEED_CUT)
    for which, name in [(B.ARR_LOCAL2GLOBAL, "local2global"), (B.ARR_ROWPTR, "rowptr"), (B.ARR_COL, "col"),
                        (B.ARR_DEG_GLOBAL, "deg_global"), (B.ARR_DAR_WEIGHT, "dar_weight")]:
        assert np.array_equal(P.host_array(which), O[name]), name
    graph = o_dropedge.full_graph(O)
    kind, dims = "gcn", wl.layer_dims()
    ids = O["local2global"]
    Xd, X64 = to_bf16(torch, inputs.node_features(ids, dims[0][0], workers=4))
    y = inputs.node_labels(ids, dims[-1][2])
    layers = inputs.model_params(kind, dims, random_bias=True)
    model = M.Model(kind, dims)
    model.load(layers)
    run = M.PartitionRunner(P, model, None, dtype="bf16")
    c = 1.0 / wl.n_nodes
    yd = torch.from_numpy(y).cuda()
    run.iteration(Xd, yd, 0, scale_c=c)
    torch.cuda.synchronize()
    progress("cfg3 x0.01: oracle iteration")
    om = to_f64_model(kind, layers)
    states = oracle_layer_states(kind, om, graph, X64, 0.0, 0, 0)
    for l, (out, _) in enumerate(states):
        assert_close(from_bf16(run.H[l + 1]), out, TOL_BF16, f"layer {l} output")
    L_ref, dlogits_ref = o_loss.weighted_softmax_ce(states[-1][0], y, O["dar_weight"], c)
    assert abs(run.loss.item() - L_ref) <= TOL_BF16 * abs(L_ref)
    G_ref = o_epoch.backward(om, graph, [sv for _, sv in states], dlogits_ref)
    force_forward_state(run, kind, states, torch)
    run.loss_backward(yd, B.W_DAR, c, 0, 0, False)
    torch.cuda.synchronize()
    for l, (got, ref) in enumerate(zip(model.grads, G_ref)):
        for name in ref:
            assert_close(got[name].cpu().numpy(), ref[name], TOL_BF16, f"layer {l} d{name}")
