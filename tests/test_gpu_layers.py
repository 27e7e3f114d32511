"""GPU parity of whole layers and whole training iterations against the oracle."""
import numpy as np
import pytest

from oracle import dropedge as o_dropedge
from oracle import epoch as o_epoch
from oracle import layers as o_layers
from oracle import loss as o_loss
from oracle import partition as o_partition
from oracle import step as o_step
from paper_2308_03209_amd import inputs
from util import assert_close, to_f64_model

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import model as M
    return dict(B=B, M=M, torch=torch)


def setup_partition(G, wl, p, part, K=0, p_drop=0.5):
    B = G["B"]
    src, dst = inputs.workload_graph(wl)
    P = B.build_partition(wl.n_nodes, src, dst, p, part, inputs.SEED_CUT)
    O = o_partition.build_partition(wl.n_nodes, src, dst, p, part, inputs.SEED_CUT)
    masks, keep = None, None
    if K:
        masks = B.dropedge_k(P, K, p_drop, inputs.SEED_MASKS)
        keep = o_dropedge.masks(O["n_edges"], K, p_drop, inputs.SEED_MASKS)
    return P, O, masks, keep


def oracle_graph(O, keep, k):
    return o_dropedge.masked_graph(O, keep[k]) if keep is not None else o_dropedge.full_graph(O)


GATE_MARGIN = 1e-5   # relative to the rms of a layer's pre-activations


def oracle_with_gate_slack(om, graph, X, y, w, c, q, seed, epoch):
    """Oracle loss / logits / gradients plus, per gradient tensor, an elementwise slack.

    A ReLU gate is a decision taken on a floating point value.  Where the oracle's float64
    pre-activation lies within float32 rounding distance of zero (|pre| < GATE_MARGIN * rms), a
    float32 evaluation may legitimately take the other branch: the forward value is unaffected
    (the activation is continuous) but the gradient that passes through that element is not.
    Both outcomes are valid, so for every such element the oracle's backward pass is repeated
    with that one gate flipped, and the absolute change of every gradient entry is added to the
    slack the comparison allows.  With no such element the slack is zero.
    """
    logits, saved = o_epoch.forward(om, graph, X, q, seed, epoch)
    L, dlogits = o_loss.weighted_softmax_ce(logits, y, w, c)
    G = o_epoch.backward(om, graph, saved, dlogits)
    slack = [{k: np.zeros_like(v) for k, v in g.items()} for g in G]
    n_amb = 0
    for l, sv in enumerate(saved):
        if not sv.get("relu", True):
            continue
        pre = sv["pre"]
        amb = np.argwhere(np.abs(pre) < GATE_MARGIN * np.sqrt((pre * pre).mean()))
        assert len(amb) <= 64, "too many near-zero pre-activations for the flip analysis"
        for (u, ch) in amb:
            n_amb += 1
            pre[u, ch] = -pre[u, ch]
            Gf = o_epoch.backward(om, graph, saved, dlogits)
            pre[u, ch] = -pre[u, ch]
            for sl, g0, g1 in zip(slack, G, Gf):
                for k in sl:
                    sl[k] += np.abs(g1[k] - g0[k])
    return L, G, logits, slack, n_amb


def assert_close_slack(got, ref, slack, tol, what):
    got = np.asarray(got, dtype=np.float64)
    assert np.all(np.isfinite(got)), f"{what}: non-finite"
    excess = np.maximum(np.abs(got - ref) - slack, 0.0)
    e_max = excess.max() / max(np.abs(ref).max(), 1e-30)
    e_fro = np.sqrt((excess * excess).sum()) / max(np.sqrt((ref * ref).sum()), 1e-30)
    assert e_max <= tol and e_fro <= tol, f"{what}: rel err max {e_max:.3e} fro {e_fro:.3e} > {tol}"


def run_iteration_parity(G, wl, kind, dims, p, part, K, q, epoch, tol=1e-4, fuse_gates=True):
    B, M, torch = G["B"], G["M"], G["torch"]
    print(f"[case] iteration {wl.name} kind={kind} dims={dims} p={p} part={part} K={K} q={q}", flush=True)
    P, O, masks, keep = setup_partition(G, wl, p, part, K)
    ids = O["local2global"]
    X = inputs.node_features(ids, dims[0][0])
    y = inputs.node_labels(ids, dims[-1][2])
    layers = inputs.model_params(kind, dims, random_bias=True)
    model = M.Model(kind, dims)
    model.load(layers)
    run = M.PartitionRunner(P, model, masks, dropout_q=q, dropout_seed=inputs.SEED_DROPOUT, fuse_gates=fuse_gates)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    c = 1.0 / wl.n_nodes
    k = run.iteration(Xd, yd, epoch, mask_seed=inputs.SEED_MASKS, scale_c=c)
    torch.cuda.synchronize()
    if K:
        assert k == o_dropedge.pick(inputs.SEED_MASKS, epoch, K)
    g = oracle_graph(O, keep, k)
    om = to_f64_model(kind, layers)
    L_ref, G_ref, logits_ref, slack, n_amb = oracle_with_gate_slack(om, g, X.astype(np.float64), y, O["dar_weight"],
                                                                    c, q, inputs.SEED_DROPOUT, epoch)
    print(f"[case] near-zero ReLU pre-activations analysed: {n_amb}", flush=True)
    assert_close(run.H[-1].cpu().numpy(), logits_ref, tol, "logits")
    assert abs(run.loss.item() - L_ref) <= tol * abs(L_ref), (run.loss.item(), L_ref)
    for l, (got, ref) in enumerate(zip(model.grads, G_ref)):
        for name in ref:
            assert_close_slack(got[name].cpu().numpy(), ref[name], slack[l][name], tol, f"layer {l} d{name}")
    return model, run, om, G_ref


@pytest.mark.parametrize("kind", ["sage", "gcn", "sage_conv"])
@pytest.mark.parametrize("q", [0.0, 0.3])
def test_single_layer_forward_backward(G, kind, q):
    """One layer in isolation, including the gradient w.r.t. its input."""
    B, torch = G["B"], G["torch"]
    wl = inputs.WORKLOADS[0]
    P, O, masks, keep = setup_partition(G, wl, 4, 1, K=2)
    g = oracle_graph(O, keep, 1)
    n = O["n_nodes"]
    rng = np.random.default_rng(3)
    for (d_in, d_msg, d_out) in [(64, 16, 8), (20, 24, 40), (33, 7, 33), (3, 2, 130), (130, 3, 1), (131, 129, 5),
                                  (128, 128, 136)]:   # last: both dP-sided weight gradients in one launch
        print(f"[case] layer kind={kind} q={q} dims={(d_in, d_msg, d_out)}", flush=True)
        prm = inputs.model_params(kind, [(d_in, d_msg, d_out)], seed=d_in, random_bias=True)[0]
        H = rng.standard_normal((n, d_in)).astype(np.float32)
        dOut = rng.standard_normal((n, d_out)).astype(np.float32)
        code = {"sage": B.SAGE_MEAN, "gcn": B.GCN, "sage_conv": B.SAGE_CONV}[kind]
        desc = B.layer_desc(code, d_in, d_msg, d_out, act=1, dropout_q=q, layer_id=2, seed=77, epoch=5)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        prm_d = {k: dev(v) for k, v in prm.items()}
        grads_d = {k: torch.full_like(v, float("nan")) for k, v in prm_d.items()}
        Hd, dOd = dev(H), dev(dOut)
        out_d = torch.empty((n, d_out), device="cuda")
        dH_d = torch.empty((n, d_in), device="cuda")
        saved = {"Z": torch.empty((n, max(d_msg, 1)), device="cuda"), "A": torch.empty((n, max(d_msg, d_in)), device="cuda")}
        ws = torch.empty(max(B.layer_workspace_bytes(desc, n, False), B.layer_workspace_bytes(desc, n, True)),
                         dtype=torch.uint8, device="cuda")
        B.layer_fwd(P, masks, 1, desc, Hd, prm_d, out_d, saved, ws)
        B.layer_bwd(P, masks, 1, desc, Hd, out_d, prm_d, saved, dOd, dH_d, grads_d, False, ws)
        torch.cuda.synchronize()
        p64 = {k: v.astype(np.float64) for k, v in prm.items()}
        drop = (q, 77, 5, 2) if q > 0 else None
        if kind == "sage":
            ref_out, sv = o_layers.sage_fwd(g, H, p64, drop)
            ref_dH, ref_g = o_layers.sage_bwd(g, p64, sv, dOut)
        elif kind == "sage_conv":
            ref_out, sv = o_layers.sage_conv_fwd(g, H, p64, True, drop)
            ref_dH, ref_g = o_layers.sage_conv_bwd(g, p64, sv, dOut)
        else:
            ref_out, sv = o_layers.gcn_fwd(g, H, p64, True, drop)
            ref_dH, ref_g = o_layers.gcn_bwd(g, p64, sv, dOut)
        assert_close(out_d.cpu().numpy(), ref_out, what="H_out")
        assert_close(dH_d.cpu().numpy(), ref_dH, what="dH_in")
        for name in ref_g:
            assert_close(grads_d[name].cpu().numpy(), ref_g[name], what=f"d{name}")
        # accumulate = 1 adds to what is there
        B.layer_bwd(P, masks, 1, desc, Hd, out_d, prm_d, saved, dOd, dH_d, grads_d, True, ws)
        torch.cuda.synchronize()
        for name in ref_g:
            assert_close(grads_d[name].cpu().numpy(), 2 * ref_g[name], what=f"accumulated d{name}")
        if kind == "sage":
            continue
        # ReLU backward of neighbouring layers carried by this call: the input gradient comes out gated by
        # [H_in > 0]; an output gradient that arrives gated by [H_out > 0] gives the same parameter gradients
        flagged = B.layer_desc(code, d_in, d_msg, d_out, act=1, dropout_q=q, layer_id=2, seed=77, epoch=5,
                               grad_flags=B.GRAD_IN_GATED | B.GRAD_OUT_GATED, dropout_q_below=0.2)
        dO_gated = dev((dOut * (out_d.cpu().numpy() > 0) / (1.0 - q)).astype(np.float32))
        dH_d.fill_(float("nan"))
        B.layer_bwd(P, masks, 1, flagged, Hd, out_d, prm_d, saved, dO_gated, dH_d, grads_d, False, ws)
        torch.cuda.synchronize()
        assert_close(dH_d.cpu().numpy(), ref_dH * (H > 0) * 1.25, what="gated dH_in")
        for name in ref_g:
            assert_close(grads_d[name].cpu().numpy(), ref_g[name], what=f"d{name} from a gated dH_out")


@pytest.mark.parametrize("kind,dims", [("gcn", [(40, 0, 72), (72, 0, 24), (24, 0, 6)]),
                                       ("sage", [(40, 48, 32), (32, 48, 6)]),
                                       ("sage_conv", [(40, 0, 72), (72, 0, 6)])])
def test_iteration_on_a_graph_with_hub_rows(G, kind, dims):
    """Whole iterations on a graph with planted hub rows (12000, 6100 and 4200 neighbours among 20k nodes), so that
    every fused epilogue of the aggregation - bias + ReLU, the ReLU gate of the messages, the gate and scale of
    the layer below - also runs in the hub launch.  DropEdge-K on, dropout on."""
    B, M, torch = G["B"], G["M"], G["torch"]
    n = 20_000
    print(f"[case] hub-row iteration kind={kind} dims={dims}", flush=True)
    src, dst = inputs.hub_graph(n, [12000, 6100, 4200], 40_000, 6)
    P = B.build_partition(n, src, dst, 1, 0, inputs.SEED_CUT)
    O = o_partition.build_partition(n, src, dst, 1, 0, inputs.SEED_CUT)
    assert (O["deg_local"] >= 4096).sum() == 3
    K, q, epoch = 2, 0.2, 3
    masks = B.dropedge_k(P, K, 0.3, inputs.SEED_MASKS)
    keep = o_dropedge.masks(O["n_edges"], K, 0.3, inputs.SEED_MASKS)
    ids = O["local2global"]
    X = inputs.node_features(ids, dims[0][0])
    y = inputs.node_labels(ids, dims[-1][2])
    layers = inputs.model_params(kind, dims, random_bias=True)
    model = M.Model(kind, dims)
    model.load(layers)
    run = M.PartitionRunner(P, model, masks, dropout_q=q, dropout_seed=inputs.SEED_DROPOUT)
    c = 1.0 / n
    k = run.iteration(torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), epoch, mask_seed=inputs.SEED_MASKS,
                      scale_c=c)
    torch.cuda.synchronize()
    assert k == o_dropedge.pick(inputs.SEED_MASKS, epoch, K)
    g = o_dropedge.masked_graph(O, keep[k])
    assert g[2].max() >= 4096 and (g[2] >= 4096).sum() < 3, "the mask must leave some hub rows and remove others"
    om = to_f64_model(kind, layers)
    L_ref, G_ref, logits_ref, slack, n_amb = oracle_with_gate_slack(om, g, X.astype(np.float64), y, O["dar_weight"],
                                                                    c, q, inputs.SEED_DROPOUT, epoch)
    assert_close(run.H[-1].cpu().numpy(), logits_ref, 1e-4, "logits")
    assert abs(run.loss.item() - L_ref) <= 1e-4 * abs(L_ref)
    for l, (got, ref) in enumerate(zip(model.grads, G_ref)):
        for name in ref:
            assert_close_slack(got[name].cpu().numpy(), ref[name], slack[l][name], 1e-4, f"layer {l} d{name}")


def test_cfg0_gcn_iteration(G):
    wl = inputs.WORKLOADS[0]
    run_iteration_parity(G, wl, "gcn", wl.layer_dims(), 4, 0, K=0, q=0.0, epoch=0)


@pytest.mark.parametrize("kind", ["gcn", "sage_conv"])
def test_iteration_with_separate_relu_backward_passes(G, kind):
    """The same iteration with every layer's ReLU backward as its own pass (no grad_flags)."""
    wl = inputs.WORKLOADS[0]
    run_iteration_parity(G, wl, kind, [(64, 0, 48), (48, 0, 32), (32, 0, 8)], 4, 1, K=2, q=0.3, epoch=2,
                         fuse_gates=False)


def test_cfg0_gcn_iteration_dropedge_dropout(G):
    wl = inputs.WORKLOADS[0]
    run_iteration_parity(G, wl, "gcn", wl.layer_dims(), 4, 3, K=4, q=0.3, epoch=6)


def test_cfg0_graph_sage_iteration(G):
    wl = inputs.WORKLOADS[0]
    run_iteration_parity(G, wl, "sage", [(64, 16, 16), (16, 16, 16), (16, 16, 8)], 4, 1, K=4, q=0.2, epoch=3)


def test_cfg0_conventional_sage_iteration(G):
    """Conventional GraphSAGE-mean layers, one widening (aggregate first) and two narrowing (transform first)."""
    wl = inputs.WORKLOADS[0]
    run_iteration_parity(G, wl, "sage_conv", [(64, 0, 80), (80, 0, 24), (24, 0, 8)], 4, 2, K=4, q=0.2, epoch=5)


def test_paper_depth_conventional_sage_scaled(G):
    """The experiments' Reddit model (4 layers, hidden 256; Appendix B) on a 1/50 node-count cfg1 graph."""
    wl = inputs.WORKLOADS[1].scaled(0.02)
    dims = [(602, 0, 256), (256, 0, 256), (256, 0, 256), (256, 0, 41)]
    run_iteration_parity(G, wl, "sage_conv", dims, 8, 1, K=2, q=0.3, epoch=2)


def test_cfg1_shape_scaled_sage(G):
    """cfg1's model shape (602 -> 256 -> 41, d_msg 256) on a 1/50 node-count version of its graph."""
    wl = inputs.WORKLOADS[1].scaled(0.02)
    run_iteration_parity(G, wl, "sage", wl.layer_dims(), 8, 0, K=0, q=0.0, epoch=0)


def test_cfg4_shape_scaled_gcn_all_partitions_accumulated(G):
    """cfg4 in miniature: GCN-4 hidden 512, every partition run back to back, gradients summed (Eq. 2),
    DropEdge-K, one update."""
    B, M, torch = G["B"], G["M"], G["torch"]
    wl = inputs.WORKLOADS[4].scaled(0.0005)
    p, K = 4, 3
    dims = wl.layer_dims()
    layers = inputs.model_params("gcn", dims, random_bias=True)
    model = M.Model("gcn", dims)
    model.load(layers)
    om = to_f64_model("gcn", layers)
    src, dst = inputs.workload_graph(wl)
    c = 1.0 / wl.n_nodes
    refs, slacks = [], []
    epoch = 2
    for i in range(p):
        print(f"[case] cfg4-mini partition {i}", flush=True)
        P = B.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        O = o_partition.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        masks = B.dropedge_k(P, K, 0.5, inputs.SEED_MASKS + i)
        keep = o_dropedge.masks(O["n_edges"], K, 0.5, inputs.SEED_MASKS + i)
        ids = O["local2global"]
        X = inputs.node_features(ids, dims[0][0])
        y = inputs.node_labels(ids, dims[-1][2])
        run = M.PartitionRunner(P, model, masks)
        k = run.iteration(torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), epoch,
                          mask_seed=inputs.SEED_MASKS + i, scale_c=c, accumulate=i > 0)
        torch.cuda.synchronize()
        assert k == o_dropedge.pick(inputs.SEED_MASKS + i, epoch, K)
        _, g_i, _, slack_i, n_amb = oracle_with_gate_slack(om, o_dropedge.masked_graph(O, keep[k]),
                                                           X.astype(np.float64), y, O["dar_weight"], c, 0.0, 0, epoch)
        print(f"[case] near-zero ReLU pre-activations analysed: {n_amb}", flush=True)
        refs.append(g_i)
        slacks.append(slack_i)
    total = o_epoch.sum_grads(refs)
    slack = o_epoch.sum_grads(slacks)
    for l, (got, ref) in enumerate(zip(model.grads, total)):
        for name in ref:
            assert_close_slack(got[name].cpu().numpy(), ref[name], slack[l][name], 1e-4, f"summed layer {l} d{name}")
    theta0 = [{k: v.cpu().numpy().astype(np.float64) for k, v in lay.items()} for lay in model.params]
    model.step(B.SGD, lr=0.5)
    torch.cuda.synchronize()
    for l, (got, ref) in enumerate(zip(model.params, total)):
        for name in ref:
            assert_close(got[name].cpu().numpy(), o_step.sgd(theta0[l][name], ref[name], 0.5), tol=1e-5,
                         what=f"theta layer {l} {name}")


def test_cfg4_at_one_fiftieth_scale_all_eight_partitions_accumulated(G):
    """cfg4 with its own partition count, mask count and widths (GCN-4, hidden 512, 8-way cut, DropEdge-K K=8,
    every partition back to back, gradients summed as in Eq. 2) on a 1/50 node-count copy of its graph: 48k
    nodes, partitions of about 37k.  Every summed gradient against the sum of eight oracle runs; the ReLU-gate
    slack is the one-pass worst-case bound (thousands of pre-activations lie within float32 rounding of zero at
    this size, too many to flip one by one)."""
    from gate_slack import worst_case_slack
    from util import progress
    B, M, torch = G["B"], G["M"], G["torch"]
    wl = inputs.WORKLOADS[4].scaled(0.02)
    p, K = wl.n_parts, wl.dropedge_K
    assert (p, K, wl.hidden) == (8, 8, 512)
    dims = wl.layer_dims()
    layers = inputs.model_params("gcn", dims, random_bias=True)
    model = M.Model("gcn", dims)
    model.load(layers)
    om = to_f64_model("gcn", layers)
    src, dst = inputs.workload_graph(wl)
    c = 1.0 / wl.n_nodes
    refs, slacks = [], []
    epoch = 5
    pool = None
    for i in range(p):
        progress(f"cfg4 x0.02: partition {i}")
        P = B.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        O = o_partition.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        masks = B.dropedge_k(P, K, wl.dropedge_p, inputs.SEED_MASKS + i)
        keep = o_dropedge.masks(O["n_edges"], K, wl.dropedge_p, inputs.SEED_MASKS + i)
        ids = O["local2global"]
        X = inputs.node_features(ids, dims[0][0])
        y = inputs.node_labels(ids, dims[-1][2])
        run = M.PartitionRunner(P, model, masks)
        k = run.iteration(torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), epoch,
                          mask_seed=inputs.SEED_MASKS + i, scale_c=c, accumulate=i > 0)
        torch.cuda.synchronize()
        assert k == o_dropedge.pick(inputs.SEED_MASKS + i, epoch, K)
        g = o_dropedge.masked_graph(O, keep[k])
        logits, saved = o_epoch.forward(om, g, X.astype(np.float64))
        assert_close(run.H[-1].cpu().numpy(), logits, 1e-4, f"partition {i} logits")
        L_ref, dlogits = o_loss.weighted_softmax_ce(logits, y, O["dar_weight"], c)
        assert abs(run.loss.item() - L_ref) <= 1e-4 * abs(L_ref)
        refs.append(o_epoch.backward(om, g, saved, dlogits))
        slack_i, n_amb = worst_case_slack(om, g, saved, dlogits, GATE_MARGIN)
        progress(f"cfg4 x0.02: partition {i}: {n_amb} pre-activations within {GATE_MARGIN} rms of zero")
        slacks.append(slack_i)
        del run, masks, P
    total = o_epoch.sum_grads(refs)
    slack = o_epoch.sum_grads(slacks)
    for l, (got, ref) in enumerate(zip(model.grads, total)):
        for name in ref:
            assert_close_slack(got[name].cpu().numpy(), ref[name], slack[l][name], 1e-4, f"summed layer {l} d{name}")


def test_iteration_is_run_to_run_identical(G):
    """No atomics and fixed-order reductions: two runs give bitwise identical gradients."""
    B, M, torch = G["B"], G["M"], G["torch"]
    wl = inputs.WORKLOADS[0]
    P, O, masks, keep = setup_partition(G, wl, 4, 0, K=2)
    dims = [(64, 16, 16), (16, 16, 8)]
    model = M.Model("sage", dims)
    model.load(inputs.model_params("sage", dims, random_bias=True))
    run = M.PartitionRunner(P, model, masks, dropout_q=0.25, dropout_seed=1)
    ids = O["local2global"]
    Xd = torch.from_numpy(inputs.node_features(ids, 64)).cuda()
    yd = torch.from_numpy(inputs.node_labels(ids, 8)).cuda()
    run.iteration(Xd, yd, 4, mask_seed=9)
    g1, l1 = model.grad.clone(), run.loss.clone()
    run.iteration(Xd, yd, 4, mask_seed=9)
    torch.cuda.synchronize()
    assert torch.equal(g1, model.grad) and torch.equal(l1, run.loss)


def test_layer_calls_reject_bad_arguments(G):
    B, torch = G["B"], G["torch"]
    P = B.build_partition(6, np.array([0, 1, 2]), np.array([1, 2, 3]), 1, 0, 1)
    n = P.num_nodes
    t = lambda *s: torch.zeros(s, device="cuda")
    prm = {"W": t(4, 3), "bW": t(4), "U": t(2, 7), "bU": t(2)}
    saved = {"Z": t(n, 4), "A": t(n, 4)}
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    good = B.layer_desc(B.SAGE_MEAN, 3, 4, 2)
    B.layer_fwd(P, None, 0, good, t(n, 3), prm, t(n, 2), saved, ws)
    for bad in [B.layer_desc(5, 3, 4, 2), B.layer_desc(B.SAGE_MEAN, 0, 4, 2), B.layer_desc(B.SAGE_MEAN, 3, 4, 2, dropout_q=1.0),
                B.layer_desc(B.SAGE_MEAN, 3, 4, 2, dtype=7)]:
        with pytest.raises(B.CofreeError) as e:
            B.layer_fwd(P, None, 0, bad, t(n, 3), prm, t(n, 2), saved, ws)
        assert e.value.code == B.EINVAL
    with pytest.raises(B.CofreeError):
        B.layer_fwd(P, None, 0, good, t(n, 3), {"W": prm["W"], "bW": prm["bW"]}, t(n, 2), saved, ws)   # U missing
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.CofreeError) as e:
        B.layer_bwd(P, None, 0, good, t(n, 3), t(n, 2), prm, saved, t(n, 2), None, {k: torch.zeros_like(v) for k, v in prm.items()},
                    False, tiny)
    assert e.value.code == B.ENOMEM
    torch.cuda.synchronize()


@pytest.mark.parametrize("kind", ["sage", "sage_conv", "gcn"])
def test_backward_on_two_streams(G, kind, monkeypatch):
    """COFREE_OVERLAP=1 moves the weight gradients that do not depend on the transposed aggregation to the
    library's second stream; gradients must not change."""
    monkeypatch.setenv("COFREE_OVERLAP", "1")
    wl = inputs.WORKLOADS[1].scaled(0.02)
    dims = [(64, 48, 32), (32, 48, 8)] if kind == "sage" else [(64, 0, 32), (32, 0, 8)]
    run_iteration_parity(G, wl, kind, dims, 8, 0, K=2, q=0.25, epoch=1)


def test_cfg1_shape_scaled_sage_sliced_gather(G, monkeypatch):
    """Same as test_cfg1_shape_scaled_sage with the XCD-sliced neighbour-group aggregation forced on (at full
    size the library picks it by itself; tests/test_gpu_fullsize.py covers that selection)."""
    monkeypatch.setenv("COFREE_AGG_SLICES", "8")
    wl = inputs.WORKLOADS[1].scaled(0.02)
    run_iteration_parity(G, wl, "sage", wl.layer_dims(), 8, 0, K=0, q=0.0, epoch=1)


@pytest.mark.parametrize("kind,dims,opt", [("sage_conv", [(64, 0, 32), (32, 0, 32), (32, 0, 8)], "adam"),
                                           ("sage", [(64, 16, 16), (16, 16, 8)], "adam"),
                                           ("gcn", [(64, 0, 16), (16, 0, 8)], "sgd")])
def test_training_driver_several_iterations(G, kind, dims, opt):
    """Algorithm 1 for several iterations on two partitions with DropEdge-K, dropout and Adam / SGD: the
    per-iteration losses and the final parameters follow the oracle's driver."""
    B, M, torch = G["B"], G["M"], G["torch"]
    from oracle import train as o_train
    from paper_2308_03209_amd import train as T
    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    p, K, q, n_iters, lr = 4, 3, 0.2, 6, 0.01
    layers = inputs.model_params(kind, dims, random_bias=True)
    model = M.Model(kind, dims)
    model.load(layers)
    om = to_f64_model(kind, layers)
    c = 1.0 / wl.n_nodes
    gpu_parts, ora_parts = [], []
    for i in (0, 2):
        print(f"[case] training driver kind={kind} partition {i}", flush=True)
        P = B.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        O = o_partition.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        masks = B.dropedge_k(P, K, 0.5, inputs.SEED_MASKS + i)
        keep = o_dropedge.masks(O["n_edges"], K, 0.5, inputs.SEED_MASKS + i)
        ids = O["local2global"]
        X = inputs.node_features(ids, dims[0][0])
        y = inputs.node_labels(ids, dims[-1][2])
        run = M.PartitionRunner(P, model, masks, dropout_q=q, dropout_seed=inputs.SEED_DROPOUT)
        gpu_parts.append(T.PartitionData(run, torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda(), 900 + i))
        ora_parts.append({"part": O, "X": X.astype(np.float64), "y": y, "w": O["dar_weight"], "keep": keep,
                          "mask_seed": 900 + i})
    f32 = lambda v: float(np.float32(v))
    hist = T.Trainer(model, gpu_parts, c, opt, lr).fit(n_iters)
    ref = o_train.train(om, ora_parts, n_iters, c, q, inputs.SEED_DROPOUT, opt, f32(lr), f32(0.9), f32(0.999), f32(1e-8))
    for t, (a, b) in enumerate(zip(hist, ref)):
        assert np.allclose(a, b, rtol=2e-4), (t, a, b)
    # parameters after n_iters updates: every update moves an entry by at most ~lr, and rounding differences of
    # the gradients enter Adam's ratio m/sqrt(v) only relatively
    for l, (got, want) in enumerate(zip(model.params, om["layers"])):
        for name in want:
            assert_close(got[name].cpu().numpy(), want[name], 1e-3, f"trained layer {l} {name}")


def test_multilabel_training_sigmoid_bce(G):
    """A Yelp-like multi-label task in miniature: conventional GraphSAGE layers, sigmoid + BCE loss with
    Degree-Aware Reweighting, Adam, two partitions; losses and trained parameters follow the oracle."""
    B, M, torch = G["B"], G["M"], G["torch"]
    from oracle import train as o_train
    from paper_2308_03209_amd import train as T
    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    kind, dims = "sage_conv", [(64, 0, 48), (48, 0, 20)]
    p, K, q, n_iters, lr = 4, 2, 0.1, 5, 0.01
    layers = inputs.model_params(kind, dims, random_bias=True)
    model = M.Model(kind, dims)
    model.load(layers)
    om = to_f64_model(kind, layers)
    c = 1.0 / wl.n_nodes
    gpu_parts, ora_parts = [], []
    for i in (1, 3):
        print(f"[case] multilabel training partition {i}", flush=True)
        P = B.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        O = o_partition.build_partition(wl.n_nodes, src, dst, p, i, inputs.SEED_CUT)
        masks = B.dropedge_k(P, K, 0.5, inputs.SEED_MASKS + i)
        keep = o_dropedge.masks(O["n_edges"], K, 0.5, inputs.SEED_MASKS + i)
        ids = O["local2global"]
        X = inputs.node_features(ids, dims[0][0])
        Y = inputs.node_multilabels(ids, dims[-1][2], 0.2)
        run = M.PartitionRunner(P, model, masks, dropout_q=q, dropout_seed=inputs.SEED_DROPOUT, loss="sigmoid_bce")
        gpu_parts.append(T.PartitionData(run, torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), 300 + i))
        ora_parts.append({"part": O, "X": X.astype(np.float64), "y": Y, "w": O["dar_weight"], "keep": keep,
                          "mask_seed": 300 + i})
    f32 = lambda v: float(np.float32(v))
    hist = T.Trainer(model, gpu_parts, c, "adam", lr).fit(n_iters)
    ref = o_train.train(om, ora_parts, n_iters, c, q, inputs.SEED_DROPOUT, "adam", f32(lr), f32(0.9), f32(0.999),
                        f32(1e-8), loss_fn=o_loss.weighted_sigmoid_bce)
    for t, (a, b) in enumerate(zip(hist, ref)):
        assert np.allclose(a, b, rtol=2e-4), (t, a, b)
    for l, (got, want) in enumerate(zip(model.params, om["layers"])):
        for name in want:
            assert_close(got[name].cpu().numpy(), want[name], 1e-3, f"trained layer {l} {name}")


@pytest.mark.parametrize("cut", ["random", "dbh"])
def test_gradient_gap_and_weight_variants(G, cut):
    """Eq. 2's objective for the three reweightings of the ablation (DAR, 1/RF, none) under both cuts: the
    library's gap follows the oracle's, and so does the replication factor."""
    B, M, torch = G["B"], G["M"], G["torch"]
    from paper_2308_03209_amd import diagnostics as D
    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    p, kind, dims = 4, "sage_conv", [(64, 0, 32), (32, 0, 8)]
    layers = inputs.model_params(kind, dims, random_bias=True)
    om = to_f64_model(kind, layers)
    Os = [o_partition.build_partition(wl.n_nodes, src, dst, p, i, 21, method=cut) for i in range(p)]
    full = o_partition.build_partition(wl.n_nodes, src, dst, 1, 0, 21)
    rf = o_partition.node_replication(wl.n_nodes, Os)
    c = 1.0 / wl.n_nodes

    def oracle_grads(O, w):
        ids = O["local2global"]
        X = inputs.node_features(ids, 64).astype(np.float64)
        return o_epoch.partition_loss_and_grads(om, o_dropedge.full_graph(O), X, inputs.node_labels(ids, 8), w, c)[1]

    g_full = oracle_grads(full, np.ones(full["n_nodes"]))
    gaps = {}
    for name, code in (("dar", B.W_DAR), ("inv_rf", B.W_INV_RF), ("none", B.W_NONE)):
        print(f"[case] gradient gap cut={cut} weights={name}", flush=True)
        ref_gap, ref_norm = o_epoch.gradient_gap(g_full, [oracle_grads(O, o_partition.loss_weights(O, name, rf)) for O in Os])
        gap, norm, rf_lib = D.gradient_gap(kind, dims, layers, wl.n_nodes, src, dst, p, 21, code, inputs.node_features,
                                           inputs.node_labels, B.CUT_DBH if cut == "dbh" else 0, c)
        assert abs(norm - ref_norm) <= 1e-4 * ref_norm, (norm, ref_norm)
        assert abs(gap - ref_gap) <= 1e-3 * ref_gap, (name, gap, ref_gap)
        assert abs(rf_lib - o_partition.replication_factor(wl.n_nodes, Os)) < 1e-12
        gaps[name] = gap
    print(f"[case] gaps {gaps}", flush=True)
    assert gaps["none"] > gaps["dar"]

def test_trainer_graph_replay_matches_eager(G):
    """Trainer(graphs=True): iterations replayed as HIP graphs (one per combination of DropEdge-K masks) give
    bit-identical parameters to the same iterations enqueued launch by launch; replays are interleaved with
    eager iterations (first sight of a mask combination) and with host synchronisations."""
    B, M, torch = G["B"], G["M"], G["torch"]
    from paper_2308_03209_amd import train as T
    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    kind, dims = "gcn", wl.layer_dims()
    finals = []
    for graphs in (False, True):
        model = M.Model(kind, dims)
        model.load(inputs.model_params(kind, dims, random_bias=True))
        parts = []
        for part in (0, 2):
            P = B.build_partition(wl.n_nodes, src, dst, 4, part, inputs.SEED_CUT)
            masks = B.dropedge_k(P, 2, 0.5, inputs.SEED_MASKS + part)
            ids = P.host_array(B.ARR_LOCAL2GLOBAL)
            X = torch.from_numpy(inputs.node_features(ids, dims[0][0])).cuda()
            y = torch.from_numpy(inputs.node_labels(ids, dims[-1][2])).cuda()
            parts.append(T.PartitionData(M.PartitionRunner(P, model, masks), X, y, mask_seed=3 + part))
        tr = T.Trainer(model, parts, scale_c=1.0 / wl.n_nodes, optimizer="sgd", lr=0.5, graphs=graphs)
        for it in range(24):
            tr.step()
            if it % 5 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        if graphs:
            assert len(tr._graphs) >= 2, "several mask combinations should have been captured"
        finals.append(model.theta.cpu().numpy().copy())
    assert np.array_equal(finals[0], finals[1])
    with pytest.raises(ValueError):
        T.Trainer(model, parts, scale_c=1.0, optimizer="adam", graphs=True)
