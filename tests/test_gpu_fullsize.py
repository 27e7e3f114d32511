"""cfg1 and cfg2 at full size, in the launch configuration bench.py times.

Every reference quantity comes from `oracle/`: the partition (structures, degrees, Degree-Aware Reweighting
weights) is built by the oracle from the same edge list at full size, and aggregations, layers, loss and all
parameter gradients are the oracle's functions evaluated on that partition - one full
`partition_loss_and_grads` run for cfg1.  Long steps write progress lines (tests/util.py)."""
import numpy as np
import pytest

from gate_slack import worst_case_slack
from oracle import dropedge as o_dropedge
from oracle import epoch as o_epoch
from oracle import layers as o_layers
from oracle import loss as o_loss
from oracle import partition as o_partition
from paper_2308_03209_amd import inputs
from util import TOL_BF16, TOL_F32, assert_close, progress, to_f64_model

pytestmark = pytest.mark.gpu

STRUCT_ARRAYS = ["local2global", "rowptr", "col", "eid", "deg_local", "deg_global", "dar_weight", "edge_lo", "edge_hi"]


def build_both(index):
    """Graph of a workload, its partition 0 from the library and from the oracle."""
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import model as M
    wl = inputs.WORKLOADS[index]
    progress(f"cfg{index} full size: generating graph")
    src, dst = inputs.workload_graph(wl)
    progress(f"cfg{index} full size: library builds partition 0")
    P = B.build_partition(wl.n_nodes, src, dst, wl.n_parts, 0, inputs.SEED_CUT)
    progress(f"cfg{index} full size: oracle builds partition 0")
    O = o_partition.build_partition(wl.n_nodes, src, dst, wl.n_parts, 0, inputs.SEED_CUT)
    progress(f"cfg{index} full size: partitions built ({O['n_nodes']} nodes, {O['nnz']} directed edges)")
    return dict(B=B, M=M, torch=torch, wl=wl, P=P, O=O)


def assert_structures_equal(B, P, O):
    codes = {"local2global": B.ARR_LOCAL2GLOBAL, "rowptr": B.ARR_ROWPTR, "col": B.ARR_COL, "eid": B.ARR_EID,
             "deg_local": B.ARR_DEG_LOCAL, "deg_global": B.ARR_DEG_GLOBAL, "dar_weight": B.ARR_DAR_WEIGHT,
             "edge_lo": B.ARR_EDGE_LO, "edge_hi": B.ARR_EDGE_HI}
    assert (P.num_nodes, P.num_edges, P.num_nnz) == (O["n_nodes"], O["n_edges"], O["nnz"])
    for name in STRUCT_ARRAYS:
        got = P.host_array(codes[name])
        assert got.dtype == O[name].dtype and np.array_equal(got, O[name]), name


@pytest.fixture(scope="module")
def full():
    return build_both(1)


def test_cfg1_structures_bit_exact_at_full_size(full):
    assert_structures_equal(full["B"], full["P"], full["O"])


def test_cfg1_aggregate_256_wide_all_rows_all_modes(full):
    """256-wide float32 aggregation over the whole 230k-row partition (the XCD-sliced kernel is selected at
    this size), every row against the oracle's aggregation functions."""
    B, P, O, torch = full["B"], full["P"], full["O"], full["torch"]
    n = O["n_nodes"]
    g = o_dropedge.full_graph(O)
    X = torch.randn((n, 256), device="cuda", generator=torch.Generator(device="cuda").manual_seed(3))
    Y = torch.empty_like(X)
    X64 = X.cpu().numpy().astype(np.float64)
    for mode, ref_fn in [(B.AGG_MEAN, o_layers.mean_aggregate), (B.AGG_MEAN_T, o_layers.mean_aggregate_bwd),
                         (B.AGG_GCN, o_layers.gcn_aggregate)]:
        progress(f"cfg1 full size: aggregate mode {mode}")
        Y.fill_(float("nan"))
        B.aggregate(P, None, 0, mode, X, Y, 256)
        torch.cuda.synchronize()
        assert_close(Y.cpu().numpy(), ref_fn(g, X64), TOL_F32, f"aggregate mode {mode}")


def test_cfg1_full_iteration_every_gradient_against_one_oracle_run(full):
    """One iteration of the benchmark workload at full size against ONE full run of the oracle: layer
    outputs, saved messages and means, logits, loss and every parameter gradient, element by element, to the
    float32 tolerance.  Gates whose float64 pre-activation lies within float32 rounding distance of zero may
    legitimately differ; the slack they add is bounded from the oracle alone (gate_slack.worst_case_slack).
    Also: a second run of the same iteration reproduces the first bit for bit (fixed-order reductions)."""
    B, M, P, O, torch, wl = full["B"], full["M"], full["P"], full["O"], full["torch"], full["wl"]
    dims = wl.layer_dims()
    layers = inputs.model_params(wl.kind, dims, random_bias=True)
    model = M.Model(wl.kind, dims)
    model.load(layers)
    run = M.PartitionRunner(P, model)
    ids = O["local2global"]
    X = inputs.node_features(ids, wl.d_feat)
    y = inputs.node_labels(ids, wl.n_classes)
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    c = 1.0 / wl.n_nodes
    progress("cfg1 full size: iteration on the GPU")
    run.iteration(Xd, yd, 0, scale_c=c)
    torch.cuda.synchronize()
    loss1, grad1 = run.loss.item(), model.grad.clone()
    run.iteration(Xd, yd, 0, scale_c=c)
    torch.cuda.synchronize()
    assert run.loss.item() == loss1 and torch.equal(grad1, model.grad)

    progress("cfg1 full size: oracle forward")
    om = to_f64_model(wl.kind, layers)
    g = o_dropedge.full_graph(O)
    logits_ref, saved = o_epoch.forward(om, g, X.astype(np.float64))
    L_ref, dlogits_ref = o_loss.weighted_softmax_ce(logits_ref, y, O["dar_weight"], c)
    progress("cfg1 full size: oracle backward")
    G_ref = o_epoch.backward(om, g, saved, dlogits_ref)
    progress("cfg1 full size: gate slack")
    slack, n_amb = worst_case_slack(om, g, saved, dlogits_ref, 1e-5)
    progress(f"cfg1 full size: {n_amb} pre-activations within 1e-5 rms of zero")

    for l, sv in enumerate(saved):
        assert_close(run.saved[l]["Z"].cpu().numpy(), sv["Z"], TOL_F32, f"layer {l} messages Z")
    assert_close(run.saved[0]["A"].cpu().numpy(), saved[0]["A"], TOL_F32, "layer 0 neighbourhood mean")
    assert_close(run.H[1].cpu().numpy(), saved[1]["H"], TOL_F32, "layer 0 output")
    assert_close(run.H[-1].cpu().numpy(), logits_ref, TOL_F32, "logits")
    assert abs(loss1 - L_ref) <= TOL_F32 * abs(L_ref), (loss1, L_ref)
    assert_close(run.dlogits.cpu().numpy(), dlogits_ref, TOL_F32, "dlogits")
    for l, (got, ref) in enumerate(zip(model.grads, G_ref)):
        for name in ref:
            gn = got[name].cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(gn)), f"layer {l} d{name}: non-finite"
            excess = np.maximum(np.abs(gn - ref[name]) - slack[l][name], 0.0)
            e_max = excess.max() / np.abs(ref[name]).max()
            e_fro = np.sqrt((excess * excess).sum()) / np.sqrt((ref[name] ** 2).sum())
            raw = np.abs(gn - ref[name]).max() / np.abs(ref[name]).max()
            progress(f"cfg1 full size: layer {l} d{name}: rel err max {raw:.2e} (beyond gate slack {e_max:.2e}), "
                     f"largest slack {slack[l][name].max() / np.abs(ref[name]).max():.2e}")
            assert e_max <= TOL_F32 and e_fro <= TOL_F32, f"layer {l} d{name}: {e_max:.3e} / {e_fro:.3e}"


# ---------------------------------------------------------------- cfg2 at full size (bf16 storage, short rows)

@pytest.fixture(scope="module")
def full2():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import model as M
    wl = inputs.WORKLOADS[2]
    print("[case] cfg2 full size: generating graph", flush=True)
    src, dst = inputs.workload_graph(wl)
    print("[case] cfg2 full size: building partition 0", flush=True)
    P = B.build_partition(wl.n_nodes, src, dst, wl.n_parts, 0, inputs.SEED_CUT)
    return dict(B=B, M=M, torch=torch, wl=wl, src=src, dst=dst, P=P)


def test_cfg2_sampled_rows_and_bf16_aggregate(full2):
    """1.9M-row partition, average degree 4: sampled CSR rows and weights against the oracle's hash, then the
    bf16 aggregation (widths 256, 100 and the ragged 47) on those rows against float64 sums."""
    B, P, torch = full2["B"], full2["P"], full2["torch"]
    l2g = P.host_array(B.ARR_LOCAL2GLOBAL)
    rowptr, col = P.host_array(B.ARR_ROWPTR), P.host_array(B.ARR_COL)
    w = P.host_array(B.ARR_DAR_WEIGHT)
    deg = np.diff(rowptr)
    rng = np.random.default_rng(9)
    # a few random rows plus the longest row
    sample = np.unique(np.r_[rng.choice(P.num_nodes, N_SAMPLES, replace=False), np.argmax(deg)])
    rows = oracle_rows(full2, l2g[sample])
    for v in sample.tolist():
        nb, dg = rows[int(l2g[v])]
        assert np.array_equal(l2g[col[rowptr[v]:rowptr[v + 1]]], nb)
        assert w[v] == np.float32(np.float64(len(nb)) / np.float64(dg))
    g2l = {int(g): i for i, g in enumerate(l2g.tolist())}
    n = P.num_nodes
    degf = deg.astype(np.float64)
    for width in (256, 100, 47):
        print(f"[case] cfg2 full size: bf16 aggregate width {width}", flush=True)
        X = torch.randn((n, width), device="cuda", generator=torch.Generator(device="cuda").manual_seed(width)).to(torch.bfloat16)
        Y = torch.empty_like(X)
        for mode in (B.AGG_MEAN, B.AGG_MEAN_T, B.AGG_GCN):
            B.aggregate(P, None, 0, mode, X, Y, width, B.BF16)
            torch.cuda.synchronize()
            Yh = Y[torch.from_numpy(sample).cuda()].float().cpu().numpy().astype(np.float64)
            for i, v in enumerate(sample.tolist()):
                nb = np.array([g2l[int(g)] for g in rows[int(l2g[v])][0]], dtype=np.int64)
                Xn = X[torch.from_numpy(nb).cuda()].float().cpu().numpy().astype(np.float64)
                if mode == B.AGG_MEAN:
                    ref = Xn.sum(0) / len(nb)
                elif mode == B.AGG_MEAN_T:
                    ref = (Xn / degf[nb][:, None]).sum(0)
                else:
                    s = 1.0 / np.sqrt(degf + 1.0)
                    ref = s[v] * (s[v] * X[v].float().cpu().numpy().astype(np.float64) + (s[nb][:, None] * Xn).sum(0))
                err = np.abs(Yh[i] - ref).max() / max(np.abs(ref).max(), 1e-30)
                assert err < 5e-3, (width, mode, v, err)      # one bf16 rounding of the float32 sum


def test_cfg2_sampled_gcn_layer_rows_large_tile(full2):
    """A bf16 GCN layer forward with ReLU (256 -> 256, and 200 -> 264 with a ragged k and a second,
    8-column tile) over the whole 1.9M-row partition - a size at which products of more than 128 columns
    take the 256x256 block tile by themselves - against relu(W agg + b) evaluated in float64 on sampled
    rows, the partition's first and last rows (ragged last tile) among them."""
    B, P, torch = full2["B"], full2["P"], full2["torch"]
    l2g = P.host_array(B.ARR_LOCAL2GLOBAL)
    rowptr = P.host_array(B.ARR_ROWPTR)
    n = P.num_nodes
    degf = np.diff(rowptr).astype(np.float64)
    rng = np.random.default_rng(17)
    sample = np.unique(np.r_[rng.choice(n, N_SAMPLES, replace=False), n - 1, n - 2, 0])
    rows = oracle_rows(full2, l2g[sample])
    g2l = {int(g): i for i, g in enumerate(l2g.tolist())}
    s = 1.0 / np.sqrt(degf + 1.0)
    for d_in, d_out in ((256, 256), (200, 264)):
        print(f"[case] cfg2 full size: bf16 GCN layer {d_in} -> {d_out}", flush=True)
        gen = torch.Generator(device="cuda").manual_seed(d_in)
        H = torch.randn((n, d_in), device="cuda", generator=gen).to(torch.bfloat16)
        W = (torch.randn((d_out, d_in), device="cuda", generator=gen) * 0.08).contiguous()
        b = (torch.randn((d_out,), device="cuda", generator=gen) * 0.1).contiguous()
        desc = B.layer_desc(B.GCN, d_in, 0, d_out, act=1, dtype=B.BF16)
        out = torch.full((n, d_out), float("nan"), device="cuda", dtype=torch.bfloat16)
        saved = {"A": torch.empty((n, d_in), device="cuda", dtype=torch.bfloat16)}
        ws = torch.empty(max(B.layer_workspace_bytes(desc, n, False), 256), dtype=torch.uint8, device="cuda")
        B.layer_fwd(P, None, 0, desc, H, {"W": W, "bW": b}, out, saved, ws)
        torch.cuda.synchronize()
        assert torch.isfinite(out.float()).all()
        W64, b64 = W.cpu().numpy().astype(np.float64), b.cpu().numpy().astype(np.float64)
        got = out[torch.from_numpy(sample).cuda()].float().cpu().numpy().astype(np.float64)
        for i, v in enumerate(sample.tolist()):
            nb = np.array([g2l[int(g)] for g in rows[int(l2g[v])][0]], dtype=np.int64)
            Hn = H[torch.from_numpy(nb).cuda()].float().cpu().numpy().astype(np.float64)
            Hv = H[v].float().cpu().numpy().astype(np.float64)
            agg = s[v] * (s[v] * Hv + (s[nb][:, None] * Hn).sum(0))
            ref = np.maximum(W64 @ agg + b64, 0.0)
            err = np.abs(got[i] - ref).max() / max(np.abs(ref).max(), 1e-30)
            assert err < 2e-2, (d_in, d_out, v, err)      # bf16 aggregate, bf16 parameters, bf16 result


def test_cfg2_full_iteration_properties(full2):
    """One full bf16 iteration with DropEdge-K at bench size: finite and repeatable bit for bit, dlogits rows
    sum to zero within bf16 rounding, the last bias gradient is the column sum of dlogits."""
    B, M, P, torch, wl = full2["B"], full2["M"], full2["P"], full2["torch"], full2["wl"]
    dims = wl.layer_dims()
    model = M.Model(wl.kind, dims)
    model.load(inputs.model_params(wl.kind, dims, random_bias=True))
    masks = B.dropedge_k(P, wl.dropedge_K, wl.dropedge_p, inputs.SEED_MASKS)
    run = M.PartitionRunner(P, model, masks, dtype="bf16")
    ids = P.host_array(B.ARR_LOCAL2GLOBAL)
    X = torch.from_numpy(inputs.node_features(ids, wl.d_feat)).to(torch.bfloat16).cuda()
    y = torch.from_numpy(inputs.node_labels(ids, wl.n_classes)).cuda()
    print("[case] cfg2 full size: iteration", flush=True)
    run.iteration(X, y, 1, mask_seed=inputs.SEED_MASKS, scale_c=1.0 / wl.n_nodes)
    torch.cuda.synchronize()
    loss1, grad1 = run.loss.item(), model.grad.clone()
    assert np.isfinite(loss1) and torch.isfinite(model.grad).all()
    wsum = float(P.host_array(B.ARR_DAR_WEIGHT).astype(np.float64).sum())
    assert 0.2 * np.log(wl.n_classes) * wsum / wl.n_nodes < loss1 < 5 * np.log(wl.n_classes) * wsum / wl.n_nodes
    dl = run.dlogits.double()
    scale = dl.abs().max().item()
    assert dl.sum(1).abs().max().item() < wl.n_classes * 2.0 ** -8 * scale
    dbU = model.grads[-1]["bU"].double()
    assert torch.allclose(dbU, dl.sum(0), rtol=1e-4, atol=1e-9)
    # the masked graphs keep about half the edges and stay symmetric in size
    for k in range(wl.dropedge_K):
        assert abs(masks.host_graph(k)[1].shape[0] / P.num_nnz - 0.5) < 0.01
    run.iteration(X, y, 1, mask_seed=inputs.SEED_MASKS, scale_c=1.0 / wl.n_nodes)
    torch.cuda.synchronize()
    assert run.loss.item() == loss1 and torch.equal(grad1, model.grad)
