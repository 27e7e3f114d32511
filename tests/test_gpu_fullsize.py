"""cfg1 at full size, in the launch configuration bench.py times: sampled outputs against values the
oracle computes one by one, plus properties that hold at any size.

The oracle cannot afford the whole 56M-edge graph inside a routine test run, so for a handful of
sampled nodes their partition rows, then their 2-hop neighbourhoods, are rebuilt from the edge list with
the oracle's own hash, and the oracle evaluates the layer definitions on those nodes only."""
import numpy as np
import pytest

from oracle import partition as o_partition
from paper_2308_03209_amd import inputs

pytestmark = pytest.mark.gpu

N_SAMPLES = 6


@pytest.fixture(scope="module")
def full():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2308_03209_amd import binding as B
    from paper_2308_03209_amd import model as M
    wl = inputs.WORKLOADS[1]
    print("[case] cfg1 full size: generating graph", flush=True)
    src, dst = inputs.workload_graph(wl)
    print("[case] cfg1 full size: building partition 0", flush=True)
    P = B.build_partition(wl.n_nodes, src, dst, wl.n_parts, 0, inputs.SEED_CUT)
    return dict(B=B, M=M, torch=torch, wl=wl, src=src, dst=dst, P=P)


def oracle_rows(full, nodes):
    """Partition-0 neighbour lists (global ids) and global degrees of `nodes`, from the edge list and the
    oracle's edge hash only."""
    wl, src, dst = full["wl"], full["src"], full["dst"]
    nodes = np.asarray(nodes, dtype=np.int64)
    touch = np.isin(src, nodes) | np.isin(dst, nodes)
    s, d = src[touch], dst[touch]
    lo, hi = np.minimum(s, d), np.maximum(s, d)
    part = o_partition.assign_edges(lo, hi, wl.n_parts, inputs.SEED_CUT)
    out = {}
    for v in nodes.tolist():
        m = (s == v) | (d == v)
        other = np.where(s[m] == v, d[m], s[m])
        out[v] = (np.sort(other[part[m] == 0]), int(m.sum()))
    return out


def test_sampled_structure_rows_and_weights(full):
    B, P, wl = full["B"], full["P"], full["wl"]
    l2g = P.host_array(B.ARR_LOCAL2GLOBAL)
    rowptr, col = P.host_array(B.ARR_ROWPTR), P.host_array(B.ARR_COL)
    w = P.host_array(B.ARR_DAR_WEIGHT)
    assert np.all(np.diff(l2g) > 0) and rowptr[-1] == P.num_nnz == 2 * P.num_edges
    sample = np.random.default_rng(5).choice(P.num_nodes, N_SAMPLES, replace=False)
    rows = oracle_rows(full, l2g[sample])
    for v in sample.tolist():
        nb, dg = rows[int(l2g[v])]
        got = l2g[col[rowptr[v]:rowptr[v + 1]]]
        assert np.array_equal(got, nb)
        assert w[v] == np.float32(np.float64(len(nb)) / np.float64(dg))
    full["sample"], full["rows"], full["l2g"] = sample, rows, l2g


def test_sampled_aggregate_rows_all_modes(full):
    """256-wide aggregation at full size (the XCD-sliced kernel is selected at this size)."""
    B, P, torch = full["B"], full["P"], full["torch"]
    if "sample" not in full:
        test_sampled_structure_rows_and_weights(full)
    sample, rows, l2g = full["sample"], full["rows"], full["l2g"]
    n = P.num_nodes
    g2l = {int(g): i for i, g in enumerate(l2g.tolist())}
    X = torch.randn((n, 256), device="cuda", generator=torch.Generator(device="cuda").manual_seed(3))
    Y = torch.empty_like(X)
    Xh = X.cpu().numpy().astype(np.float64)
    deg = np.diff(P.host_array(B.ARR_ROWPTR)).astype(np.float64)
    for mode in (B.AGG_MEAN, B.AGG_MEAN_T, B.AGG_GCN):
        B.aggregate(P, None, 0, mode, X, Y, 256)
        torch.cuda.synchronize()
        Yh = Y[torch.from_numpy(sample).cuda()].cpu().numpy()
        for i, v in enumerate(sample.tolist()):
            nb = np.array([g2l[int(g)] for g in rows[int(l2g[v])][0]], dtype=np.int64)
            if mode == B.AGG_MEAN:
                ref = Xh[nb].sum(0) / len(nb)
            elif mode == B.AGG_MEAN_T:
                ref = (Xh[nb] / deg[nb][:, None]).sum(0)
            else:
                s = 1.0 / np.sqrt(deg + 1.0)
                ref = s[v] * (s[v] * Xh[v] + (s[nb][:, None] * Xh[nb]).sum(0))
            err = np.abs(Yh[i] - ref).max() / max(np.abs(ref).max(), 1e-30)
            assert err < 1e-4, (mode, v, err)


def test_full_iteration_properties(full):
    """One full iteration at bench size: finite loss equal on two runs (fixed-order reductions), rows of
    dlogits sum to zero, and the bias gradient of the last layer equals the column sums of dlogits."""
    B, M, P, torch, wl = full["B"], full["M"], full["P"], full["torch"], full["wl"]
    dims = wl.layer_dims()
    model = M.Model(wl.kind, dims)
    model.load(inputs.model_params(wl.kind, dims, random_bias=True))
    run = M.PartitionRunner(P, model)
    ids = P.host_array(B.ARR_LOCAL2GLOBAL)
    X = torch.from_numpy(inputs.node_features(ids, wl.d_feat)).cuda()
    y = torch.from_numpy(inputs.node_labels(ids, wl.n_classes)).cuda()
    print("[case] cfg1 full size: iteration", flush=True)
    run.iteration(X, y, 0, scale_c=1.0 / wl.n_nodes)
    torch.cuda.synchronize()
    loss1, grad1 = run.loss.item(), model.grad.clone()
    assert np.isfinite(loss1) and torch.isfinite(model.grad).all()
    # uniform-ish logits at initialisation: loss close to (sum of weights / |V|) * log(C)
    wsum = float(P.host_array(B.ARR_DAR_WEIGHT).astype(np.float64).sum())
    assert 0.2 * np.log(wl.n_classes) * wsum / wl.n_nodes < loss1 < 5 * np.log(wl.n_classes) * wsum / wl.n_nodes
    dl = run.dlogits.double()
    assert dl.sum(1).abs().max().item() < 1e-9
    dbU = model.grads[-1]["bU"].double()
    assert torch.allclose(dbU, dl.sum(0), rtol=1e-4, atol=1e-9)
    run.iteration(X, y, 0, scale_c=1.0 / wl.n_nodes)
    torch.cuda.synchronize()
    assert run.loss.item() == loss1 and torch.equal(grad1, model.grad)
    full["run"], full["X"], full["model"] = run, X, model


def test_sampled_logits_two_hop_oracle(full):
    """Logits of sampled nodes: the oracle evaluates both GraphSAGE layers on the node's 2-hop neighbourhood,
    built from the edge list with the oracle's hash."""
    from oracle import layers as o_layers
    B, P, wl = full["B"], full["P"], full["wl"]
    if "run" not in full:
        test_full_iteration_properties(full)
    if "sample" not in full:
        test_sampled_structure_rows_and_weights(full)
    run, model = full["run"], full["model"]
    l2g = full["l2g"]
    prm = [{k: v.cpu().numpy().astype(np.float64) for k, v in lay.items()} for lay in model.params]
    sample = full["sample"][:3]
    targets = l2g[sample]
    hop1 = oracle_rows(full, targets)
    ring1 = np.unique(np.concatenate([hop1[int(t)][0] for t in targets] + [targets]))
    hop2 = oracle_rows(full, ring1)
    ring2 = np.unique(np.concatenate([hop2[int(t)][0] for t in ring1] + [ring1]))
    # local sub-problem over ring2 with exact rows for ring1 (rows of other nodes are not needed)
    idx = {int(g): i for i, g in enumerate(ring2.tolist())}
    X2 = inputs.node_features(ring2, wl.d_feat).astype(np.float64)

    def sage_rows(nodes, H_of, prm_l):
        """Layer output at `nodes` given a dict global id -> input row for all nodes involved."""
        W, bW, U, bU = prm_l["W"], prm_l["bW"], prm_l["U"], prm_l["bU"]
        out = {}
        for t in nodes.tolist():
            nb = hop2[int(t)][0]
            Z = np.maximum(np.stack([H_of[int(u)] for u in nb]) @ W.T + bW, 0.0)
            out[int(t)] = np.concatenate([Z.mean(0), H_of[int(t)]]) @ U.T + bU
        return out

    H0 = {int(g): X2[idx[int(g)]] for g in ring2.tolist()}
    H1 = sage_rows(ring1, H0, prm[0])
    logits = sage_rows(targets, H1, prm[1])
    got = run.H[-1][full["torch"].from_numpy(sample).cuda()].cpu().numpy()
    for i, t in enumerate(targets.tolist()):
        ref = logits[int(t)]
        err = np.abs(got[i] - ref).max() / np.abs(ref).max()
        assert err < 1e-4, (t, err)


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
