"""The loss entry point that allocates nothing (partial sums in a static device array of the library) against
the workspace-taking entry point it is a variant of: same kernels, same reduction order, so the results must be
identical bit for bit - and within the parity tolerance of the oracle.  Two calls in a row on one GPU, the
second on a smaller partition, show that nothing of the first call's scratch contents leaks into the second."""
import numpy as np
import pytest

from oracle import loss as o_loss
from oracle import partition as o_partition
from paper_2308_03209_amd import inputs
from util import assert_close

pytestmark = pytest.mark.gpu


def test_loss_static_matches_workspace_entry_point_twice():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    from paper_2308_03209_amd import binding as B

    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    # first call: a 2-way cut's partition (about 2000 nodes); second: a 16-way cut's (fewer nodes and rows)
    cases = [(2, 0, 41, B.F32), (16, 3, 7, B.F32), (2, 1, 172, B.BF16), (16, 5, 300, B.BF16)]
    sizes = []
    for p, part_id, C, dtype in cases:
        print(f"[case] static loss p={p} part={part_id} C={C} dtype={dtype}", flush=True)
        P = B.build_partition(wl.n_nodes, src, dst, p, part_id, inputs.SEED_CUT)
        O = o_partition.build_partition(wl.n_nodes, src, dst, p, part_id, inputs.SEED_CUT)
        n = O["n_nodes"]
        sizes.append(n)
        rng = np.random.default_rng(C)
        td = torch.float32 if dtype == B.F32 else torch.bfloat16
        z = torch.from_numpy((3 * rng.standard_normal((n, C))).astype(np.float32)).to(td).cuda()
        y_np = rng.integers(0, C, n).astype(np.int32)
        y = torch.from_numpy(y_np).cuda()
        tm_np = (rng.random(n) < 0.8).astype(np.uint8)
        tm = torch.from_numpy(tm_np).cuda()
        ws = torch.empty(B.loss_workspace_bytes(), dtype=torch.uint8, device="cuda")
        loss_a, loss_b = torch.zeros(1, device="cuda"), torch.full((1,), float("nan"), device="cuda")
        dz_a = torch.empty_like(z)
        dz_b = torch.full_like(z, float("nan"))
        B.loss_weighted(P, B.W_DAR, None, z, y, tm, C, 0.37, loss_a, dz_a, ws, dtype)
        B.loss_weighted_static(P, B.W_DAR, None, z, y, tm, C, 0.37, loss_b, dz_b, dtype)
        torch.cuda.synchronize()
        assert loss_a.item() == loss_b.item()
        assert torch.equal(dz_a.view(torch.int16 if dtype == B.BF16 else torch.int32),
                           dz_b.view(torch.int16 if dtype == B.BF16 else torch.int32))
        L_ref, g_ref = o_loss.weighted_softmax_ce(z.float().cpu().numpy().astype(np.float64), y_np, O["dar_weight"],
                                                  0.37, tm_np)
        assert abs(loss_b.item() - L_ref) <= 1e-4 * abs(L_ref)
        assert_close(dz_b.float().cpu().numpy(), g_ref, 1e-4 if dtype == B.F32 else 5e-3, "dlogits (static)")
    assert sizes[1] < sizes[0] and sizes[3] < sizes[2]


def test_loss_static_rejects_sizes_beyond_its_limits():
    import torch
    from paper_2308_03209_amd import binding as B
    wl = inputs.WORKLOADS[0]
    src, dst = inputs.workload_graph(wl)
    P = B.build_partition(wl.n_nodes, src, dst, 4, 0, inputs.SEED_CUT)
    n = P.num_nodes
    z = torch.zeros((n, 8), device="cuda")
    y = torch.zeros(n, dtype=torch.int32, device="cuda")
    loss = torch.zeros(1, device="cuda")
    with pytest.raises(B.CofreeError) as e:
        B.loss_weighted_static(P, B.W_DAR, None, z, y, None, 4097, 1.0, loss, z)   # rejected before any launch
    assert e.value.code == B.EINVAL and "COFREE_LOSS_STATIC_MAX_CLASSES" in str(e.value)
