"""Pins for the gate-slack helpers of the GPU parity tests (CPU only): the one-pass worst-case bound must
dominate, element by element, the sum of the absolute gradient changes obtained by flipping every ambiguous
gate by itself and repeating the oracle's backward pass (brute force), and must be exact where a flip acts
on a gradient directly."""
import numpy as np
import pytest

from gate_slack import ambiguous_gates, sampled_flip_slack, worst_case_slack
from oracle import dropedge, epoch, loss, partition
from paper_2308_03209_amd import inputs


def setup(kind, q):
    src, dst = inputs.small_random_graph(70, 200, 3)
    P = partition.build_partition(70, src, dst, 2, 0, 9)
    g = dropedge.full_graph(P)
    n = P["n_nodes"]
    dims = [(6, 5, 7), (7, 4, 6), (6, 3, 4)]
    prm = inputs.model_params(kind, dims, 5, random_bias=True)
    om = {"kind": kind, "layers": [{k: v.astype(np.float64) for k, v in l.items()} for l in prm]}
    rng = np.random.default_rng(2)
    X = rng.standard_normal((n, 6))
    y = rng.integers(0, 4, n)
    logits, saved = epoch.forward(om, g, X, q, 13, 2)
    _, dlogits = loss.weighted_softmax_ce(logits, y, P["dar_weight"], 0.1)
    return om, g, saved, dlogits


@pytest.mark.parametrize("kind", ["sage", "gcn", "sage_conv"])
@pytest.mark.parametrize("q", [0.0, 0.3])
def test_worst_case_slack_dominates_flip_by_flip_brute_force(kind, q):
    om, g, saved, dlogits = setup(kind, q)
    margin = 0.08
    slack, n_amb = worst_case_slack(om, g, saved, dlogits, margin)
    base = epoch.backward(om, g, saved, dlogits)
    brute = [{k: np.zeros_like(v) for k, v in b.items()} for b in base]
    count = 0
    for l, sv in enumerate(saved):
        if kind != "sage" and not sv["relu"]:
            continue
        for (u, ch) in np.argwhere(ambiguous_gates(sv["pre"], margin)):
            count += 1
            sv["pre"][u, ch] = -sv["pre"][u, ch]
            G = epoch.backward(om, g, saved, dlogits)
            sv["pre"][u, ch] = -sv["pre"][u, ch]
            for bl, g0, g1 in zip(brute, base, G):
                for k in bl:
                    bl[k] += np.abs(g1[k] - g0[k])
    assert count == n_amb and count > 10
    top = max(l for l, sv in enumerate(saved) if kind == "sage" or sv["relu"])
    for l, (sl, bl) in enumerate(zip(slack, brute)):
        for k in bl:
            assert np.all(sl[k] >= bl[k] - 1e-12 * (1.0 + np.abs(bl[k]))), (l, k)
            # not vacuous: within a small factor of the brute-force sum overall
            assert sl[k].sum() <= 6.0 * bl[k].sum() + 1e-12, (l, k, sl[k].sum(), bl[k].sum())
    # the topmost gated layer sees no perturbation from above: there the bound is the brute-force sum itself
    assert np.allclose(slack[top]["W"], brute[top]["W"], rtol=1e-9, atol=1e-14)
    assert np.allclose(slack[top]["bW"], brute[top]["bW"], rtol=1e-9, atol=1e-14)


def test_no_ambiguous_gate_means_no_slack():
    om, g, saved, dlogits = setup("sage", 0.0)
    slack, n_amb = worst_case_slack(om, g, saved, dlogits, 0.0)
    assert n_amb == 0 and all(np.all(v == 0.0) for sl in slack for v in sl.values())


@pytest.mark.parametrize("kind", ["sage", "gcn", "sage_conv"])
def test_sampled_flip_slack_scales_with_the_rounding_unit(kind):
    om, g, saved, dlogits = setup(kind, 0.0)
    s_small, n_small = sampled_flip_slack(om, g, saved, dlogits, epoch.backward, 1e-9)
    s_big, n_big = sampled_flip_slack(om, g, saved, dlogits, epoch.backward, 2.0 ** -9 / np.sqrt(3.0))
    assert n_small < 1e-3 and all(v == 0.0 for sl in s_small for v in sl.values())
    assert n_big > n_small and any(v > 0.0 for sl in s_big for v in sl.values())
