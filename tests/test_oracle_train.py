"""Pins for the oracle's multi-iteration driver (Algorithm 1).

A model whose graph has lost every edge is a per-node linear classifier, so training it is convex
multinomial logistic regression: the driver must reach the optimum that scipy's L-BFGS finds on that
objective written directly.  The component-aligned cut makes two partitions train exactly like the
uncut graph (Theorem 3's special case), iteration after iteration.
"""
import numpy as np
import scipy.optimize

from oracle import dropedge, partition, train
from paper_2308_03209_amd import inputs


def softmax_objective(theta, X, y, w, C):
    d = X.shape[1]
    W, b = theta[:C * d].reshape(C, d), theta[C * d:]
    z = X @ W.T + b
    z = z - z.max(1, keepdims=True)
    lse = np.log(np.exp(z).sum(1))
    return float((w * (lse - z[np.arange(len(y)), y])).sum())


def test_edgeless_gcn_training_reaches_the_logistic_regression_optimum():
    n, d, C = 60, 3, 3
    src, dst = inputs.small_random_graph(n, 120, 3)
    P = partition.build_partition(n, src, dst, 1, 0, 1)
    N = P["n_nodes"]
    rng = np.random.default_rng(0)
    X = rng.standard_normal((N, d))
    y = rng.integers(0, C, N)
    w = rng.uniform(0.5, 1.5, N)
    keep = np.zeros((1, P["n_edges"]), bool)           # the single mask drops every edge: Ahat = I
    model = {"kind": "gcn", "layers": [{"W": np.zeros((C, d)), "bW": np.zeros(C)}]}
    parts = [{"part": P, "X": X, "y": y, "w": w, "keep": keep, "mask_seed": 0}]
    hist = train.train(model, parts, 1500, c=1.0 / N, optimizer="adam", lr=0.05)
    opt = scipy.optimize.minimize(softmax_objective, np.zeros(C * d + C), args=(X, y, w / N, C), method="L-BFGS-B",
                                  options={"maxiter": 5000, "ftol": 1e-15, "gtol": 1e-10})
    assert hist[0][0] > hist[-1][0]
    assert abs(hist[-1][0] - opt.fun) < 1e-5 * abs(opt.fun), (hist[-1][0], opt.fun)
    final = softmax_objective(np.concatenate([model["layers"][0]["W"].ravel(), model["layers"][0]["bW"]]), X, y,
                              w / N, C)
    assert abs(final - opt.fun) < 1e-5 * abs(opt.fun)
    # the first recorded loss is the loss at the initial parameters: log C per unit weight
    assert np.isclose(hist[0][0], np.log(C) * w.sum() / N)


def test_component_aligned_partitions_train_like_the_uncut_graph():
    # two components, the cut follows them: no node is duplicated, all weights are 1, and the
    # summed partition gradients equal the full-graph gradient, so both runs stay identical
    edges = [(i, (i + 1) % 10) for i in range(10)] + [(0, 5), (2, 7)]
    edges += [(10 + i, 10 + (i + 3) % 10) for i in range(10)] + [(11, 12)]
    src = np.array([e[0] for e in edges])
    dst = np.array([e[1] for e in edges])
    assign = np.array([0 if e[0] < 10 else 1 for e in edges], dtype=np.int32)
    full = partition.build_partition(20, src, dst, 1, 0, 0)
    halves = [partition.build_partition(20, src, dst, 2, i, 0, assignment=assign) for i in range(2)]
    rng = np.random.default_rng(1)
    X = rng.standard_normal((20, 5))
    y = rng.integers(0, 3, 20)
    for kind, dims in [("sage", [(5, 4, 4), (4, 4, 3)]), ("sage_conv", [(5, 0, 6), (6, 0, 3)]), ("gcn", [(5, 0, 4), (4, 0, 3)])]:
        def fresh():
            prm = inputs.model_params(kind, dims, 4, random_bias=True)
            return {"kind": kind, "layers": [{k: v.astype(np.float64) for k, v in l.items()} for l in prm]}
        m_full, m_cut = fresh(), fresh()
        pf = [{"part": full, "X": X[full["local2global"]], "y": y[full["local2global"]], "w": full["dar_weight"]}]
        pc = [{"part": h, "X": X[h["local2global"]], "y": y[h["local2global"]], "w": h["dar_weight"]} for h in halves]
        assert all(np.all(h["dar_weight"] == 1.0) for h in halves)
        hf = train.train(m_full, pf, 6, c=0.05, optimizer="adam", lr=0.02)
        hc = train.train(m_cut, pc, 6, c=0.05, optimizer="adam", lr=0.02)
        for a, b in zip(hf, hc):
            assert np.isclose(a[0], sum(b), rtol=1e-10)
        for la, lb in zip(m_full["layers"], m_cut["layers"]):
            for k in la:
                assert np.allclose(la[k], lb[k], rtol=1e-7, atol=1e-10), (kind, k)
        assert hf[-1][0] < hf[0][0]


def test_sgd_driver_first_two_iterations_by_hand():
    # one node pair, 1-layer GCN, identity-free arithmetic small enough to follow by hand:
    # logits z = Ahat X W^T, Ahat = [[.5,.5],[.5,.5]], X = [[2],[4]] -> both rows see 3
    P = partition.build_partition(2, [0], [1], 1, 0, 0)
    model = {"kind": "gcn", "layers": [{"W": np.array([[0.0], [0.0]]), "bW": np.zeros(2)}]}
    parts = [{"part": P, "X": np.array([[2.0], [4.0]]), "y": np.array([0, 0]), "w": np.ones(2)}]
    hist = train.train(model, parts, 2, c=1.0, optimizer="sgd", lr=0.1)
    # iteration 0: softmax = (.5,.5) for both nodes; dz = (-.5, .5) each; dW = sum dz * 3 = (-3, 3); db = (-1, 1)
    assert np.isclose(hist[0][0], 2 * np.log(2))
    W1, b1 = np.array([[0.3], [-0.3]]), np.array([0.1, -0.1])
    z = 3 * W1[:, 0] + b1
    L1 = 2 * (np.log(np.exp(z).sum()) - z[0])
    assert np.isclose(hist[1][0], L1)
    pr = np.exp(z) / np.exp(z).sum()
    dz = pr - np.array([1.0, 0.0])
    assert np.allclose(model["layers"][0]["W"][:, 0], W1[:, 0] - 0.1 * 2 * 3 * dz)
    assert np.allclose(model["layers"][0]["bW"], b1 - 0.1 * 2 * dz)
