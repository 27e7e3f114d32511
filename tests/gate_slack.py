"""Tolerance that ReLU gates add to the gradient parity bar, computed from the oracle alone.

A ReLU gate is a decision taken on a floating-point value (the factor I(W h > 0) in the per-edge gradient of
the proof of Theorem 3).  Where the oracle's float64 pre-activation lies within the evaluation error of the
compared arithmetic, that arithmetic may take the other branch: the forward value is unaffected (ReLU is
continuous) but the gradient through the element is not, and both outcomes are valid.  Nothing here reads a
result of the HIP path: the set of gates that may differ, and how far each can move every gradient, follow
from the oracle's own state and from the rounding unit of the compared arithmetic.

Two tools:
  * worst_case_slack (float32 runs, few ambiguous gates, tight tolerance): an elementwise upper bound on the
    change of every parameter gradient when any subset of the ambiguous gates flips.  A flip of gate e
    changes the gated gradient at e by +-g_e, the gradient that arrives there; the backward pass is linear in
    that perturbation, so pushing |g_e| (for all ambiguous e at once) through a backward pass whose operands
    are replaced by their absolute values bounds the sum of the absolute changes.  One extra pass.
  * sampled_flip_slack (bfloat16 runs, a fraction of a percent of all gates ambiguous): there the worst case
    is far too pessimistic, since the flips are independent and their effects add like a random walk.  Each
    gate gets the probability of a flip that the rounding noise of its pre-activation gives it; flip patterns
    are drawn from those probabilities, the oracle's backward pass is repeated with the drawn gates, and the
    largest Frobenius deviation per gradient tensor over the draws is the slack.
"""
import numpy as np
from scipy.special import ndtr

from oracle import layers as o_layers


def _drop(d, dm):
    """Inverted-dropout backward of the oracle: `dm` = (keep, scale) or None."""
    if dm is None:
        return d
    keep, scale = dm
    return np.where(keep, d * scale, 0.0)


def ambiguous_gates(pre, margin):
    """Elements whose pre-activation lies within margin * rms(pre) of zero."""
    return np.abs(pre) < margin * np.sqrt((pre * pre).mean())


def worst_case_slack(om, graph, saved, dlogits, margin):
    """Per layer, {parameter name: elementwise bound}; also returns the number of ambiguous gates.

    om, saved: the oracle's model and the per-layer state its forward pass returned; dlogits: the oracle's
    loss gradient.  Ambiguous gates are treated as open in the absolute-value pass, so the bound also covers
    a perturbation that reaches a gate which itself flips.
    """
    kind = om["kind"]
    n_layers = len(om["layers"])
    slack = [None] * n_layers
    d = np.asarray(dlogits, dtype=np.float64)      # true gradient w.r.t. the layer output
    e = np.zeros_like(d)                           # bound on its perturbation
    n_amb = 0
    for l in range(n_layers - 1, -1, -1):
        prm, sv = om["layers"][l], saved[l]
        need = l > 0
        W = np.asarray(prm["W"], np.float64)
        if kind == "sage":
            U = np.asarray(prm["U"], np.float64)
            m = W.shape[0]
            amb = ambiguous_gates(sv["pre"], margin)
            n_amb += int(amb.sum())
            # the gradient that arrives at the gate: dZ of the true backward pass
            dP = _drop(d, sv["drop"])
            dZ = o_layers.mean_aggregate_bwd(graph, (dP @ U)[:, :m])
            # perturbation that comes from above, through |U| and the (non-negative) mean
            eP = _drop(e, sv["drop"])
            e_cat = eP @ np.abs(U)
            e_pre = np.where((sv["pre"] > 0.0) | amb, o_layers.mean_aggregate_bwd(graph, e_cat[:, :m]), 0.0)
            e_pre += np.where(amb, np.abs(dZ), 0.0)
            slack[l] = {"U": eP.T @ np.abs(sv["cat"]), "bU": eP.sum(axis=0),
                        "W": e_pre.T @ np.abs(sv["H"]), "bW": e_pre.sum(axis=0)}
            e_next = e_cat[:, m:] + e_pre @ np.abs(W) if need else None
            d_next, _ = o_layers.sage_bwd(graph, prm, sv, d, need_dH=need)
        else:
            # GCN / conventional GraphSAGE: the gate acts on the incoming gradient itself, so the bound is the
            # oracle's own backward pass on absolute-valued operands with the ambiguous gates open
            gated = bool(sv["relu"])
            amb = ambiguous_gates(sv["pre"], margin) if gated else np.zeros(sv["pre"].shape, dtype=bool)
            n_amb += int(amb.sum())
            e_in = _drop(e, sv["drop"]) + np.where(amb, np.abs(_drop(d, sv["drop"])), 0.0)
            sv_abs = dict(sv)
            sv_abs["drop"] = None
            sv_abs["pre"] = np.where((sv["pre"] > 0.0) | amb, 1.0, -1.0)
            prm_abs = {k: np.abs(np.asarray(v, np.float64)) for k, v in prm.items()}
            if kind == "gcn":
                sv_abs["AH"] = np.abs(sv["AH"])
                e_next, slack[l] = o_layers.gcn_bwd(graph, prm_abs, sv_abs, e_in, need_dH=need)
                d_next, _ = o_layers.gcn_bwd(graph, prm, sv, d, need_dH=need)
            elif kind == "sage_conv":
                sv_abs["H"], sv_abs["M"] = np.abs(sv["H"]), np.abs(sv["M"])
                e_next, slack[l] = o_layers.sage_conv_bwd(graph, prm_abs, sv_abs, e_in, need_dH=need)
                d_next, _ = o_layers.sage_conv_bwd(graph, prm, sv, d, need_dH=need)
            else:
                raise ValueError(kind)
        d, e = d_next, e_next
    return slack, n_amb


def _gate_noise_sigma(kind, prm, sv, layer, unit):
    """Standard deviation of the error of every pre-activation when its operands carry independent relative
    rounding errors of `unit` (rms): sqrt(sum_k (a_k w_k)^2) times unit, times sqrt(operands rounded).
    Layer 0 reads features the oracle sees exactly as stored, so only the parameters are rounded there; deeper
    layers read activations that were rounded on storage (and whose own inputs were), counted as one more
    rounded operand per layer."""
    W = np.asarray(prm["W"], np.float64)
    if kind == "sage":
        a = sv["H"]
    elif kind == "gcn":
        a = sv["AH"]
    else:
        a = np.concatenate([sv["H"], sv["M"]], axis=1)
    return unit * np.sqrt((a * a) @ (W * W).T) * np.sqrt(1.0 + layer)


def sampled_flip_slack(om, graph, saved, dlogits, backward, unit, draws=6, seed=0):
    """Per layer, {parameter name: Frobenius norm of the gradient change}, the largest over `draws` random gate
    patterns; also returns the expected number of flipped gates.

    backward(om, graph, saved, dlogits) is the oracle's backward pass; unit is the rms relative rounding error
    of a stored operand (bfloat16, round to nearest: 2^-9 / sqrt(3))."""
    kind = om["kind"]
    base = backward(om, graph, saved, dlogits)
    probs = []
    expected = 0.0
    for l, (prm, sv) in enumerate(zip(om["layers"], saved)):
        if kind != "sage" and not sv["relu"]:
            probs.append(None)
            continue
        sigma = _gate_noise_sigma(kind, prm, sv, l, unit)
        p = ndtr(-np.abs(sv["pre"]) / np.maximum(sigma, 1e-300))
        probs.append(p)
        expected += float(p.sum())
    rng = np.random.default_rng(seed)
    slack = [{k: 0.0 for k in g} for g in base]
    for _ in range(draws):
        flipped = []
        for sv, p in zip(saved, probs):
            s2 = dict(sv)
            if p is not None:
                s2["pre"] = np.where(rng.random(p.shape) < p, -sv["pre"], sv["pre"])
            flipped.append(s2)
        G = backward(om, graph, flipped, dlogits)
        for sl, g0, g1 in zip(slack, base, G):
            for k in sl:
                sl[k] = max(sl[k], float(np.linalg.norm(g1[k] - g0[k])))
    return slack, expected
