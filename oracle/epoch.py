"""One training iteration of Algorithm 1 on one or several partitions (oracle; test
infrastructure only).

Per partition (Algorithm 1 lines 6-12): pick a DropEdge-K mask if enabled, run the L-layer
GNN forward on the masked partition graph, evaluate the reweighted loss of Eq. 3, run
backward.  Gradients of several partitions are summed (the sum over i in Eq. 2; the paper
simulates many partitions "by accumulating gradients", Appendix C), then one update is taken.

Model description: `model = {"kind": "sage"|"gcn"|"sage_conv", "layers": [param dict per layer]}`.
GCN and the conventional GraphSAGE layer use ReLU after every layer but the last.  Dropout (rate q) acts on the output of every
layer but the last.
"""
import numpy as np

from . import layers as L
from . import loss as loss_mod


def forward(model, graph, X, q=0.0, seed=0, epoch=0):
    kind = model["kind"]
    n_layers = len(model["layers"])
    H = np.asarray(X, dtype=np.float64)
    saved = []
    for l, prm in enumerate(model["layers"]):
        last = l == n_layers - 1
        drop = None if (last or q <= 0.0) else (q, seed, epoch, l)
        if kind == "sage":
            H, sv = L.sage_fwd(graph, H, prm, drop)
        elif kind == "gcn":
            H, sv = L.gcn_fwd(graph, H, prm, relu=not last, drop=drop)
        elif kind == "sage_conv":
            H, sv = L.sage_conv_fwd(graph, H, prm, relu=not last, drop=drop)
        else:
            raise ValueError(kind)
        saved.append(sv)
    return H, saved


def backward(model, graph, saved, dlogits):
    kind = model["kind"]
    grads = [None] * len(model["layers"])
    d = dlogits
    for l in range(len(model["layers"]) - 1, -1, -1):
        prm = model["layers"][l]
        if kind == "sage":
            d, g = L.sage_bwd(graph, prm, saved[l], d, need_dH=l > 0)
        elif kind == "sage_conv":
            d, g = L.sage_conv_bwd(graph, prm, saved[l], d, need_dH=l > 0)
        else:
            d, g = L.gcn_bwd(graph, prm, saved[l], d, need_dH=l > 0)
        grads[l] = g
    return grads


def partition_loss_and_grads(model, graph, X, labels, w, c=1.0, q=0.0, seed=0, epoch=0, train_mask=None):
    """Loss of Eq. 3 on one partition graph and its parameter gradients.

    Returns (loss, grads, logits) with grads a list of per-layer dicts."""
    logits, saved = forward(model, graph, X, q, seed, epoch)
    loss, dlogits = loss_mod.weighted_softmax_ce(logits, labels, w, c, train_mask)
    grads = backward(model, graph, saved, dlogits)
    return loss, grads, logits


def sum_grads(list_of_grads):
    """Sum over partitions of per-layer gradient dicts (Eq. 2's sum over i)."""
    out = [{k: np.array(v, dtype=np.float64) for k, v in layer.items()} for layer in list_of_grads[0]]
    for g in list_of_grads[1:]:
        for lo, lg in zip(out, g):
            for k in lo:
                lo[k] += lg[k]
    return out


def gradient_gap(full_grads, partition_grads):
    """Objective of Eq. 2 for given weights: || grad on the uncut graph - sum_i grad on partition i ||_F
    over all parameters.  Returns (gap, norm of the uncut gradient)."""
    total = sum_grads(partition_grads)
    gap2, ref2 = 0.0, 0.0
    for lf, lt in zip(full_grads, total):
        for k in lf:
            d = np.asarray(lf[k], np.float64) - lt[k]
            gap2 += float((d * d).sum())
            ref2 += float((np.asarray(lf[k], np.float64) ** 2).sum())
    return np.sqrt(gap2), np.sqrt(ref2)
