"""Algorithm 1 as a whole, over several iterations (oracle; test infrastructure only).

Setup (lines 1-5): every partition comes with its graph, features, labels, loss weights and,
if DropEdge-K is on, its K masks drawn once.  Each iteration t (lines 6-12): every partition
picks one of its masks, evaluates the reweighted loss of Eq. 3 on the masked graph and its
gradient; the gradients are summed over the partitions (the sum over i of Eq. 2; the paper
itself simulates many partitions by accumulating gradients, Appendix C) and one update of
the shared parameters is taken (plain gradient step as printed, or Adam as in Appendix B).
"""
import numpy as np

from . import dropedge
from . import epoch as epoch_mod
from . import step as step_mod


def train(model, parts, n_iters, c=1.0, q=0.0, dropout_seed=0, optimizer="sgd", lr=0.01,
          b1=0.9, b2=0.999, eps=1e-8, loss_fn=None):
    """Runs n_iters iterations in place on `model` and returns the per-iteration list of per-partition losses.

    parts: list of dicts with
        "part"  : partition dict (oracle.partition.build_partition)
        "X", "y": features [n_i, d] and labels of its nodes
        "w"     : loss weight per node
        "keep"  : bool [K, n_edges] DropEdge-K masks, or None
        "mask_seed": seed of the per-iteration mask choice
    loss_fn(logits, y, w, c) -> (loss, dlogits); default weighted softmax cross-entropy.
    """
    state = None
    if optimizer == "adam":
        state = [{k: (np.zeros_like(v, dtype=np.float64), np.zeros_like(v, dtype=np.float64))
                  for k, v in layer.items()} for layer in model["layers"]]
    history = []
    for t in range(n_iters):
        losses, grads = [], []
        for p in parts:
            if p.get("keep") is not None:
                k = dropedge.pick(p["mask_seed"], t, len(p["keep"]))
                graph = dropedge.masked_graph(p["part"], p["keep"][k])
            else:
                graph = dropedge.full_graph(p["part"])
            if loss_fn is None:
                L, g, _ = epoch_mod.partition_loss_and_grads(model, graph, p["X"], p["y"], p["w"], c, q,
                                                             dropout_seed, t)
            else:
                logits, saved = epoch_mod.forward(model, graph, p["X"], q, dropout_seed, t)
                L, dlogits = loss_fn(logits, p["y"], p["w"], c)
                g = epoch_mod.backward(model, graph, saved, dlogits)
            losses.append(L)
            grads.append(g)
        total = epoch_mod.sum_grads(grads)
        for l, layer in enumerate(model["layers"]):
            for name in layer:
                if optimizer == "sgd":
                    layer[name] = step_mod.sgd(layer[name], total[l][name], lr)
                elif optimizer == "adam":
                    m, v = state[l][name]
                    layer[name], m, v = step_mod.adam(layer[name], total[l][name], m, v, lr, t + 1, b1, b2, eps)
                    state[l][name] = (m, v)
                else:
                    raise ValueError(optimizer)
        history.append(losses)
    return history
