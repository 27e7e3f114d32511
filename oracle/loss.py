"""Reweighted loss of Eq. 3 with softmax cross-entropy (oracle; test infrastructure only).

    L(f, G[i]) = c * sum over v_j[i] in V[i] of  w_ij * l(h_j[i], y_j),   w_ij = D(v_j[i]) / D(v_j)

Eq. 3 is a plain sum (c = 1).  The constant c is a caller-chosen scale (e.g. 1/|V| so that the
sum over partitions estimates the full-graph mean loss).  l is softmax cross-entropy: the
accuracy-scored datasets of Section 5.1 are single-label.  An optional 0/1 train mask selects
the nodes that contribute.  float64 throughout.

Theorem 3 is stated for binary cross-entropy on a sigmoid output, which is also what a multi-label
dataset scored by micro-F1 needs: weighted_sigmoid_bce sums the C independent binary losses of a node.
"""
import numpy as np


def weighted_softmax_ce(logits, labels, w, c=1.0, train_mask=None):
    """Returns (loss, dlogits) with dlogits[j] = c * w_j * (softmax(logits_j) - onehot(y_j))."""
    z = np.asarray(logits, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    if train_mask is not None:
        w = w * (np.asarray(train_mask) != 0)
    m = z.max(axis=1, keepdims=True)
    ez = np.exp(z - m)
    se = ez.sum(axis=1, keepdims=True)
    lse = (m + np.log(se))[:, 0]
    n = z.shape[0]
    per_node = lse - z[np.arange(n), labels]
    loss = float(c) * float(np.sum(w * per_node))
    g = ez / se
    g[np.arange(n), labels] -= 1.0
    g *= (float(c) * w)[:, None]
    return loss, g


def weighted_sigmoid_bce(logits, targets, w, c=1.0, train_mask=None):
    """Multi-label loss: l(h_j, y_j) = sum_k BCE(sigmoid(z_jk), y_jk), targets in {0, 1} of shape [n, C].

    Returns (loss, dlogits) with dlogits[j, k] = c * w_j * (sigmoid(z_jk) - y_jk).
    -log sigmoid(z) = log(1 + e^-z) and -log(1 - sigmoid(z)) = log(1 + e^z) are evaluated with logaddexp,
    which does not overflow for large |z|.
    """
    z = np.asarray(logits, dtype=np.float64)
    y = np.asarray(targets, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    if train_mask is not None:
        w = w * (np.asarray(train_mask) != 0)
    per_elem = y * np.logaddexp(0.0, -z) + (1.0 - y) * np.logaddexp(0.0, z)
    loss = float(c) * float(np.sum(w * per_elem.sum(axis=1)))
    sig = np.exp(-np.logaddexp(0.0, -z))
    g = (sig - y) * (float(c) * w)[:, None]
    return loss, g
