"""GNN layers on one (masked) partition graph, forward and backward (oracle; test infrastructure only).

GraphSAGE-mean is the layer printed in Section 3:
    h_v' = U . CONCAT( MEAN{ ReLU(W h_u) : u in N(v) }, h_v )
with N(v) the neighbours of v *in the partition* (the proof of Theorem 3 normalises an edge's
gradient by the partition-local degree D(v_j[i])).  GCN is only cited by the paper; its
textbook form (Kipf & Welling) on the partition graph is used:
    H' = act( S (A + I) S . H . W^T + b ),  S = diag(1 / sqrt(deg_v + 1)).

The conventional GraphSAGE-mean layer (the stock library layer the experiments of Section 5.1 ran;
Hamilton et al.'s mean aggregator on raw features) is
    h_v' = act( W_self h_v + W_neigh . MEAN{ h_u : u in N(v) } + b ).

Readings where the paper is silent: biases bW, bU exist; a node without neighbours has a zero
mean; there is no activation after U; inverted dropout with rate q acts on a layer's output.

All arithmetic is float64.  Graph = (rowptr, col, deg) with ascending neighbour ids per row.
The forward aggregation is a gather written row by row; the backward aggregation is the
scatter the chain rule gives (each edge (v,u) sends dA[v]/deg(v) to u).
"""
import numpy as np

from . import counter_rng as crng


def dropout_keep(n_rows, d, q, seed, epoch, layer_id):
    """bool[n_rows, d] keep decisions of inverted dropout with rate q.

    Element (r, c) has linear index i = r*d + c; it takes word i%4 of
    words(seed, DROPOUT + 256*layer_id, i div 4, epoch) and is kept iff word >= floor(q*2^32).
    """
    thr = crng.threshold(float(np.float32(q)))   # the rate is a float32 at the library boundary
    total = n_rows * d
    quads = np.arange((total + 3) // 4, dtype=np.uint64)
    w = crng.words(seed, crng.STREAM_DROPOUT + 256 * int(layer_id), quads, int(epoch) & 0xFFFFFFFF)
    flat = np.stack(w, axis=1).reshape(-1)[:total]
    return (flat >= np.uint32(thr)).reshape(n_rows, d)


def mean_aggregate(graph, Z):
    """A[v] = mean of Z[u] over u in N(v); zero for a node without neighbours."""
    rowptr, col, deg = graph
    A = np.zeros_like(Z, dtype=np.float64)
    for v in range(len(deg)):
        a, b = rowptr[v], rowptr[v + 1]
        if b > a:
            A[v] = Z[col[a:b]].sum(axis=0) / float(b - a)
    return A


def mean_aggregate_bwd(graph, dA):
    """dZ[u] = sum over v with u in N(v) of dA[v] / deg(v)."""
    rowptr, col, deg = graph
    dZ = np.zeros_like(dA, dtype=np.float64)
    for v in range(len(deg)):
        a, b = rowptr[v], rowptr[v + 1]
        if b > a:
            dZ[col[a:b]] += dA[v] / float(b - a)   # neighbour ids are distinct within a row
    return dZ


def gcn_aggregate(graph, X):
    """Y[v] = sum over u in N(v) + {v} of X[u] / sqrt((deg_u + 1)(deg_v + 1))."""
    rowptr, col, deg = graph
    s = 1.0 / np.sqrt(deg.astype(np.float64) + 1.0)
    Y = np.zeros_like(X, dtype=np.float64)
    for v in range(len(deg)):
        a, b = rowptr[v], rowptr[v + 1]
        acc = s[v] * X[v]
        if b > a:
            nb = col[a:b]
            acc = acc + (s[nb][:, None] * X[nb]).sum(axis=0)
        Y[v] = s[v] * acc
    return Y


def gcn_aggregate_bwd(graph, dY):
    """Transpose of gcn_aggregate, as a scatter: edge (v,u) sends s_v s_u dY[v] to u."""
    rowptr, col, deg = graph
    s = 1.0 / np.sqrt(deg.astype(np.float64) + 1.0)
    dX = np.zeros_like(dY, dtype=np.float64)
    for v in range(len(deg)):
        a, b = rowptr[v], rowptr[v + 1]
        dX[v] += s[v] * s[v] * dY[v]
        if b > a:
            nb = col[a:b]
            dX[nb] += (s[v] * s[nb])[:, None] * dY[v][None, :]
    return dX


def _apply_dropout(P, drop):
    if drop is None:
        return P, None
    q, seed, epoch, layer_id = drop
    if q <= 0.0:
        return P, None
    keep = dropout_keep(P.shape[0], P.shape[1], q, seed, epoch, layer_id)
    scale = 1.0 / (1.0 - float(np.float32(q)))
    return np.where(keep, P * scale, 0.0), (keep, scale)


def sage_fwd(graph, H, prm, drop=None):
    """One GraphSAGE-mean layer.  prm: W [d_msg,d_in], bW, U [d_out, d_msg+d_in], bU.

    drop = (q, seed, epoch, layer_id) or None.  Returns (H_out, saved)."""
    H = np.asarray(H, dtype=np.float64)
    W, bW, U, bU = (np.asarray(prm[k], dtype=np.float64) for k in ("W", "bW", "U", "bU"))
    pre = H @ W.T + bW
    Z = np.maximum(pre, 0.0)
    A = mean_aggregate(graph, Z)
    cat = np.concatenate([A, H], axis=1)
    P = cat @ U.T + bU
    out, dm = _apply_dropout(P, drop)
    return out, {"H": H, "pre": pre, "Z": Z, "A": A, "cat": cat, "drop": dm}


def sage_bwd(graph, prm, saved, dH_out, need_dH=True):
    """Gradients of one GraphSAGE-mean layer: returns (dH_in or None, {dW, dbW, dU, dbU})."""
    W, U = np.asarray(prm["W"], np.float64), np.asarray(prm["U"], np.float64)
    d_msg = W.shape[0]
    dP = np.asarray(dH_out, dtype=np.float64)
    if saved["drop"] is not None:
        keep, scale = saved["drop"]
        dP = np.where(keep, dP * scale, 0.0)
    dU = dP.T @ saved["cat"]
    dbU = dP.sum(axis=0)
    dcat = dP @ U
    dA, dH_self = dcat[:, :d_msg], dcat[:, d_msg:]
    dZ = mean_aggregate_bwd(graph, dA)
    dpre = np.where(saved["pre"] > 0.0, dZ, 0.0)
    dW = dpre.T @ saved["H"]
    dbW = dpre.sum(axis=0)
    dH = dH_self + dpre @ W if need_dH else None
    return dH, {"W": dW, "bW": dbW, "U": dU, "bU": dbU}


def gcn_fwd(graph, H, prm, relu=True, drop=None):
    """One GCN layer: act(Ahat H W^T + b).  prm: W [d_out, d_in], bW [d_out]."""
    H = np.asarray(H, dtype=np.float64)
    W, b = np.asarray(prm["W"], np.float64), np.asarray(prm["bW"], np.float64)
    AH = gcn_aggregate(graph, H)
    pre = AH @ W.T + b
    act = np.maximum(pre, 0.0) if relu else pre
    out, dm = _apply_dropout(act, drop)
    return out, {"AH": AH, "pre": pre, "relu": relu, "drop": dm}


def gcn_bwd(graph, prm, saved, dH_out, need_dH=True):
    W = np.asarray(prm["W"], np.float64)
    d = np.asarray(dH_out, dtype=np.float64)
    if saved["drop"] is not None:
        keep, scale = saved["drop"]
        d = np.where(keep, d * scale, 0.0)
    if saved["relu"]:
        d = np.where(saved["pre"] > 0.0, d, 0.0)
    dW = d.T @ saved["AH"]
    db = d.sum(axis=0)
    dH = gcn_aggregate_bwd(graph, d @ W) if need_dH else None
    return dH, {"W": dW, "bW": db}


def sage_conv_fwd(graph, H, prm, relu=True, drop=None):
    """One conventional GraphSAGE-mean layer: act(H W_self^T + mean_N(H) W_neigh^T + b).

    prm: W [d_out, 2 d_in] = [W_self | W_neigh] (self block first), bW [d_out]."""
    H = np.asarray(H, dtype=np.float64)
    W, b = np.asarray(prm["W"], np.float64), np.asarray(prm["bW"], np.float64)
    d_in = H.shape[1]
    M = mean_aggregate(graph, H)
    pre = H @ W[:, :d_in].T + M @ W[:, d_in:].T + b
    act = np.maximum(pre, 0.0) if relu else pre
    out, dm = _apply_dropout(act, drop)
    return out, {"H": H, "M": M, "pre": pre, "relu": relu, "drop": dm}


def sage_conv_bwd(graph, prm, saved, dH_out, need_dH=True):
    W = np.asarray(prm["W"], np.float64)
    d_in = saved["H"].shape[1]
    d = np.asarray(dH_out, dtype=np.float64)
    if saved["drop"] is not None:
        keep, scale = saved["drop"]
        d = np.where(keep, d * scale, 0.0)
    if saved["relu"]:
        d = np.where(saved["pre"] > 0.0, d, 0.0)
    dW = np.concatenate([d.T @ saved["H"], d.T @ saved["M"]], axis=1)
    db = d.sum(axis=0)
    dH = d @ W[:, :d_in] + mean_aggregate_bwd(graph, d @ W[:, d_in:]) if need_dH else None
    return dH, {"W": dW, "bW": db}
