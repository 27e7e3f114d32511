"""DropEdge-K (oracle; test infrastructure only).

Section 4.4 and Algorithm 1 lines 5-9: K DropEdge masks over the partition's edge set E[i]
are drawn once, before training; every iteration picks one of them uniformly at random and
applies it to E[i].

Readings where the paper is silent:
  * a mask has one bit per undirected edge, so both directions are kept or dropped together
    and the masked graph stays symmetric;
  * edge e is kept in mask k iff r32(seed, MASK, e, k) >= floor(p_drop * 2^32);
  * iteration t uses mask floor(r32(seed, PICK, t, 0) * K / 2^32);
  * the masked edge set simply *is* the graph of that iteration: neighbourhood means and GCN
    normalisation use the masked partition-local degrees and no 1/(1-p) rescaling is applied
    (Theorem 4's eta is not used by Algorithm 1);
  * Degree-Aware Reweighting weights are not affected by masks (Algorithm 1 computes them on
    line 4, from E[i], before the masks of line 5).
"""
import numpy as np

from . import counter_rng as crng


def masks(n_edges, K, p_drop, seed):
    """bool[K, n_edges]: True where the edge is kept."""
    if K <= 0:
        raise ValueError("K must be positive")
    thr = crng.threshold(p_drop)
    e = np.arange(n_edges, dtype=np.uint64)
    out = np.empty((K, n_edges), dtype=bool)
    for k in range(K):
        out[k] = crng.r32(seed, crng.STREAM_MASK, e, k) >= np.uint32(thr)
    return out


def pack_bits(keep):
    """uint64[ceil(E/64)] little-endian bit packing of one mask (bit e%64 of word e//64)."""
    E = keep.shape[0]
    padded = np.zeros(((E + 63) // 64) * 64, dtype=np.uint8)
    padded[:E] = keep
    return np.packbits(padded.reshape(-1, 8), axis=1, bitorder="little").reshape(-1).view("<u8").copy()


def pick(seed, t, K):
    """Index of the mask used by iteration t."""
    return int(crng.scaled_index(crng.r32(seed, crng.STREAM_PICK, np.uint64(t), 0), K))


def masked_graph(part, keep):
    """CSR of the partition graph restricted to kept edges: (rowptr int64, col int32, deg int32)."""
    sel = keep[part["eid"]]
    n = part["n_nodes"]
    rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(part["rowptr"]))[sel]
    col = part["col"][sel]
    deg = np.bincount(rows, minlength=n).astype(np.int32)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=rowptr[1:])
    return rowptr, col, deg


def full_graph(part):
    """The unmasked partition graph in the same form."""
    return part["rowptr"], part["col"], part["deg_local"]
