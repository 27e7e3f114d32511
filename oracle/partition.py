"""Random vertex cut and per-partition structures (oracle; test infrastructure only).

Follows Section 3 "Vertex Cut Partitioning": the edge set is split into p disjoint subsets
E[i] whose union is E; V[i] is the set of endpoints of E[i], so nodes are replicated.  The
only cut the paper specifies completely is the random one used in the proof of Theorem 2
(each edge goes to one of the p partitions uniformly at random); that is the cut built here.
Degree-Aware Reweighting (Section 4.3, Algorithm 1 line 4): w_ij = D(v_j[i]) / D(v_j).
Replication factor: Eq. 1.

A second, degree-aware hash cut is offered (method="dbh"): Appendix A remarks that cutting the
higher-degree vertices leaves fewer mirror vertices, and the degree-based hashing partitioner compared in
Appendix C does so by hashing every edge on its lower-degree endpoint, so that all edges of a low-degree
node land in one partition and only high-degree nodes get replicated.

Readings where the paper is silent (shared with the HIP library, implemented separately):
  * an edge's partition = floor(r32(seed, CUT, lo + 2^32 * hi, 0) * p / 2^32) with (lo, hi) the
    sorted global endpoint ids, so the cut does not depend on the order edges are listed in;
  * degree-aware cut: pivot = the endpoint of smaller global degree (the smaller id on a tie);
    partition = floor(r32(seed, CUT, pivot, 1) * p / 2^32);
  * local ids number V[i] by ascending global id;
  * CSR rows hold neighbour local ids in ascending order, both directions of every edge;
  * undirected edge id = rank of (lo_local, hi_local) in lexicographic order;
  * D(.) counts distinct neighbours; self-loops are rejected; degrees are taken before masking;
  * w = float32(float64(D_i) / float64(D)).
"""
import numpy as np

from . import counter_rng as crng


def canonical_edges(n_nodes, src, dst, dedup=False):
    """Validate an undirected edge list and return sorted unique (lo, hi) global pairs."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    if src.shape != dst.shape or src.ndim != 1:
        raise ValueError("src/dst must be 1-d arrays of equal length")
    if n_nodes <= 0 or n_nodes > (1 << 32):
        raise ValueError("n_nodes out of range")
    if src.size and (min(src.min(), dst.min()) < 0 or max(src.max(), dst.max()) >= n_nodes):
        raise ValueError("node id out of range")
    if np.any(src == dst):
        raise ValueError("self-loop")
    lo = np.minimum(src, dst)
    hi = np.maximum(src, dst)
    order = np.lexsort((hi, lo))
    lo, hi = lo[order], hi[order]
    if lo.size:
        dup = (lo[1:] == lo[:-1]) & (hi[1:] == hi[:-1])
        if dup.any():
            if not dedup:
                raise ValueError("duplicate edge")
            keep = np.r_[True, ~dup]
            lo, hi = lo[keep], hi[keep]
    return lo, hi


def assign_edges(lo, hi, n_parts, seed):
    """Partition index of every canonical edge under the seeded random cut."""
    a = lo.astype(np.uint64) | (hi.astype(np.uint64) << np.uint64(32))
    r = crng.r32(seed, crng.STREAM_CUT, a, 0)
    return crng.scaled_index(r, n_parts)


def assign_edges_dbh(lo, hi, deg_g, n_parts, seed):
    """Partition index of every canonical edge under the degree-aware hash cut."""
    pivot = np.where(deg_g[hi] < deg_g[lo], hi, lo)
    r = crng.r32(seed, crng.STREAM_CUT, pivot.astype(np.uint64), 1)
    return crng.scaled_index(r, n_parts)


def global_degrees(n_nodes, lo, hi):
    """D(v): number of distinct neighbours in the full graph."""
    return (np.bincount(lo, minlength=n_nodes) + np.bincount(hi, minlength=n_nodes)).astype(np.int64)


def build_partition(n_nodes, src, dst, n_parts, part_id, seed, assignment=None, dedup=False, method="random"):
    """Structures of partition `part_id`.

    method: "random" (the cut of the proof of Theorem 2) or "dbh" (degree-aware hash).

    assignment: optional int array giving the partition of each *input* edge (same order as
    src/dst); overrides the seeded hash (used by tests that need a hand-made cut).

    Returns a dict:
      n_nodes, n_edges, nnz           sizes of the partition (nnz = 2 * n_edges)
      local2global int64[n_nodes]     duplicated-node map (ascending)
      rowptr int64[n_nodes+1], col int32[nnz], eid int32[nnz]
      edge_lo, edge_hi int32[n_edges] local endpoints of undirected edge e (lo < hi)
      deg_local int32[n_nodes], deg_global int32[n_nodes], dar_weight float32[n_nodes]
    """
    if n_parts <= 0 or not (0 <= part_id < n_parts):
        raise ValueError("bad n_parts / part_id")
    if assignment is None:
        lo, hi = canonical_edges(n_nodes, src, dst, dedup)
        if method == "random":
            part = assign_edges(lo, hi, n_parts, seed)
        elif method == "dbh":
            part = assign_edges_dbh(lo, hi, global_degrees(n_nodes, lo, hi), n_parts, seed)
        else:
            raise ValueError(method)
    else:
        src = np.asarray(src, dtype=np.int64)
        dst = np.asarray(dst, dtype=np.int64)
        assignment = np.asarray(assignment, dtype=np.int64)
        if assignment.shape != src.shape:
            raise ValueError("assignment length")
        if assignment.size and (assignment.min() < 0 or assignment.max() >= n_parts):
            raise ValueError("assignment out of range")
        canonical_edges(n_nodes, src, dst, dedup=False)  # validation only
        lo0 = np.minimum(src, dst)
        hi0 = np.maximum(src, dst)
        order = np.lexsort((hi0, lo0))
        lo, hi, part = lo0[order], hi0[order], assignment[order]
    deg_g = global_degrees(n_nodes, lo, hi)
    mine = part == part_id
    return _structures(lo[mine], hi[mine], deg_g)


def _structures(glo, ghi, deg_g):
    """Partition dict from the partition's own edges - lexicographically sorted, unique (lo, hi) global pairs -
    and the global degree of every node of the full graph."""
    n_edges = int(glo.size)
    if 2 * n_edges >= (1 << 31):
        raise ValueError("partition too large for int32 edge ids")
    local2global = np.union1d(glo, ghi).astype(np.int64)
    n_loc = int(local2global.size)
    llo = np.searchsorted(local2global, glo).astype(np.int32)
    lhi = np.searchsorted(local2global, ghi).astype(np.int32)
    # (glo, ghi) is already lexicographically sorted and the local numbering is monotone,
    # so position in this list is the undirected edge id.
    e = np.arange(n_edges, dtype=np.int32)
    rows = np.concatenate([llo, lhi]).astype(np.int64)
    cols = np.concatenate([lhi, llo]).astype(np.int32)
    eids = np.concatenate([e, e])
    order = np.lexsort((cols, rows))
    rows, cols, eids = rows[order], cols[order], eids[order]
    deg_l = np.bincount(rows, minlength=n_loc).astype(np.int32)
    rowptr = np.zeros(n_loc + 1, dtype=np.int64)
    np.cumsum(deg_l, out=rowptr[1:])
    dg = deg_g[local2global].astype(np.int32)
    w = (deg_l.astype(np.float64) / dg.astype(np.float64)).astype(np.float32)
    return {
        "n_nodes": n_loc, "n_edges": n_edges, "nnz": 2 * n_edges,
        "local2global": local2global, "rowptr": rowptr, "col": cols, "eid": eids,
        "edge_lo": llo, "edge_hi": lhi,
        "deg_local": deg_l, "deg_global": dg, "dar_weight": w,
    }


def build_partition_chunked(n_nodes, pieces, n_parts, part_id, seed, dedup=False):
    """Partition `part_id` of the random cut when the edge list arrives in pieces (an iterable of (src, dst)
    array pairs), as for a graph too large to hold: under the random cut every edge is assigned by itself
    (proof of Theorem 2), so a piece is reduced at once to the edges it contributes to E[part_id], while the
    global degrees D(v) of Degree-Aware Reweighting are counted over everything that passes.

    Repeats inside a piece are dropped (dedup) or rejected; copies of an edge in different pieces are the
    caller's error and are detected only where they fall into this partition."""
    if n_parts <= 0 or not (0 <= part_id < n_parts):
        raise ValueError("bad n_parts / part_id")
    deg_g = np.zeros(n_nodes, dtype=np.int64)
    keep_lo, keep_hi = [], []
    for src, dst in pieces:
        lo, hi = canonical_edges(n_nodes, src, dst, dedup)
        deg_g += global_degrees(n_nodes, lo, hi)
        mine = assign_edges(lo, hi, n_parts, seed) == part_id
        keep_lo.append(lo[mine])
        keep_hi.append(hi[mine])
    glo = np.concatenate(keep_lo) if keep_lo else np.zeros(0, np.int64)
    ghi = np.concatenate(keep_hi) if keep_hi else np.zeros(0, np.int64)
    order = np.lexsort((ghi, glo))
    glo, ghi = glo[order], ghi[order]
    if glo.size and np.any((glo[1:] == glo[:-1]) & (ghi[1:] == ghi[:-1])):
        raise ValueError("an edge arrived in more than one piece")
    return _structures(glo, ghi, deg_g)


def replication_factor(n_nodes_full, partitions):
    """Eq. 1: RF = (1/|V|) * sum_i |V[i]|."""
    return sum(p["n_nodes"] for p in partitions) / float(n_nodes_full)


def node_replication(n_nodes_full, partitions):
    """RF(v_j) = number of partitions that contain v_j."""
    rf = np.zeros(n_nodes_full, dtype=np.int64)
    for p in partitions:
        rf[p["local2global"]] += 1
    return rf


def loss_weights(part, kind="dar", node_rf=None):
    """Per-node loss weights of a partition: 'dar' (Eq. 3), 'none' (all ones), or
    'inv_rf' (1 / RF(v_j), the "vanilla-inv" ablation of Table 3)."""
    if kind == "dar":
        return part["dar_weight"].copy()
    if kind == "none":
        return np.ones(part["n_nodes"], dtype=np.float32)
    if kind == "inv_rf":
        return (1.0 / node_rf[part["local2global"]].astype(np.float64)).astype(np.float32)
    raise ValueError(kind)
