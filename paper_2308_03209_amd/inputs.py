"""Seeded synthetic inputs shaped like the paper's workloads (Section 5.1 "Datasets").

The paper trains on Reddit, Yelp, ogbn-products and ogbn-papers100M.  None of
those datasets is available here, so every graph, feature matrix, label vector
and parameter set is synthetic: Chung-Lu power-law graphs with the node / edge
counts the paper states for its datasets, N(0,1) features, uniform labels and
Glorot-uniform weights.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests.  It contains no arithmetic of the method itself (no hashing of
edges to partitions, no masks, no layers): it only draws inputs with numpy's
PCG64 generator from fixed seeds.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import List, Optional, Tuple

import numpy as np

# Fixed seeds (printed by the bench).
SEED_GRAPH = 1000      # + config index
SEED_PERM = 2000       # + config index
SEED_CUT = 42
SEED_MASKS = 7
SEED_FEATURES = 99
SEED_LABELS = 100
SEED_PARAMS = 101
SEED_DROPOUT = 55


@dataclass(frozen=True)
class Workload:
    """One named training configuration (graph recipe + model shape)."""
    name: str
    index: int
    kind: str                 # "gcn" | "sage" (the layer as printed) | "sage_conv" (conventional GraphSAGE-mean)
    dtype: str                # "f32" | "bf16"  (storage of features / activations)
    n_nodes: int
    nnz_directed: int         # target number of directed adjacency entries of the full graph
    gamma: float              # power-law exponent of the degree distribution
    max_degree: Optional[int]  # cap on the largest expected degree (None: sqrt(nnz))
    d_feat: int
    hidden: int
    n_layers: int
    n_classes: int
    n_parts: int
    train_parts: Tuple[int, ...] = (0,)
    dropedge_K: int = 0       # 0: DropEdge-K off
    dropedge_p: float = 0.0
    dar: bool = True
    dropout: float = 0.0      # rate on the output of every layer but the last
    optimizer: str = "sgd"    # "sgd" (Algorithm 1 as printed) | "adam" (the experiments' optimiser)
    lr: float = 0.01
    loss: str = "softmax_ce"  # "softmax_ce" | "sigmoid_bce" (multi-label targets)
    stream: bool = False      # graph drawn by the block-wise generator (power_law_edge_stream): never held whole

    def layer_dims(self) -> List[Tuple[int, int, int]]:
        """(d_in, d_msg, d_out) per layer; d_msg = hidden for every layer (only "sage" uses it)."""
        dims = []
        d_in = self.d_feat
        for l in range(self.n_layers):
            d_out = self.n_classes if l == self.n_layers - 1 else self.hidden
            dims.append((d_in, self.hidden, d_out))
            d_in = d_out
        return dims

    def scaled(self, factor: float) -> "Workload":
        """Same recipe with node and edge counts multiplied by `factor` (average degree kept)."""
        n = max(16, int(round(self.n_nodes * factor)))
        nnz = max(2 * n, int(round(self.nnz_directed * factor)))
        md = self.max_degree
        return replace(self, name=f"{self.name}@x{factor:g}", n_nodes=n, nnz_directed=nnz, max_degree=md)


WORKLOADS = [
    Workload("cfg0-gcn2-f32-2k", 0, "gcn", "f32", 2_000, 40_000, 2.2, None, 64, 16, 2, 8, 4),
    Workload("cfg1-sage2-f32-reddit-shaped", 1, "sage", "f32", 230_000, 114_000_000, 2.1, None,
             602, 256, 2, 41, 8),
    Workload("cfg2-sage3-bf16-products-shaped", 2, "sage", "bf16", 2_400_000, 62_000_000, 2.3, None,
             100, 256, 3, 47, 8, (0,), 4, 0.5),
    Workload("cfg3-gcn3-bf16-papers100M-shaped", 3, "gcn", "bf16", 110_000_000, 1_600_000_000, 2.0,
             100_000, 128, 256, 3, 172, 16, stream=True),
    Workload("cfg4-gcn4-f32-products-shaped-allparts", 4, "gcn", "f32", 2_400_000, 62_000_000, 2.3, None,
             100, 512, 4, 47, 8, tuple(range(8)), 8, 0.5),
    # Beyond the five benchmark configurations: the models of the paper's experiments (Appendix B: depth,
    # width, dropout, Adam and its learning rate; DropEdge-K with K = 10, ratio 0.5 as in Section 5.1) with
    # conventional GraphSAGE-mean layers, on graphs of the datasets' sizes.
    Workload("ext5-sageconv4-f32-reddit-shaped", 5, "sage_conv", "f32", 230_000, 114_000_000, 2.1, None,
             602, 256, 4, 41, 8, (0,), 10, 0.5, True, 0.3, "adam", 0.01),
    Workload("ext6-sageconv3-bf16-products-shaped", 6, "sage_conv", "bf16", 2_400_000, 62_000_000, 2.3, None,
             100, 128, 3, 47, 8, (0,), 10, 0.5, True, 0.3, "adam", 0.003),
    # multi-label (micro-F1 scored in the paper): 100 independent labels, sigmoid + BCE loss
    Workload("ext7-sageconv4-f32-yelp-shaped", 7, "sage_conv", "f32", 716_000, 14_000_000, 2.4, None,
             300, 512, 4, 100, 8, (0,), 10, 0.5, True, 0.1, "adam", 0.01, "sigmoid_bce"),
]


def expected_degrees(n: int, nnz: int, gamma: float, max_degree: Optional[int]) -> np.ndarray:
    """Chung-Lu expected-degree sequence w_v = c (v + v0)^(-1/(gamma-1)), sum = nnz, max = cap."""
    alpha = 1.0 / (gamma - 1.0)
    cap = float(np.sqrt(nnz))
    if max_degree is not None:
        cap = min(cap, float(max_degree))
    cap = min(cap, float(n - 1))
    v = np.arange(n, dtype=np.float64)

    def wmax_for(v0: float) -> float:
        w = (v + v0) ** (-alpha)
        return float(nnz * w[0] / w.sum())

    lo, hi = 1e-6, float(n) * 1e3
    if wmax_for(hi) > cap:   # degenerate: nearly uniform degrees
        v0 = hi
    else:
        for _ in range(200):
            mid = np.sqrt(lo * hi)
            if wmax_for(mid) > cap:
                lo = mid
            else:
                hi = mid
        v0 = hi
    w = (v + v0) ** (-alpha)
    return w * (nnz / w.sum())


def chung_lu_edges(n: int, nnz: int, gamma: float, max_degree: Optional[int],
                   seed_graph: int, seed_perm: int, chunk: int = 1 << 24,
                   progress=None) -> Tuple[np.ndarray, np.ndarray]:
    """Undirected simple power-law graph as (src, dst) int64 arrays, one entry per edge.

    Endpoint pairs are drawn with probability proportional to w_u * w_v, self-loops and
    duplicates are dropped, and node ids are then shuffled so that degree is not
    monotone in id.  About nnz/2 undirected edges result (slightly fewer after dedup).
    progress(text), if given, is called now and then on long runs.
    """
    w = expected_degrees(n, nnz, gamma, max_degree)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    rng = np.random.Generator(np.random.PCG64(seed_graph))
    m = nnz // 2
    keys = []
    done = 0
    while done < m:
        c = min(chunk, m - done)
        a = np.searchsorted(cdf, rng.random(c), side="right")
        b = np.searchsorted(cdf, rng.random(c), side="right")
        np.minimum(a, n - 1, out=a)
        np.minimum(b, n - 1, out=b)
        lo = np.minimum(a, b)
        hi = np.maximum(a, b)
        ok = lo != hi
        keys.append(lo[ok].astype(np.int64) * n + hi[ok])
        done += c
        if progress is not None and (done == m or (done // chunk) % 4 == 0):
            progress(f"drew {done} of {m} endpoint pairs")
    key = np.concatenate(keys)
    del keys
    if progress is not None:
        progress(f"sorting {key.shape[0]} edge keys")
    key.sort()
    if key.shape[0]:
        key = key[np.r_[True, key[1:] != key[:-1]]]
    if progress is not None:
        progress(f"{key.shape[0]} distinct edges; relabelling")
    perm = np.random.Generator(np.random.PCG64(seed_perm)).permutation(n).astype(np.int64)
    src = perm[key // n]
    dst = perm[key % n]
    # random orientation of each stored pair, so that callers cannot rely on src < dst
    flip = np.random.Generator(np.random.PCG64(seed_perm + 1)).random(src.shape[0]) < 0.5
    s2 = np.where(flip, dst, src)
    d2 = np.where(flip, src, dst)
    return s2, d2


class PowerLawStream:
    """Block-wise Chung-Lu generator for graphs whose edge list is never held whole (the 1.6-billion-entry,
    papers100M-shaped workload).

    Expected degrees follow the same power law as expected_degrees(), in its integrated form: rank r (0 = the
    largest hub) has weight w_r = c * integral_r^{r+1} (x + v0)^(-alpha) dx, alpha = 1 / (gamma - 1), with c and
    v0 set so that sum w = nnz and w_0 = min(sqrt(nnz), max_degree, n - 1).  Every cumulative weight is then a
    closed form, so a partner is drawn by inverting it - no table of n entries.

    The multigraph "nnz / 2 endpoint pairs drawn with probability proportional to w_a w_b" is drawn grouped by
    the endpoint of smaller rank: rank a owns Poisson(w_a T_a / nnz) pairs, T_a = sum of the weights of the
    ranks above a, each with a partner b > a drawn proportional to w_b.  All copies of a pair therefore come
    out of the same block of ranks, where they are dropped, so the stream as a whole is duplicate-free -
    which is what lets a consumer count degrees on the fly.  Ranks are mapped to node ids by a seeded
    permutation and every pair gets a random orientation.  Block k depends on (seed, k) only.
    """

    def __init__(self, n: int, nnz: int, gamma: float, max_degree: Optional[int], seed_graph: int, seed_perm: int,
                 block_pairs: int = 1 << 24):
        self.n, self.nnz = int(n), int(nnz)
        self.alpha = 1.0 / (gamma - 1.0)
        self.seed_graph, self.seed_perm = int(seed_graph), int(seed_perm)
        cap = float(np.sqrt(nnz))
        if max_degree is not None:
            cap = min(cap, float(max_degree))
        cap = min(cap, float(n - 1))

        def w0_for(v0: float) -> float:
            return nnz * (self._G(1.0, v0) - self._G(0.0, v0)) / (self._G(float(n), v0) - self._G(0.0, v0))

        lo, hi = 1e-9, float(n) * 1e3
        if w0_for(hi) > cap:
            v0 = hi
        else:
            for _ in range(300):
                mid = float(np.sqrt(lo * hi))
                if w0_for(mid) > cap:
                    lo = mid
                else:
                    hi = mid
            v0 = hi
        self.v0 = v0
        self.G0, self.Gn = self._G(0.0, v0), self._G(float(n), v0)
        self.c = nnz / (self.Gn - self.G0)
        # block boundaries in rank space: equal shares of the expected number of pairs, from the integral of
        # w_a T_a / nnz over the ranks, (c^2 / nnz) (Fn F - F^2 / 2) with F(x) = G(x) - G(0)
        Fn = self.Gn - self.G0
        n_blocks = max(1, int(np.ceil((nnz / 2) / block_pairs)))
        share = (np.arange(1, n_blocks, dtype=np.float64) / n_blocks) * (nnz / 2)
        F = Fn - np.sqrt(np.maximum(Fn * Fn - 2.0 * nnz * share / (self.c * self.c), 0.0))
        cuts = np.floor(self._G_inv(F + self.G0)).astype(np.int64)
        self.bounds = np.unique(np.concatenate([[0], np.clip(cuts, 0, n - 1), [n - 1]]))   # rank n-1 owns nothing
        self._perm = None

    def _G(self, x, v0=None):
        """Antiderivative of (x + v0)^(-alpha)."""
        v0 = self.v0 if v0 is None else v0
        if abs(self.alpha - 1.0) < 1e-12:
            return np.log(x + v0)
        return (x + v0) ** (1.0 - self.alpha) / (1.0 - self.alpha)

    def _G_inv(self, y):
        if abs(self.alpha - 1.0) < 1e-12:
            return np.exp(y) - self.v0
        return (y * (1.0 - self.alpha)) ** (1.0 / (1.0 - self.alpha)) - self.v0

    @property
    def n_blocks(self) -> int:
        return len(self.bounds) - 1

    def perm(self) -> np.ndarray:
        if self._perm is None:
            self._perm = np.random.Generator(np.random.PCG64(self.seed_perm)).permutation(self.n).astype(np.uint32 if self.n <= (1 << 32) else np.int64)
        return self._perm

    def block(self, k: int) -> Tuple[np.ndarray, np.ndarray]:
        """(src, dst) int64 arrays of the pairs owned by the ranks of block k, duplicate-free."""
        r0, r1 = int(self.bounds[k]), int(self.bounds[k + 1])
        rng = np.random.Generator(np.random.PCG64([self.seed_graph, k]))
        a = np.arange(r0, r1, dtype=np.int64)
        G_hi = self._G(a + 1.0)
        lam = self.c * (G_hi - self._G(a.astype(np.float64))) * self.c * (self.Gn - G_hi) / self.nnz
        cnt = rng.poisson(lam)
        owner = np.repeat(a, cnt)
        G_own = np.repeat(G_hi, cnt)
        del a, lam, cnt, G_hi
        # target = G_own + u * (Gn - G_own), in place
        target = rng.random(owner.shape[0])
        np.subtract(self.Gn, G_own, out=G_own)
        target *= G_own
        np.subtract(self.Gn, G_own, out=G_own)
        target += G_own
        del G_own
        b = np.floor(self._G_inv(target)).astype(np.int64)
        del target
        np.clip(b, owner + 1, self.n - 1, out=b)
        # one 64-bit key per pair (owner rank in the high word), sorted, repeats dropped
        owner <<= 32
        owner |= b
        del b
        owner.sort()
        if owner.shape[0]:
            owner = owner[np.r_[True, owner[1:] != owner[:-1]]]
        perm = self.perm()
        src = perm[owner >> 32].astype(np.int64)
        owner &= 0xFFFFFFFF
        dst = perm[owner].astype(np.int64)
        del owner
        # random orientation: swap the two arrays where the coin says so
        flip = rng.random(src.shape[0]) < 0.5
        tmp = src[flip]
        src[flip] = dst[flip]
        dst[flip] = tmp
        return src, dst

    def blocks(self, workers: int = 1):
        """Yields the blocks in order; with workers > 1 up to that many are drawn ahead on threads (numpy
        releases the interpreter lock in its sorts, draws and elementwise loops)."""
        self.perm()
        if workers <= 1:
            for k in range(self.n_blocks):
                yield self.block(k)
            return
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=workers) as pool:
            pending = [pool.submit(self.block, k) for k in range(min(workers, self.n_blocks))]
            nxt = len(pending)
            while pending:
                out = pending.pop(0).result()
                if nxt < self.n_blocks:
                    pending.append(pool.submit(self.block, nxt))
                    nxt += 1
                yield out


def workload_stream(wl: Workload, block_pairs: int = 1 << 24) -> PowerLawStream:
    return PowerLawStream(wl.n_nodes, wl.nnz_directed, wl.gamma, wl.max_degree, SEED_GRAPH + wl.index,
                          SEED_PERM + wl.index, block_pairs)


def workload_graph(wl: Workload, progress=None) -> Tuple[np.ndarray, np.ndarray]:
    if wl.stream:   # small copies of a streamed workload: the same generator, blocks joined
        parts = list(workload_stream(wl).blocks())
        return np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])
    return chung_lu_edges(wl.n_nodes, wl.nnz_directed, wl.gamma, wl.max_degree,
                          SEED_GRAPH + wl.index, SEED_PERM + wl.index, progress=progress)


def _rng_for_rows(seed: int, block: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, block]))


FEATURE_BLOCK = 4096


def node_features(global_ids: np.ndarray, d: int, seed: int = SEED_FEATURES, workers: int = 1) -> np.ndarray:
    """N(0,1) float32 features of the given global node ids.

    Row g of the (virtual) full feature matrix depends only on (seed, g), so a
    partition's duplicated nodes get exactly the rows of their originals without the
    full matrix ever being materialised.  workers > 1 draws the blocks on threads (same values).
    """
    global_ids = np.asarray(global_ids, dtype=np.int64)
    out = np.empty((global_ids.shape[0], d), dtype=np.float32)
    blocks = global_ids // FEATURE_BLOCK
    order = np.argsort(blocks, kind="stable")
    sb = blocks[order]
    starts = np.flatnonzero(np.r_[True, sb[1:] != sb[:-1]])
    ends = np.r_[starts[1:], sb.shape[0]]

    def fill(lo: int, hi: int) -> None:
        for s, e in zip(starts[lo:hi], ends[lo:hi]):
            b = int(sb[s])
            tile = _rng_for_rows(seed, b).standard_normal((FEATURE_BLOCK, d), dtype=np.float32)
            idx = order[s:e]
            out[idx] = tile[global_ids[idx] - b * FEATURE_BLOCK]

    n_groups = len(starts)
    if workers <= 1 or n_groups < 4 * workers:
        fill(0, n_groups)
    else:
        from concurrent.futures import ThreadPoolExecutor
        cuts = np.linspace(0, n_groups, 8 * workers + 1).astype(np.int64)
        with ThreadPoolExecutor(max_workers=workers) as pool:
            list(pool.map(lambda ab: fill(int(ab[0]), int(ab[1])), zip(cuts[:-1], cuts[1:])))
    return out


def node_labels(global_ids: np.ndarray, n_classes: int, seed: int = SEED_LABELS) -> np.ndarray:
    """Uniform int32 labels, a function of (seed, global id) only."""
    global_ids = np.asarray(global_ids, dtype=np.int64)
    out = np.empty(global_ids.shape[0], dtype=np.int32)
    blocks = global_ids // FEATURE_BLOCK
    order = np.argsort(blocks, kind="stable")
    sb = blocks[order]
    starts = np.flatnonzero(np.r_[True, sb[1:] != sb[:-1]])
    ends = np.r_[starts[1:], sb.shape[0]]
    for s, e in zip(starts, ends):
        b = int(sb[s])
        tile = _rng_for_rows(seed, b).integers(0, n_classes, FEATURE_BLOCK, dtype=np.int32)
        idx = order[s:e]
        out[idx] = tile[global_ids[idx] - b * FEATURE_BLOCK]
    return out


def node_multilabels(global_ids: np.ndarray, n_classes: int, p_on: float = 0.1, seed: int = SEED_LABELS) -> np.ndarray:
    """Multi-label 0/1 targets uint8 [n, n_classes], each label on with probability p_on; a function of
    (seed, global id) only."""
    global_ids = np.asarray(global_ids, dtype=np.int64)
    out = np.empty((global_ids.shape[0], n_classes), dtype=np.uint8)
    blocks = global_ids // FEATURE_BLOCK
    order = np.argsort(blocks, kind="stable")
    sb = blocks[order]
    starts = np.flatnonzero(np.r_[True, sb[1:] != sb[:-1]])
    ends = np.r_[starts[1:], sb.shape[0]]
    for s, e in zip(starts, ends):
        b = int(sb[s])
        tile = (_rng_for_rows(seed + 1, b).random((FEATURE_BLOCK, n_classes), dtype=np.float32) < p_on).astype(np.uint8)
        idx = order[s:e]
        out[idx] = tile[global_ids[idx] - b * FEATURE_BLOCK]
    return out


def glorot(rng: np.random.Generator, fan_out: int, fan_in: int) -> np.ndarray:
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-a, a, (fan_out, fan_in)).astype(np.float32)


def model_params(kind: str, dims: List[Tuple[int, int, int]], seed: int = SEED_PARAMS,
                 random_bias: bool = False) -> List[dict]:
    """Per-layer parameter dicts of float32 arrays.

    sage: W [d_msg, d_in], bW [d_msg], U [d_out, d_msg + d_in], bU [d_out]
    gcn : W [d_out, d_in], bW [d_out]
    sage_conv: W [d_out, 2 d_in] (self block, then neighbour block), bW [d_out]
    Biases are zero unless random_bias (parity tests use non-zero biases so that a
    dropped bias term cannot go unnoticed).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    layers = []
    for (d_in, d_msg, d_out) in dims:
        if kind == "sage":
            p = {"W": glorot(rng, d_msg, d_in), "bW": np.zeros(d_msg, np.float32),
                 "U": glorot(rng, d_out, d_msg + d_in), "bU": np.zeros(d_out, np.float32)}
        elif kind == "gcn":
            p = {"W": glorot(rng, d_out, d_in), "bW": np.zeros(d_out, np.float32)}
        elif kind == "sage_conv":
            p = {"W": glorot(rng, d_out, 2 * d_in), "bW": np.zeros(d_out, np.float32)}
        else:
            raise ValueError(kind)
        if random_bias:
            for k in p:
                if k.startswith("b"):
                    p[k] = (0.1 * rng.standard_normal(p[k].shape)).astype(np.float32)
        layers.append(p)
    return layers


def small_random_graph(n: int, m: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Tiny uniform random simple graph for brute-force tests: about m undirected edges."""
    rng = np.random.Generator(np.random.PCG64(seed))
    a = rng.integers(0, n, 3 * m)
    b = rng.integers(0, n, 3 * m)
    ok = a != b
    lo = np.minimum(a, b)[ok].astype(np.int64)
    hi = np.maximum(a, b)[ok].astype(np.int64)
    key = np.unique(lo * n + hi)
    rng.shuffle(key)
    key = key[:m]
    src, dst = key // n, key % n
    flip = rng.random(key.shape[0]) < 0.5
    return np.where(flip, dst, src), np.where(flip, src, dst)


def hub_graph(n: int, hub_degrees, m_random: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """Undirected simple graph with planted hub rows: hub h (node id h) is joined to hub_degrees[h] distinct
    random other nodes; m_random more random edges connect the rest.  For tests of the kernels' handling of
    rows far longer than the average (the high-degree nodes that survive a vertex cut, Theorem 2)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    src, dst = [], []
    for h, d in enumerate(hub_degrees):
        if d > n - 1:
            raise ValueError("hub degree exceeds n - 1")
        others = rng.choice(n - 1, size=d, replace=False).astype(np.int64)
        others[others >= h] += 1          # skip the hub itself
        src.append(np.full(d, h, dtype=np.int64))
        dst.append(others)
    a = rng.integers(0, n, m_random).astype(np.int64)
    b = rng.integers(0, n, m_random).astype(np.int64)
    ok = a != b
    src.append(a[ok])
    dst.append(b[ok])
    s, d = np.concatenate(src), np.concatenate(dst)
    lo, hi = np.minimum(s, d), np.maximum(s, d)
    key = np.unique(lo * n + hi)
    rng.shuffle(key)
    s, d = key // n, key % n
    flip = rng.random(key.shape[0]) < 0.5
    return np.where(flip, d, s), np.where(flip, s, d)
