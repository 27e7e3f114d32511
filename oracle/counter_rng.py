"""Counter-based random numbers for the oracle (test infrastructure only).

The paper leaves every random choice unspecified ("randomly assigns each edge", proof of
Theorem 2; "randomly select one of the masks", Algorithm 1 line 8).  To make those choices
reproducible on two independent implementations they are drawn from Philox-4x32-10
(Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11), a
published counter-based generator: output = bijection(counter, key), no state.

Draw convention used by the method (same on the HIP side, written independently there):
    words(seed, stream, a, b) = philox4x32_10(counter = (a mod 2^32, a div 2^32, b, stream),
                                              key     = (seed mod 2^32, seed div 2^32))
with a < 2^64, b < 2^32.  `r32` is word 0.
"""
import numpy as np

STREAM_CUT = 1       # edge -> partition
STREAM_MASK = 2      # DropEdge-K mask bits
STREAM_PICK = 3      # which mask an iteration uses
STREAM_DROPOUT = 4   # dropout keep decisions (layer id in bits 8..)

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds of Philox-4x32.  c0..c3: uint32 arrays (or scalars); k0, k1: python ints.

    One round: (hi0, lo0) = M0 * c0, (hi1, lo1) = M1 * c2 as 64-bit products;
    new counter = (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key is bumped by the
    Weyl constants (W0, W1) between rounds.
    """
    c0 = np.asarray(c0, dtype=np.uint64) & _MASK32
    c1 = np.asarray(c1, dtype=np.uint64) & _MASK32
    c2 = np.asarray(c2, dtype=np.uint64) & _MASK32
    c3 = np.asarray(c3, dtype=np.uint64) & _MASK32
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for r in range(10):
        p0 = _M0 * c0
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK32
        hi1, lo1 = p1 >> _S32, p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return (c0.astype(np.uint32), c1.astype(np.uint32), c2.astype(np.uint32), c3.astype(np.uint32))


def words(seed, stream, a, b):
    """Four uint32 words for counter (a, b) on `stream` under `seed` (see module docstring)."""
    a = np.asarray(a, dtype=np.uint64)
    b = np.asarray(b, dtype=np.uint64)
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    return philox4x32_10(a & _MASK32, a >> _S32, b & _MASK32, np.uint64(stream),
                         seed & 0xFFFFFFFF, seed >> 32)


def r32(seed, stream, a, b):
    return words(seed, stream, a, b)[0]


def scaled_index(r, n):
    """Map a uniform uint32 `r` to [0, n): floor(r * n / 2^32)."""
    return ((np.asarray(r, dtype=np.uint64) * np.uint64(n)) >> _S32).astype(np.int64)


def threshold(prob):
    """uint32 threshold t with P(r32 < t) = prob (to 2^-32): t = floor(prob * 2^32), prob in [0,1)."""
    if not (0.0 <= prob < 1.0):
        raise ValueError("probability must be in [0, 1)")
    return int(np.floor(np.float64(prob) * 4294967296.0))
