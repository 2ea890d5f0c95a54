"""Which elements of a node vector are communicated (oracle side; test infrastructure).

Appendix "Compression Mechanism": the encoder sends (vector length / compression ratio) elements chosen
at random; a key shared beforehand lets the decoder know their positions. Definition 1: z in R^{n/r}.

Reading used here (the paper fixes no generator):
  * granularity is one node vector of width F: exactly k of its F elements are kept;
  * k = max(1, ceil(F / r)) with r = num/den an exact rational >= 1 (Definition 1 wants n/r integral;
    the schedules of Appendix "Scheduler" produce ratios that do not divide F);
  * the kept positions of node v at (step t, layer l) are a pure function of (key, t, l, v):
        pi_v(j) = (a_v * j + b_v) mod F,  j = 0..k-1,
    b_v uniform on [0,F), a_v uniform on the units of Z_F; k == F means the identity (lossless case);
  * (a_v, b_v) come from a counter-based integer mixer, specified below, evaluated on both sides.

Every column is kept with probability exactly k/F (b_v is uniform), which is all the moments in
Definition 1 depend on: E||x~ - x||^2 = (1 - k/F) ||x||^2.
"""
from __future__ import annotations

import math

import numpy as np

_M64 = (1 << 64) - 1
_M32 = np.uint64(0xFFFFFFFF)
_GOLDEN64 = 0x9E3779B97F4A7C15          # floor(2^64 / golden ratio), odd
_C1 = np.uint64(0x6A09E667)             # floor(2^32 * frac(sqrt 2)), odd
_C2 = np.uint64(0xBB67AE85)             # floor(2^32 * frac(sqrt 3)), odd


def _mix64(x: int) -> int:
    """splitmix64 output function (Steele, Lea, Flood 2014) on a Python int."""
    x &= _M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _M64
    x ^= x >> 31
    return x


def stream_words(key: int, step: int, layer: int) -> tuple[int, int]:
    """Two 32-bit words that select the mask family of (key, step, layer)."""
    inner = _mix64(step + _GOLDEN64 * (layer + 1))
    s = _mix64(key ^ inner)
    return s & 0xFFFFFFFF, s >> 32


def _mix32(x: np.ndarray) -> np.ndarray:
    """Bijective xorshift-multiply mixer on 32-bit words held in uint64 arrays."""
    x = x & _M32
    x = x ^ (x >> np.uint64(16))
    x = (x * _C1) & _M32
    x = x ^ (x >> np.uint64(15))
    x = (x * _C2) & _M32
    x = x ^ (x >> np.uint64(16))
    return x


def units(width: int) -> np.ndarray:
    """Ascending multipliers in [1, width) coprime with width (just [1] for width 1)."""
    u = [a for a in range(1, max(width, 2)) if math.gcd(a, width) == 1]
    return np.asarray(u, dtype=np.int64)


def affine_params(gids: np.ndarray, width: int, s0: int, s1: int) -> tuple[np.ndarray, np.ndarray]:
    """(a_v, b_v) of every node id in `gids` for vectors of `width` elements."""
    v = np.asarray(gids).astype(np.uint64) & _M32
    h1 = _mix32(v ^ np.uint64(s0))
    h2 = _mix32(h1 ^ np.uint64(s1))
    u = units(width)
    b = (h1 * np.uint64(width)) >> np.uint64(32)
    a = u[((h2 * np.uint64(u.shape[0])) >> np.uint64(32)).astype(np.int64)]
    return a.astype(np.int64), b.astype(np.int64)


def keep_count(width: int, num: int, den: int) -> int:
    """k = max(1, ceil(width * den / num)) for the ratio num/den >= 1.

    den == 0 (num > 0) stands for an unbounded ratio: nothing is communicated, k = 0. This is the
    "no communication" setting the experiments of Section V compare against, per layer: with k = 0 on every
    layer each partition trains on its own subgraph; with k = 0 only on the layers after the first, the
    input features of adjacent nodes are still exchanged but no intermediate activations.
    """
    if den == 0 and num > 0:
        return 0
    if num < den or den < 1:
        raise ValueError("compression ratio must be >= 1")
    return max(1, -((-width * den) // num))


def kept_columns(gids: np.ndarray, width: int, k: int, key: int, step: int, layer: int) -> np.ndarray:
    """Positions pi_v(0..k-1) for each node id: int64 array [len(gids), k]."""
    gids = np.asarray(gids)
    j = np.arange(k, dtype=np.int64)[None, :]
    if k == width:
        return np.broadcast_to(j, (gids.shape[0], k)).copy()
    s0, s1 = stream_words(key, step, layer)
    a, b = affine_params(gids, width, s0, s1)
    return (a[:, None] * j + b[:, None]) % width


def keep_mask(gids: np.ndarray, width: int, k: int, key: int, step: int, layer: int) -> np.ndarray:
    """0/1 matrix [len(gids), width] with exactly k ones per row."""
    cols = kept_columns(gids, width, k, key, step, layer)
    m = np.zeros((cols.shape[0], width), dtype=np.float64)
    m[np.arange(cols.shape[0])[:, None], cols] = 1.0
    return m


# ---------------------------------------------------------------------------------------------------
# ratio schedules (Section IV and Appendix "Scheduler")
# ---------------------------------------------------------------------------------------------------

def linear_ratio(c_max: int, c_min: int, slope: int, n_steps: int, step: int) -> tuple[int, int]:
    """Clamped linear schedule as an exact rational (num, den).

    The printed formula takes a min with c_min, which would pin the ratio at or below c_min from the
    first step and contradicts Section IV's requirement that the ratio start high and decrease; it is
    read as  c_k = max(c_max - slope * (c_max - c_min) * k / K, c_min).
    """
    num = c_max * n_steps - slope * (c_max - c_min) * step
    den = n_steps
    if num <= c_min * den:
        return c_min, 1
    g = math.gcd(num, den)
    return num // g, den // g


def fixed_increment_ratio(r0: int, increment: int, c_min: int, step: int) -> tuple[int, int]:
    """r_{k+1} = r_k + R with R < 0 so that the ratio decreases; clamped at c_min."""
    return max(r0 + increment * step, c_min), 1


def exponential_ratio(base: int, c_max: int, c_min: int, n_steps: int, step: int) -> tuple[int, int]:
    """Exponential schedule of Appendix "Scheduler": the communicated fraction is base^-(K - k + 1), i.e. the
    ratio is base^(K - k + 1), clamped to [c_min, c_max]. Read with an integer base >= 2 so that the ratio
    is an exact integer (a fractional base would need a rounding rule the paper does not give)."""
    if base < 2:
        raise ValueError("base must be an integer >= 2")
    exponent = max(n_steps - step + 1, 0)
    value = 1
    for _ in range(exponent):
        value *= base
        if value >= c_max:
            return c_max, 1
    return max(value, c_min), 1
