"""Pins of the oracle's compressor (Definition 1; Appendix "Compression Mechanism" / "Scheduler")."""
import math
import os

import numpy as np
import pytest

from oracle import layer as olayer
from oracle import mask as omask

KEY = 0x240617611
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- compressed size n / r -----------

@pytest.mark.parametrize("width,num,den,k", [
    (16, 4, 1, 4), (32, 4, 1, 8),                 # tiny config: ratio 4
    (128, 1, 1, 128), (128, 2, 1, 64), (128, 16, 1, 8), (256, 8, 1, 32), (40, 16, 1, 3),
    (100, 8, 1, 13), (100, 32, 1, 4), (512, 32, 1, 16),
    (100, 128, 1, 1), (7, 1000, 1, 1),            # ratio beyond the width still sends one element
    (128, 1584, 99, 8), (128, 1569, 99, 9), (128, 114, 99, 112), (128, 99, 99, 128),
])
def test_keep_count(width, num, den, k):
    assert omask.keep_count(width, num, den) == k


def test_keep_count_divisible_ratio_is_exact():
    # Definition 1: z has n/r elements whenever r divides n
    for width in (16, 100, 128, 256, 512):
        for r in range(1, width + 1):
            if width % r == 0:
                assert omask.keep_count(width, r, 1) * r == width


def test_keep_count_never_below_budget_and_rejects_expansion():
    for width in (100, 128, 255):
        for num, den in ((3, 2), (7, 3), (1584 - 15 * 37, 99)):
            k = omask.keep_count(width, num, den)
            assert k * num >= width * den and (k - 1) * num < width * den
    with pytest.raises(ValueError):
        omask.keep_count(16, 1, 2)


# ---------------------------------------------------------------- structure of the kept set -------

@pytest.mark.parametrize("width", [1, 2, 7, 16, 100, 128, 255, 256, 512])
def test_kept_columns_are_k_distinct_in_range(width):
    gids = np.arange(0, 3000, 7)
    for k in sorted({1, max(1, width // 8), max(1, width // 2), max(1, width - 1), width}):
        cols = omask.kept_columns(gids, width, k, KEY, 3, 1)
        assert cols.shape == (gids.shape[0], k)
        assert cols.min() >= 0 and cols.max() < width
        srt = np.sort(cols, axis=1)
        assert (np.diff(srt, axis=1) > 0).all()            # distinct within a row


def test_full_width_is_identity():
    cols = omask.kept_columns(np.arange(50), 100, 100, KEY, 9, 2)
    assert np.array_equal(cols, np.broadcast_to(np.arange(100), (50, 100)))


def test_units_are_exactly_the_invertible_multipliers():
    for width in (1, 2, 12, 100, 128, 255):
        u = omask.units(width)
        brute = [a for a in range(1, max(width, 2))
                 if len({(a * j) % width for j in range(width)}) == width]
        assert list(u) == brute
    assert len(omask.units(100)) == 40 and len(omask.units(256)) == 128      # Euler phi


def test_mask_depends_on_every_key_component_and_nothing_else():
    gids = np.arange(1000)
    base = omask.kept_columns(gids, 128, 16, KEY, 5, 1)
    assert np.array_equal(base, omask.kept_columns(gids, 128, 16, KEY, 5, 1))
    # a node's positions do not depend on which other nodes are asked for (destination independence)
    sub = omask.kept_columns(gids[::3][::-1], 128, 16, KEY, 5, 1)
    assert np.array_equal(sub, base[::3][::-1])
    for other in (omask.kept_columns(gids, 128, 16, KEY + 1, 5, 1),
                  omask.kept_columns(gids, 128, 16, KEY, 6, 1),
                  omask.kept_columns(gids, 128, 16, KEY, 5, 2),
                  omask.kept_columns(gids + 1000, 128, 16, KEY, 5, 1)):
        assert (other != base).any(axis=1).mean() > 0.95


def test_mixer_is_a_bijection():
    # inverse built from first principles: undo xorshifts, multiply by the modular inverses
    def unshift(x, s):
        y = x
        for _ in range(32 // s + 1):
            y = x ^ (y >> s)
        return y
    c1, c2 = 0x6A09E667, 0xBB67AE85
    i1, i2 = pow(c1, -1, 1 << 32), pow(c2, -1, 1 << 32)
    xs = np.concatenate([np.arange(4096, dtype=np.uint64),
                         np.random.default_rng(0).integers(0, 1 << 32, size=4096, dtype=np.uint64)])
    ys = omask._mix32(xs)
    for x, y in zip(xs.tolist(), ys.tolist()):
        y = unshift(y, 16)
        y = (y * i2) & 0xFFFFFFFF
        y = unshift(y, 15)
        y = (y * i1) & 0xFFFFFFFF
        y = unshift(y, 16)
        assert y == x


# ---------------------------------------------------------------- decoder semantics ---------------

def test_decompress_of_compress_is_masking_without_rescale():
    rng = np.random.default_rng(1)
    width, k = 100, 13
    x = rng.standard_normal((200, width))
    gids = rng.permutation(100000)[:200]
    cols = omask.kept_columns(gids, width, k, KEY, 0, 0)
    z = olayer.compress(x, np.arange(200), cols)
    assert z.shape == (200, k)
    xt = olayer.decompress(z, cols, width)
    mask = omask.keep_mask(gids, width, k, KEY, 0, 0)
    assert mask.sum(axis=1).tolist() == [k] * 200
    assert np.array_equal(xt, mask * x)                    # kept values verbatim, zero elsewhere
    # compress after decompress returns the message
    assert np.array_equal(olayer.compress(xt, np.arange(200), cols), z)


def test_compress_and_decompress_are_adjoint():
    rng = np.random.default_rng(2)
    width, k = 64, 20
    gids = np.arange(77)
    cols = omask.kept_columns(gids, width, k, KEY, 4, 2)
    x = rng.standard_normal((77, width))
    z = rng.standard_normal((77, k))
    lhs = (olayer.compress(x, np.arange(77), cols) * z).sum()
    rhs = (x * olayer.decompress(z, cols, width)).sum()
    assert abs(lhs - rhs) <= 1e-12 * abs(lhs)


def test_scatter_add_accumulates_at_kept_positions():
    rng = np.random.default_rng(3)
    width, k = 32, 8
    gids = np.arange(10)
    cols = omask.kept_columns(gids, width, k, KEY, 1, 1)
    rows = rng.permutation(40)[:10]
    x = rng.standard_normal((40, width))
    z = rng.standard_normal((10, k))
    want = x.copy()
    for i in range(10):
        for j in range(k):
            want[rows[i], cols[i, j]] += z[i, j]
    olayer.scatter_add(x, rows, cols, z)
    assert np.array_equal(x, want)


# ---------------------------------------------------------------- statistics (Definition 1) -------

@pytest.mark.parametrize("width,k", [(100, 13), (128, 8), (256, 32), (16, 4)])
def test_every_column_is_kept_with_probability_k_over_F(width, k):
    n = 200_000
    cols = omask.kept_columns(np.arange(n), width, k, KEY, 11, 0)
    freq = np.bincount(cols.ravel(), minlength=width) / n
    p = k / width
    sigma = math.sqrt(p * (1 - p) / n)
    assert np.abs(freq - p).max() < 5 * sigma


def test_mean_squared_error_matches_closed_form():
    # E||x~ - x||^2 = (1 - k/F) ||x||^2 ; for N(0,1) rows the mean over rows tends to F - k
    rng = np.random.default_rng(4)
    width, k, n = 100, 13, 100_000
    x = rng.standard_normal((n, width))
    mask = omask.keep_mask(np.arange(n), width, k, KEY, 2, 0)
    err = ((mask * x - x) ** 2).sum(axis=1).mean()
    assert abs(err - (width - k)) < 0.01 * (width - k)
    # lossless at ratio 1
    full = omask.keep_mask(np.arange(10), width, width, KEY, 2, 0)
    assert np.array_equal(full * x[:10], x[:10])


def test_pairs_of_steps_give_unrelated_masks():
    # fraction of positions kept at both of two steps ~ (k/F)^2 * F / k = k/F of the kept ones
    width, k, n = 128, 16, 50_000
    a = omask.keep_mask(np.arange(n), width, k, KEY, 0, 0)
    b = omask.keep_mask(np.arange(n), width, k, KEY, 1, 0)
    overlap = (a * b).sum() / (n * k)
    assert abs(overlap - k / width) < 0.01


# ---------------------------------------------------------------- golden vectors ------------------

def test_golden_mask_vectors():
    """Values written by tests/golden/make_golden.py (oracle only): guards the written mask rule."""
    path = os.path.join(GOLDEN, "mask_vectors.txt")
    n = 0
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            key, step, layer, gid, width, k, *cols = [int(t, 0) for t in line.split()]
            got = omask.kept_columns(np.array([gid]), width, k, key, step, layer)[0]
            assert got.tolist() == cols
            n += 1
    assert n >= 20


# ---------------------------------------------------------------- schedules -----------------------

def test_linear_schedule_endpoints_and_monotonicity():
    # config "16 -> 1 over 100 steps": r_t = (1584 - 15 t) / 99
    prev = None
    ks = []
    for t in range(100):
        num, den = omask.linear_ratio(16, 1, 1, 99, t)
        assert num * 99 == (1584 - 15 * t) * den
        r = num / den
        if prev is not None:
            assert r < prev                                 # Section IV: strictly decreasing
        prev = r
        ks.append(omask.keep_count(128, num, den))
    assert ks[0] == 8 and ks[1] == 9 and ks[2] == 9 and ks[-2] == 112 and ks[-1] == 128
    assert all(b >= a for a, b in zip(ks, ks[1:]))
    # paper's setting: c_max 128, c_min 1, slopes 2..7 reach and then hold the floor
    for slope in range(2, 8):
        rs = [omask.linear_ratio(128, 1, slope, 300, t) for t in range(301)]
        vals = [a / b for a, b in rs]
        assert vals[0] == 128 and vals[-1] == 1
        assert all(y <= x for x, y in zip(vals, vals[1:]))
        first_floor = next(i for i, v in enumerate(vals) if v == 1)
        assert first_floor == math.ceil(300 / slope)
