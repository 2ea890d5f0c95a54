"""Pins of the oracle's bf16 storage rounding: hand-worked values of the format's definition (8 significant
bits, ties to even), structural properties, and an independent library conversion."""
import numpy as np
import torch

from oracle.rounding import round_bf16, round_f32


def test_hand_worked_values():
    u = 2.0 ** -7                       # spacing of bf16 numbers in [1, 2)
    cases = {
        1.0: 1.0,
        1.0 + u / 2: 1.0,               # tie -> even fraction (0)
        1.0 + 3 * u / 2: 1.0 + 2 * u,   # tie -> even fraction (2)
        1.0 + u / 2 + 2.0 ** -20: 1.0 + u,
        1.0 + u / 2 - 2.0 ** -20: 1.0,
        -(1.0 + 3 * u / 2): -(1.0 + 2 * u),
        2.0 - u / 2: 2.0,               # tie at the top of a binade carries into the exponent
        (2.0 - u) * 2.0 ** 127: (2.0 - u) * 2.0 ** 127,          # the largest finite bf16
        (2.0 - u + u / 4) * 2.0 ** 127: (2.0 - u) * 2.0 ** 127,
        0.0: 0.0,
    }
    for x, want in cases.items():
        assert round_bf16(np.array([x]))[0] == want, x
    assert np.isinf(round_bf16(np.array([(2.0 - u / 4) * 2.0 ** 127]))[0])   # past the largest bf16 by more than half a step
    assert np.isnan(round_bf16(np.array([np.nan]))[0])
    assert np.signbit(round_bf16(np.array([-0.0]))[0])


def test_results_have_eight_significant_bits_and_are_nearest():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, size=20000),
                        rng.standard_normal(1000) * 1e-40])   # includes binary32 subnormals
    r = round_bf16(x)
    bits = r.astype(np.float32).view(np.uint32)
    assert np.all(bits & 0xFFFF == 0)                         # representable: low 16 bits of the binary32 are 0
    assert np.array_equal(round_bf16(r), r)                   # idempotent
    # nearest: the two bf16 neighbours of r are not closer to (the binary32 value of) x than r is
    x32 = round_f32(x)
    up = (bits.astype(np.int64) + 0x10000).astype(np.uint32).view(np.float32).astype(np.float64)
    dn = (bits.astype(np.int64) - 0x10000).clip(min=0).astype(np.uint32).view(np.float32).astype(np.float64)
    err = np.abs(r - x32)
    ok = np.isfinite(up) & (np.abs(bits.astype(np.int64) & 0x7FFFFFFF) > 0x10000)
    assert np.all(err[ok] <= np.abs(up[ok] - x32[ok])) and np.all(err[ok] <= np.abs(dn[ok] - x32[ok]))
    normal = np.abs(x32) > 1e-37
    assert np.all(err[normal] <= np.abs(x32[normal]) * 2.0 ** -8)
    # monotone
    xs = np.sort(x)
    assert np.all(np.diff(round_bf16(xs)) >= 0)


def test_matches_library_conversion():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(100000) * 10.0 ** rng.integers(-10, 10, size=100000)).astype(np.float32)
    # every tie pattern in one binade as well
    ties = (np.arange(0x3F80, 0x4000, dtype=np.uint32) << 16 | 0x8000).view(np.float32)
    x = np.concatenate([x, ties, -ties])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_bf16(x), want)
