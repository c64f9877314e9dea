"""Pins for the oracle's fp16 conversion and the two quantizers (Sec. 4.2's Q_8bit /
Q_4bit with this build's scale/zero/group reading).  None of these re-types the
oracle's formula: they use numpy's own half conversion, hand-made groups with a
known closed-form answer, brute force over all codes, and error bounds."""
import numpy as np
import pytest

import oracle as O


def test_f16_bits_match_numpy_on_every_half():
    h = np.arange(65536, dtype=np.uint16)
    f = O.f16_bits_to_f32(h)
    ref = h.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(f[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    assert np.all(np.isnan(f[nan]))
    back = O.f32_to_f16_bits(f[~nan])
    assert np.array_equal(back, h[~nan])


def test_f32_to_f16_rne_matches_numpy():
    rng = np.random.default_rng(1)
    x = np.concatenate([
        rng.standard_normal(400000).astype(np.float32),
        (rng.standard_normal(200000) * 1e-6).astype(np.float32),     # half subnormals
        (rng.standard_normal(100000) * 3e4).astype(np.float32),      # near overflow
        rng.integers(0, 2**32, 400000, dtype=np.uint64).astype(np.uint32).view(np.float32),
    ])
    x = x[~np.isnan(x)]
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(O.f32_to_f16_bits(x), ref)


def test_f32_to_f16_exact_ties_go_to_even():
    # midpoints between consecutive halves, normal and subnormal
    h = np.arange(0, 0x7bff, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).view(np.float16).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)  # midpoints are exact in fp32
    got = O.f32_to_f16_bits(mid)
    want = np.where(h % 2 == 0, h, h + 1).astype(np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(O.f32_to_f16_bits(-mid), want | 0x8000)


# ------------------------------------------------------------------ Q1

def test_q1_exact_on_power_of_two_grid():
    rng = np.random.default_rng(2)
    for e in (-10, -3, 0, 4):
        n = rng.integers(-127, 128, size=(5, 128))
        n[:, ::32] = 127                       # every group reaches amax = 127 * 2^e
        n[:, 1::32] = -127
        x = (n * 2.0 ** e).astype(np.float32)
        codes, scale = O.quant_i8(x)
        assert np.array_equal(codes, n.astype(np.int8))
        assert np.all(scale.view(np.float16) == np.float16(2.0 ** e))
        assert np.array_equal(O.dequant_i8(codes, scale), x)


def test_q1_ties_round_half_to_even_and_clamp():
    # scale 1: amax 127.  x = n + 0.5 must go to the even neighbour.
    x = np.zeros((1, 32), np.float32)
    x[0, 0] = 127.0
    x[0, 1:9] = [0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 125.5]
    codes, scale = O.quant_i8(x)
    assert scale.view(np.float16)[0, 0] == np.float16(1.0)
    assert list(codes[0, :9]) == [127, 0, 2, 2, 4, 0, -2, -2, 126]
    # fp16 rounding of the scale downwards makes x/s exceed 127 -> clamp
    x = np.zeros((1, 32), np.float32)
    x[0, 0] = 1000.3
    x[0, 1] = -1000.3
    codes, scale = O.quant_i8(x)
    s = float(scale.view(np.float16)[0, 0])
    assert s < 1000.3 / 127 and codes[0, 0] == 127 and codes[0, 1] == -127


def test_q1_degenerate_groups():
    x = np.zeros((2, 64), np.float32)
    x[1, :32] = 1e-9            # amax/127 underflows fp16 -> scale 0 -> codes 0
    x[1, 32:] = 3e-4            # scale is an fp16 subnormal, still usable
    x[1, 40] = 1e-4
    codes, scale = O.quant_i8(x)
    assert np.all(codes[0] == 0) and np.all(scale[0] == 0)
    assert np.all(codes[1, :32] == 0) and scale[1, 0] == 0
    s = scale.view(np.float16)[1, 1]
    assert 0 < float(s) < 6.2e-5
    want = np.minimum(127, np.rint(x[1, 32:] / np.float32(s)))
    assert np.array_equal(codes[1, 32:], want.astype(np.int8)) and codes[1, 40] not in (0, 127)
    assert np.all(O.dequant_i8(codes, scale)[0] == 0)
    # single outlier: everything else collapses towards 0
    x = np.full((1, 32), 0.01, np.float32)
    x[0, 7] = -50.0
    codes, scale = O.quant_i8(x)
    assert codes[0, 7] == -127 and np.all(np.delete(codes[0], 7) == 0)


def _brute_q1(x, scale_bits):
    s = scale_bits.view(np.float16).astype(np.float64)
    cand = np.arange(-127, 128, dtype=np.float64)
    err = np.abs(x.astype(np.float64)[..., None] - cand * np.repeat(s, 32, axis=-1)[..., None])
    return err


def test_q1_code_minimises_error_over_all_codes_and_bound():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((64, 128)) * rng.lognormal(0, 2, (64, 1))).astype(np.float32)
    codes, scale = O.quant_i8(x)
    err = _brute_q1(x, scale)
    best = err.min(axis=-1)
    chosen = np.take_along_axis(err, (codes.astype(np.int64) + 127)[..., None], axis=-1)[..., 0]
    assert np.all(chosen <= best * (1 + 1e-6) + 1e-30)
    s = np.repeat(scale.view(np.float16).astype(np.float64), 32, axis=-1)
    amax = np.repeat(np.abs(x).reshape(64, 4, 32).max(-1), 32, axis=-1)
    assert np.all(np.abs(O.dequant_i8(codes, scale) - x) <= s / 2 + amax * 2.0 ** -11 + 1e-30)


# ------------------------------------------------------------------ Q2

def test_q2_exact_on_grid_and_nibble_order():
    rng = np.random.default_rng(4)
    for e, z in ((-2, -1.75), (0, 3.0), (-5, 0.40625)):
        c = rng.integers(0, 16, size=(6, 128))
        c[:, ::64] = 0
        c[:, 1::64] = 15
        x = (z + c * 2.0 ** e).astype(np.float32)
        packed, scale, zero = O.quant_i4(x)
        assert np.all(scale.view(np.float16) == np.float16(2.0 ** e))
        assert np.all(zero.view(np.float16) == np.float16(z))
        assert np.array_equal(packed & 0xF, c[:, 0::2])          # even element -> low nibble
        assert np.array_equal(packed >> 4, c[:, 1::2])           # odd element -> high nibble
        assert np.array_equal(O.dequant_i4(packed, scale, zero), x)


def test_q2_ties_and_degenerate():
    x = np.zeros((1, 64), np.float32)
    x[0, 1] = 15.0
    x[0, 2:8] = [0.5, 1.5, 2.5, 13.5, 14.5, 7.5]
    packed, scale, zero = O.quant_i4(x)
    c = np.stack([packed & 0xF, packed >> 4], -1).reshape(1, 64)
    assert list(c[0, :8]) == [0, 15, 0, 2, 2, 14, 14, 8]
    x = np.abs(np.random.default_rng(0).standard_normal((2, 64))).astype(np.float32)
    x[0, 5], x[1, 5], x[1, 9] = -0.0, 0.0, -0.0   # a zero minimum: the zero point is +0 whichever zero comes first
    assert np.all(O.quant_i4(x)[2] == 0)
    x = np.full((1, 64), 2.5, np.float32)      # constant group: scale 0, codes 0, decodes to the zero point
    packed, scale, zero = O.quant_i4(x)
    assert np.all(packed == 0) and scale[0, 0] == 0 and zero.view(np.float16)[0, 0] == np.float16(2.5)
    assert np.all(O.dequant_i4(packed, scale, zero) == 2.5)


def test_q2_code_minimises_error_and_bound():
    rng = np.random.default_rng(5)
    x = (rng.standard_normal((64, 128)) * rng.lognormal(0, 1.5, (64, 1)) + rng.standard_normal((64, 1))).astype(np.float32)
    packed, scale, zero = O.quant_i4(x)
    c = np.stack([packed & 0xF, packed >> 4], -1).reshape(64, 128).astype(np.int64)
    s = np.repeat(scale.view(np.float16).astype(np.float64), 64, axis=-1)
    z = np.repeat(zero.view(np.float16).astype(np.float64), 64, axis=-1)
    cand = np.arange(16, dtype=np.float64)
    err = np.abs(x.astype(np.float64)[..., None] - (cand * s[..., None] + z[..., None]))
    chosen = np.take_along_axis(err, c[..., None], axis=-1)[..., 0]
    # the code is the nearest grid point up to fp32 rounding of (x - z)/s
    assert np.all(chosen <= err.min(-1) + 1e-5 * np.abs(x) + 1e-6 * s)
    g = x.reshape(64, 2, 64)
    lo, hi = np.repeat(g.min(-1), 64, -1), np.repeat(g.max(-1), 64, -1)
    bound = s / 2 + (np.abs(lo) + (hi - lo)) * 2.0 ** -10
    assert np.all(np.abs(O.dequant_i4(packed, scale, zero) - x) <= bound)


def test_requant_chain_equals_q2_when_q1_is_exact():
    rng = np.random.default_rng(6)
    n = rng.integers(-127, 128, size=(8, 128))
    n[:, ::32] = 127
    x = (n * 2.0 ** -4).astype(np.float32)
    chain = O.quant_i4(O.dequant_i8(*O.quant_i8(x)))
    direct = O.quant_i4(x)
    for a, b in zip(chain, direct):
        assert np.array_equal(a, b)
