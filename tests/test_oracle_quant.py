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


# ---------------------------------------------------------------- Q2 over 128 tokens per channel (keys)

def test_q2_tokens_exact_on_grid_and_nibble_order():
    """x[t][j] = z_j + c[t][j] * 2^e_j with every channel containing codes 0 and 15: scale = 2^e_j, zero = z_j,
    codes and round trip exact; channel 2i in the low nibble, 2i+1 in the high nibble of byte i of a token's row."""
    rng = np.random.default_rng(21)
    n, d = 256, 128
    c = rng.integers(0, 16, (n, d))
    for g in range(n // 128):
        for j in range(d):
            t = rng.choice(128, 2, replace=False) + g * 128
            c[t[0], j], c[t[1], j] = 0, 15
    e = rng.integers(-6, 4, d)
    z = (rng.integers(-40, 40, d) * 0.25).astype(np.float32)
    x = (z[None, :] + c * np.exp2(e)[None, :]).astype(np.float32)
    packed, scale, zero = O.quant_i4_tokens(x)
    assert packed.shape == (n, d // 2) and scale.shape == (n // 128, d) and zero.shape == (n // 128, d)
    assert np.array_equal(O.f16_bits_to_f32(scale), np.broadcast_to(np.exp2(e).astype(np.float32), (2, d)))
    assert np.array_equal(O.f16_bits_to_f32(zero), np.broadcast_to(z, (2, d)))
    assert np.array_equal(packed & 0xf, c[:, 0::2]) and np.array_equal(packed >> 4, c[:, 1::2])
    assert np.array_equal(O.dequant_i4_tokens(packed, scale, zero), x)


def test_q2_tokens_is_q2_of_the_transposed_matrix():
    """Independent of the function under test: the pinned per-token Q2 (group of 64 along the row) applied to the
    transposed block.  If every channel attains its minimum and its maximum in both halves of the 128 tokens, the
    two 64-groups of a transposed row have the scale and zero of the 128-group, so codes, scales and zeros agree."""
    rng = np.random.default_rng(22)
    d = 128
    x = rng.standard_normal((128, d)).astype(np.float32) * np.exp2(rng.integers(-3, 3, d)).astype(np.float32)[None, :]
    lo, hi = x.min(axis=0), x.max(axis=0)
    for j in range(d):
        for half in (0, 1):
            t = rng.choice(64, 2, replace=False) + 64 * half
            x[t[0], j], x[t[1], j] = lo[j], hi[j]
    packed, scale, zero = O.quant_i4_tokens(x)
    pt, st, zt = O.quant_i4(np.ascontiguousarray(x.T))          # rows = channels, columns = tokens
    assert np.array_equal(st[:, 0], st[:, 1]) and np.array_equal(zt[:, 0], zt[:, 1])
    assert np.array_equal(scale[0], st[:, 0]) and np.array_equal(zero[0], zt[:, 0])
    codes = np.empty((128, d), np.uint8)
    codes[:, 0::2], codes[:, 1::2] = packed & 0xf, packed >> 4
    codes_t = np.empty((d, 128), np.uint8)
    codes_t[:, 0::2], codes_t[:, 1::2] = pt & 0xf, pt >> 4
    assert np.array_equal(codes, codes_t.T)
    assert np.array_equal(O.dequant_i4_tokens(packed, scale, zero), O.dequant_i4(pt, st, zt).T)


def test_q2_tokens_code_minimises_error_degenerate_and_bound():
    rng = np.random.default_rng(23)
    x = rng.standard_normal((384, 128)).astype(np.float32)
    x[:, 5] *= 8.0                                     # an outlier channel
    x[:128, 7] = 0.75                                  # constant over a group
    x[128:256, 9] = 0.0                                # all zero over a group
    x[:128, 11] = np.abs(x[:128, 11])
    x[3, 11] = -0.0                                    # zero minimum with a sign
    packed, scale, zero = O.quant_i4_tokens(x)
    s = O.f16_bits_to_f32(scale).astype(np.float64)
    z = O.f16_bits_to_f32(zero).astype(np.float64)
    codes = np.empty(x.shape, np.int64)
    codes[:, 0::2], codes[:, 1::2] = packed & 0xf, packed >> 4
    S, Z = np.repeat(s, 128, axis=0), np.repeat(z, 128, axis=0)
    err = np.abs(x - (codes * S + Z))
    for c in range(16):
        alt = np.abs(x - (c * S + Z))
        assert np.all(err <= alt + 1e-7 * (1 + np.abs(x)))
    assert scale[0, 7] == 0 and np.all(codes[:128, 7] == 0) and O.f16_bits_to_f32(zero)[0, 7] == 0.75
    assert scale[1, 9] == 0 and zero[1, 9] == 0
    assert zero[0, 11] == 0                            # +0, not 0x8000
    xhat = O.dequant_i4_tokens(packed, scale, zero)
    lo, hi = x.reshape(3, 128, 128).min(axis=1), x.reshape(3, 128, 128).max(axis=1)
    bound = np.repeat(s / 2 + (np.abs(lo) + (hi - lo)) * 2.0 ** -10, 128, axis=0) + 1e-6
    assert np.all(np.abs(x - xhat) <= bound)
    # the outlier channel has its own groups: scaling it further changes nothing in any other channel
    # (per-token groups of 64 channels: the 63 neighbours lose resolution)
    x2 = x.copy()
    x2[:, 5] *= 4.0
    p2, s2, z2 = O.quant_i4_tokens(x2)
    keep = np.arange(128) != 5
    c2 = np.empty(x.shape, np.int64)
    c2[:, 0::2], c2[:, 1::2] = p2 & 0xf, p2 >> 4
    assert np.array_equal(c2[:, keep], codes[:, keep]) and np.array_equal(s2[:, keep], scale[:, keep])
    assert np.array_equal(z2[:, keep], zero[:, keep])
    others = [j for j in range(64) if j not in (5, 7, 9, 11)]
    e_tok = np.abs(x[:, others] - O.dequant_i4(*O.quant_i4(x))[:, others]).mean()
    e_tok2 = np.abs(x2[:, others] - O.dequant_i4(*O.quant_i4(x2))[:, others]).mean()
    assert e_tok2 > 2.0 * e_tok > 2.0 * np.abs(x[:, others] - xhat[:, others]).mean()
