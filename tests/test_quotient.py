"""The conversion kernels divide once per group and multiply per element (Sec. 4.2's quantizers are fixed as one
IEEE division per element followed by round-to-nearest-even): rint(x * (1 / s)) with the exact division as fallback
when x * (1 / s) lies within 5e-4 of a half-integer.  Emulated here in fp32 with numpy, against the plain division,
on scales of every fp16 magnitude and quotients placed on, next to and between the half-integers: after the clamp to
the code range the two must agree everywhere.  (The GPU tests compare the kernels' codes with the oracle's.)"""
import numpy as np
import pytest


def fast_and_exact(x, s):
    x, s = x.astype(np.float32), s.astype(np.float32)
    r = (np.float32(1.0) / s).astype(np.float32)
    t = (x * r).astype(np.float32)
    q = np.rint(t).astype(np.float32)
    exact = np.rint((x / s).astype(np.float32)).astype(np.float32)
    near = np.abs((t - q).astype(np.float32)) > np.float32(0.4995)
    return np.where(near, exact, q), exact, near


@pytest.mark.parametrize("lo,hi", [(-127, 127), (0, 15)])
def test_reciprocal_quotient_equals_the_division_after_the_clamp(lo, hi):
    g = np.random.default_rng(1976900 + hi)
    n = 4_000_000
    s = g.integers(1, 0x7BFF, n).astype(np.uint16).view(np.float16).astype(np.float32)      # every positive finite half
    k = g.integers(-300, 300, n).astype(np.float32)
    frac = np.where(g.random(n) < 0.5, 0.5, g.random(n)).astype(np.float32)                # half of them exact ties
    jitter = (1 + g.integers(-4, 5, n) * np.float32(2.0 ** -23)).astype(np.float32)        # and a few ulps around them
    x = ((k + frac) * s * jitter).astype(np.float32)
    fast, exact, near = fast_and_exact(x, s)
    assert np.array_equal(np.clip(fast, lo, hi), np.clip(exact, lo, hi))
    assert 0.3 < near.mean() < 0.7          # the adversarial mix does exercise the fallback ...
    x = g.standard_normal((200_000, 32)).astype(np.float16).astype(np.float32)
    sc = (np.abs(x).max(1, keepdims=True) / np.float32(127)).astype(np.float16).astype(np.float32)
    fast, exact, near = fast_and_exact(x.ravel(), np.repeat(sc, 32, 1).ravel())
    assert np.array_equal(fast, exact) and near.mean() < 3e-3    # ... which ordinary data takes about once in a thousand
