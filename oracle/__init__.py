"""TTKV oracle -- TEST INFRASTRUCTURE ONLY.

numpy-facing wrappers around the scalar C oracle (ttkv_oracle.c) and the tiered
cache state machine built on it (cache.py).  Nothing in the product package may
import this; it imports nothing from the product package.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) else _build.build()
        L = C.CDLL(path)
        p = C.c_void_p
        i64, i32, f64 = C.c_int64, C.c_int32, C.c_double
        L.o_f32_to_f16_array.argtypes = [p, i64, p]
        L.o_f16_to_f32_array.argtypes = [p, i64, p]
        L.o_quant_i8_sym_g32.argtypes = [p, i64, i32, p, p]
        L.o_dequant_i8_sym_g32.argtypes = [p, p, i64, i32, p]
        L.o_quant_i4_asym_g64.argtypes = [p, i64, i32, p, p, p]
        L.o_dequant_i4_asym_g64.argtypes = [p, p, p, i64, i32, p]
        L.o_quant_i4_asym_t128.argtypes = [p, i64, i32, p, p, p]
        L.o_dequant_i4_asym_t128.argtypes = [p, p, p, i64, i32, p]
        L.o_attn_partial.argtypes = [p, i32, i32, i32, p, p, i64, i64, i64, f64, p, p, p]
        L.o_merge_into.argtypes = [p, p, p, p, p, p, i32, i32]
        L.o_finalize.argtypes = [p, p, p, i32, i32, p, p]
        L.o_summary_accumulate.argtypes = [p, p, i32, i32, i64, i64, i64]
        L.o_summary_finish.argtypes = [p, i32, i32, p]
        L.o_block_score.argtypes = [p, p, i32, i32, i32]
        L.o_block_score.restype = C.c_float
        L.o_topk.argtypes = [p, i32, i32, p]
        L.o_topk.restype = i32
        _lib = L
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def f32_to_f16_bits(x):
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().o_f32_to_f16_array(_ptr(x), x.size, _ptr(out))
    return out


def f16_bits_to_f32(h):
    h = _c(h, np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().o_f16_to_f32_array(_ptr(h), h.size, _ptr(out))
    return out


def quant_i8(x):
    """Q1 on x [..., d] fp32 -> (codes int8 [..., d], scale bits uint16 [..., d/32])."""
    x = _c(x, np.float32)
    d = x.shape[-1]
    rows = x.size // d
    codes = np.empty(x.shape, np.int8)
    scale = np.empty(x.shape[:-1] + (d // 32,), np.uint16)
    lib().o_quant_i8_sym_g32(_ptr(x), rows, d, _ptr(codes), _ptr(scale))
    return codes, scale


def dequant_i8(codes, scale):
    codes = _c(codes, np.int8)
    scale = _c(scale, np.uint16)
    d = codes.shape[-1]
    out = np.empty(codes.shape, np.float32)
    lib().o_dequant_i8_sym_g32(_ptr(codes), _ptr(scale), codes.size // d, d, _ptr(out))
    return out


def quant_i4(x):
    """Q2 on x [..., d] fp32 -> (packed uint8 [..., d/2], scale bits, zero bits [..., d/64])."""
    x = _c(x, np.float32)
    d = x.shape[-1]
    rows = x.size // d
    packed = np.empty(x.shape[:-1] + (d // 2,), np.uint8)
    scale = np.empty(x.shape[:-1] + (d // 64,), np.uint16)
    zero = np.empty(x.shape[:-1] + (d // 64,), np.uint16)
    lib().o_quant_i4_asym_g64(_ptr(x), rows, d, _ptr(packed), _ptr(scale), _ptr(zero))
    return packed, scale, zero


def dequant_i4(packed, scale, zero):
    packed = _c(packed, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    d = packed.shape[-1] * 2
    out = np.empty(packed.shape[:-1] + (d,), np.float32)
    lib().o_dequant_i4_asym_g64(_ptr(packed), _ptr(scale), _ptr(zero), out.size // d, d, _ptr(out))
    return out


def quant_i4_tokens(x):
    """Q2 with groups of 128 consecutive tokens per channel, on x [..., n, d] fp32 (n a multiple of 128)
    -> (packed uint8 [..., n, d/2], scale bits, zero bits [..., n/128, d])."""
    x = _c(x, np.float32)
    n, d = x.shape[-2], x.shape[-1]
    assert n % 128 == 0
    lead = x.shape[:-2]
    packed = np.zeros(lead + (n, d // 2), np.uint8)
    scale = np.empty(lead + (n // 128, d), np.uint16)
    zero = np.empty(lead + (n // 128, d), np.uint16)
    xs, ps = x.reshape(-1, n, d), packed.reshape(-1, n, d // 2)
    ss, zs = scale.reshape(-1, n // 128, d), zero.reshape(-1, n // 128, d)
    for i in range(xs.shape[0]):
        lib().o_quant_i4_asym_t128(_ptr(xs[i]), n, d, _ptr(ps[i]), _ptr(ss[i]), _ptr(zs[i]))
    return packed, scale, zero


def dequant_i4_tokens(packed, scale, zero):
    packed = _c(packed, np.uint8)
    scale = _c(scale, np.uint16)
    zero = _c(zero, np.uint16)
    n, d = packed.shape[-2], packed.shape[-1] * 2
    out = np.empty(packed.shape[:-1] + (d,), np.float32)
    ps, os_ = packed.reshape(-1, n, d // 2), out.reshape(-1, n, d)
    ss, zs = scale.reshape(-1, n // 128, d), zero.reshape(-1, n // 128, d)
    for i in range(ps.shape[0]):
        lib().o_dequant_i4_asym_t128(_ptr(ps[i]), _ptr(ss[i]), _ptr(zs[i]), n, d, _ptr(os_[i]))
    return out


def attn_partial(q, K, V, t0, n, softmax_scale):
    """q [Hq][d], K/V [Hkv][stride][d] fp32 -> (m [Hq], l [Hq], acc [Hq][d]) fp64."""
    q = _c(q, np.float32)
    assert K.dtype == np.float32 and V.dtype == np.float32
    assert K.flags.c_contiguous and V.flags.c_contiguous and K.shape == V.shape
    Hq, d = q.shape
    Hkv, stride, d2 = K.shape
    assert d2 == d and Hq % Hkv == 0 and 0 <= t0 and t0 + n <= stride
    m = np.empty(Hq, np.float64)
    l = np.empty(Hq, np.float64)
    acc = np.empty((Hq, d), np.float64)
    lib().o_attn_partial(_ptr(q), Hq, Hkv, d, _ptr(K), _ptr(V), stride, t0, n, float(softmax_scale),
                         _ptr(m), _ptr(l), _ptr(acc))
    return m, l, acc


def empty_partial(Hq, d):
    return (np.full(Hq, -np.inf), np.zeros(Hq), np.zeros((Hq, d)))


def merge_into(a, b):
    """a <- a (+) b in place; a, b = (m, l, acc) fp64."""
    rows, d = a[2].shape
    lib().o_merge_into(_ptr(a[0]), _ptr(a[1]), _ptr(a[2]), _ptr(b[0]), _ptr(b[1]), _ptr(b[2]), rows, d)
    return a


def finalize(p):
    rows, d = p[2].shape
    out = np.empty((rows, d), np.float64)
    lse = np.empty(rows, np.float64)
    lib().o_finalize(_ptr(p[0]), _ptr(p[1]), _ptr(p[2]), rows, d, _ptr(out), _ptr(lse))
    return out, lse


def summary_accumulate(sum_, x, t0, n):
    """sum_ [Hkv][d] fp32 += x[:, t0:t0+n, :] token by token (in place)."""
    assert sum_.dtype == np.float32 and sum_.flags.c_contiguous
    assert x.dtype == np.float32 and x.flags.c_contiguous
    Hkv, stride, d = x.shape
    lib().o_summary_accumulate(_ptr(sum_), _ptr(x), Hkv, d, stride, t0, n)


def summary_finish(sum_, block_tokens):
    sum_ = _c(sum_, np.float32)
    mu = np.empty(sum_.shape, np.uint16)
    lib().o_summary_finish(_ptr(sum_), sum_.size, block_tokens, _ptr(mu))
    return mu


def block_score(q, mu, Hkv):
    q = _c(q, np.float32)
    mu = _c(mu, np.uint16)
    Hq, d = q.shape
    return float(lib().o_block_score(_ptr(q), _ptr(mu), Hq, Hkv, d))


def topk(scores, k):
    scores = _c(scores, np.float32)
    sel = np.empty(max(1, scores.size), np.int32)
    c = lib().o_topk(_ptr(scores), scores.size, k, _ptr(sel))
    assert c >= 0
    return sel[:c].copy()


from .cache import OracleCache, TierSpec  # noqa: E402,F401
