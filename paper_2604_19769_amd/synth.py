"""Seeded synthetic inputs with the shapes of the paper's workloads (long-context
decode: 4K-128K tokens, 8-32 KV heads of dimension 128).  Input preparation only:
random draws, rounding to the storage type, bit views.  None of the method's
arithmetic lives here; both the HIP path's callers and the oracle's tests use it.

Values are returned as float32 arrays that are exactly representable in the
named storage type, so the oracle (fp32 in) and the device path (fp16/bf16 bits
in) see identical numbers."""
import numpy as np

SEED_BASE = 1976900


def rng(seed):
    return np.random.Generator(np.random.Philox(int(seed)))


def round_to(x, dtype):
    """float32 array -> float32 array of values representable in dtype ('f16' | 'bf16'), round to nearest even."""
    x = np.ascontiguousarray(x, np.float32)
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32)
    raise ValueError(dtype)


def to_bits(x, dtype):
    """Exactly representable float32 values -> uint16 storage bits."""
    x = np.ascontiguousarray(x, np.float32)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        return (x.view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def normal(g, shape, dtype, scale=1.0):
    return round_to(g.standard_normal(shape, dtype=np.float32) * np.float32(scale), dtype)


def outlier_channels(g, n_heads, d, frac=0.02):
    """Seeded (head, channel) pairs that carry a x8 scale in K (2 % of all pairs)."""
    n = int(round(frac * n_heads * d))
    flat = g.choice(n_heads * d, size=n, replace=False)
    return np.stack([flat // d, flat % d], 1)


def kv(seed, n_kv_heads, n_tokens, dtype, k_outliers=None, d=128):
    """K, V [Hkv][N][d] ~ N(0,1) in `dtype`; optional x8 outlier channels on K."""
    g = rng(seed)
    k = g.standard_normal((n_kv_heads, n_tokens, d), dtype=np.float32)
    v = g.standard_normal((n_kv_heads, n_tokens, d), dtype=np.float32)
    if k_outliers is not None:
        for h, ch in k_outliers:
            k[h, :, ch] *= 8.0
    return round_to(k, dtype), round_to(v, dtype)


def queries(seed, steps, batch, n_q_heads, dtype, d=128):
    return normal(rng(seed), (steps, batch, n_q_heads, d), dtype)


def plant_blocks(g, k, q, block_tokens, n_planted, first_token, n_blocks, group, dtype, shift=1.0):
    """Shift the keys of `n_planted` seeded blocks (of the n_blocks starting at
    first_token) along the mean query of each KV head's query group, so that the
    blocks' mean keys stand out.  Returns the planted block indices."""
    planted = np.sort(g.choice(n_blocks, size=n_planted, replace=False))
    for h in range(k.shape[0]):
        u = q[h * group:(h + 1) * group].mean(0)
        u = (u / np.linalg.norm(u)).astype(np.float32)
        for j in planted:
            lo = first_token + j * block_tokens
            k[h, lo:lo + block_tokens] += np.float32(shift) * u
    k[:] = round_to(k, dtype)
    return planted
