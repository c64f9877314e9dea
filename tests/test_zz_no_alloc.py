"""ttkv_decode_attn_noalloc (the entry point for callers that cannot allocate: its split partials live in an array
inside the library's device code) against ttkv_decode_attn with a caller-owned workspace, through the C ABI: same
kernels, same plan, so the outputs must agree to the last bit.  Two calls in a row on one GPU, the second on a
smaller cache (the array keeps the first call's partials), then a selection call, then a cache whose partials
exceed the array (refused, nothing enqueued)."""
import numpy as np
import pytest
import torch

from paper_2604_19769_amd import binding as B
from paper_2604_19769_amd import synth
from paper_2604_19769_amd.cache import TierConfig, TieredCache

pytestmark = pytest.mark.gpu

DT = {"f16": torch.float16, "bf16": torch.bfloat16}


def build(batch, Hq, Hkv, dtype, lens, seed, host=True, summary=False):
    tiers = [TierConfig(dtype, dtype, 256, 64, 6),
             TierConfig("i8", "i8", 512, 128, 8),
             TierConfig("i4", "i4", 10**9, 256, max(lens) // 256 + 3, "host" if host else "device", None, summary)]
    c = TieredCache(batch, Hq, Hkv, tiers)
    for b in range(batch):
        k, v = synth.kv(seed * 31 + b, Hkv, lens[b], dtype)
        n0 = min(lens[b], 255)
        n1 = min(lens[b] - n0, 512)
        n2 = lens[b] - n0 - n1
        for t, (lo, hi) in ((2, (0, n2)), (1, (n2, n2 + n1)), (0, (n2 + n1, lens[b]))):
            if hi > lo:
                kk = torch.from_numpy(k[:, lo:hi]).to("cuda:0").to(DT[dtype]).contiguous()
                vv = torch.from_numpy(v[:, lo:hi]).to("cuda:0").to(DT[dtype]).contiguous()
                c.append(t, kk, vv, seq=b, through_tiers=True)
    torch.cuda.synchronize()
    return c


def both(c, q, sel=None):
    """(out, lse) of ttkv_decode_attn with a workspace and of ttkv_decode_attn_noalloc, on the same state."""
    q_fmt = {torch.float16: B.F16, torch.bfloat16: B.BF16}[q.dtype]
    ref_out, ref_lse = (x.clone() for x in c.decode(q, sel))
    out = torch.full_like(ref_out, float("nan"))
    lse = torch.full_like(ref_lse, float("nan"))
    sb, sc = sel if sel is not None else (None, None)
    B.ttkv_decode_attn_noalloc(c.h, c.c, q, q_fmt, out, lse, sb, sc, sb.shape[1] if sb is not None else 0,
                               torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return ref_out, ref_lse, out, lse


def test_noalloc_entry_point_matches_the_workspace_one_twice_in_a_row_then_smaller():
    g = synth.rng(synth.SEED_BASE + 500)
    big = build(3, 8, 2, "f16", [3000, 777, 2100], synth.SEED_BASE + 501)
    small = build(1, 4, 4, "bf16", [300], synth.SEED_BASE + 502, host=False)
    sparse = build(2, 8, 2, "bf16", [2900, 1800], synth.SEED_BASE + 503, summary=True)
    try:
        for rep in range(2):                                   # two calls in a row on the larger cache
            q = torch.from_numpy(synth.normal(g, (3, 8, 128), "f16")).cuda().half()
            ro, rl, o, l = both(big, q)
            assert torch.equal(ro, o) and torch.equal(rl, l), rep
            assert torch.isfinite(o).all()
        q = torch.from_numpy(synth.normal(g, (1, 4, 128), "bf16")).cuda().bfloat16()
        ro, rl, o, l = both(small, q)                          # then a smaller one: fewer rows, fewer parts
        assert torch.equal(ro, o) and torch.equal(rl, l)
        q = torch.from_numpy(synth.normal(g, (2, 8, 128), "bf16")).cuda().bfloat16()
        sel = sparse.select(q, 3)
        ro, rl, o, l = both(sparse, q, sel)                    # selected blocks of the host tier
        assert torch.equal(ro, o) and torch.equal(rl, l)
        q = torch.from_numpy(synth.normal(g, (3, 8, 128), "f16")).cuda().half()
        ro, rl, o, l = both(big, q)                            # and the larger one again
        assert torch.equal(ro, o) and torch.equal(rl, l)
    finally:
        big.close(), small.close(), sparse.close()


def test_noalloc_entry_point_refuses_partials_beyond_its_array():
    """64 sequences x 64 query heads x 9 parts x 520 B = 19 MB of partials > 16 MiB: WORKSPACE, nothing enqueued,
    the outputs untouched; the workspace entry point takes the same cache."""
    tiers = [TierConfig("f16", "f16", 10**9, 256, 10)]
    c = TieredCache(64, 64, 1, tiers)
    try:
        k = torch.zeros(64, 1, 2304, 128, dtype=torch.float16, device="cuda:0")
        c.append(0, k, k)
        B.ttkv_set_split(c.h, 1 << 20)                          # the finest split: 256-token items, 9 per sequence
        parts = B.ttkv_count_parts(c.h, c.c)
        assert parts == 9 and 64 * 64 * parts * 520 > B.TTKV_NOALLOC_SCRATCH_BYTES, parts
        q = torch.zeros(64, 64, 128, dtype=torch.float16, device="cuda:0")
        out = torch.full((64, 64, 128), 7.0, dtype=torch.float32, device="cuda:0")
        with pytest.raises(B.TTKVError) as e:
            B.ttkv_decode_attn_noalloc(c.h, c.c, q, B.F16, out, None, None, None, 0, torch.cuda.current_stream().cuda_stream)
        assert e.value.status == B.ERR_WORKSPACE
        torch.cuda.synchronize()
        assert torch.all(out == 7.0)
        ref, _ = c.decode(q)
        torch.cuda.synchronize()
        assert torch.all(ref == 0)                              # all-zero values
    finally:
        c.close()
