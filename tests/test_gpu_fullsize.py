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
from ttkv_testlib import assert_close, decode_i4c

pytestmark = pytest.mark.gpu


def sample_oracle(cache_cfg, Hq, Hkv, heads, K, V, max_tokens):
    """Oracle over KV heads `heads` only (heads are independent)."""
    G = Hq // Hkv
    ora = OracleCache(1, G * len(heads), len(heads), 128, cache_cfg, max_tokens)
    ora.load(0, K[heads].float().cpu().numpy(), V[heads].float().cpu().numpy())
    return ora


def sample_oracle_sizes(cache_cfg, Hq, Hkv, heads, K, V, max_tokens, sizes_oldest_first):
    """sample_oracle with the tiers' token counts given (oldest tier first) instead of filled by capacity."""
    G = Hq // Hkv
    ora = OracleCache(1, G * len(heads), len(heads), 128, cache_cfg, max_tokens)
    k, v = K[heads].float().cpu().numpy(), V[heads].float().cpu().numpy()
    lo = 0
    for t, n in zip(reversed(range(len(cache_cfg))), sizes_oldest_first):
        if n:
            xk, xv = ora.through_formats(k[:, lo:lo + n], v[:, lo:lo + n], t)
            ora.append(t, 0, xk, xv, lo)
        lo += n
    assert lo == k.shape[1]
    ora.total[0] = lo
    return ora


def q_rows(heads, G):
    return np.concatenate([np.arange(h * G, (h + 1) * G) for h in heads])


def compare_codes(cache, ora, b, heads, fmts):
    for t, (kf, vf) in enumerate(fmts):
        if kf == "i4t":                      # keys grouped over tokens: 128 meta rows x 4 B = {scale, zero} x 128 channels
            d = cache.dump_tier(t, b)
            s = ora.seq[t][0]
            assert int(cache.len[t][b]) == s.count and int(cache.start[t][b]) == s.first and s.first % 128 == 0
            sl, gsl = slice(s.first, s.first + s.count), slice(s.first // 128, (s.first + s.count) // 128)
            assert np.array_equal(d["k"][heads], s.kq["codes"][:, sl])
            meta = d["k_meta"][heads].reshape(len(heads), s.count // 128, 128, 4).view(np.uint16)
            assert np.array_equal(meta[..., 0], s.kq["scale"][:, gsl]) and np.array_equal(meta[..., 1], s.kq["zero"][:, gsl])
            assert np.array_equal(d["v"][heads], s.vq["codes"][:, sl])
            continue
        d = cache.dump_tier(t, b)
        s = ora.seq[t][0]
        assert int(cache.len[t][b]) == s.count and int(cache.start[t][b]) == s.first, (t, b)
        sl = slice(s.first, s.first + s.count)
        for name, fmt, hat, q in (("k", kf, s.khat, s.kq), ("v", vf, s.vhat, s.vq)):
            got = (decode_i4c(d[name]) if fmt == "i4c" else d[name])[heads]   # channel-major values: the same codes, unpacked
            if fmt in ("f16", "bf16"):
                assert np.array_equal(got.view(np.uint16), synth.to_bits(hat[:, sl], fmt)), (t, name)
            elif fmt == "i8":
                assert np.array_equal(got, q["codes"][:, sl].view(np.uint8)), (t, name)
                assert np.array_equal(d[name + "_meta"][heads].view(np.uint16), q["scale"][:, sl]), (t, name)
            else:
                assert np.array_equal(got, q["codes"][:, sl]), (t, name)
                meta = d[name + "_meta"][heads].view(np.uint16)
                assert np.array_equal(meta[:, :, 0::2], q["scale"][:, sl]) and np.array_equal(meta[:, :, 1::2], q["zero"][:, sl]), (t, name)


def compare_codes_of(cache, ora, b, heads, fmts):
    """compare_codes for an oracle that holds the whole batch and every head: view of sequence b, heads `heads`."""
    class _View:
        pass
    v = _View()
    v.seq = []
    for t in range(len(fmts)):
        s, w = ora.seq[t][b], _View()
        w.count, w.first = s.count, s.first
        w.khat, w.vhat = s.khat[heads], s.vhat[heads]
        w.kq = None if s.kq is None else {k: a[heads] for k, a in s.kq.items()}
        w.vq = None if s.vq is None else {k: a[heads] for k, a in s.vq.items()}
        v.seq.append([w])
    compare_codes(cache, v, b, heads, fmts)


def test_mha32k_full_size_every_head():
    """The HBM-bound benchmark configuration ("mha32k"): batch 4, 32 heads, 32K tokens, 2K fp16 + 30K int4 in HBM, append + attend + evict.
    The oracle holds the whole workload: every (sequence, head) row of every step is compared, element-wise and
    relative to the largest output (on N(0,1) data at 32K tokens the outputs are ~5e-3, so the absolute term of
    the element-wise tolerance alone would be most of the signal)."""
    steps = 3
    cache, (K, V), (q, kn, vn), shape = bench.build_mha32k(steps)
    try:
        B_, H = shape["B"], shape["Hq"]
        tiers = [TierSpec("f16", "f16", shape["R"], shape["bt"]), TierSpec("i4", "i4", 10**9, shape["bt"])]
        ora = OracleCache(B_, H, H, 128, tiers, [shape["R"] + 256, shape["N"] + 256])
        for b in range(B_):
            ora.load(b, K[b].float().cpu().numpy(), V[b].float().cpu().numpy())
        code_checks = [(0, [0, 31]), (2, [5, 30])]                      # (sequence, heads) whose stored bytes are compared
        for b, heads in code_checks:
            compare_codes_of(cache, ora, b, heads, [("f16", "f16"), ("i4", "i4")])
        for s in range(steps):
            out, lse = cache.step(q[s], kn[s], vn[s])
            torch.cuda.synchronize()
            ro, rl = ora.step(q[s].float().cpu().numpy(), kn[s, :, :, 0].float().cpu().numpy(), vn[s, :, :, 0].float().cpu().numpy())
            g = out.cpu().numpy()
            assert_close(g, ro, f"out step {s}")
            assert_close(lse.cpu().numpy(), rl, f"lse step {s}")
            for b in range(B_):                                        # per row: no head may hide behind another's scale
                rel = np.max(np.abs(g[b] - ro[b]), axis=1) / np.max(np.abs(ro[b]), axis=1)
                assert rel.max() < 2e-3, (s, b, int(rel.argmax()), float(rel.max()))
        for b, heads in code_checks:
            compare_codes_of(cache, ora, b, heads, [("f16", "f16"), ("i4", "i4")])
        assert cache.stats()["demotions"] == 4 and int(cache.len[0][2]) == shape["R"] - shape["bt"] + steps - 1
        assert torch.isfinite(out).all() and torch.isfinite(lse).all()
    finally:
        cache.close()


def test_mha32k_with_keys_grouped_over_tokens_full_size_sampled_heads():
    """The same workload with the old tier's keys as int4 per channel over 128 tokens (values int4 per token)."""
    steps = 3
    cache, (K, V), (q, kn, vn), shape = bench.build_mha32k(steps, slow_k="i4t")
    try:
        b, heads = 1, [7, 18]
        tiers = [TierSpec("f16", "f16", shape["R"], shape["bt"]), TierSpec("i4t", "i4", 10**9, shape["bt"])]
        ora = sample_oracle(tiers, 32, 32, heads, K[b], V[b], [shape["R"] + 256, shape["N"] + 256])
        compare_codes(cache, ora, b, heads, [("f16", "f16"), ("i4t", "i4")])
        for s in range(steps):
            out, lse = cache.step(q[s], kn[s], vn[s])
            torch.cuda.synchronize()
            ro, rl = ora.step(q[s, b][heads][None].float().cpu().numpy(), kn[s, b, heads, 0][None].float().cpu().numpy(),
                              vn[s, b, heads, 0][None].float().cpu().numpy())
            assert_close(out[b, heads].cpu().numpy(), ro[0], f"out step {s}")
            assert_close(lse[b, heads].cpu().numpy(), rl[0], f"lse step {s}")
            rel = np.max(np.abs(out[b, heads].cpu().numpy() - ro[0])) / np.max(np.abs(ro[0]))
            assert rel < 2e-3, rel
        compare_codes(cache, ora, b, heads, [("f16", "f16"), ("i4t", "i4")])
        assert cache.stats()["demotions"] == 4 and torch.isfinite(out).all()
    finally:
        cache.close()


def test_offload128k_full_size_sampled_heads():
    """The 128K offload benchmark configuration: 128K tokens, 4K bf16 + 28K int8 in HBM, 96K int4 in pinned host memory."""
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


@pytest.mark.parametrize("last_mem", ["host", "device"])
def test_serving_ragged_full_size_sampled(last_mem):
    """The ragged serving benchmark configuration: batch 16, ragged contexts in [16K, 64K], paged 256-token blocks on every tier;
    the int4 tier in pinned host memory, and (the bench's all-in-HBM variant) in HBM with its values channel-major."""
    steps = 2
    cache, kv, (q, kn, vn), shape = bench.build_serving_ragged(steps, last_mem=last_mem)
    last_fmt = ("i4", "i4c" if last_mem == "device" else "i4")
    try:
        heads, G = [0, 5], 4
        rows = q_rows(heads, G)
        ctx = shape["ctx"]
        picks = [int(np.argmin(ctx)), int(np.argmax(ctx))]           # shortest and longest sequence
        tiers = [TierSpec("f16", "f16", 4096, 256), TierSpec("i8", "i8", 12288, 256), TierSpec("i4", "i4", 10**9, 256, mem=last_mem)]
        oras = {}
        for b in picks:
            if last_mem == "device":     # the loader put whole groups of 32 tokens into the last tier: so does the oracle
                sizes = [int(cache.len[t][b]) for t in (2, 1, 0)]
                oras[b] = sample_oracle_sizes(tiers, 32, 8, heads, kv[b][0], kv[b][1], [4096 + 512, 12288 + 1024, 65536], sizes)
            else:
                oras[b] = sample_oracle(tiers, 32, 8, heads, kv[b][0], kv[b][1], [4096 + 512, 12288 + 1024, 65536])
            compare_codes(cache, oras[b], b, heads, [("f16", "f16"), ("i8", "i8"), last_fmt])
        for s in range(steps):
            out, lse = cache.step(q[s], kn[s], vn[s])
            torch.cuda.synchronize()
            for b in picks:
                ro, rl = oras[b].step(q[s, b][rows][None].float().cpu().numpy(), kn[s, b, heads, 0][None].float().cpu().numpy(),
                                      vn[s, b, heads, 0][None].float().cpu().numpy())
                assert_close(out[b, rows].cpu().numpy(), ro[0], f"out seq {b} step {s}")
                assert_close(lse[b, rows].cpu().numpy(), rl[0], f"lse seq {b} step {s}")
        for b in picks:
            compare_codes(cache, oras[b], b, heads, [("f16", "f16"), ("i8", "i8"), last_fmt])
            total = sum(int(cache.len[t][b]) for t in range(3))
            assert total == int(ctx[b]) - 1 + steps
            for pos in (0, total // 3, total - 1):
                t, blk, row, _ = cache.locate(b, pos)
                assert (t, blk, row) == tuple(int(x) for x in oras[b].locate(0, pos))
        assert torch.isfinite(out).all()
    finally:
        cache.close()


def test_sparse_recall_full_size_one_sequence():
    """The sparse recall benchmark configuration: top-64 of 96 host blocks by q . mean-key; the oracle recomputes one whole sequence
    (selection needs every head): selected block ids identical, planted blocks selected, outputs within tolerance."""
    steps = 2
    cache, kv, (q, kn, vn), shape = bench.build_sparse128k(steps)
    try:
        b = 1
        tiers = [TierSpec("bf16", "bf16", 4096, 128), TierSpec("i8", "i8", 28672, 1024),
                 TierSpec("i4", "i4", 10**9, 1024, mem="host", summary=True)]
        ora = OracleCache(1, 32, 8, 128, tiers, [4096 + 256, 28672 + 2048, 98304 + 4096])
        ora.load(0, kv[b][0].float().cpu().numpy(), kv[b][1].float().cpu().numpy())
        for blk, mu in ora.summaries(0).items():
            assert np.array_equal(cache.dump_summary(2, b, blk), mu), blk
        for s in range(steps):
            before = cache.stats()
            out, lse = cache.step(q[s], kn[s], vn[s], select_k=64)
            torch.cuda.synchronize()
            after = cache.stats()
            assert after["blocks_fetched"] - before["blocks_fetched"] == 4 * 64
            assert after["h2d_bytes"] - before["h2d_bytes"] == 4 * 64 * 1179648
            ro, rl, rsel = ora.step(q[s, b][None].float().cpu().numpy(), kn[s, b, :, 0][None].float().cpu().numpy(),
                                    vn[s, b, :, 0][None].float().cpu().numpy(), select_k=64)
            got = cache.sel_blocks.numpy()[b, :int(cache.sel_count.numpy()[b])]
            assert np.array_equal(got, rsel[0]), (got, rsel[0])
            if s == 0:     # the planted blocks were built from this step's query
                for bb in range(4):
                    sel = set(cache.sel_blocks.numpy()[bb, :64].tolist())
                    assert set(shape["planted"][bb].tolist()) <= sel, bb
            assert_close(out[b].cpu().numpy(), ro[0], f"out step {s}")
            assert_close(lse[b].cpu().numpy(), rl[0], f"lse step {s}")
    finally:
        cache.close()


@pytest.mark.parametrize("bt,k,fmt", [(128, 512, ("i4", "i4")), (1024, 64, ("i4", "i4c"))])
def test_sparse_attention_over_a_tier_in_hbm_full_size_one_sequence(bt, k, fmt):
    """bench.py's sparse_hbm rows at full size (batch 4, 128K tokens, every tier in HBM): identification, top-k (a thread
    per block, 768 of them at 128-token blocks) and attention over the selected blocks as one run whose items span
    blocks; the oracle recomputes one whole sequence: ids identical, outputs within tolerance."""
    steps = 2
    cache, kv, (q, kn, vn), shape = bench.build_sparse_hbm(steps, bt, fmt)
    try:
        b = 2
        tiers = [TierSpec("bf16", "bf16", 4096, 128), TierSpec("i8", "i8", 28672, 1024), TierSpec("i4", "i4", 10**9, bt, summary=True)]
        ora = OracleCache(1, 32, 8, 128, tiers, [4096 + 256, 28672 + 2048, 98304 + 4096])
        ora.load(0, kv[b][0].float().cpu().numpy(), kv[b][1].float().cpu().numpy())
        for s in range(steps):
            out, lse = cache.step(q[s], kn[s], vn[s], select_k=k)
            torch.cuda.synchronize()
            ro, rl, rsel = ora.step(q[s, b][None].float().cpu().numpy(), kn[s, b, :, 0][None].float().cpu().numpy(),
                                    vn[s, b, :, 0][None].float().cpu().numpy(), select_k=k)
            got = cache.sel_blocks.numpy()[b, :int(cache.sel_count.numpy()[b])]
            assert len(got) == k and np.array_equal(got, rsel[0]), (got, rsel[0])
            assert_close(out[b].cpu().numpy(), ro[0], f"out step {s}")
            assert_close(lse[b].cpu().numpy(), rl[0], f"lse step {s}")
        assert cache.stats()["h2d_bytes"] == 0
    finally:
        cache.close()
