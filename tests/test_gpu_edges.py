"""GPU parity on the degenerate and extreme cases of the path: an empty cache, one-token
sequences, the maximum batch with empty members, selection of no block and of every
block, rings that wrap many times, more query heads per KV head than any kernel groups."""
import numpy as np
import pytest
import torch

from paper_2604_19769_amd import binding as B
from paper_2604_19769_amd import synth
from ttkv_testlib import Pair, assert_close, dev
from test_gpu_parity import run_config, tiers3

pytestmark = pytest.mark.gpu


def test_empty_cache_then_single_token():
    """No live token: out = 0, lse = -inf (the identity of the merge).  After one step the only
    token carries all the weight: out equals its value row, lse its score."""
    p = Pair(2, 8, 2, tiers3("f16", host=False), "f16")
    try:
        g = synth.rng(synth.SEED_BASE + 40)
        q = synth.normal(g, (2, 8, 128), "f16")
        out, lse = p.gpu.decode(dev(q, "f16"))
        torch.cuda.synchronize()
        assert torch.all(out == 0) and torch.all(torch.isinf(lse) & (lse < 0))
        kn, vn = synth.normal(g, (2, 2, 128), "f16"), synth.normal(g, (2, 2, 128), "f16")
        r = p.step(q, kn, vn)
        assert_close(r[0], r[2], "out")
        assert_close(r[1], r[3], "lse")
        want = np.repeat(vn, 4, axis=1)                       # query head h reads KV head h // 4
        assert np.max(np.abs(r[0] - want)) <= 1e-6
        score = np.einsum("bhd,bhd->bh", q.astype(np.float64), np.repeat(kn, 4, axis=1).astype(np.float64)) / np.sqrt(128.0)
        assert np.max(np.abs(r[1] - score)) <= 1e-4
        p.assert_state_equal()
    finally:
        p.close()


def test_maximum_batch_with_empty_and_one_token_members():
    """TTKV_MAX_BATCH sequences, some empty, some with one token, the rest ragged: more (tier, sequence) runs
    than one launch table holds, empty rows merge to the identity."""
    n = B.TTKV_MAX_BATCH if hasattr(B, "TTKV_MAX_BATCH") else 64
    lens = [0 if i % 9 == 0 else 1 if i % 9 == 1 else 30 + 53 * i for i in range(n)]
    tiers = tiers3("f16", host=False, bts=(64, 64, 64), caps=(128, 256), rings=(3, 6, 60))
    run_config(n, 4, 2, tiers, "f16", None, 2, synth.SEED_BASE + 41, lens=lens)


@pytest.mark.parametrize("n_slots", [0, 2])
def test_selecting_no_block_and_every_block(n_slots):
    """k = 0: only the device tiers are attended, nothing crosses PCIe.  k >= live blocks: identical to dense."""
    tiers = tiers3("bf16", summary=True, bts=(64, 128, 128), rings=(6, 8, 40))
    for k in (0, 1000):
        p = Pair(2, 8, 2, tiers, "bf16", n_slots=n_slots)
        try:
            g = synth.rng(synth.SEED_BASE + 42)
            for b in range(2):
                kk, vv = synth.kv((synth.SEED_BASE + 42) * 31 + b, 2, 3000, "bf16")
                p.load(b, kk, vv)
            for s in range(3):
                q = synth.normal(g, (2, 8, 128), "bf16")
                kn, vn = synth.normal(g, (2, 2, 128), "bf16"), synth.normal(g, (2, 2, 128), "bf16")
                before = p.gpu.stats()["h2d_bytes"]
                r = p.step(q, kn, vn, select_k=k)
                assert_close(r[0], r[2], f"out k={k} step {s}")
                assert_close(r[1], r[3], f"lse k={k} step {s}")
                for b in range(2):
                    assert np.array_equal(r[4][b], r[5][b])
                moved = p.gpu.stats()["h2d_bytes"] - before
                if k == 0:
                    assert moved == 0 and all(len(x) == 0 for x in r[4])
                else:       # every live block of the last tier, in ascending order
                    assert moved > 0
                    for b in range(2):
                        assert len(r[4][b]) >= 16 and np.array_equal(r[4][b], np.arange(r[4][b][0], r[4][b][0] + len(r[4][b])))
            assert p.gpu.stats()["h2d_bytes"] == p.ora.h2d_bytes
        finally:
            p.close()


def test_rings_wrap_many_times():
    """Small rings on every tier (host included): 700 steps wrap the fp16 ring 11 times and the int8 ring
    5 times while blocks fall off nothing (the last tier is large enough); state compared along the way."""
    tiers = tiers3("f16", bts=(64, 64, 128), caps=(128, 256), rings=(3, 5, 12))
    run_config(2, 8, 2, tiers, "f16", None, 700, synth.SEED_BASE + 43, lens=[100, 611], check_state_every=175,
               oracle_max_tokens=[1600, 1600, 1600])     # the oracle keeps every token a tier ever held


@pytest.mark.parametrize("Hq,Hkv,dtype,fmts", [(64, 2, "f16", None), (40, 2, "bf16", None), (34, 2, "f16", None),
                                               (48, 1, "f16", (("i4", "i4"), ("i4", "i4"))),
                                               (71, 1, "f16", (("f16", "f16"), ("f16", "f16")))])
def test_many_query_heads_per_kv_head(Hq, Hkv, dtype, fmts):
    """32, 20 and 17 query heads per KV head with an int8 tier: blocks of 8 heads (the last one smaller) on the
    matrix-core kernel, each a pass over the bytes; 48 with int4 tiers and 71 with fp16 tiers (multi-query
    attention): blocks of 16."""
    tiers = tiers3(dtype, host=False) if fmts is None else tiers3(dtype, fmts=fmts, host=False)
    st = run_config(2, Hq, Hkv, tiers, dtype, None, 3, synth.SEED_BASE + 44 + Hq, lens=[333, 2100], want_stats=True)
    assert st["mfma_launches"] == 3


@pytest.mark.parametrize("Hq,Hkv,n_slots", [(4, 4, 0), (8, 2, 2)])
def test_four_tiers_the_maximum(Hq, Hkv, n_slots):
    """TTKV_MAX_TIERS tiers: fp16 -> int8 -> K 8-bit / V 4-bit in HBM -> int4 in pinned host memory; a token that
    reaches the last tier has passed through every format above it, and every boundary evicts during the run."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=128, block_tokens=64, ring_blocks=3),
             dict(k_fmt="i8", v_fmt="i8", capacity=256, block_tokens=64, ring_blocks=6),
             dict(k_fmt="i8", v_fmt="i4", capacity=384, block_tokens=128, ring_blocks=5),
             dict(k_fmt="i4", v_fmt="i4", capacity=10**9, block_tokens=256, ring_blocks=12, mem="host")]
    st = run_config(2, Hq, Hkv, tiers, "f16", None, 200, synth.SEED_BASE + 70 + Hq, lens=[90, 1900], check_state_every=100,
                    n_slots=n_slots, want_stats=True, oracle_max_tokens=[600, 1200, 1600, 3200])
    assert st["demotions"] > 8


def random_layout(seed):
    """A seeded random but valid cache: 1-4 tiers, formats that never widen from one tier to the next (values never
    wider than keys), block sizes, capacities, rings sized for the lengths, host / paged / staged variants."""
    g = synth.rng(synth.SEED_BASE + 900 + seed)
    dtype = ("f16", "bf16")[int(g.integers(2))]
    Hkv = int(g.choice([1, 2, 4]))
    G = int(g.choice([1, 1, 2, 3, 4, 6, 8]))
    B_ = int(g.integers(1, 4))
    n_tiers = int(g.integers(1, 5))
    order = [(dtype, dtype), ("i8", "i8"), ("i8", "i4"), ("i4", "i4")]
    level = 0
    tiers = []
    lens = [int(g.integers(1, 2600)) for _ in range(B_)]
    for t in range(n_tiers):
        if t > 0:
            level = int(g.integers(max(level, 0 if t < n_tiers - 1 else 0), len(order)))
        bt = int(g.choice([64, 128, 256]))
        last = t == n_tiers - 1
        cap = 10**9 if last else bt * int(g.integers(1, 5))
        prev_bt = tiers[-1]["block_tokens"] if tiers else 0            # a tier takes whole blocks of the tier above
        ring = (max(lens) + 64 + prev_bt) // bt + 3 if last else (cap + prev_bt) // bt + 2
        host = last and t > 0 and bool(g.integers(2))
        tiers.append(dict(k_fmt=order[level][0], v_fmt=order[level][1], capacity=cap, block_tokens=bt, ring_blocks=ring,
                          mem="host" if host else "device", paged_seed=int(g.integers(1, 99)) if g.integers(3) == 0 else None))
    n_slots = int(g.choice([0, 0, 2, 3])) if tiers[-1].get("mem") == "host" else 0
    return B_, Hkv * G, Hkv, tiers, dtype, lens, n_slots


@pytest.mark.parametrize("seed", range(40))
def test_randomized_layouts(seed):
    """Forty seeded random caches, loaded in bulk and stepped across evictions, against the oracle: state bit for
    bit, outputs within tolerance, locate and traffic counters equal."""
    B_, Hq, Hkv, tiers, dtype, lens, n_slots = random_layout(seed)
    run_config(B_, Hq, Hkv, tiers, dtype, None, 12, synth.SEED_BASE + 950 + seed, lens=lens, n_slots=n_slots,
               check_state_every=6, host_append_direct=bool(seed & 1), host_demote_direct=bool(seed & 2),
               one_call_step=bool(seed % 3))



def test_selection_ids_with_non_finite_scores_and_more_than_64_heads():
    """Block identification alone (ttkv_select_blocks): 72 query heads (two passes of 64 lanes) and queries that
    hold +inf, so that scores are +-inf and NaN (inf x 0 where a block's mean key has a zero channel): the ids are
    the oracle's (NaN ranks as -inf, ties to the lower id), and there are exactly min(k, live blocks) of them."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=128, block_tokens=64, ring_blocks=3),
             dict(k_fmt="f16", v_fmt="f16", capacity=10**9, block_tokens=64, ring_blocks=40, summary=True)]
    p = Pair(2, 72, 1, tiers, "f16")
    try:
        g = synth.rng(synth.SEED_BASE + 45)
        for b, n in enumerate((127 + 64 * 20 + 10, 127 + 64 * 33)):
            k, v = synth.kv((synth.SEED_BASE + 45) * 31 + b, 1, n, "f16")
            k[:, 64 * 3:64 * 7, 5] = 0.0                     # blocks 3..6: channel 5 of the mean key is exactly zero
            p.load(b, k, v)
        for trial, kk in enumerate((5, 0, 21, 1000)):
            q = synth.normal(g, (2, 72, 128), "f16")
            if trial != 1:
                q[:, 7, 5] = np.inf                          # head 7, channel 5
            if trial == 2:
                q[:, 70, 9] = -np.inf
            want = p.ora.select(q, kk)
            sb, sc = p.gpu.select(dev(q, "f16"), kk)
            for b in range(2):
                got = sb.numpy()[b, :int(sc.numpy()[b])]
                assert np.array_equal(got, want[b]), (trial, b, got, want[b])
                assert len(got) == min(kk, len(p.ora.live_blocks(1, b)))
    finally:
        p.close()


def channel_major_layout(seed):
    """random_layout(seed) with the last tier's values stored channel-major per 32 tokens, where that format applies
    (two or more heads per KV head, at least two tiers, int8 or int4 keys in the last tier); the lengths are rounded
    so that the last tier receives whole groups of 32 tokens."""
    B_, Hq, Hkv, tiers, dtype, lens, n_slots = random_layout(seed)
    last = tiers[-1]
    if Hq == Hkv or len(tiers) < 2 or (last["k_fmt"], last["v_fmt"]) not in (("i8", "i4"), ("i4", "i4")):
        return None
    last["v_fmt"] = "i4c"
    fixed = tiers[0]["capacity"] - 1 + sum(t["capacity"] for t in tiers[1:-1])
    lens = [n if n <= fixed else fixed + (n - fixed) // 32 * 32 for n in lens]
    return B_, Hq, Hkv, tiers, dtype, lens, n_slots


@pytest.mark.parametrize("seed", [s for s in range(120) if channel_major_layout(s) is not None][:16])
def test_randomized_layouts_with_channel_major_values(seed):
    """Seeded random caches (tiers, block sizes, capacities, host / paged / staged variants as in the test above)
    whose last tier stores its int4 values channel-major per 32 tokens."""
    B_, Hq, Hkv, tiers, dtype, lens, n_slots = channel_major_layout(seed)
    run_config(B_, Hq, Hkv, tiers, dtype, None, 12, synth.SEED_BASE + 1200 + seed, lens=lens, n_slots=n_slots,
               check_state_every=6, host_append_direct=bool(seed & 1), host_demote_direct=bool(seed & 2),
               one_call_step=bool(seed % 3))
