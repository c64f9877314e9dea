"""GPU parity: the HIP path through the C ABI against the CPU oracle, same seeded
inputs.  Codes / scales / zeros / fp bits / tier and block indices bit-exact;
attention outputs within 2e-3 + 1e-2*|ref| (fp32 accumulation on the device,
fp64 in the oracle)."""
import math

import numpy as np
import pytest
import torch

import oracle as O
from paper_2604_19769_amd import binding as B
from paper_2604_19769_amd import synth
from ttkv_testlib import Pair, assert_close, dev

pytestmark = pytest.mark.gpu


def tiers3(dtype, fmts=(("i8", "i8"), ("i4", "i4")), caps=(256, 512), bts=(64, 128, 256), rings=(6, 8, 16), host=True,
           summary=False, paged=False):
    return [
        dict(k_fmt=dtype, v_fmt=dtype, capacity=caps[0], block_tokens=bts[0], ring_blocks=rings[0]),
        dict(k_fmt=fmts[0][0], v_fmt=fmts[0][1], capacity=caps[1], block_tokens=bts[1], ring_blocks=rings[1],
             paged_seed=11 if paged else None),
        dict(k_fmt=fmts[1][0], v_fmt=fmts[1][1], capacity=10**9, block_tokens=bts[2], ring_blocks=rings[2],
             mem="host" if host else "device", summary=summary, paged_seed=12 if paged else None),
    ]


def edge_rows(dtype):
    """Hand-made rows that exercise ties, clamping, degenerate and denormal-scale groups."""
    rows = np.zeros((8, 128), np.float32)
    rows[0, :] = 0.0                                            # all zero
    rows[1, :] = 2.5                                            # constant
    rows[2, ::32] = 127.0
    rows[2, 1:9] = [0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 125.5]   # exact ties at scale 1
    rows[3, :] = 0.01
    rows[3, 7] = -50.0                                          # single outlier
    rows[4, :64] = 3e-4
    rows[4, 8] = 1e-4                                           # fp16-subnormal scale
    rows[4, 64:] = 1e-9                                         # underflows to scale 0
    rows[5, 0::2] = 15.0
    rows[5, 3] = 7.5
    rows[5, 5] = 0.5                                            # int4 ties: (x - 0) / 1
    rows[6, :] = np.abs(synth.normal(synth.rng(5), 128, "f16"))
    rows[6, 5] = -0.0                                           # zero minimum with a sign
    rows[7, :] = np.arange(128) - 64.0
    return synth.round_to(rows, dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("fmt", [("i8", "i8"), ("i4", "i4"), ("i8", "i4")])
def test_quantize_append_bit_exact(dtype, fmt):
    """ttkv_quantize_append into a quantized tier: codes, scales and zeros equal the oracle's Q."""
    n = 200                                       # spans 3 blocks of 64 + a ragged tail
    tiers = [dict(k_fmt=dtype, v_fmt=dtype, capacity=64, block_tokens=64, ring_blocks=2),
             dict(k_fmt=fmt[0], v_fmt=fmt[1], capacity=10**9, block_tokens=64, ring_blocks=5)]
    p = Pair(2, 4, 2, tiers, dtype)
    try:
        g = synth.rng(synth.SEED_BASE + 100)
        k = synth.normal(g, (2, 2, n, 128), dtype) * synth.round_to(np.exp2(g.integers(-6, 6, (2, 2, n, 1))).astype(np.float32), dtype)
        v = synth.normal(g, (2, 2, n, 128), dtype)
        k = synth.round_to(k, dtype)
        k[0, 0, :8] = edge_rows(dtype)
        v[1, 1, 100:108] = edge_rows(dtype)
        p.gpu.append(1, dev(k, dtype), dev(v, dtype))
        for b in range(2):
            p.ora.append(1, b, k[b], v[b], 0)
        p.assert_state_equal()
        # appending again continues at the tail (row 200 of the ring), one sequence only
        k2, v2 = synth.normal(g, (2, 37, 128), dtype), synth.normal(g, (2, 37, 128), dtype)
        p.gpu.append(1, dev(k2, dtype), dev(v2, dtype), seq=1)
        p.ora.append(1, 1, k2, v2, n)
        p.assert_state_equal()
    finally:
        p.close()


def run_config(B_, Hq, Hkv, tiers, dtype, N, steps, seed, select_k=None, overlap=True, check_state_every=None, n_slots=0,
               lens=None, peaked=False, want_stats=False, oracle_max_tokens=None, host_append_direct=False, one_call_step=True,
               host_demote_direct=False):
    p = Pair(B_, Hq, Hkv, tiers, dtype, n_slots=n_slots, oracle_max_tokens=oracle_max_tokens,
             host_append_direct=host_append_direct, one_call_step=one_call_step, host_demote_direct=host_demote_direct)
    worst = 0.0
    try:
        g = synth.rng(seed)
        for b in range(B_):
            n = N if lens is None else lens[b]
            k, v = synth.kv(seed * 31 + b, Hkv, n, dtype)
            if peaked:                                      # a few keys aligned with q -> O(1) outputs
                k[:, ::97] *= 4.0
                k = synth.round_to(k, dtype)
            p.load(b, k, v)
        p.assert_state_equal()
        for s in range(steps):
            q = synth.normal(g, (B_, Hq, 128), dtype)
            kn, vn = synth.normal(g, (B_, Hkv, 128), dtype), synth.normal(g, (B_, Hkv, 128), dtype)
            r = p.step(q, kn, vn, select_k, overlap)
            worst = max(worst, assert_close(r[0], r[2], f"out step {s}"))
            assert_close(r[1], r[3], f"lse step {s}")
            if select_k is not None:
                for b in range(B_):
                    assert np.array_equal(r[4][b], r[5][b]), (s, b, r[4][b], r[5][b])
            if check_state_every and (s + 1) % check_state_every == 0:
                p.assert_state_equal()
        p.assert_state_equal()
        for b in range(B_):
            total = sum(int(p.gpu.len[t][b]) for t in range(len(tiers)))
            p.assert_locate_equal(b, np.unique(np.concatenate([[0, total - 1], synth.rng(seed + b).integers(0, total, 64)])))
        st = p.gpu.stats()
        assert st["h2d_bytes"] == p.ora.h2d_bytes and st["blocks_fetched"] == p.ora.blocks_fetched
        assert st["demotions"] == sum(sum(d) for d in p.ora.demotions)
    finally:
        p.close()
    return st if want_stats else worst


def test_config1_tiny_fp16_plus_int8():
    """batch 1, 8 q / 2 kv heads, 4096 tokens: last 512 fp16, older 3584 int8 g32, all in HBM, one step."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=512, block_tokens=128, ring_blocks=5),
             dict(k_fmt="i8", v_fmt="i8", capacity=10**9, block_tokens=128, ring_blocks=30)]
    run_config(1, 8, 2, tiers, "f16", 4095, 1, synth.SEED_BASE + 1)


@pytest.mark.parametrize("fmt", [("f16", "f16"), ("i8", "i4"), ("i4", "i4")])
def test_config1_shape_other_slow_formats(fmt):
    """Same shape with the slow tier all-fp16 (exact attention), K 8-bit / V 4-bit (the paper's choice), int4."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=512, block_tokens=128, ring_blocks=5),
             dict(k_fmt=fmt[0], v_fmt=fmt[1], capacity=10**9, block_tokens=128, ring_blocks=30)]
    run_config(1, 8, 2, tiers, "f16", 4095, 2, synth.SEED_BASE + 2, peaked=True)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (8, 1), (12, 4)])
def test_gqa_ratios_and_ragged_lengths(Hq, Hkv):
    """Group size 1 on the vector kernel, 2 and 3 (padded to 4) and 8 (two passes of the score product for the int8
    tier) on the matrix-core kernel; lengths that are not multiples of a tile or a block."""
    st = run_config(3, Hq, Hkv, tiers3("bf16", host=False), "bf16", None, 3, synth.SEED_BASE + 3 + Hq, lens=[1, 777, 2500],
                    want_stats=True)
    assert (st["mfma_launches"] > 0) == (Hq // Hkv >= 2), st


@pytest.mark.parametrize("Hq,Hkv,dtype,slow", [(8, 1, "f16", ("i4", "i4")), (16, 2, "f16", ("i4", "i4")), (16, 1, "f16", ("f16", "f16")),
                                                (10, 2, "f16", ("f16", "f16")), (12, 2, "bf16", ("bf16", "bf16")), (8, 2, "bf16", ("i8", "i4")),
                                                (16, 4, "bf16", ("i8", "i8")), (16, 2, "f16", ("i8", "i8")), (8, 1, "bf16", ("i8", "i4")),
                                                (16, 1, "f16", ("i4", "i4")), (6, 2, "f16", ("i8", "i8")), (12, 2, "bf16", ("i4", "i4")),
                                                (10, 2, "f16", ("i8", "i4")), (4, 2, "f16", ("i8", "i4")), (24, 2, "f16", ("i4", "i4")),
                                                (7, 1, "bf16", ("i8", "i8")), (12, 1, "f16", ("i8", "i8")), (16, 1, "bf16", ("i8", "i4")),
                                                (40, 2, "bf16", ("i8", "i4")), (64, 2, "f16", ("i8", "i8")), (48, 2, "f16", ("i4", "i4"))])
def test_grouped_query_group_sizes_on_the_matrix_core_kernel(Hq, Hkv, dtype, slow):
    """Every (format, heads per KV head) case of the grouped-query kernel: int4 with 8 heads, fp16 with 16 and with
    counts that are not powers of two (5, 6), K 8-bit / V 4-bit and int8 with 4; the two-pass cases int8 and
    K 8-bit / V 4-bit with 8 heads and int4 with 16; the four-pass cases int8 and K 8-bit / V 4-bit with 12 and 16
    heads; head counts that are padded to the next of 4, 8, 16 (3, 5, 6, 7, 12) and K 8-bit / V 4-bit with 2; more
    than 16 heads per KV head cut into blocks (20 = 16 + 4, 24 = 16 + 8, 32 = 16 + 16); ragged lengths leave partial
    16-token tiles in both tiers, the rings wrap during the steps."""
    tiers = [dict(k_fmt=dtype, v_fmt=dtype, capacity=192, block_tokens=64, ring_blocks=4),
             dict(k_fmt=slow[0], v_fmt=slow[1], capacity=10**9, block_tokens=128, ring_blocks=24)]
    st = run_config(3, Hq, Hkv, tiers, dtype, None, 70, synth.SEED_BASE + 20 + Hq, lens=[5, 1033, 2890], check_state_every=35,
                    peaked=True, want_stats=True)
    assert st["mfma_launches"] == 70, st


@pytest.mark.parametrize("fast_cap,slow,n_slots,overlap", [(256, ("f16", "f16"), 0, True), (256, ("i8", "i4"), 0, True),
                                                          (64, ("i8", "i4"), 0, True), (256, ("i8", "i8"), 0, True),
                                                          (256, ("i8", "i4"), 1, False), (256, ("f16", "f16"), 2, True)])
def test_two_tier_layouts_of_the_ablation_table(fast_cap, slow, n_slots, overlap):
    """The paper's two-tier layouts (Sec. 5.4): fp16 window in HBM + everything older on the host as fp16 (the
    FP16 baseline), as K 8-bit / V 4-bit (TTKV), with no fast tier beyond one landing block, as uniform (8, 8),
    and without streaming (copies and kernels serialised on one stream)."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=fast_cap, block_tokens=64, ring_blocks=fast_cap // 64 + 1),
             dict(k_fmt=slow[0], v_fmt=slow[1], capacity=10**9, block_tokens=64, ring_blocks=50, mem="host")]
    run_config(2, 8, 2, tiers, "f16", None, 70, synth.SEED_BASE + 30 + fast_cap, lens=[900, 2777], check_state_every=35,
               n_slots=n_slots, overlap=overlap)


@pytest.mark.parametrize("n_slots", [0, 2, 3])
def test_three_tiers_with_host_streaming_and_eviction_cascade(n_slots):
    """fp16 -> int8 (HBM) -> int4 (pinned host): 150 steps cross several evictions of both device tiers;
    state compared along the way.  n_slots 0: the kernel reads the host records in place;
    2, 3: block copies into staging slots, event-chained with the attention kernels."""
    run_config(2, 8, 2, tiers3("f16"), "f16", 2900, 150 if n_slots != 3 else 20, synth.SEED_BASE + 4,
               check_state_every=50, n_slots=n_slots)


@pytest.mark.parametrize("Hq,Hkv,dtype,paged", [(4, 4, "f16", False), (8, 2, "bf16", False), (8, 2, "f16", True)])
def test_step_as_two_calls(Hq, Hkv, dtype, paged):
    """Append (ttkv_quantize_append on tier 0) and attention (ttkv_decode_attn) as separate calls; every other test
    steps through ttkv_decode_step, where the merge kernel adds the new token and stores its row."""
    run_config(2, Hq, Hkv, tiers3(dtype, paged=paged, rings=(6, 8, 16)), dtype, 2900, 70, synth.SEED_BASE + 60 + Hq,
               check_state_every=35, one_call_step=False)


@pytest.mark.parametrize("first", [("i8", "i8"), ("i8", "i4")])
def test_step_with_a_quantized_first_tier(first):
    """No fp tier at all (the ablation's "no fast tier" taken to the end): ttkv_decode_step falls back to
    quantize-append + attention, same state and outputs."""
    tiers = [dict(k_fmt=first[0], v_fmt=first[1], capacity=256, block_tokens=64, ring_blocks=6),
             dict(k_fmt="i4", v_fmt="i4", capacity=10**9, block_tokens=128, ring_blocks=30)]
    run_config(2, 8, 2, tiers, "f16", 1500, 70, synth.SEED_BASE + 62, check_state_every=35)


@pytest.mark.parametrize("variant", ["plain", "paged", "summary"])
def test_host_tier_bulk_load_written_by_the_kernels(variant):
    """The initial state of the host tier stored by the conversion kernels straight into the pinned records
    (no staging workspace, no copies): same codes, scales, zeros, summaries and outputs."""
    if variant == "plain":
        run_config(2, 8, 2, tiers3("f16"), "f16", 2900, 3, synth.SEED_BASE + 4, host_append_direct=True)
    elif variant == "paged":
        run_config(4, 8, 2, tiers3("f16", paged=True, rings=(6, 8, 12)), "f16", None, 3, synth.SEED_BASE + 5,
                   lens=[300, 1500, 2900, 2047], host_append_direct=True)
    else:
        tiers = tiers3("bf16", summary=True, bts=(64, 128, 128), rings=(6, 8, 40))
        run_config(2, 8, 2, tiers, "bf16", 3500, 3, synth.SEED_BASE + 6, select_k=6, host_append_direct=True)


@pytest.mark.parametrize("n_slots,paged", [(0, False), (2, False), (0, True)])
def test_evictions_into_the_host_tier_written_by_the_kernels(n_slots, paged):
    """ttkv_tier_demote without a workspace: the conversion kernels store the evicted blocks into the pinned records
    (no staging record, no copies, no events); the records are then read in place or copied to staging slots."""
    if paged:
        run_config(4, 8, 2, tiers3("f16", paged=True, rings=(6, 8, 12)), "f16", None, 70, synth.SEED_BASE + 5,
                   lens=[300, 1500, 2900, 2047], check_state_every=35, n_slots=n_slots, host_demote_direct=True)
    else:
        run_config(2, 8, 2, tiers3("f16"), "f16", 2900, 150, synth.SEED_BASE + 4, check_state_every=50, n_slots=n_slots,
                   host_demote_direct=True)


def test_host_tier_no_overlap_gives_the_same_result():
    run_config(2, 8, 2, tiers3("f16"), "f16", 2900, 3, synth.SEED_BASE + 4, overlap=False, n_slots=2)


@pytest.mark.parametrize("n_slots", [0, 2])
def test_paged_tiers_with_ragged_batch(n_slots):
    """Shuffled block tables (paged KV) on the int8 and host tiers, ragged contexts."""
    run_config(4, 8, 2, tiers3("f16", paged=True, rings=(6, 8, 12)), "f16", None, 70, synth.SEED_BASE + 5,
               lens=[300, 1500, 2900, 2047], check_state_every=35, n_slots=n_slots)


@pytest.mark.parametrize("n_slots,host", [(0, True), (2, True), (0, False)])
def test_sparse_block_selection(n_slots, host):
    """Block identification: mean-key summaries, phi, top-k; only selected host blocks are fetched.  With the last
    tier in HBM the selected blocks' tokens are attended as one run per sequence, in items that span blocks."""
    tiers = tiers3("bf16", summary=True, bts=(64, 128, 128), rings=(6, 8, 40), host=host)
    run_config(2, 8, 2, tiers, "bf16", 3500, 40, synth.SEED_BASE + 6, select_k=6, check_state_every=20, n_slots=n_slots)


@pytest.mark.parametrize("Hq,Hkv,fmt,k", [(4, 2, ("i4", "i4"), 100), (8, 2, ("i8", "i4c"), 37), (2, 2, ("i8", "i8"), 700)])
def test_selection_among_hundreds_of_small_blocks_in_hbm(Hq, Hkv, fmt, k):
    """The last tier in HBM in 64-token blocks, 600 to 700 of them live per sequence (the ranking runs with a thread per
    block), ragged over the batch; k of them attended as one run per sequence whose items span many blocks; k above the
    number of live blocks attends everything, the partly filled newest block included."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=128, block_tokens=64, ring_blocks=4),
             dict(k_fmt=fmt[0], v_fmt=fmt[1], capacity=10**9, block_tokens=64, ring_blocks=720, summary=True)]
    run_config(2, Hq, Hkv, tiers, "f16", None, 70, synth.SEED_BASE + 95 + k, select_k=k, check_state_every=35,
               lens=[127 + 64 * 600, 127 + 64 * 690], peaked=True)


@pytest.mark.parametrize("slow", [("i8", "i8"), ("i4", "i4c")])
def test_many_sequences_with_the_item_size_chosen_per_call(slow):
    """16 ragged sequences of a few thousand tokens, two tiers in HBM: more bytes than one round of workgroups takes in
    256-token items and more runs than fit one item each into a round, so the split plan chooses an item size between
    the two (equal items per run, a whole number of rounds) and re-fits it as the lengths grow and blocks are evicted;
    outputs, lse and the stored state against the oracle over 140 steps."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=1024, block_tokens=128, ring_blocks=9),
             dict(k_fmt=slow[0], v_fmt=slow[1], capacity=10**9, block_tokens=128, ring_blocks=80)]
    lens = [1023 + 128 * n for n in (17, 40, 23, 31, 46, 19, 28, 35, 44, 21, 38, 26, 33, 48, 24, 42)]
    st = run_config(16, 32, 8, tiers, "f16", None, 140, synth.SEED_BASE + 97, lens=lens, check_state_every=70, peaked=True,
                    want_stats=True)
    assert st["mfma_launches"] == 140 and st["demotions"] >= 16


def test_bf16_query_on_fp16_and_quantized_tiers_and_large_batch():
    """bf16 queries over int8/int4 tiers with more (tier, sequence) runs than one launch table holds."""
    tiers = tiers3("bf16", host=False, bts=(64, 64, 64), caps=(128, 192), rings=(3, 5, 8))
    run_config(48, 4, 2, tiers, "bf16", None, 2, synth.SEED_BASE + 9, lens=[50 + 11 * i for i in range(48)])


def test_summaries_match_the_oracle_bit_for_bit():
    tiers = tiers3("f16", summary=True, bts=(64, 128, 256), rings=(6, 8, 16))
    p = Pair(1, 8, 2, tiers, "f16")
    try:
        k, v = synth.kv(synth.SEED_BASE + 7, 2, 2500, "f16")
        p.load(0, k, v)
        g = synth.rng(7)
        for s in range(130):
            p.step(synth.normal(g, (1, 8, 128), "f16"), synth.normal(g, (1, 2, 128), "f16"), synth.normal(g, (1, 2, 128), "f16"))
        want = p.ora.summaries(0)
        assert len(want) >= 7
        for blk, mu in want.items():
            assert np.array_equal(p.gpu.dump_summary(2, 0, blk), mu), blk
    finally:
        p.close()


def test_head_pairs_on_the_vector_kernel():
    """Eight query heads per KV head with an int8 tier (two passes of the score product on the matrix cores) and a last
    tier whose keys are grouped over tokens: the one combination the matrix-core kernel has no case for, so the vector
    kernel serves the heads in pairs, each pair a pass of its own over the bytes."""
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=256, block_tokens=128, ring_blocks=3),
             dict(k_fmt="i8", v_fmt="i8", capacity=512, block_tokens=128, ring_blocks=6),
             dict(k_fmt="i4t", v_fmt="i4", capacity=10**9, block_tokens=128, ring_blocks=30)]
    p = Pair(2, 16, 2, tiers, "f16")
    try:
        g = synth.rng(synth.SEED_BASE + 70)
        for b, n in enumerate((255 + 512 + 128 * 9, 255 + 512 + 128 * 14)):   # whole token groups in the last tier
            k, v = synth.kv((synth.SEED_BASE + 70) * 31 + b, 2, n, "f16")
            p.load(b, k, v)
        p.assert_state_equal()
        for s_ in range(3):
            q = synth.normal(g, (2, 16, 128), "f16")
            kn, vn = synth.normal(g, (2, 2, 128), "f16"), synth.normal(g, (2, 2, 128), "f16")
            r = p.step(q, kn, vn)
            assert_close(r[0], r[2], f"out step {s_}")
            assert_close(r[1], r[3], f"lse step {s_}")
        p.assert_state_equal()
        assert p.gpu.stats()["mfma_launches"] == 0
    finally:
        p.close()


@pytest.mark.parametrize("rows,P,stride", [(37, 19, 24), (9, 700, 704), (5, 257, 257), (4, 1, 1)])
def test_merge_partials_standalone(rows, P, stride):
    """ttkv_merge_partials against the oracle's merge: random partials, empty parts, ragged part counts; one part,
    and more parts than one pass of the workgroup takes (several batches, halves with different batch counts)."""
    g = synth.rng(synth.SEED_BASE + 8)
    m = (g.standard_normal((rows, stride)) * 5).astype(np.float32)
    l = (g.random((rows, stride)) * 50 + 0.1).astype(np.float32)
    acc = (g.standard_normal((rows, stride, 128)) * 30).astype(np.float32)
    m[3, min(4, P - 1)] = -np.inf
    l[3, min(4, P - 1)] = 0
    acc[3, min(4, P - 1)] = 0
    m[2, :] = -np.inf
    l[2, :] = 0
    acc[2] = 0
    cnt = g.integers(1, P + 1, rows).astype(np.int32)
    cnt[1] = 0
    cnt[0] = P
    h = B.ttkv_create()
    try:
        for counts in (None, cnt):
            out = torch.empty(rows, 128, dtype=torch.float32, device="cuda:0")
            lse = torch.empty(rows, dtype=torch.float32, device="cuda:0")
            B.ttkv_merge_partials(h, torch.from_numpy(m).cuda(), torch.from_numpy(l).cuda(), torch.from_numpy(acc).cuda(), P, stride,
                                  None if counts is None else torch.from_numpy(counts).cuda(), rows, out, lse, None)
            torch.cuda.synchronize()
            for r in range(rows):
                n = P if counts is None else int(counts[r])
                acc_p = O.empty_partial(1, 128)
                for i in range(n):
                    O.merge_into(acc_p, (m[r, i:i + 1].astype(np.float64), l[r, i:i + 1].astype(np.float64),
                                         acc[r, i:i + 1].astype(np.float64)))
                ro, rl = O.finalize(acc_p)
                got = out[r].cpu().numpy()
                assert np.max(np.abs(got - ro[0])) <= 1e-5 * (1 + np.max(np.abs(ro[0]))), r
                gl = float(lse[r])
                assert (gl == rl[0]) if not np.isfinite(rl[0]) else abs(gl - rl[0]) < 1e-5 * (1 + abs(rl[0])), r
    finally:
        B.ttkv_destroy(h)


def test_capacity_error_leaves_state_untouched():
    tiers = [dict(k_fmt="f16", v_fmt="f16", capacity=64, block_tokens=64, ring_blocks=1)]
    p = Pair(1, 2, 2, tiers, "f16")
    try:
        k = dev(np.zeros((1, 2, 64, 128), np.float32), "f16")
        p.gpu.append(0, k, k)
        with pytest.raises(B.TTKVError) as e:
            p.gpu.append(0, k[:, :, :1].contiguous(), k[:, :, :1].contiguous())
        assert e.value.status == B.ERR_CAPACITY and int(p.gpu.len[0][0]) == 64
    finally:
        p.close()


@pytest.mark.parametrize("Hq,Hkv,dtype,host,n_slots", [(4, 4, "f16", False, 0), (4, 2, "f16", False, 0), (8, 2, "bf16", False, 0),
                                                       (4, 4, "f16", True, 0), (16, 2, "f16", False, 0), (10, 2, "f16", True, 0),
                                                       (4, 4, "f16", True, 2), (8, 2, "f16", True, 3)])
def test_keys_grouped_over_tokens_per_channel(Hq, Hkv, dtype, host, n_slots):
    """Last tier with int4 keys that have one (scale, zero) per channel and 128 tokens (values int4 per token):
    bulk load of whole groups, eviction of whole 128-token blocks, codes / scales / zeros bit-exact, outputs within
    tolerance with outlier channels on the keys; one query head per KV head on the vector kernel, two, four, five
    and eight on the matrix-core kernel; HBM and pinned host (read in place and through staging slots)."""
    tiers = [dict(k_fmt=dtype, v_fmt=dtype, capacity=256, block_tokens=128, ring_blocks=3),
             dict(k_fmt="i4t", v_fmt="i4", capacity=10**9, block_tokens=128 if not host else 256, ring_blocks=30,
                  mem="host" if host else "device")]
    p = Pair(2, Hq, Hkv, tiers, dtype, n_slots=n_slots, host_append_direct=host and n_slots == 3)   # one case: bulk load stored by the kernels
    try:
        g = synth.rng(synth.SEED_BASE + 50 + Hq)
        for b, n in enumerate((128 * 9 + 255, 128 * 20 + 130)):       # tier 0 takes the newest 255 / 130... rest whole groups
            k, v = synth.kv((synth.SEED_BASE + 50) * 31 + b, Hkv, n, dtype)
            k[:, :, 5::37] *= 8.0                                       # outlier channels
            k = synth.round_to(k, dtype)
            # the oracle's loader puts cap - 1 = 255 tokens into tier 0; the rest must be whole groups
            n_old = n - 255
            n_old -= n_old % 128
            k, v = k[:, -(n_old + 255):], v[:, -(n_old + 255):]
            p.load(b, k, v)
        p.assert_state_equal()
        worst = 0.0
        for s in range(300):
            q = synth.normal(g, (2, Hq, 128), dtype)
            kn, vn = synth.normal(g, (2, Hkv, 128), dtype), synth.normal(g, (2, Hkv, 128), dtype)
            kn[:, :, 5::37] *= 8.0
            kn = synth.round_to(kn, dtype)
            r = p.step(q, kn, vn)
            assert_close(r[0], r[2], f"out step {s}")
            assert_close(r[1], r[3], f"lse step {s}")
            worst = max(worst, float(np.max(np.abs(r[0] - r[2]) / (2e-3 + 1e-2 * np.abs(r[2])))))
            if s % 100 == 99:
                p.assert_state_equal()
        p.assert_state_equal()
        print(f"worst error / tolerance: {worst:.3f}")
        assert worst < (0.5 if Hq // Hkv >= 2 else 0.25)   # scaled queries as fp16 hi + lo: as accurate as the other formats of each kernel
        st = p.gpu.stats()
        assert st["demotions"] == sum(sum(d) for d in p.ora.demotions) >= 4
        assert (st["mfma_launches"] > 0) == (Hq // Hkv >= 2)
    finally:
        p.close()


@pytest.mark.parametrize("Hq,Hkv,dtype,kfmt,host,n_slots", [(8, 2, "f16", "i8", False, 0), (8, 2, "f16", "i4", False, 0), (4, 2, "bf16", "i8", False, 0),
                                                            (6, 2, "f16", "i4", False, 0), (16, 2, "f16", "i8", False, 0), (16, 2, "bf16", "i4", False, 0),
                                                            (32, 2, "f16", "i4", False, 0), (8, 2, "f16", "i8", True, 0), (8, 2, "bf16", "i4", True, 2),
                                                            (8, 2, "f16", "i4", True, 3), (32, 2, "f16", "i8", True, 0),
                                                            (16, 1, "bf16", "i8", True, 2)])
def test_values_stored_channel_major_per_32_tokens(Hq, Hkv, dtype, kfmt, host, n_slots):
    """Last tier with Q_4bit values stored channel-major per 32 tokens (the matrix cores take them without a
    transposition): the codes, decoded from that packing, and the scales / zeros equal the oracle's Q_4bit bit for
    bit -- bulk load of whole groups, evictions of 64-token blocks, through an int8 tier in the three-tier cases --
    and the outputs stay within tolerance with peaked softmax; int8 and int4 keys, 2 to 16 heads per KV head (one-,
    two- and four-pass cases), HBM and pinned host (read in place, through staging slots, bulk load stored by the kernels)."""
    three = host
    tiers = [dict(k_fmt=dtype, v_fmt=dtype, capacity=256, block_tokens=64, ring_blocks=6)]
    if three:
        tiers.append(dict(k_fmt="i8", v_fmt="i8", capacity=512, block_tokens=128, ring_blocks=8))
    tiers.append(dict(k_fmt=kfmt, v_fmt="i4c", capacity=10**9, block_tokens=256 if host else 128, ring_blocks=30,
                      mem="host" if host else "device"))
    p = Pair(3, Hq, Hkv, tiers, dtype, n_slots=n_slots, host_append_direct=host and n_slots == 3)
    try:
        g = synth.rng(synth.SEED_BASE + 80 + Hq)
        fixed = 255 + (512 if three else 0)
        for b, n_old in enumerate((32 * 1, 32 * 33, 32 * 90 + 64)):       # whole groups of 32 in the last tier
            k, v = synth.kv((synth.SEED_BASE + 80) * 31 + b, Hkv, fixed + n_old, dtype)
            k[:, ::97] *= 4.0                                              # a few keys aligned with nothing in particular: O(1) weights
            p.load(b, synth.round_to(k, dtype), v)
        p.assert_state_equal()
        worst = 0.0
        for s in range(200):
            q = synth.normal(g, (3, Hq, 128), dtype)
            kn, vn = synth.normal(g, (3, Hkv, 128), dtype), synth.normal(g, (3, Hkv, 128), dtype)
            r = p.step(q, kn, vn)
            worst = max(worst, assert_close(r[0], r[2], f"out step {s}"))
            assert_close(r[1], r[3], f"lse step {s}")
            if s % 100 == 99:
                p.assert_state_equal()
        st = p.gpu.stats()
        assert st["demotions"] == sum(sum(d) for d in p.ora.demotions) >= 6
        assert st["mfma_launches"] > 0 and st["h2d_bytes"] == p.ora.h2d_bytes
        for b in range(3):
            total = sum(int(p.gpu.len[t][b]) for t in range(len(tiers)))
            p.assert_locate_equal(b, [0, total // 2, total - 1])
    finally:
        p.close()


def test_channel_major_values_are_refused_where_no_kernel_takes_them():
    """One query head per KV head runs on the vector kernel, which reads token-major rows only; the format is for
    the last tier and for whole groups of 32 tokens."""
    ok = [dict(k_fmt="f16", v_fmt="f16", capacity=256, block_tokens=64, ring_blocks=6),
          dict(k_fmt="i8", v_fmt="i4c", capacity=10**9, block_tokens=128, ring_blocks=8)]
    p = Pair(1, 4, 4, ok, "f16")           # 4 q / 4 kv heads
    try:
        k = dev(np.zeros((1, 4, 64, 128), np.float32), "f16")
        with pytest.raises(B.TTKVError) as e:
            p.gpu.append(1, k, k)
        assert e.value.status == B.ERR_UNSUPPORTED
    finally:
        p.close()
    p = Pair(1, 8, 4, ok, "f16")
    try:
        k = dev(np.zeros((1, 4, 48, 128), np.float32), "f16")
        with pytest.raises(B.TTKVError) as e:
            p.gpu.append(1, k, k)            # 48 tokens: not whole groups of 32
        assert e.value.status == B.ERR_INVALID_ARG and int(p.gpu.len[1][0]) == 0
        middle = [ok[0], dict(k_fmt="i8", v_fmt="i4c", capacity=512, block_tokens=128, ring_blocks=8),
                  dict(k_fmt="i4", v_fmt="i4", capacity=10**9, block_tokens=128, ring_blocks=8)]
    finally:
        p.close()
    p = Pair(1, 8, 4, middle, "f16")
    try:
        with pytest.raises(B.TTKVError) as e:
            p.gpu.append(0, k, k)
        assert e.value.status == B.ERR_UNSUPPORTED    # a middle tier: values would have to pass through it
    finally:
        p.close()


@pytest.mark.parametrize("n_slots,paged,host", [(0, False, True), (2, False, True), (0, True, True), (0, False, False), (0, True, False)])
def test_block_selection_over_channel_major_values(n_slots, paged, host):
    """Block identification + top-k + attention of the selected host blocks when the host tier's values are stored
    channel-major per 32 tokens: ids left on the device (the kernel looks the blocks up and takes the newest one's
    live length, a multiple of 32, from the launch arguments), ids on the host with staged copies, paged records."""
    tiers = tiers3("bf16", fmts=(("i8", "i8"), ("i4", "i4c")), summary=True, bts=(64, 128, 128), rings=(6, 8, 40), paged=paged, host=host)
    run_config(2, 8, 2, tiers, "bf16", 255 + 512 + 32 * 85, 40, synth.SEED_BASE + 90, select_k=6, check_state_every=20, n_slots=n_slots)
