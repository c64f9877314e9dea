"""Pins for the oracle's attention partials, log-sum-exp merge, tier state machine,
block index, selection and traffic counter (Sec. 4.1, 4.3, Alg. 1).  Pins are the
plain definition of softmax attention over the union of attended tokens (brute
force, fp64), torch's own scaled_dot_product_attention, closed forms and
invariants -- not the oracle's own formulas."""
import math

import numpy as np
import pytest
import torch

import oracle as O
from oracle import OracleCache, TierSpec


def brute_attention(q, K, V, scale):
    """softmax(scale * q K^T) V straight from the definition, fp64, one pass."""
    Hq, Hkv = q.shape[0], K.shape[0]
    G = Hq // Hkv
    out = np.zeros((Hq, K.shape[2]))
    lse = np.zeros(Hq)
    for h in range(Hq):
        s = scale * (K[h // G].astype(np.float64) @ q[h].astype(np.float64))
        w = np.exp(s - s.max())
        out[h] = (w / w.sum()) @ V[h // G].astype(np.float64)
        lse[h] = s.max() + math.log(w.sum())
    return out, lse


def rand(rng, *shape):
    return rng.standard_normal(shape).astype(np.float16).astype(np.float32)


@pytest.mark.parametrize("Hq,Hkv,d,N", [(8, 2, 128, 37), (4, 4, 64, 64), (6, 1, 128, 5)])
def test_partial_plus_finalize_is_textbook_attention(Hq, Hkv, d, N):
    rng = np.random.default_rng(10)
    q, K, V = rand(rng, Hq, d), rand(rng, Hkv, N, d), rand(rng, Hkv, N, d)
    scale = 1 / math.sqrt(d)
    out, lse = O.finalize(O.attn_partial(q, K, V, 0, N, scale))
    ref, ref_lse = brute_attention(q, K, V, scale)
    assert np.max(np.abs(out - ref)) < 1e-12 and np.max(np.abs(lse - ref_lse)) < 1e-12
    # independent library routine, fp32
    G = Hq // Hkv
    tq = torch.from_numpy(q)[None, :, None, :]
    tk = torch.from_numpy(np.repeat(K, G, axis=0))[None]
    tv = torch.from_numpy(np.repeat(V, G, axis=0))[None]
    sd = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=scale)[0, :, 0].numpy()
    assert np.max(np.abs(out - sd)) < 2e-6


def test_partial_respects_range_and_gqa_mapping():
    rng = np.random.default_rng(11)
    q, K, V = rand(rng, 8, 128), rand(rng, 2, 50, 128), rand(rng, 2, 50, 128)
    out, _ = O.finalize(O.attn_partial(q, K, V, 13, 21, 0.1))
    ref, _ = brute_attention(q, K[:, 13:34], V[:, 13:34], 0.1)
    assert np.max(np.abs(out - ref)) < 1e-12
    # heads 0-3 read KV head 0, heads 4-7 KV head 1: zero out KV head 1's values
    V2 = V.copy()
    V2[1] = 0
    out2, _ = O.finalize(O.attn_partial(q, K, V2, 0, 50, 0.1))
    assert np.all(out2[4:] == 0) and np.max(np.abs(out2[:4])) > 0


def test_closed_forms():
    rng = np.random.default_rng(12)
    K, V = rand(rng, 2, 40, 128), rand(rng, 2, 40, 128)
    # q = 0: uniform weights -> mean of V, lse = ln N
    out, lse = O.finalize(O.attn_partial(np.zeros((4, 128), np.float32), K, V, 0, 40, 0.3))
    assert np.max(np.abs(out - np.repeat(V.astype(np.float64).mean(1), 2, axis=0))) < 1e-13
    assert np.max(np.abs(lse - math.log(40))) < 1e-13
    # all keys equal -> mean of V whatever q is
    Keq = np.broadcast_to(K[:, :1], K.shape).copy()
    out, _ = O.finalize(O.attn_partial(rand(rng, 4, 128), Keq, V, 0, 40, 0.3))
    assert np.max(np.abs(out - np.repeat(V.astype(np.float64).mean(1), 2, axis=0))) < 1e-12
    # one key far ahead (score +60 over the rest) -> that token's value
    q = np.zeros((2, 128), np.float32)
    q[:, 0] = 1
    K0 = np.zeros((2, 40, 128), np.float32)
    K0[:, 17, 0] = 60
    out, lse = O.finalize(O.attn_partial(q, K0, V, 0, 40, 1.0))
    assert np.max(np.abs(out - V[:, 17])) < 1e-20 + 40 * math.exp(-60) * 10
    assert np.max(np.abs(lse - 60)) < 1e-12


def test_merge_is_partition_and_order_independent_with_identity():
    rng = np.random.default_rng(13)
    q, K, V = rand(rng, 8, 128), rand(rng, 2, 200, 128) * 3, rand(rng, 2, 200, 128)
    scale = 0.2
    ref, ref_lse = brute_attention(q, K, V, scale)
    for trial in range(6):
        cuts = np.sort(rng.choice(np.arange(1, 200), size=rng.integers(1, 12), replace=False))
        bounds = [0, *cuts, 200]
        parts = [O.attn_partial(q, K, V, a, b - a, scale) for a, b in zip(bounds[:-1], bounds[1:])]
        parts.insert(int(rng.integers(0, len(parts))), O.empty_partial(8, 128))   # identity element
        parts.append(O.attn_partial(q, K, V, 5, 0, scale))                          # empty range
        order = rng.permutation(len(parts))
        P = O.empty_partial(8, 128)
        for i in order:
            O.merge_into(P, parts[i])
        out, lse = O.finalize(P)
        assert np.max(np.abs(out - ref) / (np.abs(ref) + 1e-3)) < 1e-9
        assert np.max(np.abs(lse - ref_lse)) < 1e-10
    out, lse = O.finalize(O.empty_partial(3, 128))
    assert np.all(out == 0) and np.all(lse == -np.inf)


# ------------------------------------------------------------------ state machine

def make_cache(B=2, caps=(64, 128), bts=(16, 32, 64), fmts=("f16", "i8", "i4"), maxtok=4096, summary=False):
    tiers = [TierSpec(fmts[0], fmts[0], caps[0], bts[0]),
             TierSpec(fmts[1], fmts[1], caps[1], bts[1]),
             TierSpec(fmts[2], fmts[2], 10**9, bts[2], mem="host", summary=summary)]
    return OracleCache(B, 8, 2, 128, tiers, maxtok)


def run_steps(c, T, rng, keep=None):
    for t in range(T):
        q, k, v = rand(rng, c.B, 8, 128), rand(rng, c.B, 2, 128), rand(rng, c.B, 2, 128)
        if keep is not None:
            keep.append((q, k, v))
        yield c.step(q, k, v)


def test_tier_invariants_and_demotion_counts():
    rng = np.random.default_rng(14)
    c = make_cache()
    T = 700
    for t, _ in enumerate(run_steps(c, T, rng), 1):
        for b in range(c.B):
            ranges = [c.tier_range(i, b) for i in range(3)]
            live = [r for r in ranges if r is not None and r[1] > r[0]]
            assert sum(r[1] - r[0] for r in live) == t                      # partition covers [0, t)
            assert live[0][1] == t and live[-1][0] == 0
            for newer, older in zip(live[:-1], live[1:]):
                assert older[1] == newer[0]                                  # adjacent, ordered oldest -> newest
            n0 = c.seq[0][b].count
            assert n0 < 64 and (t < 64 or n0 >= 64 - 16)                     # after evicting: (cap - B_blk, cap)
            # closed form: tier 0 evicts one block each time it reaches 64 = every 16 appends from t = 64
            d0 = 0 if t < 64 else (t - 64) // 16 + 1
            assert c.demotions[0][b] == d0
            n1_in = 16 * d0
            d1 = 0 if n1_in < 128 else (n1_in - 128) // 32 + 1
            assert c.demotions[1][b] == d1 and c.seq[2][b].count == 32 * d1


def test_locate_matches_direct_enumeration():
    rng = np.random.default_rng(15)
    c = make_cache(B=1)
    list(run_steps(c, 500, rng))
    # enumerate: tier 2 got tokens 0.. in 32-token evictions into 64-token blocks, etc.
    r2, r1, r0 = c.tier_range(2, 0), c.tier_range(1, 0), c.tier_range(0, 0)
    for pos in range(500):
        t, blk, off = c.locate(0, pos)
        if pos < r2[1]:
            assert (t, blk, off) == (2, pos // 64, pos % 64)
        elif pos < r1[1]:
            assert (t, blk, off) == (1, pos // 32, pos % 32)      # tier 1's stream also starts at position 0
        else:
            assert (t, blk, off) == (0, pos // 16, pos % 16)
    with pytest.raises(KeyError):
        c.locate(0, 500)


def test_step_equals_brute_force_over_decompressed_union():
    """A full tiered step equals plain softmax attention over what the tiers hold."""
    rng = np.random.default_rng(16)
    c = make_cache(B=2)
    hist = []
    list(run_steps(c, 300, rng, hist))
    # replay all but the last step, then append + attend by hand so the pre-eviction state is visible
    c2 = make_cache(B=2)
    for q, k, v in hist[:-1]:
        c2.step(q, k, v)
    q, k, v = hist[-1]
    for b in range(2):
        c2.append(0, b, k[b][:, None], v[b][:, None], c2.total[b])
        c2.total[b] += 1
    out, lse = c2.attend(q)
    for b in range(2):
        Ks, Vs = [], []
        for t in (2, 1, 0):
            s = c2.seq[t][b]
            Ks.append(s.khat[:, s.first:s.first + s.count])
            Vs.append(s.vhat[:, s.first:s.first + s.count])
        K, V = np.concatenate(Ks, 1), np.concatenate(Vs, 1)
        assert K.shape[1] == 300
        ref, ref_lse = brute_attention(q[b], K, V, c2.scale)
        assert np.max(np.abs(out[b] - ref)) < 1e-12 and np.max(np.abs(lse[b] - ref_lse)) < 1e-11


def test_all_fp16_tiers_equal_exact_attention_on_raw_inputs():
    """With every tier full precision the tiered step is attention with no approximation."""
    rng = np.random.default_rng(17)
    c = make_cache(B=1, fmts=("f16", "f16", "f16"))
    hist = []
    outs = list(run_steps(c, 260, rng, hist))
    K = np.stack([h[1][0] for h in hist], 1)
    V = np.stack([h[2][0] for h in hist], 1)
    ref, _ = brute_attention(hist[-1][0][0], K, V, c.scale)
    assert np.max(np.abs(outs[-1][0][0] - ref)) < 1e-12


def test_stored_codes_follow_the_format_chain():
    """A token that went fp16 -> int8 -> int4 holds Q2(D1(Q1(x)))."""
    rng = np.random.default_rng(18)
    c = make_cache(B=1)
    hist = []
    list(run_steps(c, 400, rng, hist))
    s2 = c.seq[2][0]
    assert s2.count > 0
    k_raw = np.stack([h[1][0] for h in hist], 1)[:, :s2.count]
    want = O.quant_i4(O.dequant_i8(*O.quant_i8(k_raw)))
    assert np.array_equal(s2.kq["codes"][:, :s2.count], want[0])
    assert np.array_equal(s2.kq["scale"][:, :s2.count], want[1])
    assert np.array_equal(s2.kq["zero"][:, :s2.count], want[2])


def test_load_distributes_newest_first_through_the_format_chain():
    rng = np.random.default_rng(19)
    N = 500
    K, V = rand(rng, 2, N, 128), rand(rng, 2, N, 128)
    c = make_cache(B=1, caps=(64, 128))
    spans = c.load(0, K, V)
    assert spans == [(437, 500), (309, 437), (0, 309)]          # cap0-1 newest, cap1 next, rest oldest
    assert [c.tier_range(t, 0) for t in range(3)] == spans
    s2 = c.seq[2][0]
    want = O.quant_i4(O.dequant_i8(*O.quant_i8(K[:, :309])))    # reached tier 2 through tier 1's int8
    assert np.array_equal(s2.kq["codes"][:, :309], want[0]) and np.array_equal(s2.kq["scale"][:, :309], want[1])
    assert np.array_equal(c.seq[1][0].vq["codes"][:, :128], O.quant_i8(V[:, 309:437])[0])
    assert np.array_equal(c.seq[0][0].khat[:, :63], K[:, 437:])
    # the next step appends -> tier 0 reaches its capacity exactly -> attends N+1 tokens -> evicts
    q, k, v = rand(rng, 1, 8, 128), rand(rng, 1, 2, 128), rand(rng, 1, 2, 128)
    c.step(q, k, v)
    assert [c.seq[t][0].count for t in range(3)] == [48, 128 + 16 - 32, 309 + 32] and c.demotions == [[1], [1], [0]]


# ------------------------------------------------------------------ selection, traffic

def planted_cache(rng, n_blocks=12, planted=(3, 7)):
    c = OracleCache(1, 8, 2, 128, [TierSpec("f16", "f16", 32, 16), TierSpec("i4", "i4", 10**9, 64, mem="host", summary=True)], 2048)
    q = rand(rng, 1, 8, 128)
    N = n_blocks * 64
    K, V = rand(rng, 2, N, 128), rand(rng, 2, N, 128)
    for j in planted:                       # shift the block's keys along the mean query of each KV head's group
        for h in range(2):
            u = q[0, 4 * h:4 * h + 4].mean(0)
            K[h, 64 * j:64 * j + 64] += (2.0 * u / np.linalg.norm(u)).astype(np.float32)
    K = K.astype(np.float16).astype(np.float32)
    c.append(1, 0, K, V, 0)
    c.total[0] = N
    return c, q


def test_selection_properties():
    rng = np.random.default_rng(20)
    c, q = planted_cache(rng)
    sel = c.select(q, 4)[0]
    assert len(sel) == 4 and np.all(np.diff(sel) > 0) and {3, 7} <= set(sel.tolist())
    dense, _ = c.attend(q)
    every, _ = c.attend(q, c.select(q, 100))              # k >= n_blocks: identical to dense
    assert np.array_equal(dense, every)
    none, lse = c.attend(q, c.select(q, 0))               # k = 0 and empty tier 0: nothing attended
    assert np.all(none == 0) and np.all(lse == -np.inf)
    # ties go to the lower index
    assert O.topk(np.array([1, 5, 5, 0, 5], np.float32), 2).tolist() == [1, 2]
    assert O.topk(np.array([2, 2, 2], np.float32), 2).tolist() == [0, 1]


def token_order_mean_bits(K, lo, hi, block_tokens):
    """fp16 bits of (fp32 sum of K[:, lo:hi] in token order) * (1 / block_tokens): the mean key as Alg. 1's
    identification step reads it, written out with numpy (each `+` below is one IEEE fp32 addition per element)."""
    s = np.zeros((K.shape[0], K.shape[2]), np.float32)
    for t in range(lo, hi):
        s = s + K[:, t]
    return (s * np.float32(1.0 / block_tokens)).astype(np.float16).view(np.uint16)


def test_summary_accumulate_token_range_and_head_stride():
    """The accumulator adds exactly tokens [t0, t0 + n) of every head, in token order, to what it held."""
    rng = np.random.default_rng(23)
    x = rand(rng, 3, 50, 128)                                  # 3 KV heads, 50 tokens held (stride 50)
    for t0, n in ((0, 50), (7, 1), (7, 0), (13, 29), (49, 1)):
        acc = rng.standard_normal((3, 128)).astype(np.float32)
        want = acc.copy()
        for t in range(t0, t0 + n):
            want = want + x[:, t]
        O.summary_accumulate(acc, x, t0, n)
        assert np.array_equal(acc, want), (t0, n)
    # integer-valued keys: every partial sum is exact, so the result is the exact sum whatever the order
    xi = rng.integers(-8, 9, (2, 40, 128)).astype(np.float32)
    acc = np.zeros((2, 128), np.float32)
    O.summary_accumulate(acc, xi, 5, 30)
    assert np.array_equal(acc, xi[:, 5:35].sum(1))
    # one token off at either end, or the other head's rows, is a different number
    assert not np.array_equal(acc, xi[:, 4:34].sum(1)) and not np.array_equal(acc, xi[:, 5:36].sum(1))
    assert not np.array_equal(acc[0], xi[1, 5:35].sum(0))


@pytest.mark.parametrize("pieces", [[768], [40, 100, 300, 328], [64, 64, 1, 63, 200, 376], [1] * 70 + [698]])
def test_block_summaries_are_token_order_means_of_the_keys(pieces):
    """Mean keys of a tier fed by appends that straddle block boundaries, fill a block in several calls, or
    stop inside a block: each equals the token-order fp32 mean of that block's keys, bit for bit, for both KV
    heads; a partly filled newest block divides by B_blk as well."""
    rng = np.random.default_rng(24)
    bt, N = 64, sum(pieces) - 24                               # the last block holds 40 of 64 tokens
    pieces = pieces[:-1] + [pieces[-1] - 24]
    c = OracleCache(1, 8, 2, 128, [TierSpec("f16", "f16", 32, 16), TierSpec("i4", "i4", 10**9, bt, mem="host", summary=True)], 2048)
    K, V = rand(rng, 2, N, 128), rand(rng, 2, N, 128)
    o = 0
    for n in pieces:
        c.append(1, 0, K[:, o:o + n], V[:, o:o + n], o)
        o += n
    c.total[0] = N
    mu = c.summaries(0)
    assert sorted(mu) == list(range((N + bt - 1) // bt))
    for j in mu:
        want = token_order_mean_bits(K, j * bt, min(N, (j + 1) * bt), bt)
        assert np.array_equal(mu[j], want), j
        # and it is the mean key: within fp16 rounding + fp32 summation error of the fp64 mean
        ref = K[:, j * bt:min(N, (j + 1) * bt)].astype(np.float64).sum(1) / bt
        assert np.max(np.abs(O.f16_bits_to_f32(mu[j]) - ref)) <= np.abs(ref).max() * 2.0 ** -10 + 1e-5


def test_block_summaries_after_eviction_are_means_of_what_the_quantizer_received():
    """Blocks that reach the summarised tier by eviction (Alg. 1, evict & compress) out of an fp16 tier with a
    smaller block: the mean is over the values that entered that tier's quantizer (the stored fp16 keys), in
    token order, several evictions filling one block."""
    rng = np.random.default_rng(25)
    tiers = [TierSpec("f16", "f16", 64, 32), TierSpec("i4", "i4", 10**9, 128, mem="host", summary=True)]
    c = OracleCache(1, 4, 2, 128, tiers, [2048, 2048])
    ks = []
    for _ in range(500):
        q, k, v = rand(rng, 1, 4, 128), rand(rng, 1, 2, 128), rand(rng, 1, 2, 128)
        ks.append(k[0])
        c.step(q, k, v)
    K = np.stack(ks, 1)                                         # [Hkv][500][128]
    n1 = c.seq[1][0].count
    assert n1 == 448 and c.seq[1][0].first == 0                 # 14 evictions of 32 tokens
    mu = c.summaries(0)
    assert sorted(mu) == [0, 1, 2, 3]
    for j in mu:
        assert np.array_equal(mu[j], token_order_mean_bits(K, j * 128, min(n1, (j + 1) * 128), 128)), j


def test_block_score_is_the_plain_dot_product():
    rng = np.random.default_rng(21)
    q = rand(rng, 8, 128)
    mu = rng.standard_normal((2, 128)).astype(np.float16)
    got = O.block_score(q, mu.view(np.uint16), 2)
    ref = sum(float(q[h].astype(np.float64) @ mu[h // 4].astype(np.float64)) for h in range(8))
    assert abs(got - ref) < 1e-4 * (1 + abs(ref))


def test_block_score_order_free_cases_and_head_mapping():
    """Integer-valued queries and mean keys: every product and partial sum is exact in fp32, so phi must be
    the exact integer sum whatever the accumulation order; and query head h reads KV head h // G."""
    rng = np.random.default_rng(26)
    q = rng.integers(-4, 5, (8, 128)).astype(np.float32)
    mu = rng.integers(-4, 5, (2, 128)).astype(np.float16)
    want = sum(int(q[h].astype(np.int64) @ mu[h // 4].astype(np.int64)) for h in range(8))
    assert O.block_score(q, mu.view(np.uint16), 2) == float(want)
    wrong = sum(int(q[h].astype(np.int64) @ mu[h % 2].astype(np.int64)) for h in range(8))
    assert wrong != want
    # one head alone is the left-to-right fused chain over its channels (single rounding per step)
    q1 = rand(rng, 1, 128)
    m1 = rng.standard_normal((1, 128)).astype(np.float16)
    s = 0.0
    for i in range(128):       # exact product in fp64 (24 x 11 bits), one rounding of product + sum to fp32 = fmaf
        s = float(np.float32(float(q1[0, i]) * float(m1[0, i]) + s))
    assert O.block_score(q1, m1.view(np.uint16), 1) == s


def test_topk_against_brute_force_including_nan_scores():
    """The k chosen are exactly those with fewer than k blocks ahead of them (larger score, or equal score and
    lower index); NaN counts as -inf; always min(k, n) ids, ascending."""
    rng = np.random.default_rng(27)
    for trial in range(200):
        n = int(rng.integers(1, 40))
        sc = rng.integers(-3, 4, n).astype(np.float32)           # many ties
        if trial % 3 == 0:
            sc[rng.integers(0, n, 2)] = np.nan
        if trial % 5 == 0:
            sc[rng.integers(0, n)] = -np.inf
        k = int(rng.integers(0, n + 3))
        key = np.where(np.isnan(sc), -np.inf, sc)
        want = [j for j in range(n) if sum((key[i] > key[j]) or (key[i] == key[j] and i < j) for i in range(n)) < k]
        got = O.topk(sc, k).tolist()
        assert got == want and len(got) == min(k, n), (sc, k, got, want)


def test_h2d_traffic_closed_form():
    # 128K offload shape: 96 records of 1024 tokens x 8 KV heads x 144 B = 1,179,648 B each
    c = OracleCache(1, 32, 8, 128, [TierSpec("bf16", "bf16", 4096, 128), TierSpec("i8", "i8", 28672, 128),
                                    TierSpec("i4", "i4", 10**9, 1024, mem="host")], [8, 8, 8])
    assert c.record_bytes(2) == 1179648 and 96 * c.record_bytes(2) == 113246208
    assert c.record_bytes(1) == 128 * 8 * 272 and c.record_bytes(0) == 128 * 8 * 512
    rng = np.random.default_rng(22)
    c, q = planted_cache(rng)
    c.attend(q)
    assert c.blocks_fetched == 12 and c.h2d_bytes == 12 * 64 * 2 * 144
    c.attend(q, c.select(q, 5))
    assert c.blocks_fetched == 17


def test_two_tier_cache_with_keys_grouped_over_tokens():
    """fp16 window of one 128-token block in front of a tier whose keys are int4 with one (scale, zero) per
    channel and 128 tokens: whole blocks arrive by eviction, the stored codes are that quantizer's on the raw
    keys, and a step equals plain softmax attention over the decompressed union."""
    rng = np.random.default_rng(31)
    tiers = [TierSpec("f16", "f16", 128, 128), TierSpec("i4t", "i4", 10**9, 128)]
    c = OracleCache(1, 4, 2, 128, tiers, [1024, 1024])
    hist = []
    for _ in range(400):
        q, k, v = rand(rng, 1, 4, 128), rand(rng, 1, 2, 128), rand(rng, 1, 2, 128)
        hist.append((q, k, v))
        out, lse = c.step(q, k, v)
    s1, s0 = c.seq[1][0], c.seq[0][0]
    assert s1.count == 384 and s0.count == 16 and c.demotions[0][0] == 3
    k_raw = np.stack([h[1][0] for h in hist], 1)[:, :384]
    want = O.quant_i4_tokens(k_raw)
    assert np.array_equal(s1.kq["codes"][:, :384], want[0]) and np.array_equal(s1.kq["scale"][:, :3], want[1])
    assert np.array_equal(s1.kq["zero"][:, :3], want[2])
    K = np.concatenate([s1.khat[:, :384], s0.khat[:, s0.first:s0.first + 16]], 1)
    V = np.concatenate([s1.vhat[:, :384], s0.vhat[:, s0.first:s0.first + 16]], 1)
    ref, ref_lse = brute_attention(hist[-1][0][0], K, V, c.scale)
    assert np.max(np.abs(out[0] - ref)) < 1e-12 and np.max(np.abs(lse[0] - ref_lse)) < 1e-11
    assert c.record_bytes(1) == 2 * 128 * (68 + 72)
