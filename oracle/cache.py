"""Tiered KV cache state machine of the oracle -- TEST INFRASTRUCTURE ONLY.

Follows the paper's Sec. 4.1 (tier layout, block index, FIFO tier management),
Sec. 4.2 (what is stored per tier) and Alg. 1 (one decode step: attend the fast
tier, attend [selected] slow-tier blocks, accumulate, evict when full).  The
paper has two tiers; here a cache is a list of tiers, newest first, each with
its own precision, so that the paper's layout {FP16 in HBM, K 8-bit / V 4-bit in
host DRAM} is one instance.

Storage is deliberately naive: per tier and sequence one flat array indexed by
the token's ordinal in that tier's lifetime stream (no ring, no pages, no
packing beyond the nibble pairs Q2 defines).  Order of one step (Alg. 1):
append -> attend -> while len >= capacity: evict the oldest block to the next
tier (quantizing what it held, stored or decompressed, into that tier's format).
"""
from dataclasses import dataclass

import numpy as np

import oracle as O

FP_FORMATS = ("f16", "bf16")


@dataclass
class TierSpec:
    k_fmt: str            # 'f16' | 'bf16' | 'i8' (Q1) | 'i4' (Q2) | 'i4t' (Q2 over 128 tokens per channel; keys only)
    v_fmt: str
    capacity: int         # tokens; eviction threshold (L_fast for tier 0)
    block_tokens: int     # B_blk of this tier: eviction unit out of it, attention / fetch unit in it
    mem: str = "device"   # 'device' | 'host'
    summary: bool = False  # keep a per-block mean-key summary (for phi)


def bytes_per_token_head(fmt, d):
    """Stored bytes of one token of one KV head for K or V alone."""
    if fmt in FP_FORMATS:
        return 2 * d
    if fmt == "i8":
        return d + 2 * (d // 32)
    if fmt == "i4":
        return d // 2 + 4 * (d // 64)
    if fmt == "i4t":
        return d // 2 + 4 * d // 128          # one (scale, zero) pair per channel and 128 tokens
    raise ValueError(fmt)


class _Seq:
    """One tier of one sequence."""

    def __init__(self, spec, Hkv, d, max_tokens):
        M = max_tokens
        self.M = M
        self.khat = np.zeros((Hkv, M, d), np.float32)
        self.vhat = np.zeros((Hkv, M, d), np.float32)
        self.kq = self._alloc_q(spec.k_fmt, Hkv, M, d)
        self.vq = self._alloc_q(spec.v_fmt, Hkv, M, d)
        self.first = 0     # ordinal of the oldest live token
        self.count = 0     # live tokens
        self.p0 = None     # sequence position of ordinal 0
        nblk = (M + spec.block_tokens - 1) // spec.block_tokens
        self.ksum = np.zeros((nblk, Hkv, d), np.float32) if spec.summary else None

    @staticmethod
    def _alloc_q(fmt, Hkv, M, d):
        if fmt == "i8":
            return {"codes": np.zeros((Hkv, M, d), np.int8), "scale": np.zeros((Hkv, M, d // 32), np.uint16)}
        if fmt == "i4":
            return {"codes": np.zeros((Hkv, M, d // 2), np.uint8), "scale": np.zeros((Hkv, M, d // 64), np.uint16),
                    "zero": np.zeros((Hkv, M, d // 64), np.uint16)}
        if fmt == "i4t":
            return {"codes": np.zeros((Hkv, M, d // 2), np.uint8), "scale": np.zeros((Hkv, (M + 127) // 128, d), np.uint16),
                    "zero": np.zeros((Hkv, (M + 127) // 128, d), np.uint16)}
        return None


def _store(fmt, x, hat, q, lo, hi):
    """Write x [Hkv][n][d] (fp32) into ordinals [lo, hi) in format fmt."""
    if fmt in FP_FORMATS:
        hat[:, lo:hi] = x
    elif fmt == "i8":
        codes, scale = O.quant_i8(x)
        q["codes"][:, lo:hi] = codes
        q["scale"][:, lo:hi] = scale
        hat[:, lo:hi] = O.dequant_i8(codes, scale)
    elif fmt == "i4":
        codes, scale, zero = O.quant_i4(x)
        q["codes"][:, lo:hi] = codes
        q["scale"][:, lo:hi] = scale
        q["zero"][:, lo:hi] = zero
        hat[:, lo:hi] = O.dequant_i4(codes, scale, zero)
    elif fmt == "i4t":
        assert lo % 128 == 0 and (hi - lo) % 128 == 0, "token groups of 128 arrive whole and aligned"
        codes, scale, zero = O.quant_i4_tokens(x)
        q["codes"][:, lo:hi] = codes
        q["scale"][:, lo // 128:hi // 128] = scale
        q["zero"][:, lo // 128:hi // 128] = zero
        hat[:, lo:hi] = O.dequant_i4_tokens(codes, scale, zero)
    else:
        raise ValueError(fmt)


class OracleCache:
    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, tiers, max_tokens, softmax_scale=None):
        assert n_q_heads % n_kv_heads == 0 and head_dim % 64 == 0
        self.B, self.Hq, self.Hkv, self.d = batch, n_q_heads, n_kv_heads, head_dim
        self.tiers = list(tiers)
        if isinstance(max_tokens, int):
            max_tokens = [max_tokens] * len(self.tiers)
        self.seq = [[_Seq(s, n_kv_heads, head_dim, m) for _ in range(batch)] for s, m in zip(self.tiers, max_tokens)]
        self.scale = float(softmax_scale) if softmax_scale is not None else 1.0 / float(np.sqrt(head_dim))
        self.total = [0] * batch                       # tokens ever appended per sequence
        self.demotions = [[0] * batch for _ in self.tiers]
        self.h2d_bytes = 0                             # host-tier record bytes fetched by attend()
        self.blocks_fetched = 0

    # ------------------------------------------------------------- layout
    def record_bytes(self, t):
        """Bytes of one block record (all KV heads) of tier t."""
        s = self.tiers[t]
        return self.Hkv * s.block_tokens * (bytes_per_token_head(s.k_fmt, self.d) + bytes_per_token_head(s.v_fmt, self.d))

    def tier_range(self, t, b):
        """Sequence positions [lo, hi) tier t holds for sequence b."""
        s = self.seq[t][b]
        if s.p0 is None:
            return None
        return (s.p0 + s.first, s.p0 + s.first + s.count)

    def locate(self, b, pos):
        """Block index of Eq. (1): position -> (tier, block id, offset in block).
        Block ids count blocks of the tier's lifetime stream from 0."""
        for t, spec in enumerate(self.tiers):
            r = self.tier_range(t, b)
            if r is not None and r[0] <= pos < r[1]:
                o = pos - self.seq[t][b].p0
                return (t, o // spec.block_tokens, o % spec.block_tokens)
        raise KeyError(pos)

    def live_blocks(self, t, b):
        """[(block id, first ordinal, n tokens)] of the live tokens of tier t."""
        s, bt = self.seq[t][b], self.tiers[t].block_tokens
        out = []
        if s.count == 0:
            return out
        for blk in range(s.first // bt, (s.first + s.count - 1) // bt + 1):
            lo = max(s.first, blk * bt)
            hi = min(s.first + s.count, (blk + 1) * bt)
            out.append((blk, lo, hi - lo))
        return out

    # ------------------------------------------------------------- append
    def append(self, t, b, xk, xv, pos):
        """Append n tokens (xk, xv [Hkv][n][d] fp32; sequence positions pos..pos+n-1)
        at the tail of tier t, stored in the tier's formats."""
        spec, s = self.tiers[t], self.seq[t][b]
        xk = np.ascontiguousarray(xk, np.float32)
        xv = np.ascontiguousarray(xv, np.float32)
        n = xk.shape[1]
        if s.p0 is None:
            s.p0 = pos
        assert pos == s.p0 + s.first + s.count, "tiers must hold adjacent, ordered position ranges"
        lo, hi = s.first + s.count, s.first + s.count + n
        assert hi <= s.M, "oracle array too small for this test's horizon"
        _store(spec.k_fmt, xk, s.khat, s.kq, lo, hi)
        _store(spec.v_fmt, xv, s.vhat, s.vq, lo, hi)
        if s.ksum is not None:
            bt = spec.block_tokens
            o = lo
            while o < hi:
                blk = o // bt
                e = min(hi, (blk + 1) * bt)
                O.summary_accumulate(s.ksum[blk], xk, o - lo, e - o)
                o = e
        s.count += n

    def load(self, b, k, v):
        """Bulk initial state (not a step of Alg. 1): distribute k, v [Hkv][N][d]
        over the tiers newest-first: tier 0 takes the newest min(N, cap_0 - 1)
        tokens (so that the next append fills it exactly), tier i the next
        cap_i, the last tier the rest.  Tokens reach tier i through the formats
        of the tiers above it, Q_i(D_{i-1}(... Q_1(x))), as they would by
        eviction.  Returns the position span per tier."""
        N = k.shape[1]
        sizes, rest = [], N
        for t, spec in enumerate(self.tiers):
            if t == len(self.tiers) - 1:
                take = rest
            else:
                take = min(rest, spec.capacity - 1 if t == 0 else spec.capacity)
            sizes.append(take)
            rest -= take
        hi = N
        spans = []
        for t, n in enumerate(sizes):
            spans.append((hi - n, hi))
            hi -= n
        for t in reversed(range(len(self.tiers))):
            lo, hi = spans[t]
            if hi > lo:
                xk, xv = self.through_formats(k[:, lo:hi], v[:, lo:hi], t)
                self.append(t, b, xk, xv, lo)
        self.total[b] = N
        return spans

    def through_formats(self, xk, xv, t):
        """Values a token holds on arrival at tier t after passing tiers 1..t-1."""
        xk = np.ascontiguousarray(xk, np.float32)
        xv = np.ascontiguousarray(xv, np.float32)
        for u in range(1, t):
            xk = _roundtrip(self.tiers[u].k_fmt, xk)
            xv = _roundtrip(self.tiers[u].v_fmt, xv)
        return xk, xv

    # ------------------------------------------------------------- attend
    def select(self, q, k):
        """Block identification (Alg. 1): per sequence, the k best blocks of the
        last tier by phi = sum_h q_h . mean-key.  Returns block ids ascending."""
        t = len(self.tiers) - 1
        out = []
        for b in range(self.B):
            blocks = self.live_blocks(t, b)
            sc = np.array([O.block_score(q[b], O.summary_finish(self.seq[t][b].ksum[blk], self.tiers[t].block_tokens),
                                         self.Hkv) for blk, _, _ in blocks], np.float32)
            idx = O.topk(sc, k) if len(blocks) else np.zeros(0, np.int32)
            out.append(np.array([blocks[i][0] for i in idx], np.int32))
        return out

    def summaries(self, b):
        """fp16 bit patterns of the mean-key summaries of the last tier's live blocks."""
        t = len(self.tiers) - 1
        return {blk: O.summary_finish(self.seq[t][b].ksum[blk], self.tiers[t].block_tokens)
                for blk, _, _ in self.live_blocks(t, b)}

    def attend(self, q, selected=None):
        """Alg. 1 (one decode step) for every sequence.  q [B][Hq][d] fp32.  selected:
        None (every slow block) or per sequence the block ids of the last tier to
        attend.  Returns (out [B][Hq][d], lse [B][Hq]) fp64."""
        out = np.empty((self.B, self.Hq, self.d), np.float64)
        lse = np.empty((self.B, self.Hq), np.float64)
        last = len(self.tiers) - 1
        for b in range(self.B):
            P = O.empty_partial(self.Hq, self.d)
            for t, spec in enumerate(self.tiers):
                s = self.seq[t][b]
                if t == 0:
                    parts = [(None, s.first, s.count)] if s.count else []
                else:
                    parts = self.live_blocks(t, b)
                    if selected is not None and t == last:
                        keep = set(int(x) for x in selected[b])
                        parts = [p for p in parts if p[0] in keep]
                for blk, lo, n in parts:
                    O.merge_into(P, O.attn_partial(q[b], s.khat, s.vhat, lo, n, self.scale))
                    if spec.mem == "host":
                        self.h2d_bytes += self.record_bytes(t)
                        self.blocks_fetched += 1
            out[b], lse[b] = O.finalize(P)
        return out, lse

    # ------------------------------------------------------------- demote
    def demote(self):
        """FIFO tier management: while a tier holds >= capacity tokens, move its
        oldest block to the tail of the next tier in that tier's format."""
        for t in range(len(self.tiers) - 1):
            spec = self.tiers[t]
            for b in range(self.B):
                s = self.seq[t][b]
                while s.count >= spec.capacity:
                    n = spec.block_tokens
                    assert s.count >= n
                    xk = s.khat[:, s.first:s.first + n].copy()
                    xv = s.vhat[:, s.first:s.first + n].copy()
                    self.append(t + 1, b, xk, xv, s.p0 + s.first)
                    s.first += n
                    s.count -= n
                    self.demotions[t][b] += 1

    def step(self, q, k_new, v_new, select_k=None):
        """One decode step: append the new token's k, v ([B][Hkv][d]) to tier 0,
        attend, evict.  Returns (out, lse[, selected])."""
        for b in range(self.B):
            self.append(0, b, k_new[b][:, None, :], v_new[b][:, None, :], self.total[b])
            self.total[b] += 1
        sel = self.select(q, select_k) if select_k is not None else None
        out, lse = self.attend(q, sel)
        self.demote()
        return (out, lse) if sel is None else (out, lse, sel)


def _roundtrip(fmt, x):
    if fmt in FP_FORMATS:
        return x
    if fmt == "i8":
        return O.dequant_i8(*O.quant_i8(x))
    if fmt == "i4":
        return O.dequant_i4(*O.quant_i4(x))
    raise ValueError(fmt)     # 'i4t' is a last-tier format: nothing passes through it
