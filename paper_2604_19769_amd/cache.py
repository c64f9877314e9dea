"""Caller-side plumbing around libttkv: allocates the tiers' record pools
(torch tensors: HBM or pinned host memory), fills the ttkv_cache descriptor and
forwards to the C ABI.  No arithmetic of the method lives here; every step of
the hot path runs in the library's kernels."""
import ctypes as C
from dataclasses import dataclass

import numpy as np
import torch

from . import binding as B


@dataclass
class TierConfig:
    k_fmt: str                 # 'f16' | 'bf16' | 'i8' | 'i4' | 'i4t' (keys of the last tier: int4 grouped over 128 tokens per channel)
    v_fmt: str                 # the same, or 'i4c' (last tier, >= 2 query heads per KV head: int4 as 'i4', stored channel-major per 32 tokens)
    capacity: int              # eviction threshold in tokens (L_fast for tier 0)
    block_tokens: int          # B_blk
    ring_blocks: int           # records per sequence ring
    mem: str = "device"        # 'device' | 'host'
    paged_seed: int = None     # not None: shuffled block table over a shared pool (paged KV)
    summary: bool = False      # keep mean-key summaries (block identification)


_SECTION_BYTES = {"f16": (256, 0), "bf16": (256, 0), "i8": (128, 8), "i4": (64, 8), "i4t": (64, 4), "i4c": (64, 8)}


class TieredCache:
    def __init__(self, batch, n_q_heads, n_kv_heads, tiers, device="cuda:0", softmax_scale=None, n_slots=0):
        self.B, self.Hq, self.Hkv = batch, n_q_heads, n_kv_heads
        self.cfg = list(tiers)
        self.device = torch.device(device)
        self.n_slots = n_slots
        self.device_topk = True           # step() with select_k: the chosen ids stay on the device (ttkv_decode_step_topk)
        self.one_call_step = True         # step(): append + attend through ttkv_decode_step; False: the two calls
        self.host_demote_direct = False   # True: evictions into a host tier are stored by the kernels (no staging, no copies)
        self.host_append_direct = True    # bulk appends to a host tier are stored by the kernels; False: staging record + copies
        self.h = B.ttkv_create()
        self.c = B.ttkv_cache()
        c = self.c
        c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.n_tiers = batch, n_q_heads, n_kv_heads, 128, len(self.cfg)
        c.softmax_scale = float(softmax_scale) if softmax_scale is not None else 1.0 / float(np.sqrt(128.0))
        self._keep = []          # tensors / arrays the descriptor points into
        self.start, self.len, self.pool, self.table = [], [], [], []
        for t, cfg in enumerate(self.cfg):
            T = c.tier[t]
            T.k_fmt, T.v_fmt = B.FMT_NAMES[cfg.k_fmt], B.FMT_NAMES[cfg.v_fmt]
            T.mem = B.MEM_HOST_PINNED if cfg.mem == "host" else B.MEM_DEVICE
            T.block_tokens, T.capacity_tokens, T.ring_blocks = cfg.block_tokens, cfg.capacity, cfg.ring_blocks
            T.pool_blocks = batch * cfg.ring_blocks
            rec = B.ttkv_record_bytes(c, t)
            assert rec > 0
            nbytes = T.pool_blocks * rec
            if cfg.mem == "host":
                pool = torch.zeros(nbytes, dtype=torch.uint8, pin_memory=True)
            else:
                pool = torch.zeros(nbytes, dtype=torch.uint8, device=self.device)
            T.data = pool.data_ptr()
            start = np.zeros(batch, np.int64)
            ln = np.zeros(batch, np.int64)
            T.start, T.len = start.ctypes.data, ln.ctypes.data
            table = None
            if cfg.paged_seed is not None:
                table = np.random.Generator(np.random.Philox(cfg.paged_seed)).permutation(T.pool_blocks).astype(np.int32)
                table = np.ascontiguousarray(table.reshape(batch, cfg.ring_blocks))
                tdev = torch.from_numpy(table).to(self.device)
                T.block_table, T.block_table_dev = table.ctypes.data, tdev.data_ptr()
                self._keep.append(tdev)
            if cfg.summary:
                ksum = torch.zeros(T.pool_blocks * n_kv_heads * 128, dtype=torch.float32, device=self.device)
                kmu = torch.zeros(T.pool_blocks * n_kv_heads * 128, dtype=torch.float16, device=self.device)
                T.k_sum, T.k_summary = ksum.data_ptr(), kmu.data_ptr()
                self._keep += [ksum, kmu]
                self.ksum, self.kmu = ksum, kmu
            self.start.append(start)
            self.len.append(ln)
            self.pool.append(pool)
            self.table.append(table)
        self.copy_stream = torch.cuda.Stream(device=self.device)
        self.ws = None
        self.ws_parts = 0
        self.demote_ws = None
        self._demote_need = None          # per tier: bytes of staging ttkv_tier_demote wants (constant for a cache)
        self._parts_age = None            # dense steps since the parts per row were last counted (None: never)
        self._until_evict = 0             # steps until some sequence's tier 0 can have filled (0: ask the library)
        self.sel_blocks = self.sel_count = self.sel_scratch = None
        self.out = torch.empty(batch, n_q_heads, 128, dtype=torch.float32, device=self.device)
        self.lse = torch.empty(batch, n_q_heads, dtype=torch.float32, device=self.device)

    def close(self):
        if self.h is not None:
            torch.cuda.synchronize(self.device)
            B.ttkv_destroy(self.h)
            self.h = None

    # ------------------------------------------------------------------ streams
    def _compute(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    def _copy(self, overlap=True):
        return self.copy_stream.cuda_stream if overlap else self._compute()

    # ------------------------------------------------------------------ calls
    def record_bytes(self, t):
        return B.ttkv_record_bytes(self.c, t)

    def locate(self, b, pos):
        return B.ttkv_locate(self.c, b, pos)

    def stats(self):
        return B.ttkv_get_stats(self.h)

    def append(self, tier, k, v, seq=-1, through_tiers=False):
        """k, v: device tensors [B][Hkv][n][128] (seq=-1) or [Hkv][n][128], f16 / bf16 / f32."""
        fmt = {torch.float16: B.F16, torch.bfloat16: B.BF16, torch.float32: B.F32}[k.dtype]
        assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape and k.dtype == v.dtype
        n = k.shape[-2]
        self._parts_age = None            # lengths jump: count the parts again at the next step
        self._until_evict = 0
        if self.cfg[tier].mem == "host" and self.host_append_direct:
            # no staging: the conversion kernels store into the pinned records
            B.ttkv_quantize_append_host(self.h, self.c, tier, seq, k, v, fmt, n, int(through_tiers), None, 0, self._compute())
        elif self.cfg[tier].mem == "host":
            need = B.ttkv_append_host_workspace_bytes(self.c, tier, seq, n)
            ws = torch.empty(need, dtype=torch.uint8, device=self.device)
            B.ttkv_quantize_append_host(self.h, self.c, tier, seq, k, v, fmt, n, int(through_tiers), ws, need, self._compute())
            torch.cuda.current_stream(self.device).synchronize()   # ws goes out of scope
        else:
            B.ttkv_quantize_append(self.h, self.c, tier, seq, k, v, fmt, n, int(through_tiers), self._compute())

    def demote(self, overlap=True):
        """Cascade eviction through all tiers (Alg. 1, last lines)."""
        if self._demote_need is None:
            self._demote_need = [B.ttkv_demote_workspace_bytes(self.c, t) for t in range(len(self.cfg) - 1)]
        for t in range(len(self.cfg) - 1):
            need = 0 if self.host_demote_direct else self._demote_need[t]
            if need and (self.demote_ws is None or self.demote_ws.numel() < need):
                self.demote_ws = torch.empty(need, dtype=torch.uint8, device=self.device)
            B.ttkv_tier_demote(self.h, self.c, t, 0, self.demote_ws if need else None, need, self._compute(),
                               self._copy(overlap))

    def _workspace(self, parts):
        if self.ws is None or parts > self.ws_parts or self.ws_slots != self.n_slots:
            parts = max(parts + 16, int(parts * 1.25))
            need = B.ttkv_workspace_bytes(self.c, parts, self.n_slots)
            assert need > 0
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.device)
            self.ws_parts, self.ws_slots = parts, self.n_slots
        return self.ws

    def decode(self, q, selected=None, overlap=True, new=None):
        """q [B][Hq][128] f16/bf16 on the device.  selected: None or (sel_blocks, sel_count) pinned int32 tensors.
        new: None, or (k_new, v_new) [B][Hkv][1][128] of the step's token, appended to tier 0 by the same call."""
        q_fmt = {torch.float16: B.F16, torch.bfloat16: B.BF16}[q.dtype]
        assert q.is_contiguous() and tuple(q.shape) == (self.B, self.Hq, 128)
        sb = sc = None
        stride = 0
        if selected is not None:
            sb, sc = selected
            stride = sb.shape[1]
        # Parts per row: counted by the library.  A dense decode step adds one token per sequence, i.e. at most one
        # part per tier every 256 steps, and the workspace is sized with 16 parts to spare: inside step() the count is
        # therefore refreshed only every 64 steps (the library still checks the workspace on every call).
        if selected is None and new is not None and self.ws is not None and self._parts_age is not None and self._parts_age < 64 \
                and self.ws_slots == self.n_slots:
            self._parts_age += 1
            ws = self.ws
        else:
            if new is not None:
                self.len[0] += 1            # size the workspace for the lengths the attention may see
            parts = B.ttkv_count_parts(self.h, self.c, sb, sc, stride, self.n_slots)
            if new is not None:
                self.len[0] -= 1
            if parts < 0:
                raise B.TTKVError(B.ERR_INVALID_ARG, "ttkv_count_parts")
            ws = self._workspace(max(parts, 1))
            self._parts_age = 0 if (selected is None and new is not None) else None
        if new is not None:
            k_new, v_new = new
            fmt = {torch.float16: B.F16, torch.bfloat16: B.BF16}[k_new.dtype]
            assert k_new.is_contiguous() and v_new.is_contiguous() and k_new.dtype == v_new.dtype
            assert tuple(k_new.shape) == tuple(v_new.shape) == (self.B, self.Hkv, 1, 128)
            try:
                B.ttkv_decode_step(self.h, self.c, q, q_fmt, k_new, v_new, fmt, self.out, self.lse, sb, sc, stride, ws, ws.numel(),
                                   self.n_slots, self._compute(), self._copy(overlap))
            except B.TTKVError as e:
                if e.status != B.ERR_WORKSPACE or self._parts_age in (None, 0):
                    raise
                self._parts_age = None    # the split changed under a cached count (nothing was enqueued): count and go again
                return self.decode(q, selected, overlap, new)
        else:
            B.ttkv_decode_attn(self.h, self.c, q, q_fmt, self.out, self.lse, sb, sc, stride, ws, ws.numel(), self.n_slots,
                               self._compute(), self._copy(overlap))
        return self.out, self.lse

    def select(self, q, k):
        q_fmt = {torch.float16: B.F16, torch.bfloat16: B.BF16}[q.dtype]
        stride = self._select_buffers(k)
        B.ttkv_select_blocks(self.h, self.c, q, q_fmt, k, self.sel_blocks, self.sel_count, stride, self.sel_scratch,
                             self.sel_scratch.numel(), self._compute())
        return self.sel_blocks, self.sel_count

    def _select_buffers(self, k):
        stride = max(1, k)
        if self.sel_blocks is None or self.sel_blocks.shape[1] != stride:
            self.sel_blocks = torch.zeros(self.B, stride, dtype=torch.int32, pin_memory=True)
            self.sel_count = torch.zeros(self.B, dtype=torch.int32, pin_memory=True)
            self.sel_scratch = torch.empty(self.B * (1024 * 4 + (stride + 1) * 4) + 512, dtype=torch.uint8, device=self.device)
        return stride

    def step_topk(self, q, k_new, v_new, k):
        """append -> identify + top-k + attend with the chosen ids left on the device (no host round trip)."""
        q_fmt = {torch.float16: B.F16, torch.bfloat16: B.BF16}[q.dtype]
        fmt = {torch.float16: B.F16, torch.bfloat16: B.BF16}[k_new.dtype]
        assert q.is_contiguous() and k_new.is_contiguous() and v_new.is_contiguous()
        assert tuple(k_new.shape) == tuple(v_new.shape) == (self.B, self.Hkv, 1, 128)
        stride = self._select_buffers(k)
        # parts: every other tier as usual; the last one min(k, live blocks) blocks of fixed items -- an upper bound
        # is what a dense pass over everything would use, at the lengths the attention will see
        self.len[0] += 1
        parts = B.ttkv_count_parts(self.h, self.c, None, None, 0, 0)
        self.len[0] -= 1
        last = self.cfg[-1]
        per_block = max(1, last.block_tokens // (2048 if last.mem == "host" else 256))
        parts += per_block * min(k, int(max((l + last.block_tokens - 1) // last.block_tokens for l in self.len[-1]))) + 1
        ws = self._workspace(max(parts, 1))
        B.ttkv_decode_step_topk(self.h, self.c, q, q_fmt, k_new, v_new, fmt, self.out, self.lse, k, self.sel_blocks,
                                self.sel_count, stride, self.sel_scratch, self.sel_scratch.numel(), ws, ws.numel(),
                                self._compute())
        return self.out, self.lse

    def _evict_if_due(self, overlap):
        """Alg. 1's eviction check after a step that appended one token per sequence.  A tier below the first only grows
        when the one above evicts, so nothing can be due before some sequence's tier 0 has filled: until then the
        library is not asked (every call validates the whole descriptor)."""
        self._until_evict -= 1
        if self._until_evict > 0:
            return
        self.demote(overlap)
        self._until_evict = max(1, int((self.cfg[0].capacity - self.len[0]).min()))

    def step(self, q, k_new, v_new, select_k=None, overlap=True):
        """One decode step (Alg. 1): append -> [identify blocks] -> attend -> evict.  k_new, v_new [B][Hkv][1][128]."""
        if select_k is not None and self.device_topk and self.one_call_step and self.n_slots == 0:
            out, lse = self.step_topk(q, k_new, v_new, select_k)
            self._evict_if_due(overlap)
            return out, lse
        if not self.one_call_step:
            self.append(0, k_new, v_new)
            sel = self.select(q, select_k) if select_k is not None else None
            out, lse = self.decode(q, sel, overlap)
        else:
            sel = self.select(q, select_k) if select_k is not None else None
            out, lse = self.decode(q, sel, overlap, new=(k_new, v_new))
        self._evict_if_due(overlap)
        return out, lse

    # ------------------------------------------------------------------ inspection (layout decoding only)
    def dump_tier(self, t, b):
        """Live rows of tier t, sequence b, oldest first, as raw bytes:
        {'k': uint8 [Hkv][n][kc], 'k_meta': uint8 [Hkv][n][km], 'v': ..., 'v_meta': ...}."""
        torch.cuda.synchronize(self.device)
        cfg = self.cfg[t]
        bt, ring = cfg.block_tokens, cfg.ring_blocks
        kc, km = _SECTION_BYTES[cfg.k_fmt]
        vc, vm = _SECTION_BYTES[cfg.v_fmt]
        head_bytes = bt * (kc + km + vc + vm)
        pool = self.pool[t].cpu().numpy().reshape(-1, self.Hkv, head_bytes)
        o = int(self.start[t][b]) + np.arange(int(self.len[t][b]), dtype=np.int64)
        r = (o // bt) % ring
        rec = self.table[t][b][r] if self.table[t] is not None else b * ring + r
        row = o % bt
        out, off = {}, 0
        for name, w in (("k", kc), ("k_meta", km), ("v", vc), ("v_meta", vm)):
            sec = pool[:, :, off:off + bt * w].reshape(pool.shape[0], self.Hkv, bt, w)
            out[name] = np.ascontiguousarray(sec[rec, :, row].transpose(1, 0, 2)) if w else None
            off += bt * w
        return out

    def dump_summary(self, t, b, block_id):
        torch.cuda.synchronize(self.device)
        ring = self.cfg[t].ring_blocks
        r = block_id % ring
        rec = int(self.table[t][b][r]) if self.table[t] is not None else b * ring + r
        return self.kmu.view(-1, self.Hkv, 128)[rec].cpu().numpy().view(np.uint16)
