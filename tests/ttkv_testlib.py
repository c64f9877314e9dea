"""Shared helpers of the GPU parity tests: build the device cache and the oracle
cache from one description, feed both the same seeded inputs, compare."""
import numpy as np
import torch

import oracle as O
from oracle import OracleCache, TierSpec
from paper_2604_19769_amd import synth
from paper_2604_19769_amd.cache import TierConfig, TieredCache

TORCH_DT = {"f16": torch.float16, "bf16": torch.bfloat16}

# |gpu - oracle| <= ABS_TOL + REL_TOL * |oracle|, element-wise, on fp32-accumulated outputs; and, because on
# N(0,1) data over thousands of tokens the outputs are only ~1e-2 and the absolute term alone would be most of
# the signal, max|gpu - oracle| <= NORM_TOL * max|oracle| as well
ABS_TOL, REL_TOL, NORM_TOL = 2e-3, 1e-2, 2e-3


def dev(x, dtype, device="cuda:0"):
    """float32 numpy values (representable in dtype) -> device tensor of dtype."""
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(device).to(TORCH_DT[dtype]).contiguous()


def oracle_fmt(fmt):
    """'i4c' is Q_4bit exactly as 'i4' (same codes, scales, zeros); only the device's record packing differs."""
    return "i4" if fmt == "i4c" else fmt


def decode_i4c(raw):
    """Value codes stored channel-major per 32 tokens -> the token-major packing of 'i4' (element 2i in the low
    nibble of byte i).  raw: uint8 [Hkv][n][64], the V code section's bytes in token order, n a multiple of 32; every
    32 rows are one 2 KiB group of 512 32-bit words: word d belongs to piece p = d / 4 = 64 hh + 16 kg + c and is its
    word w = d % 4: channel 16 (4 hh + w) + c, nibble j = token {0, 2, 16, 18, 1, 3, 17, 19}[j] + 4 kg of the group
    (the layout include/ttkv.h documents)."""
    Hkv, n, _ = raw.shape
    assert n % 32 == 0
    words = np.ascontiguousarray(raw).reshape(Hkv, n // 32, 2048).view(np.uint32)          # [Hkv][groups][512]
    d = np.arange(512)
    p, w = d >> 2, d & 3
    hh, kg, c = p >> 6, (p >> 4) & 3, p & 15
    ch = 16 * (4 * hh + w) + c
    tokmap = np.array([0, 2, 16, 18, 1, 3, 17, 19])
    codes = np.full((Hkv, n // 32, 32, 128), 255, np.uint8)
    for j in range(8):
        codes[:, :, tokmap[j] + 4 * kg, ch] = (words >> np.uint32(4 * j)) & np.uint32(15)
    assert codes.max() <= 15                                                                # every (token, channel) was written
    codes = codes.reshape(Hkv, n, 128)
    return codes[..., 0::2] | (codes[..., 1::2] << 4)


class Pair:
    """tiers: list of dicts(k_fmt, v_fmt, capacity, block_tokens, ring_blocks, mem, paged_seed, summary)."""

    def __init__(self, B, Hq, Hkv, tiers, dtype, oracle_max_tokens=None, n_slots=0, host_append_direct=False, one_call_step=True,
                 host_demote_direct=False):
        self.B, self.Hq, self.Hkv, self.dtype = B, Hq, Hkv, dtype
        self.tiers = tiers
        self.gpu = TieredCache(B, Hq, Hkv, [TierConfig(t["k_fmt"], t["v_fmt"], t["capacity"], t["block_tokens"],
                                                        t["ring_blocks"], t.get("mem", "device"), t.get("paged_seed"),
                                                        t.get("summary", False)) for t in tiers], n_slots=n_slots)
        self.gpu.host_append_direct = host_append_direct   # bulk loads of a host tier written by the kernels
        self.gpu.host_demote_direct = host_demote_direct   # evictions into a host tier stored by the kernels
        self.gpu.one_call_step = one_call_step             # append + attend in one call (ttkv_decode_step) or in two
        if oracle_max_tokens is None:
            oracle_max_tokens = [t["ring_blocks"] * t["block_tokens"] * 4 for t in tiers]
        self.ora = OracleCache(B, Hq, Hkv, 128,
                               [TierSpec(t["k_fmt"], oracle_fmt(t["v_fmt"]), t["capacity"], t["block_tokens"], t.get("mem", "device"),
                                         t.get("summary", False)) for t in tiers], oracle_max_tokens)

    def close(self):
        self.gpu.close()

    # -------------------------------------------------------------- feeding
    def load(self, b, k, v):
        """Bulk initial state of sequence b from k, v [Hkv][N][128] (float32, representable in dtype)."""
        spans = self.ora.load(b, k, v)
        for t in reversed(range(len(self.tiers))):
            lo, hi = spans[t]
            if hi > lo:
                self.gpu.append(t, dev(k[:, lo:hi], self.dtype), dev(v[:, lo:hi], self.dtype), seq=b, through_tiers=True)
        return spans

    def step(self, q, k_new, v_new, select_k=None, overlap=True):
        """q [B][Hq][128], k_new/v_new [B][Hkv][128] float32.  Returns (gpu_out, gpu_lse, ora_out, ora_lse[, sel])."""
        res = self.ora.step(q, k_new, v_new, select_k)
        out, lse = self.gpu.step(dev(q, self.dtype), dev(k_new[:, :, None, :], self.dtype), dev(v_new[:, :, None, :], self.dtype),
                                 select_k, overlap)
        torch.cuda.synchronize()
        r = (out.cpu().numpy().copy(), lse.cpu().numpy().copy(), res[0], res[1])
        if select_k is not None:
            sb, sc = self.gpu.sel_blocks.numpy(), self.gpu.sel_count.numpy()
            r = r + ([sb[b, :sc[b]].copy() for b in range(self.B)], res[2])
        return r

    # -------------------------------------------------------------- comparing
    def assert_state_equal(self):
        """Codes, scales, zeros, fp bits and tier/block indices: bit-exact."""
        for t, spec in enumerate(self.tiers):
            for b in range(self.B):
                s = self.ora.seq[t][b]
                assert int(self.gpu.len[t][b]) == s.count, (t, b, int(self.gpu.len[t][b]), s.count)
                assert int(self.gpu.start[t][b]) == s.first, (t, b)
                if s.count == 0:
                    continue
                d = self.gpu.dump_tier(t, b)
                sl = slice(s.first, s.first + s.count)
                for name, fmt, hat, q in (("k", spec["k_fmt"], s.khat, s.kq), ("v", spec["v_fmt"], s.vhat, s.vq)):
                    if fmt in ("f16", "bf16"):
                        want = synth.to_bits(hat[:, sl], fmt)
                        assert np.array_equal(d[name].view(np.uint16), want), (t, b, name, "fp bits")
                    elif fmt == "i4t":      # 128 meta rows x 4 B of a token group = {scale, zero} x 128 channels
                        assert s.first % 128 == 0 and s.count % 128 == 0
                        assert np.array_equal(d[name], q["codes"][:, sl]), (t, b, name, "codes")
                        meta = d[name + "_meta"].reshape(self.Hkv, s.count // 128, 128, 4).view(np.uint16)
                        gsl = slice(s.first // 128, (s.first + s.count) // 128)
                        assert np.array_equal(meta[..., 0], q["scale"][:, gsl]), (t, b, name, "scale")
                        assert np.array_equal(meta[..., 1], q["zero"][:, gsl]), (t, b, name, "zero")
                    elif fmt == "i8":
                        assert np.array_equal(d[name], q["codes"][:, sl].view(np.uint8)), (t, b, name, "codes")
                        assert np.array_equal(d[name + "_meta"].view(np.uint16), q["scale"][:, sl]), (t, b, name, "scale")
                    else:
                        got = decode_i4c(d[name]) if fmt == "i4c" else d[name]
                        assert np.array_equal(got, q["codes"][:, sl]), (t, b, name, "codes")
                        meta = d[name + "_meta"].view(np.uint16)
                        assert np.array_equal(meta[:, :, 0::2], q["scale"][:, sl]), (t, b, name, "scale")
                        assert np.array_equal(meta[:, :, 1::2], q["zero"][:, sl]), (t, b, name, "zero")

    def assert_locate_equal(self, b, positions):
        for pos in positions:
            t, blk, row, _ = self.gpu.locate(b, int(pos))
            assert (t, blk, row) == tuple(int(x) for x in self.ora.locate(b, int(pos))), pos


def assert_close(gpu, ora, what=""):
    gpu = np.asarray(gpu, np.float64)
    ora = np.asarray(ora, np.float64)
    fin = np.isfinite(ora)
    assert np.array_equal(np.isfinite(gpu), fin), what
    err = np.abs(gpu[fin] - ora[fin])
    lim = ABS_TOL + REL_TOL * np.abs(ora[fin])
    assert np.all(err <= lim), f"{what}: max err {err.max():.3e} (max |ref| {np.abs(ora[fin]).max():.3e}, worst ratio {(err / lim).max():.3f})"
    if err.size:
        top = np.abs(ora[fin]).max()
        assert err.max() <= NORM_TOL * top + 1e-6, f"{what}: max err {err.max():.3e} against max |ref| {top:.3e}: normalised {err.max() / max(top, 1e-30):.2e}"
    return float(err.max()) if err.size else 0.0
