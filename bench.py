#!/usr/bin/env python3
"""Benchmark of the tiered decode-attention hot path on one MI355X.

A step = append the new token's K/V -> streaming decode attention over every
tier (split-K partials + log-sum-exp merge) -> evict when the fast tier is full
(Alg. 1 of the TTKV paper).  Inputs are seeded synthetic tensors resident in HBM
(and, for the offload workload, in pinned host memory, which is where the
method keeps its slow tier) before the timed region starts.

Main workload `mha32k`: batch 4, 32 heads (MHA), head_dim 128, 32K context,
recent 2K fp16 + 30K int4 (group 64, scale+zero), all in HBM -- the HBM-bound
configuration.  Extra object `offload_128k`: batch 1, 32 q / 8 kv heads, 128K
context, 4K bf16 + 28K int8 in HBM + 96K int4 in pinned host DRAM streamed in
1024-token blocks -- the PCIe-bound configuration (microseconds per token).

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
# HBM bytes per mha32k attention launch from rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy
# kernel's reading (profiles/attn_fused_mha32k_hbm_traffic_pmc.txt): 702.03 MB for 700.38 MB of algorithmic bytes.
# A profile constant, not a reading of this run: the object gives the factor and where it is from, and applies it to
# the run's own bytes per launch.
MHA32K_TRAFFIC_FACTOR = 1.0024
MHA32K_TRAFFIC_SOURCE = ("1.0024 x the algorithmic bytes of the timed launches: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this kernel at "
                         "this workload, profiles/attn_fused_mha32k_hbm_traffic_pmc.txt")
PCIE_PEAK_GBS = 64.0        # PCIe Gen5 x16 per direction, nominal
SEED = 1976900


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="mha32k", choices=["mha32k", "offload128k", "tiny", "serving_ragged", "sparse128k", "sparse_hbm", "gqa_hbm", "ablation", "grid"])
    ap.add_argument("--grid-rows", default="", help="grid only: comma-separated q/kv head counts, e.g. 64/4,64/2 (default: the whole table)")
    ap.add_argument("--gqa-formats", default="", help="gqa_hbm only: comma-separated K/V formats to run, e.g. i8/i4,i4/i4 (default: all)")
    ap.add_argument("--mode", default="all", choices=["all", "staged"],
                    help="offload128k only: 'staged' runs nothing but attention calls in the staged-copy mode (for a trace)")
    ap.add_argument("--overlap-from-trace", metavar="DIR", help="no GPU work: summarise the copy/compute overlap of a rocprofv3 "
                    "--kernel-trace --memory-copy-trace csv output in DIR (files <prefix>_kernel_trace.csv, <prefix>_memory_copy_trace.csv)")
    ap.add_argument("--trace-prefix", default="kt")
    ap.add_argument("--no-offload", action="store_true", help="skip the 128K offload object")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--offload-steps", type=int, default=20)
    ap.add_argument("--no-extra", action="store_true", help="skip the ragged-serving and sparse-recall objects")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="first run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def device_normal(gen, shape, dtype):
    import torch
    return torch.randn(shape, generator=gen, device=gen.device, dtype=torch.float32).to(dtype)


def sync_time():
    import torch
    torch.cuda.synchronize()
    return time.perf_counter()


SETTLE_LAUNCHES = 192


def settle(cache, q, launches=SETTLE_LAUNCHES):
    """Untimed attention launches on the cache as it stands (no append, no eviction: the cache state is untouched)
    before a measurement: after idle time the launch durations of these kernels drift for about 15 ms of continuous
    work (first short, then up to 20 % long, then steady: the device's clock management), and a decode loop lives
    in the steady state.  192 launches of ~0.1 ms cover that."""
    for i in range(launches):
        cache.decode(q[i % len(q)])


def timed_steps(cache, q, kn, vn, first, count, overlap=True, keep=None, sample_every=0):
    """Run steps [first, first+count) and return seconds, bracketed by full synchronisation.
    sample_every > 0: every sample_every-th step has its attention launch timed by a HIP event pair."""
    from paper_2604_19769_amd import binding as B
    t0 = sync_time()
    for s in range(first, first + count):
        sampled = sample_every > 0 and (s - first) % sample_every == sample_every - 1
        if sampled:
            B.ttkv_time_attn(cache.h, count)
        out, lse = cache.step(q[s], kn[s], vn[s], overlap=overlap)
        if sampled:
            B.ttkv_time_attn(cache.h, 0)
        if keep is not None:
            keep.append(out.clone())
    return sync_time() - t0


def step_latencies(cache, q, kn, vn, first, count):
    """Per-step times in seconds of steps [first, first+count): one HIP event recorded on the stream after every
    step, no host synchronisation in between.  Each event leaves a few microseconds of idle stream, so the median
    reads higher than the back-to-back mean of timed_steps; the spread (p95) is what this is for."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(count + 1)]
    torch.cuda.synchronize()
    ev[0].record()
    for i, s in enumerate(range(first, first + count)):
        cache.step(q[s], kn[s], vn[s])
        ev[i + 1].record()
    torch.cuda.synchronize()
    return sorted(ev[i].elapsed_time(ev[i + 1]) * 1e-3 for i in range(count))


# ------------------------------------------------------------------ workload: MHA 32K, int4 in HBM

def build_mha32k(steps_total, N=32768, slow_k="i4"):
    import numpy as np
    import torch
    from paper_2604_19769_amd import synth
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    B, H, R, bt = 4, 32, 2048, 128
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 2)
    tiers = [TierConfig("f16", "f16", R, bt, R // bt + 1),
             TierConfig(slow_k, "i4", 10**9, bt, (N - R) // bt + 2 + steps_total // bt + 1)]
    cache = TieredCache(B, H, H, tiers)
    K = torch.randn((B, H, N - 1, 128), generator=gen, device=dev, dtype=torch.float32)
    V = torch.randn((B, H, N - 1, 128), generator=gen, device=dev, dtype=torch.float32)
    outl = synth.outlier_channels(synth.rng(SEED + 2), H, 128, 0.02)      # 82 (head, channel) pairs, x8 on K
    for h, ch in outl:
        K[:, h, :, ch] *= 8.0
    K, V = K.to(torch.float16), V.to(torch.float16)
    n_old = N - R                                                       # 30720 tokens -> int4 tier
    cache.append(1, K[:, :, :n_old].contiguous(), V[:, :, :n_old].contiguous(), through_tiers=True)
    cache.append(0, K[:, :, n_old:].contiguous(), V[:, :, n_old:].contiguous())
    q = device_normal(gen, (steps_total, B, H, 128), torch.float16)
    kn = device_normal(gen, (steps_total, B, H, 1, 128), torch.float16)
    vn = device_normal(gen, (steps_total, B, H, 1, 128), torch.float16)
    for h, ch in outl:
        kn[:, :, h, :, ch] *= 8.0
    torch.cuda.synchronize()
    return cache, (K, V), (q, kn, vn), dict(B=B, Hq=H, Hkv=H, N=N, R=R, bt=bt)


def algorithmic_bytes(cache):
    """Stored bytes the step must read: codes + scales + zeros + fp K/V of every live token."""
    per = {"f16": 256, "bf16": 256, "i8": 136, "i4": 72, "i4t": 68, "i4c": 72}
    total, by_tier = 0, []
    for t, cfg in enumerate(cache.cfg):
        n = int(cache.len[t].sum()) * cache.Hkv * (per[cfg.k_fmt] + per[cfg.v_fmt])
        by_tier.append(n)
        total += n
    return total, by_tier


def cpu_baseline_mha32k(kv, steps, shape, gpu_outs):
    """The oracle as it stands, timed on this machine's host cores on the same workload (whole batch; the warm-up
    steps, each compared with the GPU's output, then further steps up to ~10 s of oracle time)."""
    import numpy as np
    import oracle as O
    from oracle import OracleCache, TierSpec
    K, V = kv
    q, kn, vn = steps
    B, H, N, R, bt = shape["B"], shape["Hq"], shape["N"], shape["R"], shape["bt"]
    cores = len(os.sched_getaffinity(0))
    ora = OracleCache(B, H, H, 128, [TierSpec("f16", "f16", R, bt), TierSpec("i4", "i4", 10**9, bt)], [R + bt, N + bt])
    for b in range(B):
        ora.load(b, K[b].float().cpu().numpy(), V[b].float().cpu().numpy())
    # the compared steps first, then further steps of the same inputs for the timing alone: ~10 s of oracle work
    n_cmp, n_steps, secs, bytes_, err = len(gpu_outs), 0, 0.0, 0, 0.0
    for s in range(q.shape[0]):
        if s >= n_cmp and secs >= 10.0:
            break
        n_steps += 1
        qs = q[s].float().cpu().numpy()
        ks, vs = kn[s, :, :, 0].float().cpu().numpy(), vn[s, :, :, 0].float().cpu().numpy()
        # same accounting as the GPU line: stored bytes of every token the step attends (incl. the new one)
        bytes_ += sum((ora.seq[0][b].count + 1) * H * 512 + ora.seq[1][b].count * H * 144 for b in range(B))
        t0 = time.perf_counter()
        out, _ = ora.step(qs, ks, vs)
        secs += time.perf_counter() - t0
        if s < n_cmp:
            g = gpu_outs[s].cpu().numpy()
            err = max(err, float(np.max(np.abs(g - out) / (2e-3 + 1e-2 * np.abs(out)))))
    return {"value": round(bytes_ / secs / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"whole workload (batch {B}, {H} heads, {N} tokens), {n_steps} decode steps incl. append+evict "
                      f"({secs:.1f} s of oracle time), the first {n_cmp} compared with the GPU's outputs",
            "ms_per_step": round(secs / n_steps * 1e3, 1), "gpu_vs_oracle_worst_err_over_tol": round(err, 4)}



# ------------------------------------------------------------------ shared: sampled oracle baselines, PCIe roofline

def host_tier_live_bytes(cache):
    """Stored bytes of the live rows of the host tiers: what actually crosses PCIe when the kernel reads them in
    place (the library's h2d counter counts whole block records, as the oracle's does)."""
    total, by_tier = algorithmic_bytes(cache)
    return sum(n for n, cfg in zip(by_tier, cache.cfg) if cfg.mem == "host")


def pcie_roofline(host_bytes, seconds, what):
    gbs = host_bytes / seconds / 1e9
    return {"bound": "pcie", "kernel": what, "achieved": round(gbs, 2), "peak": PCIE_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / PCIE_PEAK_GBS, 4), "traffic": None, "bytes_per_step": int(host_bytes),
            "note": "host-tier bytes of live rows / attention time; traffic: no PCIe counter is read"}


def oracle_sample(tier_specs, max_tokens, Hq, Hkv, heads, seqs, steps_in, step, gpu_out, what, select_k=None):
    """The oracle as it stands on a sample of the workload: for each (sequence index b, K, V) in seqs, KV heads
    `heads` (all their query heads, every token), loaded in bulk, then one decode step timed on this machine's host
    cores and compared with the GPU's output of that step, and up to 32 further steps (until ~2 s) for the timing.  Returns the cpu_baseline object (GB/s of stored bytes)."""
    import numpy as np
    from oracle import OracleCache
    q, kn, vn = steps_in
    G = Hq // Hkv
    rows = np.concatenate([np.arange(h * G, (h + 1) * G) for h in heads])
    cores = min(len(os.sched_getaffinity(0)), len(rows))      # the oracle's threads run over query heads
    secs, bytes_, err, n_steps = 0.0, 0, 0.0, 0
    per = {"f16": 256, "bf16": 256, "i8": 136, "i4": 72, "i4t": 68, "i4c": 72}
    for b, K, V in seqs:
        ora = OracleCache(1, G * len(heads), len(heads), 128, tier_specs, max_tokens)
        ora.load(0, K[heads].float().cpu().numpy(), V[heads].float().cpu().numpy())
        # the compared step, then up to 32 further steps of the same inputs for the timing alone (~2 s of oracle work)
        mine = 0.0
        for s in range(step, min(step + 33, q.shape[0])):
            if s > step and mine >= 2.0:
                break
            args = (q[s, b][rows][None].float().cpu().numpy(), kn[s, b, heads, 0][None].float().cpu().numpy(),
                    vn[s, b, heads, 0][None].float().cpu().numpy())
            t0 = time.perf_counter()
            r = ora.step(*args) if select_k is None else ora.step(*args, select_k=select_k)
            mine += time.perf_counter() - t0
            n_steps += 1
            if select_k is None:
                bytes_ += sum(ora.seq[t][0].count * len(heads) * (per[sp.k_fmt] + per[sp.v_fmt]) for t, sp in enumerate(tier_specs))
            else:   # only the selected blocks of the last tier are attended
                last = len(tier_specs) - 1
                bytes_ += sum(ora.seq[t][0].count * len(heads) * (per[sp.k_fmt] + per[sp.v_fmt]) for t, sp in enumerate(tier_specs[:-1]))
                bytes_ += len(r[2][0]) * tier_specs[last].block_tokens * len(heads) * (per[tier_specs[last].k_fmt] + per[tier_specs[last].v_fmt])
            if s == step:
                g = gpu_out[b][rows].float().cpu().numpy()
                err = max(err, float(np.max(np.abs(g - r[0][0]) / (2e-3 + 1e-2 * np.abs(r[0][0])))))
        secs += mine
        del ora
    return {"value": round(bytes_ / secs / 1e9, 3), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": what + f"; compared with the GPU's output, then {n_steps - len(seqs)} further steps for the timing alone",
            "seconds": round(secs, 2), "steps_timed": n_steps, "gpu_vs_oracle_worst_err_over_tol": round(err, 4)}

# ------------------------------------------------------------------ workload: 128K offload

def build_offload128k(steps_total):
    import torch
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    B, Hq, Hkv, N = 1, 32, 8, 131072
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 3)
    tiers = [TierConfig("bf16", "bf16", 4096, 128, 33),
             TierConfig("i8", "i8", 28672, 128, 28672 // 128 + 2),
             TierConfig("i4", "i4", 10**9, 1024, 98304 // 1024 + 2, mem="host")]
    cache = TieredCache(B, Hq, Hkv, tiers)
    K = device_normal(gen, (B, Hkv, N - 1, 128), torch.bfloat16)
    V = device_normal(gen, (B, Hkv, N - 1, 128), torch.bfloat16)
    a, b = 98304, 98304 + 28672
    parts = [(2, K[:, :, :a].contiguous(), V[:, :, :a].contiguous(), True), (1, K[:, :, a:b].contiguous(), V[:, :, a:b].contiguous(), True),
             (0, K[:, :, b:].contiguous(), V[:, :, b:].contiguous(), False)]
    # prefill-side tiering of the whole prompt: every token through the formats of the tiers above its own,
    # the oldest 96K quantized to int4 on the device and copied to the pinned host pool
    for t, kk, vv, through in parts:
        cache.append(t, kk, vv, through_tiers=through)
    torch.cuda.synchronize()
    # timed on two further caches (everything warm): the host tier's records stored by the conversion kernels
    # themselves (the default: no staging record, no device-to-host copies), and through a staging record + copies
    tiering = {}
    for direct in (True, False):
        other = TieredCache(B, Hq, Hkv, tiers)
        other.host_append_direct = direct
        t0 = sync_time()
        for t, kk, vv, through in parts:
            other.append(t, kk, vv, through_tiers=through)
        tiering[direct] = sync_time() - t0
        assert torch.equal(other.pool[2], cache.pool[2]), "host records differ between the two bulk paths"
        other.close()
        del other
    q = device_normal(gen, (steps_total, B, Hq, 128), torch.bfloat16)
    kn = device_normal(gen, (steps_total, B, Hkv, 1, 128), torch.bfloat16)
    vn = device_normal(gen, (steps_total, B, Hkv, 1, 128), torch.bfloat16)
    torch.cuda.synchronize()
    return cache, (K, V), (q, kn, vn), dict(B=B, Hq=Hq, Hkv=Hkv, N=N, tiering_s=tiering[True], tiering_staged_s=tiering[False],
                                                    d2h_bytes=cache.stats()["d2h_bytes"])


def offload128k_all_in_hbm(steps, warmup):
    """The same 128K context and formats with the int4 tier in HBM as well (113 MB of 288 GB), its values stored
    channel-major: microseconds per token and the time to tier the prompt when nothing crosses PCIe."""
    import torch
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    B, Hq, Hkv, N = 1, 32, 8, 131072
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 3)
    tiers = [TierConfig("bf16", "bf16", 4096, 128, 33), TierConfig("i8", "i8", 28672, 128, 28672 // 128 + 2),
             TierConfig("i4", "i4c", 10**9, 1024, 98304 // 1024 + 2)]
    K = device_normal(gen, (B, Hkv, N - 1, 128), torch.bfloat16)
    V = device_normal(gen, (B, Hkv, N - 1, 128), torch.bfloat16)
    a, b = 98304, 98304 + 28672
    parts = [(2, K[:, :, :a].contiguous(), V[:, :, :a].contiguous(), True), (1, K[:, :, a:b].contiguous(), V[:, :, a:b].contiguous(), True),
             (0, K[:, :, b:].contiguous(), V[:, :, b:].contiguous(), False)]
    tier_s = []
    for rep in range(3):                     # the last build is the one that is kept
        cache = TieredCache(B, Hq, Hkv, tiers)
        t0 = sync_time()
        for t, kk, vv, through in parts:
            cache.append(t, kk, vv, through_tiers=through)
        tier_s.append(sync_time() - t0)
        if rep < 2:
            cache.close()
    try:
        total_steps = steps + warmup
        q = device_normal(gen, (total_steps, B, Hq, 128), torch.bfloat16)
        kn = device_normal(gen, (total_steps, B, Hkv, 1, 128), torch.bfloat16)
        vn = device_normal(gen, (total_steps, B, Hkv, 1, 128), torch.bfloat16)
        settle(cache, q, 96)
        timed_steps(cache, q, kn, vn, 0, warmup)
        total, _ = algorithmic_bytes(cache)
        t = timed_steps(cache, q, kn, vn, warmup, steps) / steps
        return {"us_per_token": round(t * 1e6, 1), "bytes_per_step": int(total), "effective_kv_GBs": round(total / t / 1e9, 1),
                "frac_of_hbm_peak": round(total / t / 1e9 / HBM_PEAK_GBS, 4), "prefill_tiering_ms": round(min(tier_s) * 1e3, 3)}
    finally:
        cache.close()


# ------------------------------------------------------------------ workload: ragged paged serving batch

def build_serving_ragged(steps_total, batch=16, last_mem="host"):
    """The ragged serving benchmark configuration: batch 16, 32 q / 8 kv heads, contexts uniform in [16K, 64K], 256-token pages with
    shuffled page tables; 4K fp16 + 12K int8 in HBM, the rest int4 in pinned host memory (last_mem "device": in HBM too)."""
    import numpy as np
    import torch
    from paper_2604_19769_amd import synth
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    Hq, Hkv, page = 32, 8, 256
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 4)
    ctx = synth.rng(SEED + 4).integers(16384, 65537, batch)
    tiers = [TierConfig("f16", "f16", 4096, page, 4096 // page + 1, paged_seed=SEED + 40),
             TierConfig("i8", "i8", 12288, page, 12288 // page + 2, paged_seed=SEED + 41),
             TierConfig("i4", "i4c" if last_mem == "device" else "i4", 10**9, page, (65536 - 16384) // page + 4, mem=last_mem,
                        paged_seed=SEED + 42)]   # in HBM: the same int4 codes stored channel-major per 32 tokens
    cache = TieredCache(batch, Hq, Hkv, tiers)
    kv = []
    for b in range(batch):
        n = int(ctx[b]) - 1
        K = device_normal(gen, (Hkv, n, 128), torch.float16)
        V = device_normal(gen, (Hkv, n, 128), torch.float16)
        n2 = n - 4095 - 12288                      # oldest tokens -> host tier (>= 0 since ctx >= 16384)
        if last_mem == "device":
            n2 = n2 // 32 * 32                     # channel-major values arrive in whole groups of 32 tokens
        if n2 > 0:
            cache.append(2, K[:, :n2].contiguous(), V[:, :n2].contiguous(), seq=b, through_tiers=True)
        cache.append(1, K[:, n2:n2 + 12288].contiguous(), V[:, n2:n2 + 12288].contiguous(), seq=b, through_tiers=True)
        cache.append(0, K[:, n2 + 12288:].contiguous(), V[:, n2 + 12288:].contiguous(), seq=b)
        kv.append((K, V))
    q = device_normal(gen, (steps_total, batch, Hq, 128), torch.float16)
    kn = device_normal(gen, (steps_total, batch, Hkv, 1, 128), torch.float16)
    vn = device_normal(gen, (steps_total, batch, Hkv, 1, 128), torch.float16)
    torch.cuda.synchronize()
    return cache, kv, (q, kn, vn), dict(B=batch, Hq=Hq, Hkv=Hkv, ctx=ctx)


def serving_ragged_all_in_hbm(steps, warmup):
    """The same sequences, pages and formats with the int4 tier in HBM as well (1.3 GB of 288): what the placement costs."""
    cache, kv, (q, kn, vn), shape = build_serving_ragged(steps + warmup, last_mem="device")
    try:
        del kv
        settle(cache, q, 64)
        timed_steps(cache, q, kn, vn, 0, warmup)
        total, _ = algorithmic_bytes(cache)
        t = timed_steps(cache, q, kn, vn, warmup, steps) / steps
        return {"ms_per_step": round(t * 1e3, 4), "tokens_per_s": round(shape["B"] / t, 1), "bytes_per_step": int(total),
                "effective_kv_GBs": round(total / t / 1e9, 1), "frac_of_hbm_peak": round(total / t / 1e9 / HBM_PEAK_GBS, 4)}
    finally:
        cache.close()


def run_serving_ragged(steps, warmup, cpu_baseline=True):
    from oracle import TierSpec
    cache, kv, steps_in, shape = build_serving_ragged(steps + warmup)
    q, kn, vn = steps_in
    try:
        keep = []
        timed_steps(cache, q, kn, vn, 0, 1, keep=keep)                   # the first step is also the oracle's
        timed_steps(cache, q, kn, vn, 1, warmup - 1)
        total, by_tier = algorithmic_bytes(cache)
        live0 = host_tier_live_bytes(cache)
        s0 = cache.stats()
        t = timed_steps(cache, q, kn, vn, warmup, steps) / steps
        live = (live0 + host_tier_live_bytes(cache)) / 2
        h2d = (cache.stats()["h2d_bytes"] - s0["h2d_bytes"]) / steps
        cpu = None
        if cpu_baseline:
            import numpy as np
            b = int(np.argmin(shape["ctx"]))
            tiers = [TierSpec("f16", "f16", 4096, 256), TierSpec("i8", "i8", 12288, 256), TierSpec("i4", "i4", 10**9, 256, mem="host")]
            cpu = oracle_sample(tiers, [4096 + 512, 12288 + 1024, 65536], 32, 8, [0, 5], [(b, kv[b][0], kv[b][1])], steps_in, 0, keep[0],
                                f"sequence {b} (the shortest, {int(shape['ctx'][b])} tokens) of 16, KV heads 0 and 5 of 8 (8 query "
                                f"heads), the first decode step incl. append+evict")
        hbm = serving_ragged_all_in_hbm(steps, warmup)
        return {"workload": "batch 16, 32 q / 8 kv heads, contexts U[16K, 64K] (mean %d), 256-token pages, 4K fp16 + 12K int8 in HBM, "
                            "rest int4 in pinned host memory" % int(shape["ctx"].mean()),
                "same_cache_all_in_hbm": hbm,
                "steps": steps, "ms_per_step": round(t * 1e3, 3), "tokens_per_s": round(shape["B"] / t, 1),
                "host_tier_record_bytes_per_step": int(h2d), "host_tier_live_bytes_per_step": int(live),
                "device_tier_bytes_per_step": int(by_tier[0] + by_tier[1]),
                "effective_kv_GBs": round(total / t / 1e9, 2),
                "roofline": pcie_roofline(live, t, "attn_mfma_kernel<4>: every tier in one launch, host pages read in place"),
                "cpu_baseline": cpu}
    finally:
        cache.close()


# ------------------------------------------------------------------ workload: sparse recall of the host tier

def build_sparse128k(steps_total, batch=4, planted=8):
    """The sparse recall benchmark configuration: batch 4, 128K tokens, tiers as the offload workload (1024-token host blocks) plus fp16
    mean-key summaries; only the top-64 of 96 host blocks by q . summary are fetched.  `planted` seeded host blocks per
    sequence have their keys shifted along the mean query of each KV head's group (of the first step's query)."""
    import numpy as np
    import torch
    from paper_2604_19769_amd import synth
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    Hq, Hkv, N = 32, 8, 131072
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 5)
    tiers = [TierConfig("bf16", "bf16", 4096, 128, 33),
             TierConfig("i8", "i8", 28672, 1024, 28672 // 1024 + 2),
             TierConfig("i4", "i4", 10**9, 1024, 98304 // 1024 + 3, mem="host", summary=True)]
    cache = TieredCache(batch, Hq, Hkv, tiers)
    q = device_normal(gen, (steps_total, batch, Hq, 128), torch.bfloat16)
    g = synth.rng(SEED + 5)
    kv, plant_ids = [], []
    a, b2 = 98304, 98304 + 28672
    for b in range(batch):
        K = torch.randn((Hkv, N - 1, 128), generator=gen, device=dev, dtype=torch.float32)
        V = device_normal(gen, (Hkv, N - 1, 128), torch.bfloat16)
        ids = np.sort(g.choice(96, size=planted, replace=False))
        u = q[0, b].float().view(Hkv, Hq // Hkv, 128).mean(1)
        u = u / u.norm(dim=1, keepdim=True)
        for j in ids:
            K[:, j * 1024:(j + 1) * 1024] += u[:, None, :]
        K = K.to(torch.bfloat16)
        cache.append(2, K[:, :a].contiguous(), V[:, :a].contiguous(), seq=b, through_tiers=True)
        cache.append(1, K[:, a:b2].contiguous(), V[:, a:b2].contiguous(), seq=b, through_tiers=True)
        cache.append(0, K[:, b2:].contiguous(), V[:, b2:].contiguous(), seq=b)
        kv.append((K, V))
        plant_ids.append(ids)
    kn = device_normal(gen, (steps_total, batch, Hkv, 1, 128), torch.bfloat16)
    vn = device_normal(gen, (steps_total, batch, Hkv, 1, 128), torch.bfloat16)
    torch.cuda.synchronize()
    return cache, kv, (q, kn, vn), dict(B=batch, Hq=Hq, Hkv=Hkv, N=N, planted=plant_ids)


def run_sparse128k(steps, warmup, k=64, cpu_baseline=True):
    from oracle import TierSpec
    cache, kv, steps_in, shape = build_sparse128k(steps + warmup)
    q, kn, vn = steps_in
    try:
        first = None
        for s in range(warmup):
            out, _ = cache.step(q[s], kn[s], vn[s], select_k=k)
            if s == 0:
                first = out.clone()
        total, by_tier = algorithmic_bytes(cache)
        s0 = cache.stats()
        t0 = sync_time()
        for s in range(warmup, warmup + steps):
            cache.step(q[s], kn[s], vn[s], select_k=k)
        t = (sync_time() - t0) / steps
        st = cache.stats()
        h2d = (st["h2d_bytes"] - s0["h2d_bytes"]) / steps
        # selected blocks: whole 1024-token records except a partly filled newest one (none here: the host tier only
        # grows by whole blocks), so live bytes = record bytes
        cpu = None
        if cpu_baseline:
            tiers = [TierSpec("bf16", "bf16", 4096, 128), TierSpec("i8", "i8", 28672, 1024),
                     TierSpec("i4", "i4", 10**9, 1024, mem="host", summary=True)]
            cpu = oracle_sample(tiers, [4096 + 256, 28672 + 2048, 98304 + 4096], 32, 8, list(range(8)), [(1, kv[1][0], kv[1][1])],
                                steps_in, 0, first, "sequence 1 of 4, all 8 KV heads (block identification sums over every head), the "
                                "first decode step: scoring + top-64 of 96 + attention + append+evict", select_k=k)
        return {"workload": "batch 4, 32 q / 8 kv heads, 131072 tokens: 4K bf16 + 28K int8 in HBM, 96K int4 on the host in "
                            "1024-token blocks with mean-key summaries; top-64 of 96 blocks fetched per sequence",
                "steps": steps, "ms_per_step": round(t * 1e3, 3), "blocks_fetched_per_step": (st["blocks_fetched"] - s0["blocks_fetched"]) / steps,
                "host_tier_bytes_per_step": int(h2d), "dense_host_tier_bytes": 4 * 96 * 1179648,
                "device_tier_bytes_per_step": int(by_tier[0] + by_tier[1]),
                "effective_kv_GBs": round((h2d + by_tier[0] + by_tier[1]) / t / 1e9, 2),
                "roofline": pcie_roofline(h2d, t, "score_kernel + topk_kernel + attn_mfma_kernel<4> (selected host blocks read in place)"),
                "cpu_baseline": cpu}
    finally:
        cache.close()


# ------------------------------------------------------------------ workload: tiny (launch-latency floor)

def run_tiny(steps=200, warmup=20, cpu_baseline=True):
    """The smallest benchmark configuration ("tiny"): batch 1, 8 q / 2 kv heads, 4096 tokens, recent 512 fp16 + 3584 int8 (group 32), all in HBM.
    2.5 MB per step: 0.3 us at the HBM peak, so the step is launch latency (two launches: attention, merge)."""
    import numpy as np
    import torch
    from oracle import TierSpec
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    Hq, Hkv, N, R, bt = 8, 2, 4096, 512, 128
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 1)
    total_steps = steps + warmup
    cache = TieredCache(1, Hq, Hkv, [TierConfig("f16", "f16", R, bt, R // bt + 1),
                                     TierConfig("i8", "i8", 10**9, bt, (N - R + 2 * total_steps) // bt + 3)])
    try:
        K = device_normal(gen, (1, Hkv, N - 1, 128), torch.float16)
        V = device_normal(gen, (1, Hkv, N - 1, 128), torch.float16)
        cache.append(1, K[:, :, :N - R].contiguous(), V[:, :, :N - R].contiguous(), through_tiers=True)
        cache.append(0, K[:, :, N - R:].contiguous(), V[:, :, N - R:].contiguous())
        q = device_normal(gen, (total_steps, 1, Hq, 128), torch.float16)
        kn = device_normal(gen, (total_steps, 1, Hkv, 1, 128), torch.float16)
        vn = device_normal(gen, (total_steps, 1, Hkv, 1, 128), torch.float16)
        keep = []
        timed_steps(cache, q, kn, vn, 0, 1, keep=keep)
        timed_steps(cache, q, kn, vn, 1, warmup - 1)
        total, by_tier = algorithmic_bytes(cache)
        t = timed_steps(cache, q, kn, vn, warmup, steps) / steps
        lat = step_latencies(cache, q, kn, vn, warmup, steps)       # replays the same inputs on the grown cache: timing only
        cpu = None
        if cpu_baseline:
            tiers = [TierSpec("f16", "f16", R, bt), TierSpec("i8", "i8", 10**9, bt)]
            cpu = oracle_sample(tiers, [R + 256, N + 512], Hq, Hkv, [0, 1], [(0, K[0], V[0])], (q, kn, vn), 0, keep[0],
                                "the whole workload (1 sequence, both KV heads), the first decode step incl. append+evict")
        gbs = total / t / 1e9
        return {"workload": "batch 1, 8 q / 2 kv heads, 4096 tokens: recent 512 fp16 + 3584 int8 (group 32) in HBM",
                "steps": steps, "us_per_step": round(t * 1e6, 2), "us_per_step_p50_p95_event_timed":
                    [round(lat[len(lat) // 2] * 1e6, 1), round(lat[int(0.95 * len(lat))] * 1e6, 1)],
                "bytes_per_step": int(total), "effective_kv_GBs": round(gbs, 1),
                "roofline": {"bound": "hbm", "kernel": "attn_mfma_kernel<4> + merge_kernel: launch-latency floor (0.3 us of traffic at the peak)",
                             "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 5),
                             "traffic": None},
                "cpu_baseline": cpu}
    finally:
        cache.close()


def measure_h2d_peak():
    """Pinned host -> device copy rate of one 1 GiB hipMemcpyAsync (what the link delivers at best)."""
    import torch
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, pin_memory=True)
    dst = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    dst.copy_(src, non_blocking=True)
    t0 = sync_time()
    for _ in range(3):
        dst.copy_(src, non_blocking=True)
    dt = (sync_time() - t0) / 3
    return n / dt / 1e9


def measure_hbm_read_peak(h):
    """Rate of the library's load-only kernel (the attention kernels' access pattern) over 2 GiB of device
    memory, HIP events on the launching stream: the practical ceiling beside the nominal 8 TB/s."""
    import torch
    from paper_2604_19769_amd import binding as B
    n = 2 << 30
    buf = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        B.ttkv_stream_read(h, buf.data_ptr(), n, sink.data_ptr(), stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    e0.record()
    for _ in range(reps):
        B.ttkv_stream_read(h, buf.data_ptr(), n, sink.data_ptr(), stream)
    e1.record()
    torch.cuda.synchronize()
    return n * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def measure_hbm_read_same_size(h, n):
    """The load-only kernel over n bytes, one HIP event pair per launch (median of 15): the time a kernel that
    only streams the attention launch's bytes needs, measured the way the attention launch is."""
    import torch
    from paper_2604_19769_amd import binding as B
    n = n // 4096 * 4096
    buf = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(3):
        B.ttkv_stream_read(h, buf.data_ptr(), n, sink.data_ptr(), stream)
    ts = []
    for _ in range(15):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.ttkv_stream_read(h, buf.data_ptr(), n, sink.data_ptr(), stream)
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) * 1e-3)
    return sorted(ts)[len(ts) // 2]


def decode_only_seconds(cache, q, reps):
    """Attention alone (no append, no eviction), mean over reps, bracketed by full synchronisation."""
    for i in range(2):
        cache.decode(q[i % len(q)])
    t0 = sync_time()
    for i in range(reps):
        cache.decode(q[i % len(q)])
    return (sync_time() - t0) / reps


def spread(xs):
    xs = sorted(xs)
    return [round(xs[len(xs) // 2] * 1e6, 1), round(xs[0] * 1e6, 1), round(xs[-1] * 1e6, 1)]      # median, min, max in us


def run_offload128k(steps, warmup, cpu_baseline=True, staged_only=False):
    """128K context with the oldest 96K tokens in pinned host DRAM.  Reported for the default mode
    (the attention kernel reads the host records in place over PCIe) and for the staged mode
    (hipMemcpyAsync of runs of block records into staging slots, event-chained with the kernels).
    staged_only: nothing but `steps` attention calls in the staged mode after the warm-up (the run a
    rocprofv3 kernel + memory-copy trace is taken of)."""
    from oracle import TierSpec
    from paper_2604_19769_amd import binding as B
    cache, kv, steps_in, shape = build_offload128k(2 * (steps + warmup) + 4)
    q, kn, vn = steps_in
    try:
        if staged_only:
            cache.n_slots = 4
            decode_only_seconds(cache, q, warmup)
            t = decode_only_seconds(cache, q, steps)
            live = host_tier_live_bytes(cache)
            return {"mode": "staged copies, 4 slots", "attn_only_us": round(t * 1e6, 1), "steps": steps,
                    "roofline": pcie_roofline(live, t, "hipMemcpyAsync x4 + attn_mfma_kernel<4> per copy, event-chained")}
        keep = []
        timed_steps(cache, q, kn, vn, 0, 1, keep=keep)
        timed_steps(cache, q, kn, vn, 1, warmup - 1)
        total, by_tier = algorithmic_bytes(cache)
        s0 = cache.stats()
        # every step bracketed by a HIP event pair on its stream as well: median and p95 (Sec. 5.1 item 4)
        import torch
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = sync_time()
        for s in range(steps):
            evs[s][0].record()
            cache.step(q[warmup + s], kn[warmup + s], vn[warmup + s])
            evs[s][1].record()
        t_step = (sync_time() - t0) / steps
        per_step = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
        h2d_per_step = (cache.stats()["h2d_bytes"] - s0["h2d_bytes"]) / steps
        live = host_tier_live_bytes(cache)      # the state the attention-only figures below are measured on
        # In-place mode: copy and compute are ONE launch, so there are no copy and kernel intervals to intersect.
        # What can be shown: the attention launch alone (HIP event pair on its stream) over the host tier only, the
        # device tiers only, and everything, in interleaved rounds.  The device tiers are ~1 % of the launch, less
        # than the spread of the other two, so a fraction is not resolvable from them; the three durations are.
        t_all = decode_only_seconds(cache, q, steps)
        keep_len = [cache.len[t].copy() for t in range(3)]
        rounds, per = 7, max(4, steps // 4)
        ts = {"all": [], "dev": [], "host": []}

        def launch_seconds():
            B.ttkv_time_attn(cache.h, per)
            decode_only_seconds(cache, q, per)
            ms = sorted(B.ttkv_read_attn_timing(cache.h))
            return ms[len(ms) // 2] * 1e-3

        for _ in range(rounds):
            ts["all"].append(launch_seconds())
            cache.len[2][:] = 0
            ts["dev"].append(launch_seconds())
            cache.len[2][:] = keep_len[2]
            cache.len[0][:] = 0
            cache.len[1][:] = 0
            ts["host"].append(launch_seconds())
            cache.len[0][:] = keep_len[0]
            cache.len[1][:] = keep_len[1]
        peak = measure_h2d_peak()
        # staged mode on the same cache: 4 copies of up to 27 records (32 MiB), one slot each
        cache.n_slots = 4
        decode_only_seconds(cache, q, 4)
        t_staged = decode_only_seconds(cache, q, max(3, steps // 2))
        cache.n_slots = 0
        cpu = None
        if cpu_baseline:
            tiers = [TierSpec("bf16", "bf16", 4096, 128), TierSpec("i8", "i8", 28672, 128), TierSpec("i4", "i4", 10**9, 1024, mem="host")]
            cpu = oracle_sample(tiers, [4096 + 256, 28672 + 512, 98304 + 2048], 32, 8, [1, 6], [(0, kv[0][0], kv[1][0])], steps_in, 0,
                                keep[0], "KV heads 1 and 6 of 8 (8 query heads), all 131072 tokens, the first decode step incl. append+evict")
        hbm = offload128k_all_in_hbm(64, 8)
        roof = pcie_roofline(live, t_all, "attn_mfma_kernel<4>: device tiers + host records read in place, one launch")
        roof["frac_of_measured_link_peak"] = round(live / t_all / 1e9 / peak, 4)
        roof["measured_link_peak_GBs"] = round(peak, 2)
        return {
            "workload": "batch 1, 32 q / 8 kv heads, 131072 tokens: 4K bf16 + 28K int8 in HBM, 96K int4 in pinned host "
                        "DRAM in 1024-token block records",
            "us_per_token": round(t_step * 1e6, 1),
            "us_per_token_p50": round(per_step[len(per_step) // 2], 1),
            "us_per_token_p95": round(per_step[min(len(per_step) - 1, int(0.95 * len(per_step)))], 1),
            "attn_only_us": round(t_all * 1e6, 1),
            "host_tier_record_bytes_per_step": int(h2d_per_step),
            "host_tier_live_bytes_per_step": int(live),
            "device_tier_bytes_per_step": int(by_tier[0] + by_tier[1]),
            "effective_kv_GBs": round(total / t_step / 1e9, 2),
            "roofline": roof,
            "cpu_baseline": cpu,
            "in_place_overlap": {
                "attn_launch_us_median_min_max": spread(ts["all"]),
                "host_tier_alone_us_median_min_max": spread(ts["host"]),
                "device_tiers_alone_us_median_min_max": spread(ts["dev"]),
                "note": "copy and compute are one launch: PCIe loads of some waves are in flight while others compute; the device "
                        "tiers' time is smaller than the run-to-run spread of the launch, so no overlap fraction is derived here"},
            "staged_copy_mode": {
                "n_slots": 4, "attn_only_us": round(t_staged * 1e6, 1),
                "pcie_GBs": round(live / t_staged / 1e9, 2), "pcie_frac_of_nominal_64": round(live / t_staged / 1e9 / PCIE_PEAK_GBS, 4),
                "overlap_fraction": "from a rocprofv3 kernel + memory-copy trace: profiles/offload128k_staged_overlap_trace.txt"},
            "prefill_tiering_ms": round(shape["tiering_s"] * 1e3, 2),
            "prefill_tiering_tokens_per_s": round((shape["N"] - 1) / shape["tiering_s"], 0),
            "prefill_d2h_GBs": round(shape["d2h_bytes"] / shape["tiering_s"] / 1e9, 2),
            "prefill_tiering_staged_ms": round(shape["tiering_staged_s"] * 1e3, 2),
            "same_cache_all_in_hbm": hbm,
        }
    finally:
        cache.close()


def overlap_from_trace(trace_dir, prefix):
    """Copy/compute overlap of the staged mode from a rocprofv3 --kernel-trace --memory-copy-trace run (csv output):
    per attention call, T_copy = union of the host-to-device copy intervals, T_compute = union of the kernel
    intervals, T_step = first start to last end; overlap = (T_copy + T_compute - T_step) / min(T_copy, T_compute).
    A call = the copies and kernels between two merge kernels.  Prints a summary (what profiles/ keeps)."""
    import csv

    def union(iv):
        tot, end = 0, None
        for a, b in sorted(iv):
            if end is None or a > end:
                tot += b - a
                end = b
            elif b > end:
                tot += b - end
                end = b
        return tot

    ks = list(csv.DictReader(open(os.path.join(trace_dir, prefix + "_kernel_trace.csv"))))
    cs = list(csv.DictReader(open(os.path.join(trace_dir, prefix + "_memory_copy_trace.csv"))))
    ev = [(int(r["Start_Timestamp"]), int(r["End_Timestamp"]), "k", r["Kernel_Name"]) for r in ks]
    ev += [(int(r["Start_Timestamp"]), int(r["End_Timestamp"]), "c", r.get("Direction", "")) for r in cs
           if "HOST_TO_DEVICE" in r.get("Direction", "").upper() or "H2D" in r.get("Direction", "").upper()]
    ev.sort()
    calls, cur = [], []
    for e in ev:
        cur.append(e)
        if e[2] == "k" and "merge_kernel" in e[3]:
            calls.append(cur)
            cur = []
    def merged(iv):
        out = []
        for a, b in sorted(iv):
            if out and a <= out[-1][1]:
                out[-1][1] = max(out[-1][1], b)
            else:
                out.append([a, b])
        return out

    def intersection(x, y):
        tot = 0
        for a, b in merged(x):
            for c, d in merged(y):
                tot += max(0, min(b, d) - max(a, c))
        return tot

    rows = []
    for call in calls:
        cop = [(a, b) for a, b, k, _ in call if k == "c"]
        ker = [(a, b) for a, b, k, n in call if k == "k" and ("attn_" in n or "merge_kernel" in n)]
        if len(cop) < 2 or not ker:
            continue                       # not a staged attention call
        t_copy, t_comp = union(cop), union(ker)
        t_step = max(b for _, b in cop + ker) - min(a for a, _ in cop + ker)
        rows.append((t_copy, t_comp, t_step, (t_copy + t_comp - t_step) / min(t_copy, t_comp), len(cop), len(ker),
                     intersection(cop, ker) / t_comp, t_step - union(cop + ker)))
    rows = rows[len(rows) // 4:]           # the first quarter is warm-up
    med = lambda i: sorted(r[i] for r in rows)[len(rows) // 2]
    print(f"staged attention calls analysed: {len(rows)} (copies per call {rows[0][4]}, kernels per call {rows[0][5]})")
    print(f"T_copy    (union of H2D copy intervals)  median {med(0) / 1e3:9.1f} us")
    print(f"T_compute (union of kernel intervals)    median {med(1) / 1e3:9.1f} us")
    print(f"T_step    (first start .. last end)      median {med(2) / 1e3:9.1f} us")
    print(f"idle inside the step (neither a copy nor a kernel running) median {med(7) / 1e3:.1f} us")
    print(f"overlap = (T_copy + T_compute - T_step) / min(T_copy, T_compute): median {med(3):.3f}, "
          f"min {min(r[3] for r in rows):.3f}, max {max(r[3] for r in rows):.3f}")
    print(f"share of the kernel time that ran while a copy was in flight: median {med(6):.3f}")
    print(f"exposed beyond the copies (T_step - T_copy) median {(med(2) - med(0)) / 1e3:.1f} us")
    call = calls[len(calls) // 2]
    t0 = call[0][0]
    print("timeline of one call (us from its first operation): start, end, what")
    for a, b, k, n in call:
        name = "copy H2D" if k == "c" else next((x for x in ("attn_mfma_kernel", "attn_fused_kernel", "merge_kernel") if x in n), n[:40])
        print(f"  {(a - t0) / 1e3:8.1f} {(b - t0) / 1e3:8.1f}  {name}")


# ------------------------------------------------------------------ workload: grouped-query tiers resident in HBM

def run_gqa_hbm(reps=12, only=None):
    """32 q / 8 kv heads, batch 4, one HBM-resident tier per case (~0.55-0.6 GB per launch): the attention
    launch alone (HIP event pair), i.e. the matrix-core kernel's rate per stored format."""
    import torch
    from paper_2604_19769_amd import binding as B
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 7)
    rows = []
    for fmt, N, dt in ((("i8", "i8"), 65536, torch.float16), (("i8", "i4"), 81920, torch.float16), (("i4", "i4"), 131072, torch.float16),
                       (("i8", "i4c"), 81920, torch.float16), (("i4", "i4c"), 131072, torch.float16),
                       (("f16", "f16"), 32768, torch.float16), (("bf16", "bf16"), 32768, torch.bfloat16)):
        if only and "/".join(fmt) not in only:
            continue
        fp = "f16" if dt == torch.float16 else "bf16"
        tiers = [TierConfig(fp, fp, 10**9, 128, N // 128 + 2)] if fmt[0] in ("f16", "bf16") else \
                [TierConfig(fp, fp, 256, 128, 3), TierConfig(fmt[0], fmt[1], 10**9, 128, N // 128 + 2)]
        cache = TieredCache(4, 32, 8, tiers)
        try:
            K, V = device_normal(gen, (4, 8, N, 128), dt), device_normal(gen, (4, 8, N, 128), dt)
            cache.append(len(tiers) - 1, K, V, through_tiers=True)
            if len(tiers) == 2:
                cache.append(0, K[:, :, :128].contiguous(), V[:, :, :128].contiguous())
            q = device_normal(gen, (4, 4, 32, 128), dt)
            total, _ = algorithmic_bytes(cache)
            settle(cache, q)
            s0 = cache.stats()
            # the launch four times back to back between one event pair (the pair's own cost, a few microseconds of
            # marker dispatch, spread over four launches: what rocprofv3 reports as the kernel's duration), `reps` samples
            B.ttkv_time_attn_repeat(cache.h, 4)
            B.ttkv_time_attn(cache.h, reps)
            for i in range(reps):
                cache.decode(q[i % 4])
            ms = sorted(B.ttkv_read_attn_timing(cache.h))
            B.ttkv_time_attn(cache.h, 0)
            B.ttkv_time_attn_repeat(cache.h, 1)
            us = ms[len(ms) // 2] * 1e3
            rows.append({"tier": f"K {fmt[0]} / V {fmt[1]} x {N} tokens", "bytes_per_launch": int(total), "kernel_us": round(us, 1),
                         "GBs": round(total / us / 1e3, 1), "frac_of_hbm_peak": round(total / us / 1e3 / HBM_PEAK_GBS, 4),
                         "kernel_us_min_max": [round(ms[0] * 1e3, 1), round(ms[-1] * 1e3, 1)],
                         "matrix_core_launches": cache.stats()["mfma_launches"] - s0["mfma_launches"]})
        finally:
            cache.close()
            del K, V
            torch.cuda.empty_cache()
    return {"workload": "batch 4, 32 q / 8 kv heads (4 query heads per KV head), one tier in HBM per row, attention launch alone "
                        f"(x4 back to back per event pair, median of 12 samples, after {SETTLE_LAUNCHES} untimed launches)",
            "rows": rows}


# ------------------------------------------------------------------ workload: int4 keys grouped over tokens

def run_key_grouping(steps=12):
    """The mha32k workload (keys with x8 on 2 % of the (head, channel) pairs) with the old tier's int4 keys grouped
    per token over 64 channels, or per channel over 128 tokens: step time, attention launch rate and the
    attention-output error of each against the same cache held entirely in fp16."""
    import torch
    from paper_2604_19769_amd import binding as B
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    rows, ref = [], None
    for name, slow_k in (("fp16 everywhere (reference)", None), ("int4 keys, groups of 64 channels per token", "i4"),
                         ("int4 keys, groups of 128 tokens per channel", "i4t")):
        if slow_k is None:
            cache, (K, V), (q, kn, vn), shape = build_mha32k(steps + 4)
            cache.close()
            cache = TieredCache(4, 32, 32, [TierConfig("f16", "f16", 10**9, 128, 32768 // 128 + 2)])
            cache.append(0, K, V)
        else:
            cache, (K, V), (q, kn, vn), shape = build_mha32k(steps + 4, slow_k=slow_k)
        try:
            del K, V
            out0 = cache.decode(q[0])[0].clone()
            torch.cuda.synchronize()
            if ref is None:
                ref = out0
            err = float((out0 - ref).abs().max() / ref.abs().max())
            rms = float(((out0 - ref).pow(2).mean() / ref.pow(2).mean()).sqrt())
            total, _ = algorithmic_bytes(cache)
            if slow_k is None:
                rows.append({"keys": name, "bytes_per_launch": int(total)})
            else:
                settle(cache, q)
                timed_steps(cache, q, kn, vn, 0, 3)
                B.ttkv_read_attn_timing(cache.h)
                secs = timed_steps(cache, q, kn, vn, 3, steps, sample_every=4)
                ms = sorted(B.ttkv_read_attn_timing(cache.h))
                us = ms[len(ms) // 2] * 1e3
                rows.append({"keys": name, "bytes_per_launch": int(total), "us_per_step": round(secs / steps * 1e6, 1),
                             "attn_launch_us": round(us, 1), "attn_GBs": round(total / us / 1e3, 1),
                             "out_err_vs_fp16_rel_max": round(err, 5), "out_err_vs_fp16_rel_rms": round(rms, 5)})
        finally:
            cache.close()
            torch.cuda.empty_cache()
    return {"workload": "mha32k shapes and data (batch 4, 32 heads, 32768 tokens, recent 2048 fp16), the old tier's keys in two "
                        "int4 groupings; error = attention output vs the all-fp16 cache", "rows": rows}


# ------------------------------------------------------------------ workload: formats x head groupings in HBM

def run_grid(only=None):
    """One HBM-resident tier of ~560 MB (plus a 256-token fp16 window for the quantized ones), batch 4, every stored
    format against head groupings from multi-head to multi-query: attention launch issued four times back to back
    between one event pair, median of six samples.  Effective TB/s of stored bytes; which kernel served it."""
    import torch
    from paper_2604_19769_amd import binding as B
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 9)
    per = {("f16", "f16"): 512, ("i8", "i8"): 272, ("i8", "i4"): 208, ("i4", "i4"): 144, ("i8", "i4c"): 208, ("i4", "i4c"): 144}
    rows = []
    for Hq, Hkv in ((32, 32), (32, 16), (24, 8), (32, 8), (48, 8), (28, 4), (64, 8), (48, 4), (64, 4), (64, 2)):
        if only and f"{Hq}/{Hkv}" not in only:
            continue
        row = {"q_heads": Hq, "kv_heads": Hkv}
        for (kf, vf), bytes_per in per.items():
            if vf == "i4c" and Hq == Hkv:
                continue              # values channel-major per 32 tokens: a layout for two or more heads per KV head
            N = int(560e6 / (4 * Hkv * bytes_per)) // 256 * 256
            tiers = [TierConfig(kf, vf, 10**9, 128, N // 128 + 2)] if kf == "f16" else \
                    [TierConfig("f16", "f16", 256, 128, 3), TierConfig(kf, vf, 10**9, 128, N // 128 + 2)]
            cache = TieredCache(4, Hq, Hkv, tiers)
            K = device_normal(gen, (4, Hkv, N, 128), torch.float16)
            V = device_normal(gen, (4, Hkv, N, 128), torch.float16)
            cache.append(len(tiers) - 1, K, V, through_tiers=True)
            del K, V
            q = device_normal(gen, (4, 4, Hq, 128), torch.float16)
            total, _ = algorithmic_bytes(cache)
            settle(cache, q)
            B.ttkv_time_attn_repeat(cache.h, 4)
            B.ttkv_time_attn(cache.h, 6)
            for i in range(6):
                cache.decode(q[i % 4])
            B.ttkv_time_attn(cache.h, 0)
            B.ttkv_time_attn_repeat(cache.h, 1)
            ms = sorted(B.ttkv_read_attn_timing(cache.h))
            row[f"K {kf} / V {vf}"] = {"TBs": round(total / ms[3] / 1e9, 2),
                                      "kernel": "matrix-core" if cache.stats()["mfma_launches"] else "vector"}
            cache.close()
            del cache
        rows.append(row)
    return {"workload": "one HBM-resident tier of ~560 MB, batch 4; attention launch x4 back to back per sample", "rows": rows}


# ------------------------------------------------------------------ workload: block-sparse attention over a tier in HBM

SPARSE_HBM_ROWS = ((1024, 64, ("i4", "i4")), (1024, 64, ("i4", "i4c")), (256, 256, ("i4", "i4")), (128, 512, ("i4", "i4")),
                   (128, 64, ("i4", "i4")))     # block tokens, k, formats of the int4 tier


def build_sparse_hbm(steps_total, bt, fmt, batch=4):
    """The sparse-recall layout with the old tier in HBM: batch 4, 32 q / 8 kv heads, 128K tokens = 4096 bf16 + 28672 int8
    + 98304 int4 in blocks of bt tokens with mean-key summaries."""
    import torch
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 11)
    Hq, Hkv, N, n_last = 32, 8, 131072, 98304
    tiers = [TierConfig("bf16", "bf16", 4096, 128, 33), TierConfig("i8", "i8", 28672, 1024, 30),
             TierConfig(fmt[0], fmt[1], 10**9, bt, n_last // bt + 1024 // bt + 3, summary=True)]
    cache = TieredCache(batch, Hq, Hkv, tiers)
    kv = []
    for b in range(batch):
        K = device_normal(gen, (Hkv, N - 1, 128), torch.bfloat16)
        V = device_normal(gen, (Hkv, N - 1, 128), torch.bfloat16)
        a, b2 = n_last, n_last + 28672
        cache.append(2, K[:, :a].contiguous(), V[:, :a].contiguous(), seq=b, through_tiers=True)
        cache.append(1, K[:, a:b2].contiguous(), V[:, a:b2].contiguous(), seq=b, through_tiers=True)
        cache.append(0, K[:, b2:].contiguous(), V[:, b2:].contiguous(), seq=b)
        kv.append((K, V))
    q = device_normal(gen, (steps_total, batch, Hq, 128), torch.bfloat16)
    kn = device_normal(gen, (steps_total, batch, Hkv, 1, 128), torch.bfloat16)
    vn = device_normal(gen, (steps_total, batch, Hkv, 1, 128), torch.bfloat16)
    torch.cuda.synchronize()
    return cache, kv, (q, kn, vn), dict(B=batch, Hq=Hq, Hkv=Hkv, N=N, n_last=n_last)


def run_sparse_hbm(steps=32, warmup=8):
    """Block-sparse attention with the old tier in HBM instead of pinned host memory (what 288 GB allow); per step block
    identification + top-k on the device, attention over the dense tiers and the selected blocks, append, evict.
    Selecting 2/3 of the blocks (the sparse-recall benchmark's 64 of 96) in blocks of 1024, 256 and the paper's own B_blk = 128 tokens."""
    import torch
    per = {"i4": 72, "i8": 136, "i4c": 72}
    rows = []
    for bt, k, fmt in SPARSE_HBM_ROWS:
        cache, kv, (q, kn, vn), shape = build_sparse_hbm(steps + warmup, bt, fmt)
        del kv
        batch, Hkv, n_last = shape["B"], shape["Hkv"], shape["n_last"]
        for s in range(warmup):
            cache.step(q[s], kn[s], vn[s], select_k=k)
        t0 = sync_time()
        for s in range(warmup, steps + warmup):
            cache.step(q[s], kn[s], vn[s], select_k=k)
        dt = (sync_time() - t0) / steps
        attended = batch * Hkv * (4096 * 512 + 28672 * 272 + min(k, n_last // bt) * bt * (per[fmt[0]] + per[fmt[1]]))
        rows.append({"block_tokens": bt, "k": k, "of_blocks": n_last // bt, "last_tier": f"K {fmt[0]} / V {fmt[1]}",
                     "us_per_step": round(dt * 1e6, 1), "attended_MB": round(attended / 1e6, 1),
                     "effective_TBs": round(attended / dt / 1e12, 2)})
        cache.close()
        del cache
        torch.cuda.empty_cache()
    return {"workload": "batch 4, 32 q / 8 kv heads, 128K tokens, all tiers in HBM, top-k blocks of the int4 tier per step "
                        "(identification + top-k + attention + merge + append + evict)", "rows": rows}


# ------------------------------------------------------------------ workload: ablation variants (Sec. 5.4, Table 6)

def run_ablation(steps, warmup):
    """The ablation table's variants as cache configurations on one synthetic 64K context (32 q / 8 kv heads,
    recent window 4096, 128-token blocks): per-step latency (median, p95), host-to-GPU bytes per step and, in
    place of task accuracy, the attention-output error against the all-fp16 cache on the same keys and values."""
    import torch
    from paper_2604_19769_amd.cache import TierConfig, TieredCache
    B, Hq, Hkv, N, R, bt = 1, 32, 8, 65536, 4096, 128
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED + 6)
    K = device_normal(gen, (B, Hkv, N - 1, 128), torch.float16)
    V = device_normal(gen, (B, Hkv, N - 1, 128), torch.float16)
    total = steps + warmup + 2
    q = device_normal(gen, (total, B, Hq, 128), torch.float16)
    kn = device_normal(gen, (total, B, Hkv, 1, 128), torch.float16)
    vn = device_normal(gen, (total, B, Hkv, 1, 128), torch.float16)
    ring = N // bt + 4
    variants = {
        "fp16 (recent window in HBM, the rest fp16 on the host)":
            ([TierConfig("f16", "f16", R, bt, R // bt + 1), TierConfig("f16", "f16", 10**9, bt, ring, mem="host")], 0, True),
        "single tier (no fast tier beyond one landing block; K 8-bit / V 4-bit on the host)":
            ([TierConfig("f16", "f16", bt, bt, 2), TierConfig("i8", "i4", 10**9, bt, ring, mem="host")], 0, True),
        "uniform quantization (8, 8) on the host":
            ([TierConfig("f16", "f16", R, bt, R // bt + 1), TierConfig("i8", "i8", 10**9, bt, ring, mem="host")], 0, True),
        "no streaming attention (block copies and kernels serialised on one stream)":
            ([TierConfig("f16", "f16", R, bt, R // bt + 1), TierConfig("i8", "i4", 10**9, bt, ring, mem="host")], 1, False),
        "TTKV as in the paper (fp16 recent window, K 8-bit / V 4-bit on the host)":
            ([TierConfig("f16", "f16", R, bt, R // bt + 1), TierConfig("i8", "i4", 10**9, bt, ring, mem="host")], 0, True),
        "three tiers (fp16 4K, int8 12K in HBM, int4 on the host)":
            ([TierConfig("f16", "f16", R, bt, R // bt + 1), TierConfig("i8", "i8", 12288, bt, 12288 // bt + 2),
              TierConfig("i4", "i4", 10**9, 1024, N // 1024 + 2, mem="host")], 0, True),
    }
    rows, ref = [], None
    for name, (tiers, n_slots, overlap) in variants.items():
        cache = TieredCache(B, Hq, Hkv, tiers, n_slots=n_slots)
        try:
            # N - 1 tokens: tier 0 one short of its capacity, middle tiers full, the oldest rest in the last tier
            # (whole blocks), every token having passed through the formats of the tiers above its own
            counts = [tiers[0].capacity - 1] + [t.capacity for t in tiers[1:-1]]
            counts.append(N - 1 - sum(counts))
            assert counts[-1] % tiers[-1].block_tokens == 0
            lo = 0
            for t in range(len(tiers) - 1, -1, -1):
                hi = lo + counts[t]
                cache.append(t, K[:, :, lo:hi].contiguous(), V[:, :, lo:hi].contiguous(), through_tiers=t > 0)
                lo = hi
            torch.cuda.synchronize()
            out0 = cache.decode(q[0], None, overlap)[0].clone()
            torch.cuda.synchronize()
            if ref is None:
                ref = out0
            err = float((out0 - ref).abs().max() / ref.abs().max())
            for s in range(warmup):
                cache.step(q[s], kn[s], vn[s], overlap=overlap)
            s0 = cache.stats()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
            for s in range(steps):
                evs[s][0].record()
                cache.step(q[warmup + s], kn[warmup + s], vn[warmup + s], overlap=overlap)
                evs[s][1].record()
            torch.cuda.synchronize()
            us = sorted(a.elapsed_time(b) * 1e3 for a, b in evs)
            h2d = (cache.stats()["h2d_bytes"] - s0["h2d_bytes"]) / steps
            rows.append({"variant": name, "us_per_step_p50": round(us[len(us) // 2], 1),
                         "us_per_step_p95": round(us[min(len(us) - 1, int(0.95 * len(us)))], 1),
                         "h2d_MB_per_step": round(h2d / 1e6, 2), "out_err_vs_fp16_rel_max": round(err, 5)})
            print("ablation:", rows[-1], file=sys.stderr, flush=True)
        finally:
            cache.close()
            torch.cuda.empty_cache()
    return {"workload": "batch 1, 32 q / 8 kv heads, 65536 tokens, recent window 4096, 128-token blocks, one layer's decode "
                        "attention per step (append + attend + evict); error = max |out - out_fp16| / max |out_fp16|",
            "rows": rows}


# ------------------------------------------------------------------ main

def main():
    args = parse()
    if args.overlap_from_trace:
        overlap_from_trace(args.overlap_from_trace, args.trace_prefix)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2604_19769_amd import binding as B
    B.lib()      # fails loudly if the HIP library has not been built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    W, K = args.warmup, args.steps
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB per launch
        torch.cuda.synchronize()
        del src, dst

    if args.workload == "grid":
        r = run_grid([x for x in args.grid_rows.split(",") if x] or None)
        best = max(v["TBs"] for row in r["rows"] for k, v in row.items() if isinstance(v, dict))
        line = {"metric": "decode-attn effective KV TB/s by stored format and head grouping (HBM-resident)", "value": best,
                "unit": "TB/s", "n_gpus": 1, "steps": 24, "warmup": 3, "ms_per_step": None, "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": "f16/int8/int4 -> f32", "data": "synthetic",
                "config": {"workload": "grid: " + r["workload"]}, "grid": r}
        print(json.dumps(line))
        return
    if args.workload == "sparse_hbm":
        r = run_sparse_hbm()
        line = {"metric": "block-sparse decode attention over tiers in HBM: us per step", "value": r["rows"][0]["us_per_step"],
                "unit": "us", "n_gpus": 1, "steps": 32, "warmup": 8, "ms_per_step": round(r["rows"][0]["us_per_step"] / 1e3, 4),
                "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16/int8/int4 -> f32",
                "data": "synthetic", "config": {"workload": "sparse_hbm: " + r["workload"]}, "sparse_hbm": r}
        print(json.dumps(line))
        return
    if args.workload == "gqa_hbm":
        r = run_gqa_hbm(12, [x for x in args.gqa_formats.split(",") if x] or None)
        worst = min(row["GBs"] for row in r["rows"])
        line = {"metric": "decode-attn effective KV GB/s of the grouped-query kernel per stored format (HBM-resident)", "value": worst,
                "unit": "GB/s", "n_gpus": 1, "steps": 12, "warmup": 3, "ms_per_step": None, "higher_is_better": True,
                "scaling": "weak", "vs_baseline": None, "dtype": "f16/int8/int4 -> f32", "data": "synthetic",
                "config": {"workload": "gqa_hbm: " + r["workload"]}, "gqa_hbm": r}
        print(json.dumps(line))
        return
    if args.workload == "ablation":
        r = run_ablation(K, W)
        ttkv = [x for x in r["rows"] if x["variant"].startswith("TTKV")][0]
        line = {"metric": "decode-attn us/step at 64K per ablation variant (Table 6 shape)", "value": ttkv["us_per_step_p50"],
                "unit": "us", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ttkv["us_per_step_p50"] / 1e3, 4),
                "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f16/int8/int4 -> f32",
                "data": "synthetic", "config": {"workload": "ablation: " + r["workload"]}, "ablation": r}
        print(json.dumps(line))
        return
    base = {"n_gpus": 1, "steps": K, "warmup": W, "scaling": "weak", "vs_baseline": None, "data": "synthetic"}
    cpu_on = not args.no_cpu_baseline
    if args.workload == "offload128k":
        r = run_offload128k(K, W, cpu_on, staged_only=args.mode == "staged")
        roof = r["roofline"]
        t_us = r["attn_only_us"] if args.mode == "staged" else r["us_per_token"]
        line = dict(base, metric="decode-attn effective KV GB/s (HBM & PCIe % peak), us/token at 128K", value=roof["achieved"],
                    unit="GB/s", ms_per_step=round(t_us / 1e3, 4), higher_is_better=True, dtype="bf16/int8/int4 -> f32",
                    config={"workload": "offload128k" + (" (staged copies only)" if args.mode == "staged" else ": " + r["workload"])},
                    roofline=roof, cpu_baseline=r.get("cpu_baseline"), offload_128k=r)
        print(json.dumps(line))
        return
    if args.workload in ("tiny", "serving_ragged", "sparse128k"):
        r = {"tiny": lambda: run_tiny(K, W, cpu_on), "serving_ragged": lambda: run_serving_ragged(K, W, cpu_on),
             "sparse128k": lambda: run_sparse128k(K, W, 64, cpu_on)}[args.workload]()
        ms = r["us_per_step"] / 1e3 if "us_per_step" in r else r["ms_per_step"]
        line = dict(base, metric="decode-attn effective KV GB/s (HBM & PCIe % peak), us/token at 128K", value=r["effective_kv_GBs"],
                    unit="GB/s", ms_per_step=round(ms, 4), higher_is_better=True, dtype="f16/bf16/int8/int4 -> f32",
                    config={"workload": args.workload + ": " + r["workload"]}, roofline=r["roofline"], cpu_baseline=r["cpu_baseline"])
        line[args.workload] = r
        print(json.dumps(line))
        return

    L = 64                                                   # further steps timed one by one (median, p95)
    cache, kv, steps_in, shape = build_mha32k(W + K + L)
    q, kn, vn = steps_in
    keep = []
    settle(cache, q)
    timed_steps(cache, q, kn, vn, 0, W, keep=keep)
    total_bytes, by_tier = algorithmic_bytes(cache)        # state at the start of the timed region
    # the attention launch of every 4th timed step is bracketed by a HIP event pair on its stream (each pair
    # leaves ~6 us of idle stream on either side of the launch, so timing every step would cost the step 8 %)
    secs = timed_steps(cache, q, kn, vn, W, K, sample_every=4)
    kernel_ms = B.ttkv_read_attn_timing(cache.h)
    total_bytes_end, by_tier_end = algorithmic_bytes(cache)
    step_bytes = (total_bytes + total_bytes_end) / 2 + shape["B"] * shape["Hkv"] * 512   # + the appended token
    ms = secs / K * 1e3
    value = step_bytes / (secs / K) / 1e9
    kms = sum(kernel_ms) / len(kernel_ms)
    k_bytes = (total_bytes + total_bytes_end) / 2      # the fused launch streams every tier once
    roofline = {"bound": "hbm", "kernel": "attn_fused_kernel<G=1>: fp16 tier + int4 tier in one launch",
                "achieved": round(k_bytes / (kms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(k_bytes / (kms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                "traffic_source": MHA32K_TRAFFIC_SOURCE,
                "kernel_us": round(kms * 1e3, 2), "bytes_per_launch": int(k_bytes), "launches_timed": len(kernel_ms)}
    hbm_read = measure_hbm_read_peak(cache.h)
    roofline["load_only_kernel_GBs"] = round(hbm_read, 1)
    lat = step_latencies(cache, q, kn, vn, W + K, L)
    # the attention launch eight times back to back between one event pair, eight samples: the pair's own cost
    # (dispatch of the markers, a few microseconds) spread over eight launches
    B.ttkv_time_attn_repeat(cache.h, 8)
    B.ttkv_time_attn(cache.h, 8)
    for i in range(8):
        cache.decode(q[i])
    B.ttkv_time_attn(cache.h, 0)
    B.ttkv_time_attn_repeat(cache.h, 1)
    b2b = B.ttkv_read_attn_timing(cache.h)
    b2b_ms = sum(b2b) / len(b2b)
    b2b_bytes = algorithmic_bytes(cache)[0]
    # the headline figures of the object are the back-to-back ones (they agree with rocprofv3's duration of the
    # kernel); the single pair inside the timed region, which also spans the dispatch of its two markers, stays beside
    roofline["kernel_us_single_pair_in_timed_region"] = roofline["kernel_us"]
    roofline["achieved_single_pair_in_timed_region"] = roofline["achieved"]
    roofline["kernel_us"] = round(b2b_ms * 1e3, 2)
    roofline["bytes_per_launch"] = int(b2b_bytes)
    roofline["traffic"] = int(MHA32K_TRAFFIC_FACTOR * b2b_bytes)
    roofline["achieved"] = round(b2b_bytes / (b2b_ms * 1e-3) / 1e9, 1)
    roofline["frac"] = round(b2b_bytes / (b2b_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
    roofline["launches_timed"] = 8 * len(b2b)
    roofline["frac_of_load_only_kernel"] = round(roofline["achieved"] / hbm_read, 4)
    same = measure_hbm_read_same_size(cache.h, int(k_bytes))
    roofline["load_only_same_bytes_us"] = round(same * 1e6, 2)
    roofline["frac_of_load_only_same_bytes"] = round(same / (kms * 1e-3), 4)   # both with a single event pair per launch
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline_mha32k(kv, steps_in, shape, keep[:min(len(keep), 24)])   # the warm-up steps: ~0.1 s of oracle each
    cache.close()
    del cache, kv
    torch.cuda.empty_cache()
    off = None
    if not args.no_offload:
        off = run_offload128k(args.offload_steps, 3, cpu_on)
    line = {
        "metric": "decode-attn effective KV GB/s (HBM & PCIe % peak), us/token at 128K",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16/int4 -> f32", "data": "synthetic",
        "config": {"workload": "mha32k: batch 4, 32 heads MHA, head_dim 128, 32768 tokens, recent 2048 fp16 + 30720 int4 "
                               "(group 64, asymmetric) in HBM, append + attend + evict per step",
                   "algorithmic_bytes_per_step": int(step_bytes), "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
                   "fp16_equivalent_GBs": round(shape["B"] * shape["Hkv"] * shape["N"] * 512 / (secs / K) / 1e9, 1),
                   "step_us_p50_p95_of_64_event_timed": [round(lat[len(lat) // 2] * 1e6, 1),
                                                         round(lat[int(0.95 * len(lat))] * 1e6, 1)],
                   "settle": f"{SETTLE_LAUNCHES} untimed attention launches (~20 ms, cache state untouched) precede the {W} warm-up "
                             "steps: after idle the launch durations drift for ~15 ms (clock management) before they are steady"},
        "roofline": roofline, "cpu_baseline": cpu, "offload_128k": off,
        "tiny": None if args.no_extra else run_tiny(200, 20, cpu_on),
        "serving_ragged": None if args.no_extra else run_serving_ragged(64, 2, cpu_on),
        "sparse_recall_128k": None if args.no_extra else run_sparse128k(8, 2, 64, cpu_on),
        "gqa_hbm": None if args.no_extra else run_gqa_hbm(),
        "key_grouping": None if args.no_extra else run_key_grouping(),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
