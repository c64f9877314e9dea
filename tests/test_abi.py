"""CPU-only checks of the C ABI: the library loads, exports every function the
header declares, sizes records as the format table says, and turns bad arguments
into status codes before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2604_19769_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions(name="ttkv.h"):
    text = open(os.path.join(ROOT, "include", name)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ttkv_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    L = B.lib()
    names = header_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names
    aids = header_functions("ttkv_bench.h")               # measurement / inspection aids: their own header
    assert len(aids) == 5 and not set(aids) & set(names)
    for n in aids:
        assert hasattr(L, n), n
    assert sorted(B.BENCH_EXPORTS) == aids


def host_cache(batch=2, Hq=8, Hkv=2, fmts=(("f16", "f16"), ("i8", "i8"), ("i4", "i4")), bt=(128, 128, 1024)):
    """A descriptor whose pointers are host memory: good enough for everything that must fail before a launch."""
    c = B.ttkv_cache()
    c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.n_tiers = batch, Hq, Hkv, 128, len(fmts)
    c.softmax_scale = 0.088
    keep = []
    for t, ((kf, vf), b) in enumerate(zip(fmts, bt)):
        T = c.tier[t]
        T.k_fmt, T.v_fmt, T.mem, T.block_tokens = B.FMT_NAMES[kf], B.FMT_NAMES[vf], B.MEM_DEVICE, b
        T.capacity_tokens, T.ring_blocks, T.pool_blocks = 4 * b, 8, 8 * batch
        buf = np.zeros(16, np.uint8)
        s, l = np.zeros(batch, np.int64), np.zeros(batch, np.int64)
        T.data, T.start, T.len = buf.ctypes.data, s.ctypes.data, l.ctypes.data
        keep += [buf, s, l]
    c._keep = keep
    return c


def test_record_bytes_follow_the_format_table():
    c = host_cache(Hkv=8)
    assert B.ttkv_record_bytes(c, 0) == 128 * 8 * 512          # fp16 K+V: 512 B per token-head
    assert B.ttkv_record_bytes(c, 1) == 128 * 8 * 272          # int8 g32: 2 x (128 + 4 x 2)
    assert B.ttkv_record_bytes(c, 2) == 1024 * 8 * 144 == 1179648   # int4 g64: 2 x (64 + 2 x 4)
    c.tier[1].v_fmt = B.I4_ASYM_G64                              # K 8-bit / V 4-bit
    assert B.ttkv_record_bytes(c, 1) == 128 * 8 * 208
    assert B.ttkv_record_bytes(c, 3) == 0 and B.ttkv_record_bytes(c, -1) == 0


def test_invalid_arguments_are_status_codes():
    h = B.ttkv_create()
    L = B.lib()
    c = host_cache()
    null = C.c_void_p()
    dummy = C.c_void_p(c._keep[0].ctypes.data)
    # NULL handle / NULL pointers
    assert L.ttkv_decode_attn(None, C.byref(c), dummy, B.F16, dummy, None, None, None, 0, dummy, 1 << 20, 2, None, None) == B.ERR_INVALID_ARG
    assert L.ttkv_decode_attn(h, C.byref(c), None, B.F16, dummy, None, None, None, 0, dummy, 1 << 20, 2, None, None) == B.ERR_INVALID_ARG
    assert L.ttkv_decode_attn(h, C.byref(c), dummy, B.I8_SYM_G32, dummy, None, None, None, 0, dummy, 1 << 20, 2, None, None) == B.ERR_INVALID_ARG
    # workspace too small for even one part
    assert L.ttkv_decode_attn(h, C.byref(c), dummy, B.F16, dummy, None, None, None, 0, dummy, 64, 2, None, None) == B.ERR_WORKSPACE
    # head_dim
    c.head_dim = 64
    assert L.ttkv_decode_attn(h, C.byref(c), dummy, B.F16, dummy, None, None, None, 0, dummy, 1 << 20, 2, None, None) == B.ERR_UNSUPPORTED
    c.head_dim = 128
    # more KV heads than a launch grid's third dimension indexes together with the batch
    c.n_q_heads, c.n_kv_heads = 1024, 1024
    assert L.ttkv_decode_attn(h, C.byref(c), dummy, B.F16, dummy, None, None, None, 0, dummy, 1 << 20, 2, None, None) == B.ERR_UNSUPPORTED
    c.n_q_heads, c.n_kv_heads = 8, 2
    # unsupported format pair (V wider than K)
    c.tier[1].k_fmt, c.tier[1].v_fmt = B.I4_ASYM_G64, B.I8_SYM_G32
    assert L.ttkv_count_parts(h, C.byref(c), None, None, 0, 0) == -1
    assert L.ttkv_quantize_append(h, C.byref(c), 1, -1, dummy, dummy, B.F16, 4, 0, None) == B.ERR_UNSUPPORTED
    c.tier[1].k_fmt = c.tier[1].v_fmt = B.I8_SYM_G32
    # values stored channel-major per 32 tokens: a value format of the last tier, int8 or int4 keys, >= 2 heads per KV
    # head, whole groups of 32 tokens
    c.tier[2].v_fmt = B.I4_ASYM_G64_T32
    assert B.ttkv_record_bytes(c, 2) == 1024 * 2 * 144
    assert L.ttkv_quantize_append(h, C.byref(c), 2, -1, dummy, dummy, B.F16, 48, 0, None) == B.ERR_INVALID_ARG
    assert L.ttkv_quantize_append(h, C.byref(c), 2, -1, dummy, dummy, B.F16, 0, 0, None) == B.OK
    c._keep[8][:] = 40                                                     # tier 2's len[]: not whole groups
    assert L.ttkv_count_parts(h, C.byref(c), None, None, 0, 0) == -1
    c._keep[8][:] = 0
    c.tier[2].k_fmt = B.F16
    assert L.ttkv_count_parts(h, C.byref(c), None, None, 0, 0) == -1        # fp16 keys with int4 values: no kernel
    c.tier[2].k_fmt = B.I4_ASYM_G64_T32
    assert L.ttkv_count_parts(h, C.byref(c), None, None, 0, 0) == -1        # not a key format
    c.tier[2].k_fmt = B.I8_SYM_G32
    assert L.ttkv_count_parts(h, C.byref(c), None, None, 0, 0) == 0         # K 8-bit + these values: fine (nothing cached yet)
    c.n_q_heads = c.n_kv_heads
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 1, 0, None) == B.ERR_UNSUPPORTED   # one head per KV head
    c.n_q_heads = 8
    c.tier[2].k_fmt = c.tier[2].v_fmt = B.I4_ASYM_G64
    c.tier[1].v_fmt = B.I4_ASYM_G64_T32
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 1, 0, None) == B.ERR_UNSUPPORTED   # a middle tier
    c.tier[1].v_fmt = B.I8_SYM_G32
    # block_tokens not a multiple of 64, batch out of range, GQA ratio
    c.tier[0].block_tokens = 100
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 1, 0, None) == B.ERR_INVALID_ARG
    c.tier[0].block_tokens = 128
    c.batch = 65
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 1, 0, None) == B.ERR_INVALID_ARG
    c.batch = 2
    c.n_q_heads = 7
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 1, 0, None) == B.ERR_INVALID_ARG
    c.n_q_heads = 8
    # fp tier only takes its own format; ring overflow; bad tier / seq
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.BF16, 1, 0, None) == B.ERR_UNSUPPORTED
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 8 * 128 + 1, 0, None) == B.ERR_CAPACITY
    assert L.ttkv_quantize_append(h, C.byref(c), 3, -1, dummy, dummy, B.F16, 1, 0, None) == B.ERR_INVALID_ARG
    assert L.ttkv_quantize_append(h, C.byref(c), 0, 2, dummy, dummy, B.F16, 1, 0, None) == B.ERR_INVALID_ARG
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 0, 0, None) == B.OK     # nothing to do
    # one-call step: NULL token, a format the fp tier does not have, a full ring; no length changes on refusal
    tail = (dummy, None, None, None, 0, dummy, 1 << 20, 0, None, None)     # out, lse, selection, workspace, slots, streams
    assert L.ttkv_decode_step(h, C.byref(c), dummy, B.F16, None, dummy, B.F16, *tail) == B.ERR_INVALID_ARG
    assert L.ttkv_decode_step(h, C.byref(c), dummy, B.F16, dummy, dummy, B.I8_SYM_G32, *tail) == B.ERR_INVALID_ARG
    assert L.ttkv_decode_step(h, C.byref(c), dummy, B.F16, dummy, dummy, B.BF16, *tail) == B.ERR_UNSUPPORTED
    assert L.ttkv_decode_step(None, C.byref(c), dummy, B.F16, dummy, dummy, B.F16, *tail) == B.ERR_INVALID_ARG
    lens = c._keep[2]                       # tier 0's len[]
    lens[:] = 8 * 128
    assert L.ttkv_decode_step(h, C.byref(c), dummy, B.F16, dummy, dummy, B.F16, *tail) == B.ERR_CAPACITY
    lens[:] = 5
    assert L.ttkv_decode_step(h, C.byref(c), None, B.F16, dummy, dummy, B.F16, *tail) == B.ERR_INVALID_ARG      # no query
    assert L.ttkv_decode_step(h, C.byref(c), dummy, B.F16, dummy, dummy, B.F16, dummy, None, None, None, 0, dummy, 64, 0,
                              None, None) == B.ERR_WORKSPACE
    assert lens.tolist() == [5, 5]
    lens[:] = 0
    # identify + top-k + attend in one call: no mean keys on the last tier, half a pair of output pointers
    topk_tail = (dummy, None, 4, None, None, 4, dummy, 1 << 16, dummy, 1 << 20, None)
    assert L.ttkv_decode_step_topk(h, C.byref(c), dummy, B.F16, dummy, dummy, B.F16, *topk_tail) == B.ERR_UNSUPPORTED
    assert L.ttkv_decode_step_topk(None, C.byref(c), dummy, B.F16, dummy, dummy, B.F16, *topk_tail) == B.ERR_INVALID_ARG
    assert L.ttkv_decode_step_topk(h, C.byref(c), dummy, B.F16, dummy, None, B.F16, *topk_tail) == B.ERR_INVALID_ARG
    assert L.ttkv_decode_step_topk(h, C.byref(c), dummy, B.F16, dummy, dummy, B.F16, dummy, None, 4, dummy, None, 4, dummy,
                                   1 << 16, dummy, 1 << 20, None) == B.ERR_INVALID_ARG
    # a paged host tier written by the kernels needs the device copy of its block table
    tbl = np.arange(16, dtype=np.int32)
    c.tier[2].mem, c.tier[2].block_table = B.MEM_HOST_PINNED, tbl.ctypes.data
    assert L.ttkv_quantize_append_host(h, C.byref(c), 2, -1, dummy, dummy, B.F16, 4, 0, None, 0, None) == B.ERR_INVALID_ARG
    c.tier[2].mem, c.tier[2].block_table = B.MEM_DEVICE, None
    # keys grouped over tokens: a key format of the last tier only, whole groups of 128 tokens
    c.tier[2].k_fmt = B.I4_ASYM_T128
    assert L.ttkv_quantize_append_host is not None
    assert L.ttkv_quantize_append(h, C.byref(c), 2, -1, dummy, dummy, B.F16, 100, 0, None) == B.ERR_INVALID_ARG
    assert L.ttkv_quantize_append(h, C.byref(c), 2, -1, dummy, dummy, B.F16, 0, 0, None) == B.OK
    c.tier[2].v_fmt = B.I8_SYM_G32
    assert L.ttkv_quantize_append(h, C.byref(c), 2, -1, dummy, dummy, B.F16, 128, 0, None) == B.ERR_UNSUPPORTED   # V must be int4 g64
    c.tier[2].v_fmt = B.I4_ASYM_T128
    assert L.ttkv_quantize_append(h, C.byref(c), 2, -1, dummy, dummy, B.F16, 128, 0, None) == B.ERR_UNSUPPORTED   # not a value format
    c.tier[2].k_fmt = c.tier[2].v_fmt = B.I4_ASYM_G64
    c.tier[1].k_fmt, c.tier[1].v_fmt = B.I4_ASYM_T128, B.I4_ASYM_G64
    assert L.ttkv_quantize_append(h, C.byref(c), 0, -1, dummy, dummy, B.F16, 1, 0, None) == B.ERR_UNSUPPORTED     # nothing passes through it
    c.tier[1].k_fmt = c.tier[1].v_fmt = B.I8_SYM_G32
    assert B.ttkv_record_bytes(c, 2) == 1024 * 2 * 144
    c.tier[2].k_fmt = B.I4_ASYM_T128
    assert B.ttkv_record_bytes(c, 2) == 1024 * 2 * 140          # 64 + 4 bytes of keys per token-head
    c.tier[2].k_fmt = B.I4_ASYM_G64
    # nothing is due: demote is a no-op; src tier out of range
    assert L.ttkv_tier_demote(h, C.byref(c), 0, 0, None, 0, None, None) == B.OK
    assert L.ttkv_tier_demote(h, C.byref(c), 2, 0, None, 0, None, None) == B.ERR_INVALID_ARG
    # destination ring overflow is found before anything is enqueued
    c._keep[2][:] = 4 * 128            # tier 0 len = capacity -> due
    c._keep[5][:] = 8 * 128            # tier 1 ring full
    assert L.ttkv_tier_demote(h, C.byref(c), 0, 0, None, 0, None, None) == B.ERR_CAPACITY
    assert list(c._keep[2]) == [512, 512] and list(c._keep[5]) == [1024, 1024]    # no state change
    # selection lists
    c._keep[2][:] = 0
    c._keep[5][:] = 0
    cnt = np.array([3, 0], np.int32)
    ids = np.zeros((2, 2), np.int32)
    assert L.ttkv_count_parts(h, C.byref(c), ids.ctypes.data, cnt.ctypes.data, 2, 0) == -1   # count > stride
    assert L.ttkv_count_parts(h, C.byref(c), ids.ctypes.data, None, 2, 0) == -1
    # locate on an empty cache, merge argument checks
    t = C.c_int32()
    assert L.ttkv_locate(C.byref(c), 0, 0, C.byref(t), None, None, None) == B.ERR_INVALID_ARG
    assert L.ttkv_merge_partials(h, dummy, dummy, dummy, 4, 2, None, 1, dummy, None, None) == B.ERR_INVALID_ARG
    assert B.status_string(B.ERR_CAPACITY) == "tier capacity"
    B.ttkv_destroy(h)


def test_locate_and_part_count_are_host_arithmetic():
    c = host_cache(batch=1)
    # tier 2 holds the oldest 2048 tokens (start ordinal 1024), tier 1 the next 300, tier 0 the newest 70
    c._keep[7][0], c._keep[8][0] = 1024, 2048
    c._keep[4][0], c._keep[5][0] = 256, 300
    c._keep[1][0], c._keep[2][0] = 0, 70
    assert B.ttkv_locate(c, 0, 0) == (2, 1, 0, 1)
    assert B.ttkv_locate(c, 0, 2047) == (2, 2, 1023, 2)
    assert B.ttkv_locate(c, 0, 2048) == (1, 2, 0, 2)
    assert B.ttkv_locate(c, 0, 2048 + 299) == (1, 4, 43, 4)
    assert B.ttkv_locate(c, 0, 2048 + 300 + 69) == (0, 0, 69, 0)
    with pytest.raises(B.TTKVError):
        B.ttkv_locate(c, 0, 2048 + 300 + 70)
    h = B.ttkv_create()
    assert B.ttkv_count_parts(h, c) >= 3
    B.ttkv_destroy(h)
    assert B.ttkv_workspace_bytes(c, 8, 2) >= 1 * 8 * 8 * 130 * 4


def golden_sizes():
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "tier_sizes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, kf, vf, hkv, tokens, nbytes, _ = [x.strip() for x in line.split("|")]
        rows.append((name, kf, vf, int(hkv), int(tokens), int(nbytes)))
    return rows


def test_sizes_of_the_layout_formula():
    """Sec. 4.1's M = L x d_kv x b with the stored formats' byte widths, worked out by hand in
    tests/golden/tier_sizes.txt: the library's record size and the oracle's agree with it."""
    from oracle import OracleCache, TierSpec
    rows = golden_sizes()
    assert len(rows) >= 9
    for name, kf, vf, hkv, tokens, nbytes in rows:
        bt = 128 if tokens % 1024 else 1024
        assert tokens % bt == 0
        c = host_cache(batch=1, Hq=hkv, Hkv=hkv, fmts=((kf if kf != "i4t" else "f16", vf if kf != "i4t" else "f16"), (kf, vf)), bt=(128, bt))
        assert B.ttkv_record_bytes(c, 1) * (tokens // bt) == nbytes, name
        fp = "bf16" if kf == "bf16" else "f16"
        ora = OracleCache(1, hkv, hkv, 128, [TierSpec(fp, fp, 128, 128), TierSpec(kf, vf, 10**9, bt)], [128, 128])
        assert ora.record_bytes(1) * (tokens // bt) == nbytes, name


def test_header_is_plain_c(tmp_path):
    """include/ttkv.h is the boundary: it must compile as C99 on its own (no C++ or HIP types in the signatures)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "hdr.c"
    src.write_text('#include "ttkv.h"\nint main(void) { ttkv_cache c; ttkv_stats s; (void)c; (void)s; return 0; }\n')
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-c", str(src), "-o",
                    str(tmp_path / "hdr.o")], check=True)



def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N above 1 exits with a message that says so (before touching a GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2", "--steps", "1", "--warmup", "0"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_block_table_entries_are_checked_per_call_unless_switched_off():
    """Paged tiers: an entry beyond pool_blocks is refused by every call that takes the handle; with the per-call check
    switched off (ttkv_set_table_check, for pools of millions of pages) the same descriptor is taken as the caller
    wrote it -- shown with ttkv_count_parts, which enqueues nothing -- and the switch can be turned back on."""
    h = B.ttkv_create()
    try:
        c = host_cache()
        T = c.tier[2]
        T.mem = B.MEM_HOST_PINNED
        table = np.arange(2 * 8, dtype=np.int32)
        T.block_table = table.ctypes.data
        lens = np.array([3000, 500], np.int64)
        T.len = lens.ctypes.data
        c._keep += [table, lens]
        good = B.ttkv_count_parts(h, c)
        assert good > 0
        table[5] = 16                      # == pool_blocks: one past the last record
        assert B.ttkv_count_parts(h, c) == -1
        B.ttkv_set_table_check(h, 0)
        assert B.ttkv_count_parts(h, c) == good
        B.ttkv_set_table_check(h, 1)
        assert B.ttkv_count_parts(h, c) == -1
        assert B.lib().ttkv_set_table_check(h, 2) == B.ERR_INVALID_ARG
        assert B.lib().ttkv_set_table_check(None, 0) == B.ERR_INVALID_ARG
    finally:
        B.ttkv_destroy(h)


def plan_cache(batch, Hq, Hkv, tiers):
    """tiers: (k_fmt, v_fmt, block_tokens, tokens per sequence); device tiers, pointers never dereferenced."""
    c = B.ttkv_cache()
    c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.n_tiers = batch, Hq, Hkv, 128, len(tiers)
    c.softmax_scale = 0.088
    keep = []
    for t, (kf, vf, bt, n) in enumerate(tiers):
        T = c.tier[t]
        T.k_fmt, T.v_fmt, T.mem, T.block_tokens = B.FMT_NAMES[kf], B.FMT_NAMES[vf], B.MEM_DEVICE, bt
        lens = np.full(batch, n, np.int64) if np.isscalar(n) else np.asarray(n, np.int64)
        T.capacity_tokens, T.ring_blocks = 10**9, int(lens.max()) // bt + 2
        T.pool_blocks = T.ring_blocks * batch
        buf, s = np.zeros(16, np.uint8), np.zeros(batch, np.int64)
        T.data, T.start, T.len = buf.ctypes.data, s.ctypes.data, lens.ctypes.data
        keep += [buf, s, lens]
    c._keep = keep
    return c


def test_split_plan_equal_items_and_whole_rounds():
    """The split-K plan (how Alg. 1's sum over blocks is cut; host arithmetic only): one long run per tier and
    sequence keeps the kernel's default number of workgroups; many short runs get finer, equal items instead of one
    unequal item per run; a forced target is taken as given; no item is shorter than 256 or longer than 8192 tokens."""
    h = B.ttkv_create()
    try:
        # batch 4, 32 q / 8 kv heads, 256-token window + one long int8 tier: one round of 768 workgroups = 24 items per run
        c = plan_cache(4, 32, 8, [("f16", "f16", 128, 255), ("i8", "i8", 128, 65536)])
        assert B.ttkv_count_parts(h, c) == 1 + 24
        # the multi-head workload: 2.5 rounds of 1024 -> 4 + 16 items of 512 and 1920 tokens (262 and 276 KB)
        c = plan_cache(4, 32, 32, [("f16", "f16", 128, 2048), ("i4", "i4", 128, 30720)])
        assert B.ttkv_count_parts(h, c) == 4 + 16
        # 64 sequences of 1024 fp16 + 3072 int8 tokens: one item per run would be 524 and 835 KB on 1024 workgroups for
        # 768 slots; the plan goes to 2 + 3 items (262 and 278 KB)
        c = plan_cache(64, 32, 8, [("f16", "f16", 128, 1024), ("i8", "i8", 128, 3072)])
        assert B.ttkv_count_parts(h, c) == 2 + 3
        B.ttkv_set_split(h, 768)
        assert B.ttkv_count_parts(h, c) == 1 + 1
        B.ttkv_set_split(h, 1 << 20)
        assert B.ttkv_count_parts(h, c) == 1024 // 256 + 3072 // 256
        B.ttkv_set_split(h, 1)
        c = plan_cache(1, 8, 8, [("f16", "f16", 128, 100000)])
        assert B.ttkv_count_parts(h, c) == -(-100000 // 8192)
        B.ttkv_set_split(h, 0)
        # ragged lengths: every sequence's parts cover its tokens in items of 256..8192 tokens
        lens = [300, 5000, 70000, 129, 8192, 64, 33333, 2048]
        c = plan_cache(8, 32, 8, [("bf16", "bf16", 128, 200), ("i4", "i4", 128, lens)])
        parts = B.ttkv_count_parts(h, c)
        assert 1 + -(-70000 // 8192) <= parts <= 1 + 70000 // 256
    finally:
        B.ttkv_destroy(h)
