"""ctypes binding of libttkv.so: the same names as include/ttkv.h, argument
marshalling only.  The library must have been built (python -m
paper_2604_19769_amd.build, or __graft_entry__.build()); there is no fallback
path of any kind: a missing library is an error."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libttkv.so")

TTKV_MAX_TIERS = 4
TTKV_MAX_BATCH = 64
TTKV_MAX_SLOTS = 16
TTKV_NOALLOC_SCRATCH_BYTES = 16 << 20

OK, ERR_INVALID_ARG, ERR_CAPACITY, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = range(6)
F16, BF16, I8_SYM_G32, I4_ASYM_G64, F32, I4_ASYM_T128, I4_ASYM_G64_T32 = range(7)
MEM_DEVICE, MEM_HOST_PINNED = 0, 1
FMT_NAMES = {"f16": F16, "bf16": BF16, "i8": I8_SYM_G32, "i4": I4_ASYM_G64, "f32": F32, "i4t": I4_ASYM_T128,
             "i4c": I4_ASYM_G64_T32}   # i4c: values as i4, codes stored channel-major per 32 tokens


class ttkv_tier(C.Structure):
    _fields_ = [
        ("k_fmt", C.c_int32), ("v_fmt", C.c_int32), ("mem", C.c_int32), ("block_tokens", C.c_int32),
        ("capacity_tokens", C.c_int64), ("ring_blocks", C.c_int64), ("pool_blocks", C.c_int64),
        ("data", C.c_void_p), ("block_table", C.c_void_p), ("block_table_dev", C.c_void_p),
        ("k_sum", C.c_void_p), ("k_summary", C.c_void_p), ("start", C.c_void_p), ("len", C.c_void_p),
    ]


class ttkv_cache(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
        ("n_tiers", C.c_int32), ("softmax_scale", C.c_float), ("tier", ttkv_tier * TTKV_MAX_TIERS),
    ]


class ttkv_stats(C.Structure):
    _fields_ = [
        ("h2d_bytes", C.c_uint64), ("d2h_bytes", C.c_uint64), ("blocks_fetched", C.c_uint64),
        ("kernels", C.c_uint64), ("demotions", C.c_uint64), ("mfma_launches", C.c_uint64),
        ("last_hip_error", C.c_int32),
    ]


EXPORTS = [
    "ttkv_create", "ttkv_destroy", "ttkv_get_stats", "ttkv_reset_stats", "ttkv_status_string", "ttkv_record_bytes",
    "ttkv_locate", "ttkv_workspace_bytes", "ttkv_demote_workspace_bytes", "ttkv_append_host_workspace_bytes",
    "ttkv_count_parts", "ttkv_quantize_append", "ttkv_quantize_append_host", "ttkv_tier_demote", "ttkv_decode_attn",
    "ttkv_decode_step", "ttkv_decode_step_topk", "ttkv_decode_attn_noalloc",
    "ttkv_merge_partials", "ttkv_select_blocks", "ttkv_set_split", "ttkv_set_table_check",
]
# include/ttkv_bench.h: measurement and inspection aids, not part of the boundary
BENCH_EXPORTS = ["ttkv_time_attn", "ttkv_time_attn_repeat", "ttkv_read_attn_timing", "ttkv_stream_read", "ttkv_staged_schedule"]
OP_COPY, OP_ATTEND, OP_RECORD, OP_WAIT, OP_MERGE = range(5)


class ttkv_chain_op(C.Structure):
    _fields_ = [("kind", C.c_int32), ("stream", C.c_int32), ("event", C.c_int32), ("slot", C.c_int32), ("fetch", C.c_int32),
                ("bytes", C.c_uint64)]


_lib = None


class TTKVError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


def lib():
    """Load libttkv.so.  Raises if it has not been built: nothing replaces it."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_19769_amd.build`")
        L = C.CDLL(LIB_PATH)
        p, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        cp = C.POINTER(ttkv_cache)
        L.ttkv_create.argtypes = [C.POINTER(p)]
        L.ttkv_destroy.argtypes = [p]
        L.ttkv_get_stats.argtypes = [p, C.POINTER(ttkv_stats)]
        L.ttkv_get_stats.restype = None
        L.ttkv_reset_stats.argtypes = [p]
        L.ttkv_reset_stats.restype = None
        L.ttkv_status_string.argtypes = [i32]
        L.ttkv_status_string.restype = C.c_char_p
        L.ttkv_record_bytes.argtypes = [cp, i32]
        L.ttkv_record_bytes.restype = sz
        L.ttkv_locate.argtypes = [cp, i32, i64, C.POINTER(i32), C.POINTER(i64), C.POINTER(i32), C.POINTER(i64)]
        L.ttkv_workspace_bytes.argtypes = [cp, i32, i32]
        L.ttkv_workspace_bytes.restype = sz
        L.ttkv_demote_workspace_bytes.argtypes = [cp, i32]
        L.ttkv_demote_workspace_bytes.restype = sz
        L.ttkv_append_host_workspace_bytes.argtypes = [cp, i32, i32, i64]
        L.ttkv_append_host_workspace_bytes.restype = sz
        L.ttkv_count_parts.argtypes = [p, cp, p, p, i32, i32]
        L.ttkv_set_split.argtypes = [p, i32]
        L.ttkv_set_table_check.argtypes = [p, i32]
        L.ttkv_count_parts.restype = i32
        L.ttkv_quantize_append.argtypes = [p, cp, i32, i32, p, p, i32, i64, i32, p]
        L.ttkv_quantize_append_host.argtypes = [p, cp, i32, i32, p, p, i32, i64, i32, p, sz, p]
        L.ttkv_tier_demote.argtypes = [p, cp, i32, i32, p, sz, p, p]
        L.ttkv_decode_attn.argtypes = [p, cp, p, i32, p, p, p, p, i32, p, sz, i32, p, p]
        L.ttkv_decode_attn_noalloc.argtypes = [p, cp, p, i32, p, p, p, p, i32, p]
        L.ttkv_decode_step.argtypes = [p, cp, p, i32, p, p, i32, p, p, p, p, i32, p, sz, i32, p, p]
        L.ttkv_decode_step_topk.argtypes = [p, cp, p, i32, p, p, i32, p, p, i32, p, p, i32, p, sz, p, sz, p]
        L.ttkv_merge_partials.argtypes = [p, p, p, p, i32, i32, p, i32, p, p, p]
        L.ttkv_select_blocks.argtypes = [p, cp, p, i32, i32, p, p, i32, p, sz, p]
        L.ttkv_time_attn.argtypes = [p, i32]
        L.ttkv_time_attn_repeat.argtypes = [p, i32]
        L.ttkv_stream_read.argtypes = [p, p, sz, p, p]
        L.ttkv_read_attn_timing.argtypes = [p, C.POINTER(C.c_float), i32, C.POINTER(i32)]
        L.ttkv_staged_schedule.argtypes = [p, cp, p, p, i32, i32, i32, C.POINTER(ttkv_chain_op), i32, C.POINTER(i32)]
        for name in EXPORTS + BENCH_EXPORTS:
            f = getattr(L, name)
            if name not in ("ttkv_get_stats", "ttkv_reset_stats", "ttkv_status_string", "ttkv_record_bytes",
                            "ttkv_workspace_bytes", "ttkv_demote_workspace_bytes",
                            "ttkv_append_host_workspace_bytes", "ttkv_count_parts"):
                f.restype = i32
        _lib = L
    return _lib


def status_string(status):
    return lib().ttkv_status_string(int(status)).decode()


def _check(status, what):
    if status != OK:
        raise TTKVError(status, what)


def _p(x):
    """Pointer of a torch tensor / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return C.c_void_p(x)
    return C.c_void_p(x.data_ptr())


def ttkv_create():
    h = C.c_void_p()
    _check(lib().ttkv_create(C.byref(h)), "ttkv_create")
    return h


def ttkv_destroy(h):
    _check(lib().ttkv_destroy(h), "ttkv_destroy")


def ttkv_get_stats(h):
    s = ttkv_stats()
    lib().ttkv_get_stats(h, C.byref(s))
    return {k: getattr(s, k) for k, _ in ttkv_stats._fields_}


def ttkv_reset_stats(h):
    lib().ttkv_reset_stats(h)


def ttkv_record_bytes(cache, tier):
    return lib().ttkv_record_bytes(C.byref(cache), tier)


def ttkv_locate(cache, b, pos):
    t, blk, row, rec = C.c_int32(), C.c_int64(), C.c_int32(), C.c_int64()
    _check(lib().ttkv_locate(C.byref(cache), b, pos, C.byref(t), C.byref(blk), C.byref(row), C.byref(rec)), "ttkv_locate")
    return t.value, blk.value, row.value, rec.value


def ttkv_workspace_bytes(cache, max_parts, n_slots):
    return lib().ttkv_workspace_bytes(C.byref(cache), max_parts, n_slots)


def ttkv_demote_workspace_bytes(cache, src_tier):
    return lib().ttkv_demote_workspace_bytes(C.byref(cache), src_tier)


def ttkv_append_host_workspace_bytes(cache, tier, seq, n_tokens):
    return lib().ttkv_append_host_workspace_bytes(C.byref(cache), tier, seq, n_tokens)


def ttkv_count_parts(h, cache, sel_blocks=None, sel_count=None, sel_stride=0, n_slots=0):
    return lib().ttkv_count_parts(h, C.byref(cache), _p(sel_blocks), _p(sel_count), sel_stride, n_slots)


def ttkv_stream_read(h, src, nbytes, sink, stream):
    _check(lib().ttkv_stream_read(h, _p(src), nbytes, _p(sink), _p(stream)), "ttkv_stream_read")


def ttkv_set_split(h, target_items):
    _check(lib().ttkv_set_split(h, target_items), "ttkv_set_split")


def ttkv_set_table_check(h, on):
    _check(lib().ttkv_set_table_check(h, int(on)), "ttkv_set_table_check")


def ttkv_quantize_append(h, cache, tier, seq, k_src, v_src, src_fmt, n_tokens, through_tiers, stream):
    _check(lib().ttkv_quantize_append(h, C.byref(cache), tier, seq, _p(k_src), _p(v_src), src_fmt, n_tokens,
                                      through_tiers, _p(stream)), "ttkv_quantize_append")


def ttkv_quantize_append_host(h, cache, tier, seq, k_src, v_src, src_fmt, n_tokens, through_tiers, workspace,
                              ws_bytes, stream):
    _check(lib().ttkv_quantize_append_host(h, C.byref(cache), tier, seq, _p(k_src), _p(v_src), src_fmt, n_tokens,
                                           through_tiers, _p(workspace), ws_bytes, _p(stream)),
           "ttkv_quantize_append_host")


def ttkv_tier_demote(h, cache, src_tier, max_blocks, workspace, ws_bytes, compute, copy):
    _check(lib().ttkv_tier_demote(h, C.byref(cache), src_tier, max_blocks, _p(workspace), ws_bytes, _p(compute),
                                  _p(copy)), "ttkv_tier_demote")


def ttkv_decode_attn(h, cache, q, q_fmt, out, lse, sel_blocks, sel_count, sel_stride, workspace, ws_bytes, n_slots,
                     compute, copy):
    _check(lib().ttkv_decode_attn(h, C.byref(cache), _p(q), q_fmt, _p(out), _p(lse), _p(sel_blocks), _p(sel_count),
                                  sel_stride, _p(workspace), ws_bytes, n_slots, _p(compute), _p(copy)),
           "ttkv_decode_attn")


def ttkv_decode_attn_noalloc(h, cache, q, q_fmt, out, lse, sel_blocks, sel_count, sel_stride, stream):
    _check(lib().ttkv_decode_attn_noalloc(h, C.byref(cache), _p(q), q_fmt, _p(out), _p(lse), _p(sel_blocks), _p(sel_count),
                                          sel_stride, _p(stream)), "ttkv_decode_attn_noalloc")


def ttkv_decode_step(h, cache, q, q_fmt, k_new, v_new, new_fmt, out, lse, sel_blocks, sel_count, sel_stride, workspace,
                     ws_bytes, n_slots, compute, copy):
    _check(lib().ttkv_decode_step(h, C.byref(cache), _p(q), q_fmt, _p(k_new), _p(v_new), new_fmt, _p(out), _p(lse),
                                  _p(sel_blocks), _p(sel_count), sel_stride, _p(workspace), ws_bytes, n_slots,
                                  _p(compute), _p(copy)), "ttkv_decode_step")


def ttkv_decode_step_topk(h, cache, q, q_fmt, k_new, v_new, new_fmt, out, lse, k, sel_blocks_out, sel_count_out, sel_stride,
                          sel_scratch, sel_scratch_bytes, workspace, ws_bytes, stream):
    _check(lib().ttkv_decode_step_topk(h, C.byref(cache), _p(q), q_fmt, _p(k_new), _p(v_new), new_fmt, _p(out), _p(lse), k,
                                       _p(sel_blocks_out), _p(sel_count_out), sel_stride, _p(sel_scratch), sel_scratch_bytes,
                                       _p(workspace), ws_bytes, _p(stream)), "ttkv_decode_step_topk")


def ttkv_merge_partials(h, m, l, acc, n_parts, part_stride, n_parts_row, rows, out, lse, stream):
    _check(lib().ttkv_merge_partials(h, _p(m), _p(l), _p(acc), n_parts, part_stride, _p(n_parts_row), rows, _p(out),
                                     _p(lse), _p(stream)), "ttkv_merge_partials")


def ttkv_select_blocks(h, cache, q, q_fmt, k, sel_blocks, sel_count, sel_stride, scratch, scratch_bytes, stream):
    _check(lib().ttkv_select_blocks(h, C.byref(cache), _p(q), q_fmt, k, _p(sel_blocks), _p(sel_count), sel_stride,
                                    _p(scratch), scratch_bytes, _p(stream)), "ttkv_select_blocks")


def ttkv_time_attn(h, max_samples):
    _check(lib().ttkv_time_attn(h, max_samples), "ttkv_time_attn")


def ttkv_time_attn_repeat(h, repeat):
    _check(lib().ttkv_time_attn_repeat(h, repeat), "ttkv_time_attn_repeat")


def ttkv_read_attn_timing(h, capacity=4096):
    ms = (C.c_float * capacity)()
    n = C.c_int32()
    _check(lib().ttkv_read_attn_timing(h, ms, capacity, C.byref(n)), "ttkv_read_attn_timing")
    return [ms[i] for i in range(n.value)]


def ttkv_staged_schedule(h, cache, sel_blocks=None, sel_count=None, sel_stride=0, n_slots=2, same_stream=False, capacity=1 << 16):
    """The stream operations ttkv_decode_attn would issue, as a list of dicts (host only: nothing runs)."""
    ops = (ttkv_chain_op * capacity)()
    n = C.c_int32()
    _check(lib().ttkv_staged_schedule(h, C.byref(cache), _p(sel_blocks), _p(sel_count), sel_stride, n_slots, int(same_stream), ops,
                                      capacity, C.byref(n)), "ttkv_staged_schedule")
    assert n.value <= capacity
    return [{k: getattr(ops[i], k) for k, _ in ttkv_chain_op._fields_} for i in range(n.value)]
