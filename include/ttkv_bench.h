/*
 * libttkv -- measurement and inspection aids.  NOT part of the boundary (ttkv.h): nothing here computes a
 * step of the method.  The benchmark uses the timing calls and the load-only kernel for its roofline
 * figures; the tests use ttkv_staged_schedule to check the order of the copy/compute chain on the CPU.
 * Same conventions as ttkv.h ([host] / [device] pointers, status codes, no allocation of device memory).
 */
#ifndef TTKV_BENCH_H
#define TTKV_BENCH_H

#include "ttkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid (roofline of the attention kernel; Sec. 5.1 item 4 "latency is
 * measured on the GPU with events"): from now on every ttkv_decode_attn records a
 * HIP event pair around its fused attention launch(es) on the compute stream, for
 * at most max_samples calls (<= 4096) in total; max_samples <= 0 pauses it (the
 * samples taken so far are kept, so a caller can time every n-th step: each event
 * pair costs a few microseconds of idle stream around the launch).  Creates HIP
 * events only.  ttkv_read_attn_timing BLOCKS until the recorded kernels have
 * finished, writes their durations in milliseconds (oldest first, at most
 * `capacity`), returns the count in *n_out and clears the samples. */
ttkv_status ttkv_time_attn(ttkv_handle h, int32_t max_samples);
/* Measurement aid: a timed call issues its attention launch(es) `repeat` times (1..64) back to back between
 * the two events -- same arguments, the same partials written again -- and its sample is the duration
 * divided by `repeat`, so that the event pair's own cost (a few microseconds per sample) is spread over
 * several launches.  1 restores the single launch.  Calls that are not timed are unaffected. */
ttkv_status ttkv_time_attn_repeat(ttkv_handle h, int32_t repeat);
/* Measurement aid: enqueue a load-only kernel that streams `bytes` (rounded down to a
 * multiple of 64 KiB) of [device] memory at `src` with the attention kernels' access
 * pattern (128-bit loads, eight in flight per lane, four wave64 per workgroup).  Timed by
 * the caller, it gives the read rate the memory system delivers to such a kernel, the
 * practical ceiling beside the nominal HBM peak.  sink: [device] 4 writable bytes. */
ttkv_status ttkv_stream_read(ttkv_handle h, const void *src, size_t bytes, void *sink, void *stream);
ttkv_status ttkv_read_attn_timing(ttkv_handle h, float *ms, int32_t capacity, int32_t *n_out);


/* One stream operation of an attention call, in the order the host issues it. */
enum {
  TTKV_OP_COPY = 0,   /* hipMemcpyAsync of `bytes` host-tier bytes (fetch number `fetch`) into staging slot `slot` */
  TTKV_OP_ATTEND = 1, /* attention launch: on slot `slot` for fetch `fetch`, or (fetch -1) on the tiers read in place */
  TTKV_OP_RECORD = 2, /* hipEventRecord(event) on the stream */
  TTKV_OP_WAIT = 3,   /* hipStreamWaitEvent(stream, event): waits for the event's latest record issued before it */
  TTKV_OP_MERGE = 4   /* merge launch */
};
typedef struct ttkv_chain_op {
  int32_t kind;   /* TTKV_OP_* */
  int32_t stream; /* 0 = compute, 1 = copy */
  int32_t event;  /* RECORD / WAIT: 0 = fence, 1 + s = ready[s], 1 + TTKV_MAX_SLOTS + s = freed[s]; else -1 */
  int32_t slot, fetch;
  uint64_t bytes;
} ttkv_chain_op;

/* The stream operations ttkv_decode_attn would issue for this cache state with these selection lists and
 * n_slots (Sec. 4.3, Alg. 1 "AsyncPrefetch": copy i + 1 runs while attention reads copy i), recorded instead of
 * executed: the same issuing code runs against a recorder, nothing is enqueued, no device is touched, no
 * pointer of the cache is dereferenced except its [host] arrays.  same_stream != 0: as with copy == compute.
 * ops [host] receives at most `capacity` operations; *n_out the number issued (may exceed capacity). */
ttkv_status ttkv_staged_schedule(ttkv_handle h, const ttkv_cache *c, const int32_t *sel_blocks, const int32_t *sel_count,
                                 int32_t sel_stride, int32_t n_slots, int32_t same_stream, ttkv_chain_op *ops,
                                 int32_t capacity, int32_t *n_out);

#ifdef __cplusplus
}
#endif
#endif /* TTKV_BENCH_H */
