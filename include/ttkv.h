/*
 * libttkv -- tiered decode attention for gfx950 (MI355X), C ABI.
 *
 * The data-parallel hot path of TTKV ("Temporal-Tiered KV Cache"): block-wise
 * streaming decode attention over a KV cache split into temporal tiers.  Tier 0
 * holds the most recent tokens in fp16/bf16 in HBM (Sec. 4.1, fast tier); older
 * tiers hold low-bit codes with per-group fp16 scale/zero (Sec. 4.2,
 * differential quantization) in HBM or in pinned host DRAM, organised in blocks
 * of B_blk tokens (Sec. 4.1, block-wise organisation) that are fetched,
 * decompressed in registers and attended block by block while later blocks are
 * still in flight (Sec. 4.3, Alg. 1).
 *
 * Conventions
 *   - Every pointer is tagged [host], [pinned] (page-locked host) or [device].
 *   - All memory is allocated and owned by the caller.  The library never
 *     allocates or frees device memory and never synchronises the device,
 *     except where a call says it blocks.
 *   - Streams are passed as void* holding a hipStream_t (NULL = default stream).
 *   - Every call validates its arguments on the host and returns a status
 *     before enqueuing anything; on error nothing was enqueued and no tier
 *     state changed.  There are no exceptions and no aborts.
 *   - head_dim is fixed to 128.  batch <= TTKV_MAX_BATCH.
 *
 * Block record (the unit of storage, eviction and DMA; Sec. 4.1 "blocks B_j")
 *   A tier's `data` is a pool of `pool_blocks` records of ttkv_record_bytes()
 *   bytes.  One record holds block_tokens tokens of every KV head:
 *     record = [n_kv_heads] x head part
 *     head part = K codes [block_tokens][kc] | K meta [block_tokens][km]
 *               | V codes [block_tokens][vc] | V meta [block_tokens][vm]
 *   per token-head:  F16/BF16: codes = 128 x 2 B, no meta
 *                    I8_SYM_G32: codes = 128 x int8, meta = 4 x fp16 scale
 *                    I4_ASYM_G64: codes = 64 B (element 2i low nibble, 2i+1 high
 *                                 nibble of byte i), meta = fp16 {s0, z0, s1, z1}
 *                    I4_ASYM_G64_T32 (V): Q_4bit exactly as I4_ASYM_G64 (same codes, same meta rows),
 *                                 but the codes of 32 consecutive tokens (aligned to multiples of 32
 *                                 in the block) are stored as one 2 KiB group in the operand order
 *                                 of the matrix cores: the group's 16-byte piece p = 64 hh + 16 kg + c
 *                                 (hh 0..1, kg 0..3, c 0..15) holds four 32-bit words w = 0..3; word w
 *                                 carries channel 16 (4 hh + w) + c of eight tokens, nibble j (bits
 *                                 4j..4j+3) = token {0, 2, 16, 18, 1, 3, 17, 19}[j] + 4 kg of the group
 *                    I4_ASYM_T128 (K): codes as I4_ASYM_G64; km = 4: the meta rows of
 *                                 tokens [128 g, 128 g + 128) of a block together hold
 *                                 fp16 {scale, zero} x 128 channels of token group g
 *   Sequence b's token with lifetime ordinal o (o = start[b] + i for its i-th
 *   live token) sits in ring block r = (o / block_tokens) % ring_blocks at row
 *   o % block_tokens of record  block_table ? block_table[b*ring_blocks + r]
 *                                           : b*ring_blocks + r.
 *   o / block_tokens is the block id of Eq. (1).
 */
#ifndef TTKV_H
#define TTKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TTKV_MAX_TIERS 4
#define TTKV_MAX_BATCH 64
#define TTKV_MAX_KV_HEADS 1023   /* n_kv_heads beyond this: TTKV_ERR_UNSUPPORTED */
#define TTKV_HEAD_DIM 128
#define TTKV_MAX_SLOTS 16
#define TTKV_NOALLOC_SCRATCH_BYTES (16u << 20) /* split partials of ttkv_decode_attn_noalloc, per GPU */

typedef enum {
  TTKV_OK = 0,
  TTKV_ERR_INVALID_ARG = 1, /* NULL / out-of-range / inconsistent argument */
  TTKV_ERR_CAPACITY = 2,    /* a tier ring would overflow, or too few tokens to evict */
  TTKV_ERR_UNSUPPORTED = 3, /* head_dim != 128, format combination without a kernel */
  TTKV_ERR_WORKSPACE = 4,   /* workspace smaller than ttkv_workspace_bytes() */
  TTKV_ERR_HIP = 5          /* a HIP launch / copy / event call failed; code in ttkv_stats */
} ttkv_status;

typedef enum {
  TTKV_F16 = 0,
  TTKV_BF16 = 1,
  TTKV_I8_SYM_G32 = 2,  /* Q_8bit: symmetric int8, group 32 along head_dim, fp16 scale */
  TTKV_I4_ASYM_G64 = 3, /* Q_4bit: asymmetric int4, group 64, fp16 scale + zero */
  TTKV_F32 = 4,         /* source format of ttkv_quantize_append only */
  TTKV_I4_ASYM_G64_T32 = 6, /* values only: Q_4bit (Sec. 4.2) with the codes of every 32 tokens stored channel-major
                           ("Block record" above), so that the grouped-query kernel feeds them to the matrix cores
                           without transposing them: the decompressed values are those of I4_ASYM_G64 bit for bit.
                           For caches with >= 2 query heads per KV head (UNSUPPORTED otherwise); K of the tier:
                           I8_SYM_G32 or I4_ASYM_G64; tokens arrive in whole aligned groups of 32 (eviction of whole
                           blocks, appends of multiples of 32); last tier of a chain only. */
  TTKV_I4_ASYM_T128 = 5 /* keys only: asymmetric int4 where a group is one channel over 128 consecutive
                           tokens (keys carry the larger dynamic range, Sec. 3 / 4.2, in a few channels:
                           such a channel then sets no scale but its own).  V of the tier: I4_ASYM_G64.
                           block_tokens a multiple of 128; tokens arrive in whole aligned groups (by
                           eviction of whole blocks, or appends of multiples of 128); nothing passes
                           THROUGH this format: it belongs to the last tier of a chain. */
} ttkv_fmt;

typedef enum { TTKV_MEM_DEVICE = 0, TTKV_MEM_HOST_PINNED = 1 } ttkv_mem;

/* One temporal tier.  Tier 0 is the newest (the paper's fast tier). */
typedef struct ttkv_tier {
  int32_t k_fmt, v_fmt;      /* ttkv_fmt of keys / values (set separately: K 8-bit + V 4-bit is Sec. 4.2's choice) */
  int32_t mem;               /* ttkv_mem: where `data` lives */
  int32_t block_tokens;      /* B_blk: tokens per record; multiple of 64 */
  int64_t capacity_tokens;   /* eviction threshold per sequence (L_fast for tier 0): a tier is due when len >= capacity */
  int64_t ring_blocks;       /* records per sequence ring; ring_blocks*block_tokens >= the largest len ever held */
  int64_t pool_blocks;       /* records in `data` */
  void *data;                /* [device] or [pinned] per `mem`: pool_blocks records */
  const int32_t *block_table;     /* [host] [batch][ring_blocks] record index per ring block, or NULL = b*ring_blocks + r */
  const int32_t *block_table_dev; /* [device] copy of block_table; required when block_table != NULL and kernels address the
                                     pool: a device tier, a host tier read in place (n_slots 0) or written without a workspace */
  float *k_sum;              /* [device] fp32 [pool_blocks][n_kv_heads][128] running key sums, or NULL (no summaries) */
  void *k_summary;           /* [device] fp16 [pool_blocks][n_kv_heads][128] mean keys; required iff k_sum != NULL */
  int64_t *start;            /* [host] [batch] lifetime ordinal of the oldest live token (library updates) */
  int64_t *len;              /* [host] [batch] live tokens (library updates) */
} ttkv_tier;

typedef struct ttkv_cache {
  int32_t batch, n_q_heads, n_kv_heads, head_dim, n_tiers;
  float softmax_scale; /* multiplies q.k; 1/sqrt(head_dim) in the usual case */
  ttkv_tier tier[TTKV_MAX_TIERS];
} ttkv_cache;

typedef struct ttkv_stats {
  uint64_t h2d_bytes;       /* host-tier record bytes fetched (Sec. 5.1 item 5: host-to-GPU KV traffic) */
  uint64_t d2h_bytes;       /* bytes written to host tiers by eviction */
  uint64_t blocks_fetched;  /* host-tier records fetched */
  uint64_t kernels;         /* kernels launched */
  uint64_t demotions;       /* blocks evicted, all tiers and sequences */
  uint64_t mfma_launches;   /* attention launches served by the grouped-query matrix-core kernel */
  int32_t last_hip_error;   /* hipError_t of the last failed HIP call, 0 if none */
} ttkv_stats;

typedef struct ttkv_handle_s *ttkv_handle; /* events for the copy/compute chain + stats; one per calling thread */

/* Create / destroy a handle (host memory only; the HIP events of the copy/compute
 * chain are created on the device current at the first call that needs them). */
ttkv_status ttkv_create(ttkv_handle *out);
ttkv_status ttkv_destroy(ttkv_handle h);
void ttkv_get_stats(ttkv_handle h, ttkv_stats *out);
void ttkv_reset_stats(ttkv_handle h);
const char *ttkv_status_string(ttkv_status s); /* utility: a status code as text (no passage of the paper applies) */

/* Bytes of one block record of `tier` (all KV heads). 0 on invalid formats. */
size_t ttkv_record_bytes(const ttkv_cache *c, int32_t tier);

/* Position -> block index, Eq. (1).  pos counts the sequence's tokens from the
 * oldest live one (0) to the newest (sum of len - 1) at the time of the call.
 * Outputs: tier, block id (lifetime ordinal / block_tokens), row in the block,
 * record index in the tier's pool.  INVALID_ARG if pos is not live. */
ttkv_status ttkv_locate(const ttkv_cache *c, int32_t b, int64_t pos, int32_t *tier, int64_t *block_id,
                        int32_t *row, int64_t *record);

/* Utilities around Alg. 1's accumulation "o <- o + Attn(q, K_j, V_j)": the un-normalised partials of its terms live in
 * a caller-owned workspace until the merge.
 * [device] workspace ttkv_decode_attn needs for this cache: split partials for
 * up to max_parts parts per (sequence, query head) plus n_slots staging slots, each
 * holding the largest run of adjacent host-tier records one copy moves (up to 32 MiB or 64 records).  ttkv_tier_demote needs batch records of its
 * destination tier when that is a host tier (always covered when n_slots >= batch,
 * else use ttkv_demote_workspace_bytes). */
size_t ttkv_workspace_bytes(const ttkv_cache *c, int32_t max_parts, int32_t n_slots);
size_t ttkv_demote_workspace_bytes(const ttkv_cache *c, int32_t src_tier);
/* Parts per (sequence, query head) ttkv_decode_attn would use right now with this n_slots. */
int32_t ttkv_count_parts(ttkv_handle h, const ttkv_cache *c, const int32_t *sel_blocks, const int32_t *sel_count,
                         int32_t sel_stride, int32_t n_slots);
/* Split-K granularity (how many terms Alg. 1's sum over blocks is cut into; the result is the same up to fp32
 * rounding, Sec. 4.3): ttkv_decode_attn cuts the device-resident tiers into about
 * target_items workgroups of equal bytes, counted over all sequences and KV heads; every
 * (tier, sequence) run is cut into items of equal size (multiples of 64 tokens, 256 to 8192).
 * 0 restores the default: chosen per call from the lengths -- the number of rounds of resident
 * workgroups that suits the kernel the cache's formats and head counts select, raised in steps
 * until the items of all runs are within 10 % of each other and the last round is filled.
 * More items: better balance over 256 CUs, more partials. */
ttkv_status ttkv_set_split(ttkv_handle h, int32_t target_items);
/* Paged tiers (Eq. (1): the index maps a block to where it is stored): by default every call that takes the handle
 * checks every entry of every host block table against pool_blocks before it enqueues anything -- batch x
 * ring_blocks comparisons per table per call, which a pool of millions of pages makes longer than the step itself.
 * on = 0 switches the per-call check off for this handle: the entries are then trusted as the caller's allocator
 * wrote them (a wrong entry is an out-of-bounds access on the device); on = 1 restores it.  Everything else is
 * still validated on every call. */
ttkv_status ttkv_set_table_check(ttkv_handle h, int32_t on);

/* Append n_tokens at the tail of `tier` (Sec. 4.1 "newly generated tokens are
 * appended to the fast tier"; also the bulk loader of any device tier).
 *   seq  -1: every sequence, k_src/v_src [device] [batch][n_kv_heads][n_tokens][128];
 *        >= 0: that sequence only, k_src/v_src [device] [n_kv_heads][n_tokens][128].
 *   src_fmt F16, BF16 or F32.  An fp tier takes only its own format (plain
 *   copy); a quantized tier applies Q of Sec. 4.2.
 *   through_tiers != 0: the values first pass through the formats of tiers
 *   1..tier-1 (quantize + decompress each), i.e. arrive as eviction would have
 *   delivered them; 0: quantized directly.
 * Updates len[].  CAPACITY if a ring would overflow.  Enqueues on `stream`;
 * the sources must stay valid until it has run. */
ttkv_status ttkv_quantize_append(ttkv_handle h, ttkv_cache *c, int32_t tier, int32_t seq, const void *k_src,
                                 const void *v_src, int32_t src_fmt, int64_t n_tokens, int32_t through_tiers,
                                 void *stream);

/* The same for a host tier: quantizes into `workspace` [device]
 * (ttkv_append_host_workspace_bytes) and copies the touched rows of the touched
 * records to the pinned pool on `stream`.  workspace NULL (ws_bytes ignored): no
 * staging and no copies, the conversion kernels store into the pinned records
 * themselves, so the transfer over PCIe runs while they compute (the bulk path
 * for tiering a whole prompt, Sec. 3 "prefilling and decoding"). */
ttkv_status ttkv_quantize_append_host(ttkv_handle h, ttkv_cache *c, int32_t tier, int32_t seq, const void *k_src,
                                      const void *v_src, int32_t src_fmt, int64_t n_tokens, int32_t through_tiers,
                                      void *workspace, size_t ws_bytes, void *stream);
size_t ttkv_append_host_workspace_bytes(const ttkv_cache *c, int32_t tier, int32_t seq, int64_t n_tokens);

/* FIFO tier management (Sec. 4.1; Alg. 1 "evict & compress"): for every
 * sequence whose src_tier holds >= capacity_tokens, move its oldest block
 * (src block_tokens tokens; values as stored or decompressed) to the tail of
 * tier src_tier+1 in that tier's formats, repeating while still due, at most
 * max_blocks times per sequence (<= 0: no limit).  Host destination: quantized
 * into `workspace` [device] (ttkv_demote_workspace_bytes) on `compute`, then
 * copied device->pinned on `copy` after an event; workspace NULL: the kernels
 * store into the pinned records themselves, on `compute`, no copies.  Updates
 * start[], len[] of both tiers and the destination's key summaries.  CAPACITY
 * if a destination ring would overflow. */
ttkv_status ttkv_tier_demote(ttkv_handle h, ttkv_cache *c, int32_t src_tier, int32_t max_blocks, void *workspace,
                             size_t ws_bytes, void *compute, void *copy);

/* One decode step of streaming attention (Alg. 1, Sec. 4.3) for every
 * sequence: partial (max, sum-exp, weighted V) over each part of every tier,
 * merged by log-sum-exp.
 *   q    [device] [batch][n_q_heads][128], q_fmt F16 or BF16 (a BF16 tier needs BF16
 *        queries; for the other tiers |q| must stay below 65504)
 *   out  [device] [batch][n_q_heads][128] fp32;  lse [device] [batch][n_q_heads] fp32 or NULL
 *   sel_blocks [host] [batch][sel_stride] block ids (Eq. 1) of the LAST tier to
 *        attend, ascending, sel_count [host] [batch] how many; both NULL = every
 *        live block (dense).
 *   n_slots == 0: host tiers are read in place by the attention kernel (loads
 *        over PCIe stay in flight while other waves compute: the prefetch/compute
 *        overlap of Sec. 4.3 inside one launch); `copy` is not used.
 *   n_slots >= 1 (<= TTKV_MAX_SLOTS): host-tier records are copied with hipMemcpyAsync
 *        on `copy` into n_slots staging slots of `workspace` (adjacent records of a
 *        dense tier merged up to 32 MiB per copy: every copy carries a fixed cost of tens of microseconds), event-chained so that copy i+1 runs
 *        while `compute` attends copy i (both streams equal: nothing overlaps).  A
 *        slot is reused only after the kernel that read it has finished; enough slots
 *        for a whole step avoid those waits.
 * Returns after enqueuing; `out` is complete when `compute` has drained. */
ttkv_status ttkv_decode_attn(ttkv_handle h, const ttkv_cache *c, const void *q, int32_t q_fmt, float *out,
                             float *lse, const int32_t *sel_blocks, const int32_t *sel_count, int32_t sel_stride,
                             void *workspace, size_t ws_bytes, int32_t n_slots, void *compute, void *copy);

/* ttkv_decode_attn for callers that cannot allocate or hand over device memory for the call: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results as ttkv_decode_attn with n_slots = 0 (host tiers read in place) and both streams = `stream`, but the
 * split partials live in an array of TTKV_NOALLOC_SCRATCH_BYTES (16 MiB) that is part of the library's device
 * code: each GPU the library runs on holds its own copy from the first call on it until the process ends.  The
 * call allocates nothing on the device and calls no allocating routine.  WORKSPACE if the partials this cache
 * needs right now, batch x n_q_heads x ttkv_count_parts(.., n_slots 0) x 520 bytes, exceed the array; nothing
 * is enqueued then.  All calls on one GPU share that GPU's array: two calls whose kernels may overlap on one
 * GPU (different streams, different threads) race; calls on one stream are ordered and safe.  Nothing in the
 * array needs clearing between calls (every part the merge reads is written by the same call first). */
ttkv_status ttkv_decode_attn_noalloc(ttkv_handle h, const ttkv_cache *c, const void *q, int32_t q_fmt, float *out,
                                     float *lse, const int32_t *sel_blocks, const int32_t *sel_count,
                                     int32_t sel_stride, void *stream);

/* The "append" and "attend" lines of Alg. 1 for one decode step in one call: the step's new token
 * (k_new, v_new [device] [batch][n_kv_heads][128], new_fmt F16 or BF16) is appended to tier 0 of every
 * sequence and attended together with everything cached; len[] of tier 0 grows by one.  Same result and
 * same arguments otherwise as ttkv_quantize_append(tier 0, seq -1, n_tokens 1) followed by
 * ttkv_decode_attn.  When tier 0 is an fp16/bf16 device tier (new_fmt must be its format, else
 * UNSUPPORTED) the step takes one launch fewer: the attention kernels run over the tokens already
 * cached, and the merge kernel adds the new token's own term (score q.k_new, weight 1, value v_new)
 * and stores its row.  Any other first tier: the two calls, one after the other.  CAPACITY if tier
 * 0's ring has no room; nothing is enqueued and no length changes when a status other than OK or
 * HIP is returned.  Eviction (ttkv_tier_demote) stays the caller's next call. */
ttkv_status ttkv_decode_step(ttkv_handle h, ttkv_cache *c, const void *q, int32_t q_fmt, const void *k_new,
                             const void *v_new, int32_t new_fmt, float *out, float *lse, const int32_t *sel_blocks,
                             const int32_t *sel_count, int32_t sel_stride, void *workspace, size_t ws_bytes,
                             int32_t n_slots, void *compute, void *copy);

/* "Identify", "TopK" and the attention of Alg. 1 in one call with no host round trip: the blocks of the LAST
 * tier are scored against its mean keys and the k best per sequence chosen as by ttkv_select_blocks, the ids
 * stay on the device, and the attention kernels look them up themselves (the host only needs their number,
 * min(k, live blocks)); every other tier is attended whole.  The last tier is read in place (no staging
 * slots).  k_new, v_new as in ttkv_decode_step or both NULL (attend only); with a token, tier 0 must be an
 * fp16/bf16 device tier of format new_fmt (UNSUPPORTED otherwise).
 *   sel_scratch [device] as for ttkv_select_blocks; it holds the ids until the call's kernels have run.
 *   sel_blocks_out [pinned] [batch][sel_stride], sel_count_out [pinned] [batch], or both NULL: copies of the
 *   chosen ids and counts for the caller's information, enqueued behind the attention; valid once `stream`
 *   has drained.
 * Same results as ttkv_select_blocks + ttkv_decode_step with its lists.  Enqueues on `stream` only and does
 * not block. */
ttkv_status ttkv_decode_step_topk(ttkv_handle h, ttkv_cache *c, const void *q, int32_t q_fmt, const void *k_new,
                                  const void *v_new, int32_t new_fmt, float *out, float *lse, int32_t k,
                                  int32_t *sel_blocks_out, int32_t *sel_count_out, int32_t sel_stride,
                                  void *sel_scratch, size_t sel_scratch_bytes, void *workspace, size_t ws_bytes,
                                  void *stream);

/* Log-sum-exp merge of n_parts partials per row (the "+" of Alg. 1):
 *   m, l [device] [rows][part_stride] fp32;  acc [device] [rows][part_stride][128] fp32;
 *   n_parts_row [device] [rows] int32 parts to merge per row, or NULL = n_parts for all.
 *   out [device] [rows][128] fp32 = sum_p acc_p e^(m_p-m*) / sum_p l_p e^(m_p-m*);
 *   lse [device] [rows] = m* + ln(sum) or NULL.  Parts with m = -inf count as empty;
 *   a row with no non-empty part gives out = 0, lse = -inf. */
ttkv_status ttkv_merge_partials(ttkv_handle h, const float *m, const float *l, const float *acc, int32_t n_parts,
                                int32_t part_stride, const int32_t *n_parts_row, int32_t rows, float *out,
                                float *lse, void *stream);

/* Block identification (Alg. 1, the identification step): phi(q, B_j) = sum over query heads of
 * q_h . mean-key_j for every live block of the LAST tier (needs k_summary), then
 * the k best per sequence, ties to the lower block id.  sel_blocks [pinned]
 * [batch][sel_stride] block ids ascending, sel_count [pinned] [batch];
 * scratch [device] >= batch*(max live blocks)*8 + batch*(sel_stride+1)*4 bytes.
 * BLOCKS until the ids are on the host. */
ttkv_status ttkv_select_blocks(ttkv_handle h, const ttkv_cache *c, const void *q, int32_t q_fmt, int32_t k,
                               int32_t *sel_blocks, int32_t *sel_count, int32_t sel_stride, void *scratch,
                               size_t scratch_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TTKV_H */
