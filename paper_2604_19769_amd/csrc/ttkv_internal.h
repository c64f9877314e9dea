// Internal declarations shared by the translation units of libttkv (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include <vector>

#include "ttkv.h"
#include "ttkv_bench.h"

namespace ttkv {

// ---------------------------------------------------------------- layout
// Per token-head byte counts of one format (K or V alone).
struct FmtBytes {
  int code, meta;
};
inline FmtBytes fmt_bytes(int fmt) {
  switch (fmt) {
    case TTKV_F16:
    case TTKV_BF16: return {256, 0};
    case TTKV_I8_SYM_G32: return {128, 8};
    case TTKV_I4_ASYM_G64:
    case TTKV_I4_ASYM_G64_T32: return {64, 8};
    case TTKV_I4_ASYM_T128: return {64, 4};   // 128 tokens x 4 B = 128 channels x fp16 {scale, zero}
    default: return {0, 0};
  }
}

// Byte geometry of one block record of a tier (see the header's "Block record").
struct Layout {
  int32_t bt;          // tokens per record
  int32_t kc, km, vc, vm;
  int32_t k_meta_off;  // offsets inside one head part
  int32_t v_off, v_meta_off;
  int32_t head_bytes;
  int64_t rec_bytes;
};
inline Layout make_layout(const ttkv_tier &t, int n_kv_heads) {
  Layout L{};
  FmtBytes k = fmt_bytes(t.k_fmt), v = fmt_bytes(t.v_fmt);
  L.bt = t.block_tokens;
  L.kc = k.code; L.km = k.meta; L.vc = v.code; L.vm = v.meta;
  L.k_meta_off = L.bt * L.kc;
  L.v_off = L.k_meta_off + L.bt * L.km;
  L.v_meta_off = L.v_off + L.bt * L.vc;
  L.head_bytes = L.v_meta_off + L.bt * L.vm;
  L.rec_bytes = (int64_t)L.head_bytes * n_kv_heads;
  return L;
}

// What a kernel needs to find a token of a tier (or of a staging slot that holds
// a few consecutive records of it).
struct TierView {
  uint8_t *base;          // record pool (device) or staging slot
  const int32_t *table;   // device block table or nullptr
  int64_t rec_bytes;
  int32_t head_bytes, k_meta_off, v_off, v_meta_off;
  int32_t bt, ring_blocks;
  int32_t k_fmt, v_fmt;
  int32_t in_host;        // the records are pinned host memory, read over PCIe
};

// Per-launch sequence table, passed by value in the kernel arguments so that no
// host->device copy is needed per step.
struct SeqTable {
  int32_t n_seq;
  int32_t seq_id[TTKV_MAX_BATCH];       // sequence (batch index) of entry j
  int32_t rec_base[TTKV_MAX_BATCH];     // record index of ring block 0 when there is no block table
  int32_t first_tok[TTKV_MAX_BATCH];    // ring token index of the entry's first token (multiple of 64)
  int32_t len[TTKV_MAX_BATCH];          // tokens
  int32_t item_start[TTKV_MAX_BATCH + 1];  // prefix sum of work items (chunks) per entry
  int32_t part_base[TTKV_MAX_BATCH];    // first partial index this launch writes for the entry
};

// ---------------------------------------------------------------- the split-K plan of one attention call
// One run of consecutive tokens of one (tier, sequence) attended by the fused
// kernel in place: a device tier, a host tier read over PCIe by the kernel itself,
// or a run of selected blocks.
struct Run {
  int tier, b;
  int32_t rec_base, first_tok, len;
  bool no_table;
  bool selected;   // blocks named by the device-side selection (rec_base: index of the first id, first_tok: newest block
                   // id; len: their number for a host tier, their tokens for a tier in HBM)
  int part_base, n_chunks;
};
// Selection left on the device by the top-k kernel: ids [batch][stride], min(k, live blocks) of them per sequence.
struct DevSel {
  const int32_t *ids;
  int32_t k, stride;
};
// One staged copy: consecutive pool records of a host tier brought into a slot.
struct Fetch {
  int tier, b;
  int64_t rec;     // first pool record
  int nrec;        // consecutive records in this copy
  int ntok;        // live tokens covered
  int part_base;
  int chunk;
};
// Lives in the handle and is rebuilt by every call: the vectors keep their storage, so a call allocates host
// memory only when its plan is larger than any before it (ttkv_create reserves TTKV_PLAN_RESERVE entries).
#define TTKV_PLAN_RESERVE 4096
// What the search for the split-K item size settled on, kept while the cache keeps its shape.
struct SplitMemo {
  bool valid;
  uint32_t sig;      // tiers, formats, head counts, batch
  int n_runs;
  bool sel;          // the last tier was a device-side selection
  int step;          // index into the table of rounds
  int64_t bytes;     // bytes of one pass over one KV head when it was chosen
};
struct Plan {
  SplitMemo memo;
  std::vector<Run> runs;
  std::vector<Fetch> fetch;
  std::vector<const Run *> order;   // launch order of `runs`
  int chunk[TTKV_MAX_TIERS];
  bool even[TTKV_MAX_TIERS];   // the tier's runs are cut into items of equal size each (chunk[] is then the size aimed at)
  int parts[TTKV_MAX_BATCH];
  int max_parts;
  size_t slot_bytes;
  ttkv_status status;
};

// ---------------------------------------------------------------- handle
struct Handle {
  Plan plan;
  int device;
  bool have_events;
  hipEvent_t ready[TTKV_MAX_SLOTS];
  hipEvent_t freed[TTKV_MAX_SLOTS];
  hipEvent_t fence;     // orders the copy stream behind earlier compute work
  hipEvent_t fence2;    // orders device->host eviction copies behind the quantize kernel
  ttkv_stats stats;
  // optional per-call timing of one device tier's partial kernel
  bool time_on;
  int target_items;     // split-K granularity of the fused launch
  bool check_tables;    // every call checks every host block-table entry against pool_blocks
  int time_max, time_n;
  hipEvent_t *time_ev;  // 2 * time_max events
  int32_t *time_reps;   // launches between the events of each sample
  int time_repeat;      // how often a timed call issues its attention launch(es)
};

#define TTKV_HIP(h, expr)                                   \
  do {                                                      \
    hipError_t e_ = (expr);                                 \
    if (e_ != hipSuccess) {                                 \
      if (h) (h)->stats.last_hip_error = (int32_t)e_;       \
      return TTKV_ERR_HIP;                                  \
    }                                                       \
  } while (0)

inline bool is_fp(int f) { return f == TTKV_F16 || f == TTKV_BF16; }
inline bool is_tier_fmt(int f) {
  return (f >= TTKV_F16 && f <= TTKV_I4_ASYM_G64) || f == TTKV_I4_ASYM_T128 || f == TTKV_I4_ASYM_G64_T32;
}

ttkv_status validate_cache(const ttkv_cache *c, bool check_tables = true);

// ---------------------------------------------------------------- launchers (defined in the .hip files)
struct ConvSource {
  // flat source [n_seq][Hkv][n][128] indexed by launch entry, or a tier view
  const void *k_flat, *v_flat;
  int32_t flat_fmt;
  int32_t from_tier;    // 0: flat source, 1: read rows of `src`
  TierView src;
  int32_t src_first_tok[TTKV_MAX_BATCH];  // ring token index of the first row to read, per entry
  int32_t src_rec_base[TTKV_MAX_BATCH];
};
struct ConvArgs {
  ConvSource s;
  TierView dst;
  int32_t n_seq, Hkv, n_tokens;            // rows per entry and head
  int32_t seq_id[TTKV_MAX_BATCH];
  int32_t dst_first_tok[TTKV_MAX_BATCH];   // ring token index where the first row lands
  int32_t dst_rec_base[TTKV_MAX_BATCH];
  int32_t which0;                          // first of {0: K, 1: V} the row kernel converts (1: V only)
  int32_t n_via;                           // intermediate formats a value passes through first
  int32_t via_k[TTKV_MAX_TIERS], via_v[TTKV_MAX_TIERS];
  // summaries of the destination tier (nullable)
  float *k_sum;
  uint16_t *k_summary;
  const int32_t *sum_table;                // device block table of the destination pool for the summaries
  int32_t sum_rec_base[TTKV_MAX_BATCH];
  int32_t sum_ring_blocks;
  float inv_bt;
};
hipError_t launch_convert(const ConvArgs &a, hipStream_t s, int *n_kernels);
hipError_t launch_summary(const ConvArgs &a, hipStream_t s, int *n_kernels);

// One launch of the fused attention kernel: up to TTKV_MAX_ENTRIES runs of tokens,
// each belonging to one (tier, sequence), all passed by value (no per-step upload).
#define TTKV_MAX_ENTRIES 120
struct Entry {
  int32_t tier_seq;     // bit 24: ignore the block table (rec_base is a pool record); bits 16-23 tier; low 16 sequence
                        // bit 25: the run is made of blocks named by the device-side selection: rec_base = index of
                        // its first id in FusedArgs::sel_ids, first_tok = id of the tier's newest live block, len =
                        // the number of blocks (tier cut into fixed items) or their tokens (equal items)
  int32_t rec_base;     // record of ring block 0 (no table) or of the run's first block
  int32_t first_tok;    // ring token index of the run's first token (multiple of 64)
  int32_t len;          // tokens
  int32_t item_start;   // first work item (chunk) of the run in this launch
  int32_t part_base;    // first partial index of the run
};
// A run of `len` tokens cut into n items of equal size, a multiple of 64 tokens (the last item may be shorter).
// The host plans with it and the kernels derive an item's size from the run's length and item count with it.
__host__ __device__ inline int even_chunk(int len, int n) { return ((len + n - 1) / n + 63) / 64 * 64; }
struct FusedArgs {
  TierView tv[TTKV_MAX_TIERS];
  int32_t chunk[TTKV_MAX_TIERS];   // tokens per item of the tier's runs; 0: every run in items of equal size (even_chunk)
  Entry e[TTKV_MAX_ENTRIES];
  int32_t n_entries, n_items;
  const void *q;
  int32_t q_fmt;
  float *pm, *pl, *pacc;
  int32_t part_stride;
  int32_t Hq, Hkv;
  float scale;
  int32_t mfma_heads;   // set by the matrix-core launcher: query heads one workgroup serves
  const int32_t *sel_ids;                    // device: block ids (Eq. 1) chosen by the top-k kernel, for runs with bit 25
  int32_t sel_last_ntok[TTKV_MAX_BATCH];     // live tokens in the newest block of the selected tier, per sequence
};
static_assert(sizeof(FusedArgs) <= 4096, "kernel arguments are passed by value");
hipError_t launch_attn(const FusedArgs &a, hipStream_t s, int *n_kernels, int *n_mfma);
bool attn_supported(int k_fmt, int v_fmt, int G);
int attn_group_width(int Gtot);
// Grouped-query kernel on the matrix cores: all query heads of a KV head in one pass over its bytes.
bool attn_mfma_fits(int k_fmt, int v_fmt, int G);
bool attn_mfma_pays(int G, bool has_mixed_or_t128);
bool attn_mfma_eligible(const FusedArgs &a);
hipError_t launch_attn_mfma(const FusedArgs &a, hipStream_t s);

struct MergeArgs {
  const float *m, *l, *acc;
  int32_t n_parts, part_stride, rows;
  const int32_t *n_parts_row;   // device, nullable
  int32_t rows_per_seq;         // > 0: use cnt[row / rows_per_seq]
  int32_t cnt[TTKV_MAX_BATCH];
  float *out, *lse;
  // The step's new token (k_new nullable; then rows = batch x Hq): its term (score q.k_new, weight 1, value
  // v_new) joins the merge, and its row is stored at the tail of tier 0, whose fp format it has.
  const void *q, *k_new, *v_new;   // q [batch][Hq][128]; k_new, v_new [batch][Hkv][128]
  int32_t q_fmt, new_fmt, Hq, Hkv;
  float scale;
  TierView dst;                       // tier 0
  int32_t new_tok[TTKV_MAX_BATCH];    // ring token index where the sequence's row lands
};
hipError_t launch_merge(const MergeArgs &a, hipStream_t s);

struct SelectArgs {
  const void *q;
  int32_t q_fmt;
  const uint16_t *k_summary;
  const int32_t *table;          // device block table of the last tier or nullptr
  int32_t ring_blocks, Hq, Hkv, k, sel_stride, n_seq;
  int32_t rec_base[TTKV_MAX_BATCH];
  int32_t first_block[TTKV_MAX_BATCH];   // ring index of the oldest live block
  int64_t first_block_id[TTKV_MAX_BATCH];  // its block id (Eq. 1)
  int32_t n_blocks[TTKV_MAX_BATCH];
  int32_t max_blocks;
  float *scores;                 // [n_seq][max_blocks]
  int32_t *sel_out;              // [n_seq][sel_stride + 1]: count then ids relative to first_block_id
};
hipError_t launch_select(const SelectArgs &a, hipStream_t s);

// Load-only kernel over `bytes` (rounded down to 64 KiB) of device memory; sink: 4 writable bytes.
hipError_t launch_stream_read(const void *src, int64_t bytes, uint32_t *sink, hipStream_t s);

}  // namespace ttkv
