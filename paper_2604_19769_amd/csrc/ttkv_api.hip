// Host side of libttkv: argument validation, tier bookkeeping (Sec. 4.1), the
// split-K plan, and the copy/compute event chain of streaming attention
// (Sec. 4.3, Alg. 1).  No device memory is allocated here.
#include "ttkv_internal.h"

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

using namespace ttkv;

namespace ttkv {

ttkv_status validate_cache(const ttkv_cache *c, bool check_tables) {
  if (!c) return TTKV_ERR_INVALID_ARG;
  if (c->head_dim != TTKV_HEAD_DIM) return TTKV_ERR_UNSUPPORTED;
  if (c->batch < 1 || c->batch > TTKV_MAX_BATCH) return TTKV_ERR_INVALID_ARG;
  if (c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads || c->n_q_heads % c->n_kv_heads) return TTKV_ERR_INVALID_ARG;
  if (c->n_kv_heads > TTKV_MAX_KV_HEADS) return TTKV_ERR_UNSUPPORTED;   // (sequence, KV head) pairs index a launch grid's third dimension
  if (c->n_tiers < 1 || c->n_tiers > TTKV_MAX_TIERS) return TTKV_ERR_INVALID_ARG;
  if (!(c->softmax_scale > 0.0f)) return TTKV_ERR_INVALID_ARG;
  for (int t = 0; t < c->n_tiers; ++t) {
    const ttkv_tier &T = c->tier[t];
    if (!is_tier_fmt(T.k_fmt) || !is_tier_fmt(T.v_fmt)) return TTKV_ERR_INVALID_ARG;
    if (!attn_supported(T.k_fmt, T.v_fmt, c->n_q_heads / c->n_kv_heads)) return TTKV_ERR_UNSUPPORTED;
    if (T.mem != TTKV_MEM_DEVICE && T.mem != TTKV_MEM_HOST_PINNED) return TTKV_ERR_INVALID_ARG;
    if (T.block_tokens < 64 || T.block_tokens % 64) return TTKV_ERR_INVALID_ARG;
    if (T.v_fmt == TTKV_I4_ASYM_T128 || T.k_fmt == TTKV_I4_ASYM_G64_T32) return TTKV_ERR_UNSUPPORTED;   // a key / a value format
    if (T.v_fmt == TTKV_I4_ASYM_G64_T32) {
      if (t == 0 || t + 1 < c->n_tiers) return TTKV_ERR_UNSUPPORTED;          // whole groups arrive; nothing passes through
      for (int b = 0; b < c->batch; ++b)
        if (T.len[b] % 32) return TTKV_ERR_INVALID_ARG;
    }
    if (T.k_fmt == TTKV_I4_ASYM_T128) {
      if (T.block_tokens % 128) return TTKV_ERR_INVALID_ARG;
      if (t == 0 || t + 1 < c->n_tiers) return TTKV_ERR_UNSUPPORTED;          // whole groups arrive; nothing passes through
      for (int b = 0; b < c->batch; ++b)
        if (T.len[b] % 128) return TTKV_ERR_INVALID_ARG;
    }
    if (T.ring_blocks < 1 || T.pool_blocks < 1 || !T.data || !T.start || !T.len) return TTKV_ERR_INVALID_ARG;
    if (T.ring_blocks * (int64_t)T.block_tokens >= (int64_t)1 << 30) return TTKV_ERR_INVALID_ARG;
    if (T.pool_blocks >= (int64_t)1 << 31) return TTKV_ERR_INVALID_ARG;
    if (T.capacity_tokens < T.block_tokens) return TTKV_ERR_INVALID_ARG;
    if (!T.block_table && T.pool_blocks < (int64_t)c->batch * T.ring_blocks) return TTKV_ERR_INVALID_ARG;
    if (T.block_table && (T.mem == TTKV_MEM_DEVICE || T.k_sum) && !T.block_table_dev) return TTKV_ERR_INVALID_ARG;
    if (T.k_sum && !T.k_summary) return TTKV_ERR_INVALID_ARG;
    if (T.block_table && check_tables)   // O(batch x ring_blocks) per call: the caller may take the responsibility (ttkv_set_table_check)
      for (int64_t i = 0; i < (int64_t)c->batch * T.ring_blocks; ++i)
        if (T.block_table[i] < 0 || T.block_table[i] >= T.pool_blocks) return TTKV_ERR_INVALID_ARG;
    for (int b = 0; b < c->batch; ++b) {
      if (T.len[b] < 0 || T.len[b] > T.ring_blocks * T.block_tokens) return TTKV_ERR_INVALID_ARG;
      if (T.start[b] < 0 || T.start[b] % T.block_tokens) return TTKV_ERR_INVALID_ARG;
    }
  }
  return TTKV_OK;
}

}  // namespace ttkv

namespace {

TierView make_view(const ttkv_tier &T, const Layout &L) {
  TierView v{};
  v.base = (uint8_t *)T.data;
  v.table = T.block_table_dev;
  v.rec_bytes = L.rec_bytes;
  v.head_bytes = L.head_bytes;
  v.k_meta_off = L.k_meta_off;
  v.v_off = L.v_off;
  v.v_meta_off = L.v_meta_off;
  v.bt = L.bt;
  v.ring_blocks = (int32_t)T.ring_blocks;
  v.k_fmt = T.k_fmt;
  v.v_fmt = T.v_fmt;
  v.in_host = T.mem == TTKV_MEM_HOST_PINNED;
  return v;
}

// A staging area holding `nrec` consecutive records in the tier's layout.
TierView make_slot_view(const ttkv_tier &T, const Layout &L, void *slot, int nrec) {
  TierView v = make_view(T, L);
  v.base = (uint8_t *)slot;
  v.table = nullptr;
  v.ring_blocks = nrec;
  v.in_host = 0;
  return v;
}

inline int64_t ring_tokens(const ttkv_tier &T) { return T.ring_blocks * (int64_t)T.block_tokens; }
inline int64_t record_of(const ttkv_tier &T, int b, int64_t ring_block) {
  return T.block_table ? (int64_t)T.block_table[(int64_t)b * T.ring_blocks + ring_block] : (int64_t)b * T.ring_blocks + ring_block;
}
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Consecutive pool records merged into one copy when adjacent (dense, unpaged tiers): up to
// TTKV_COPY_GRANULE_MIB per copy.  Every hipMemcpyAsync carries a fixed cost of some tens of
// microseconds (set-up, its event hop to the compute stream), so the copies want to be few and
// large; yet more than one, so that attention on copy i runs under copy i + 1.
#ifndef TTKV_COPY_GRANULE_MIB
#define TTKV_COPY_GRANULE_MIB 32
#endif
int copy_granule(int64_t rec_bytes) {
  int64_t g = ((int64_t)TTKV_COPY_GRANULE_MIB << 20) / rec_bytes;
  return (int)std::max<int64_t>(1, std::min<int64_t>(64, g));
}

// Default split-K granularity, in workgroups resident at once on 256 CUs: 2.5 rounds of 4 per CU for the vector
// kernel (flat between 1 and 3 rounds, measured), exactly one round of 3 per CU for the grouped-query matrix-core
// kernel (int4: 5.1 TB/s against 4.4-4.7 with two rounds; the other formats are indifferent).
int default_items(const ttkv_cache *c) {
  const int G = c->n_q_heads / c->n_kv_heads;
  bool special = false;   // K 8-bit / V 4-bit or keys grouped over tokens
  for (int t = 0; t < c->n_tiers; ++t) {
    const ttkv_tier &T = c->tier[t];
    if (!attn_mfma_fits(T.k_fmt, T.v_fmt, G)) return 2560;
    special |= T.k_fmt == TTKV_I4_ASYM_T128 || (T.k_fmt == TTKV_I8_SYM_G32 && T.v_fmt != T.k_fmt);
  }
  if (!attn_mfma_pays(G, special)) return 2560;
  for (int t = 0; t < c->n_tiers; ++t)
    if (G > 8 && (c->tier[t].k_fmt == TTKV_I4_ASYM_G64 || c->tier[t].k_fmt == TTKV_I8_SYM_G32))
      return 512;   // the 16-head cases run 2 workgroups per CU (64 q / 4 kv heads, int8 keys: 6.06 against 5.8 TB/s with 768)
  return 768;
}

inline int per_token_bytes(const ttkv_tier &U) {
  return fmt_bytes(U.k_fmt).code + fmt_bytes(U.k_fmt).meta + fmt_bytes(U.v_fmt).code + fmt_bytes(U.v_fmt).meta;
}

// Items of a run of `len` tokens when about `want` are asked for: the count that its own equal item size gives.
int even_items(int len, int want) {
  int n = std::max(1, want);
  for (;;) {
    const int c = even_chunk(len, n), n2 = (len + c - 1) / c;
    if (n2 == n) return n;
    n = n2;
  }
}
// Items for a run of `len` tokens of `per_token` bytes when an item should stream about item_bytes: at most 8192
// tokens each, and no more items than 256-token ones would give.
int items_for(int64_t len, int per_token, double item_bytes) {
  const int64_t lo = (len + 8191) / 8192, hi = (len + 255) / 256;
  const int64_t want = (int64_t)((double)len * per_token / item_bytes + 0.5);
  return even_items((int)len, (int)std::max(lo, std::min(hi, want)));
}

// How the tiers read in place from HBM are cut into work items: bytes per item (one KV head's share of a chunk of
// tokens), the same for every tier, so that all workgroups of the fused launch stream about the same amount.
// Every run (tier, sequence) is cut into items of equal size, and a run cannot share an item with another, so with
// many runs the item sizes and the number of workgroups come out in steps.  What costs time, measured at 16 and 64
// sequences of a few thousand tokens: items of unequal size (one round of workgroups with 524 and 745 KB items
// 5.45 TB/s, the same bytes as 350 and 331 KB items 5.98), and a last round of resident workgroups that is mostly
// empty when there are few rounds (1024 workgroups on 768 slots 3.98-4.6 TB/s, 3072 on 768 4.9-5.7) -- fewer
// workgroups per CU hide less latency, so the partly filled round does not run proportionally faster.  The
// target is therefore raised from the kernel's default (default_items) in steps until the items are within 10 % of
// their mean and the last round is filled (or there are at least three rounds); failing that, the candidate with
// the smallest estimated loss is taken.  target_items != 0 (ttkv_set_split) is taken as given.
double choose_item_bytes(const ttkv_cache *c, const bool *dense, int target_items, const int64_t *last_tokens, SplitMemo *memo) {
  // last_tokens: null, or the tokens of the last tier that are attended, per sequence (its selected blocks)
  // The runs, gathered once: length and bytes per token (at most batch x tiers of them).
  struct RunShape { int32_t len, per_token, finest; };
  RunShape runs[TTKV_MAX_BATCH * TTKV_MAX_TIERS];
  int n_runs = 0;
  int64_t S = 0;   // bytes one pass over one KV head's tokens streams
  uint32_t sig = (uint32_t)c->batch * 31u + (uint32_t)c->n_tiers * 7u + (uint32_t)c->n_q_heads * 131u + (uint32_t)c->n_kv_heads * 17u;
  for (int t = 0; t < c->n_tiers; ++t) {
    sig = sig * 33u + (uint32_t)(c->tier[t].k_fmt * 8 + c->tier[t].v_fmt) * 2u + (dense[t] ? 1u : 0u);
    if (!dense[t]) continue;
    const int pt = per_token_bytes(c->tier[t]);
    for (int b = 0; b < c->batch; ++b) {
      const int64_t len = last_tokens && t == c->n_tiers - 1 ? last_tokens[b] : c->tier[t].len[b];
      if (len == 0) continue;
      runs[n_runs++] = RunShape{(int32_t)len, pt, (int32_t)((len + 255) / 256)};
      S += len * pt;
    }
  }
  if (S == 0) return 1.0;
  const int Hkv = c->n_kv_heads, G = c->n_q_heads / Hkv;
  if (target_items) return std::max(1.0, (double)S * Hkv / target_items);
  const int legacy = default_items(c);
  const bool vector_kernel = legacy == 2560;
  const int resident = vector_kernel ? 1024 : legacy;                             // workgroups on the chip at once
  const int per_item = Hkv * (vector_kernel ? G / attn_group_width(G) : (G + 15) / 16);   // workgroups per item
  // the vector kernel's default of 2.5 rounds is as fast as one round when the items are equal (measured)
  static const float steps_v[] = {2.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 5.0f, 6.0f};
  static const float steps_m[] = {1.0f, 1.5f, 2.0f, 2.5f, 3.0f, 4.0f, 5.0f, 6.0f};
  const float *steps = vector_kernel ? steps_v : steps_m;

  struct Fit { double b, largest, sum_b, sum_b2, n_big; bool all_max; };
  // Item size for `want_rounds` rounds.  The item counts come out in steps: if the large items (at least half the
  // largest) overshoot the rounds aimed at, slightly larger items are asked for, up to three times.
  auto fit = [&](double want_rounds) {
    Fit f{};
    f.b = std::max(1.0, (double)S * Hkv / (resident * want_rounds));
    double item[TTKV_MAX_BATCH * TTKV_MAX_TIERS];
    int count[TTKV_MAX_BATCH * TTKV_MAX_TIERS];
    double n_big_before = -1.0;
    for (int attempt = 0; attempt < 4; ++attempt) {
      if (attempt) f.b *= 1.03;
      f.largest = f.sum_b = f.sum_b2 = f.n_big = 0.0;
      f.all_max = true;
      for (int r = 0; r < n_runs; ++r) {
        count[r] = items_for(runs[r].len, runs[r].per_token, f.b);
        item[r] = (double)even_chunk(runs[r].len, count[r]) * runs[r].per_token;
        f.sum_b += count[r] * item[r];
        f.sum_b2 += count[r] * item[r] * item[r];
        f.largest = std::max(f.largest, item[r]);
        f.all_max &= count[r] >= runs[r].finest;
      }
      bool all_min = true;   // every run in one item already: larger items change nothing
      for (int r = 0; r < n_runs; ++r) {
        if (2.0 * item[r] >= f.largest) f.n_big += count[r];
        all_min &= count[r] == 1;
      }
      if (f.n_big * per_item <= resident * want_rounds || f.all_max || all_min || f.n_big == n_big_before) break;
      n_big_before = f.n_big;   // the same count as before: the steps are coarser than the nudge
    }
    return f;
  };

  // The search over the number of rounds is remembered (in the handle's plan) while the cache keeps its shape: the
  // same tiers, formats and runs, the bytes within 1/32 of what they were; a call then only fits the item size.
  if (memo && memo->valid && memo->sig == sig && memo->n_runs == n_runs && memo->sel == (last_tokens != nullptr) &&
      std::llabs(S - memo->bytes) <= memo->bytes / 32)
    return fit(steps[memo->step]).b;

  double best_b = 0.0, best_loss = 1e30;
  int best_step = 0;
  for (int k = 0; k < 8; ++k) {
    const Fit f = fit(steps[k]);
    // Short items (a 256-token window beside a long tier) neither unbalance a launch nor fill a round: the mean
    // weighs an item by its bytes, the rounds count only the items of at least half the largest size.
    const double imbalance = f.largest / (f.sum_b2 / f.sum_b);
    const double rounds = f.n_big * per_item / resident;
    const double frac = rounds - std::floor(rounds);
    const double fill = frac == 0.0 ? 1.0 : frac;
    const bool filled = rounds >= 3.0 || fill >= (vector_kernel ? 0.45 : 0.75) || (rounds < 1.0 && (f.all_max || rounds >= 0.75));
    const double loss = imbalance <= 1.10 && filled ? 0.0 : imbalance * (1.0 + (1.0 - fill) / std::max(1.0, std::ceil(rounds)));
    if (loss < best_loss) {
      best_loss = loss;
      best_b = f.b;
      best_step = k;
    }
    if (loss == 0.0 || f.all_max) break;   // good enough, or finer targets change nothing
  }
  if (memo) *memo = SplitMemo{true, sig, n_runs, last_tokens != nullptr, best_step, S};
  return best_b;
}

// staged: host tiers are copied block by block into staging slots (one kernel per
// copy); otherwise the fused kernel reads them in place.
void build_plan(const ttkv_cache *c, const int32_t *sel_blocks, const int32_t *sel_count, int32_t sel_stride, bool staged,
                int target_items, Plan *P, const DevSel *ds = nullptr) {
  P->status = TTKV_OK;
  P->slot_bytes = 0;
  P->max_parts = 0;
  P->runs.clear();
  P->fetch.clear();
  for (int b = 0; b < c->batch; ++b) P->parts[b] = 0;
  const int last = c->n_tiers - 1;
  // tiers in HBM are cut into items of equal size per run; so are the blocks a device-side selection names
  for (int t = 0; t < c->n_tiers; ++t) P->even[t] = c->tier[t].mem != TTKV_MEM_HOST_PINNED && !(sel_blocks && t == last);
  int64_t sel_tokens[TTKV_MAX_BATCH];
  if (ds)
    for (int b = 0; b < c->batch; ++b) {
      const ttkv_tier &T = c->tier[last];
      const int64_t live = T.len[b] ? (T.start[b] + T.len[b] + T.block_tokens - 1) / T.block_tokens - T.start[b] / T.block_tokens : 0;
      sel_tokens[b] = std::max<int64_t>(0, std::min<int64_t>(std::min(ds->k, ds->stride), live)) * T.block_tokens;
    }
  const double item_bytes = choose_item_bytes(c, P->even, target_items, ds ? sel_tokens : nullptr, &P->memo);
  for (int t = 0; t < c->n_tiers; ++t) {
    const ttkv_tier &T = c->tier[t];
    const Layout L = make_layout(T, c->n_kv_heads);
    const bool sparse = sel_blocks && t == last;
    const bool host = T.mem == TTKV_MEM_HOST_PINNED;
    // host rows read in place: few large sequential items keep the PCIe read stream efficient (measured); staged
    // slots: 256-token items for parallelism; tiers in HBM, dense or selected on the device: equal items per run (0)
    P->chunk[t] = (host && !staged) ? 2048 : (host || sparse) ? 256 : 0;
    if (ds && t == last) P->chunk[t] = host ? 2048 : 0;
    if (!host && sparse && t == last) {
      // Blocks of a tier in HBM that the caller selected (ids on the host): one item per block once the selection
      // alone fills the chip, finer items, down to 256 tokens, when few blocks are selected.
      int64_t n_sel = 0;
      for (int b = 0; b < c->batch; ++b) n_sel += sel_count[b];
      const int legacy = default_items(c), resident = legacy == 2560 ? 1024 : legacy;
      const int64_t wgs = std::max<int64_t>(1, n_sel * c->n_kv_heads);
      const int ipb = (int)std::min<int64_t>(L.bt / 256, std::max<int64_t>(1, (resident + wgs - 1) / wgs));
      P->chunk[t] = ((L.bt + ipb - 1) / ipb + 63) / 64 * 64;
    }
    const int chunk = P->chunk[t];
    if (ds && t == last) {
      // the kernel looks the block ids up itself: the host only knows how many there are
      const int ipb = host ? (L.bt + chunk - 1) / chunk : 0;   // items per block
      for (int b = 0; b < c->batch; ++b) {
        const int64_t first_id = T.start[b] / L.bt;
        const int64_t end_id = (T.start[b] + T.len[b] + L.bt - 1) / L.bt;  // exclusive
        const int count = (int)std::min<int64_t>(std::min(ds->k, ds->stride), end_id - first_id);
        if (T.len[b] == 0 || count <= 0) continue;
        Run r{};
        r.tier = t; r.b = b;
        r.rec_base = (int32_t)((int64_t)b * ds->stride);
        r.first_tok = (int32_t)(end_id - 1);
        r.len = host ? count : count * L.bt;     // blocks in fixed items, or their tokens as one run in equal items
        r.selected = true;
        r.part_base = P->parts[b];
        r.n_chunks = host ? count * ipb : items_for((int64_t)count * L.bt, per_token_bytes(T), item_bytes);
        P->parts[b] += r.n_chunks;
        P->runs.push_back(r);
      }
      continue;
    }
    if (!sparse && !(host && staged)) {
      for (int b = 0; b < c->batch; ++b) {
        if (T.len[b] == 0) continue;
        Run r{};
        r.tier = t; r.b = b;
        r.rec_base = (int32_t)((int64_t)b * T.ring_blocks);
        r.first_tok = (int32_t)(T.start[b] % ring_tokens(T));
        r.len = (int32_t)T.len[b];
        r.no_table = false;
        r.part_base = P->parts[b];
        r.n_chunks = P->even[t] ? items_for(T.len[b], per_token_bytes(T), item_bytes) : (int)((T.len[b] + chunk - 1) / chunk);
        P->parts[b] += r.n_chunks;
        P->runs.push_back(r);
      }
      continue;
    }
    // block by block: selected blocks of the last tier, or staged host blocks
    const int gran = host && staged ? copy_granule(L.rec_bytes) : (1 << 20);
    if (host && staged) P->slot_bytes = std::max(P->slot_bytes, align256((size_t)gran * L.rec_bytes));
    for (int b = 0; b < c->batch; ++b) {
      if (T.len[b] == 0 && !sparse) continue;
      const int64_t first_id = T.start[b] / L.bt;
      const int64_t end_id = (T.start[b] + T.len[b] + L.bt - 1) / L.bt;  // exclusive
      const int64_t n_ids = sparse ? sel_count[b] : end_id - first_id;
      int64_t prev_id = -1;
      for (int64_t i = 0; i < n_ids; ++i) {
        const int64_t id = sparse ? (int64_t)sel_blocks[(int64_t)b * sel_stride + i] : first_id + i;
        if (id < first_id || id >= end_id || id <= prev_id) {
          P->status = TTKV_ERR_INVALID_ARG;
          return;
        }
        prev_id = id;
        const int64_t rec = record_of(T, b, id % T.ring_blocks);
        const int ntok = (int)std::min<int64_t>(L.bt, T.start[b] + T.len[b] - id * L.bt);
        const int nparts = (ntok + chunk - 1) / chunk;
        if (host && staged) {
          if (!P->fetch.empty()) {
            Fetch &f = P->fetch.back();
            if (f.tier == t && f.b == b && f.nrec < gran && f.rec + f.nrec == rec && f.ntok == f.nrec * L.bt) {
              // the merged copy is cut into chunks as one run of tokens: recount its parts
              P->parts[b] -= (f.ntok + chunk - 1) / chunk;
              f.nrec += 1;
              f.ntok += ntok;
              P->parts[b] += (f.ntok + chunk - 1) / chunk;
              continue;
            }
          }
          Fetch f{};
          f.tier = t; f.b = b; f.rec = rec; f.nrec = 1; f.ntok = ntok; f.chunk = chunk;
          f.part_base = P->parts[b];
          P->parts[b] += nparts;
          P->fetch.push_back(f);
        } else {
          if (!P->runs.empty()) {
            Run &r = P->runs.back();
            if (r.tier == t && r.b == b && r.no_table && (int64_t)r.rec_base + r.len / L.bt == rec && r.len % L.bt == 0) {
              P->parts[b] -= r.n_chunks;
              r.len += ntok;
              r.n_chunks = (r.len + chunk - 1) / chunk;
              P->parts[b] += r.n_chunks;
              continue;
            }
          }
          Run r{};
          r.tier = t; r.b = b;
          r.rec_base = (int32_t)rec;
          r.first_tok = 0;
          r.len = ntok;
          r.no_table = true;
          r.part_base = P->parts[b];
          r.n_chunks = nparts;
          P->parts[b] += nparts;
          P->runs.push_back(r);
        }
      }
    }
  }
  P->max_parts = 0;
  for (int b = 0; b < c->batch; ++b) P->max_parts = std::max(P->max_parts, P->parts[b]);
}

ttkv_status check_sel(const ttkv_cache *c, const int32_t *sel_blocks, const int32_t *sel_count, int32_t sel_stride) {
  if ((sel_blocks == nullptr) != (sel_count == nullptr)) return TTKV_ERR_INVALID_ARG;
  if (sel_blocks) {
    if (sel_stride < 0) return TTKV_ERR_INVALID_ARG;
    for (int b = 0; b < c->batch; ++b)
      if (sel_count[b] < 0 || sel_count[b] > sel_stride) return TTKV_ERR_INVALID_ARG;
  }
  return TTKV_OK;
}

// Rows were described by `a` (their destination may be a staging view); update the
// running key sums / mean keys of tier t, whose ring position is taken from its
// start/len before they are advanced.
hipError_t run_summary(const ConvArgs &a, const ttkv_cache *c, int t, hipStream_t s, int *nk) {
  const ttkv_tier &T = c->tier[t];
  if (!T.k_sum) return hipSuccess;
  ConvArgs u = a;
  u.dst = make_view(T, make_layout(T, c->n_kv_heads));
  u.k_sum = T.k_sum;
  u.k_summary = (uint16_t *)T.k_summary;
  u.sum_table = T.block_table_dev;
  u.sum_ring_blocks = (int32_t)T.ring_blocks;
  u.inv_bt = 1.0f / (float)T.block_tokens;
  for (int j = 0; j < a.n_seq; ++j) {
    const int b = a.seq_id[j];
    u.dst_first_tok[j] = (int32_t)((T.start[b] + T.len[b]) % ring_tokens(T));
    u.sum_rec_base[j] = (int32_t)((int64_t)b * T.ring_blocks);
  }
  return launch_summary(u, s, nk);
}

void fill_via(ConvArgs &a, const ttkv_cache *c, int tier, bool through) {
  a.n_via = 0;
  if (!through) return;
  for (int u = 1; u < tier; ++u) {
    a.via_k[a.n_via] = c->tier[u].k_fmt;
    a.via_v[a.n_via] = c->tier[u].v_fmt;
    ++a.n_via;
  }
}

// Device->pinned copies of rows [row_lo, row_hi) of one record (all heads, all sections).
ttkv_status copy_rows_to_host(Handle *h, const Layout &L, int Hkv, uint8_t *host_rec, const uint8_t *dev_rec, int row_lo,
                              int row_hi, hipStream_t s) {
  if (row_lo == 0 && row_hi == L.bt) {
    TTKV_HIP(h, hipMemcpyAsync(host_rec, dev_rec, (size_t)L.rec_bytes, hipMemcpyDeviceToHost, s));
    h->stats.d2h_bytes += (uint64_t)L.rec_bytes;
    return TTKV_OK;
  }
  const int off[4] = {0, L.k_meta_off, L.v_off, L.v_meta_off};
  const int rowb[4] = {L.kc, L.km, L.vc, L.vm};
  for (int sct = 0; sct < 4; ++sct) {
    if (!rowb[sct]) continue;
    const size_t o = (size_t)off[sct] + (size_t)row_lo * rowb[sct];
    const size_t width = (size_t)(row_hi - row_lo) * rowb[sct];
    TTKV_HIP(h, hipMemcpy2DAsync(host_rec + o, (size_t)L.head_bytes, dev_rec + o, (size_t)L.head_bytes, width, (size_t)Hkv,
                                 hipMemcpyDeviceToHost, s));
    h->stats.d2h_bytes += (uint64_t)width * Hkv;
  }
  return TTKV_OK;
}

ttkv_status append_impl(Handle *h, ttkv_cache *c, int32_t tier, int32_t seq, const void *k_src, const void *v_src,
                        int32_t src_fmt, int64_t n_tokens, int32_t through, void *workspace, size_t ws_bytes,
                        hipStream_t stream, bool host_variant) {
  if (!h) return TTKV_ERR_INVALID_ARG;
  ttkv_status st = validate_cache(c, h->check_tables);
  if (st != TTKV_OK) return st;
  if (tier < 0 || tier >= c->n_tiers || seq < -1 || seq >= c->batch || !k_src || !v_src || n_tokens < 0)
    return TTKV_ERR_INVALID_ARG;
  if (src_fmt != TTKV_F16 && src_fmt != TTKV_BF16 && src_fmt != TTKV_F32) return TTKV_ERR_INVALID_ARG;
  ttkv_tier &T = c->tier[tier];
  if ((T.mem == TTKV_MEM_HOST_PINNED) != host_variant) return TTKV_ERR_INVALID_ARG;
  if ((is_fp(T.k_fmt) && T.k_fmt != src_fmt) || (is_fp(T.v_fmt) && T.v_fmt != src_fmt)) return TTKV_ERR_UNSUPPORTED;
  if (n_tokens == 0) return TTKV_OK;
  if (T.k_fmt == TTKV_I4_ASYM_T128 && n_tokens % 128) return TTKV_ERR_INVALID_ARG;   // whole token groups only
  if (T.v_fmt == TTKV_I4_ASYM_G64_T32 && n_tokens % 32) return TTKV_ERR_INVALID_ARG;
  const int b0 = seq < 0 ? 0 : seq, b1 = seq < 0 ? c->batch : seq + 1;
  for (int b = b0; b < b1; ++b)
    if (T.len[b] + n_tokens > ring_tokens(T)) return TTKV_ERR_CAPACITY;
  const Layout L = make_layout(T, c->n_kv_heads);

  ConvArgs a{};
  a.s.k_flat = k_src;
  a.s.v_flat = v_src;
  a.s.flat_fmt = src_fmt;
  a.s.from_tier = 0;
  a.n_seq = b1 - b0;
  a.Hkv = c->n_kv_heads;
  a.n_tokens = (int32_t)n_tokens;
  fill_via(a, c, tier, through != 0);

  // host tier without a workspace: the kernels store into the pinned records themselves (PCIe writes)
  const bool direct = host_variant && workspace == nullptr;
  if (direct && T.block_table && !T.block_table_dev) return TTKV_ERR_INVALID_ARG;   // the kernels look the records up
  int max_touched = 0;
  if (!host_variant || direct) {
    a.dst = make_view(T, L);
    for (int b = b0; b < b1; ++b) {
      const int j = b - b0;
      a.seq_id[j] = b;
      a.dst_rec_base[j] = (int32_t)((int64_t)b * T.ring_blocks);
      a.dst_first_tok[j] = (int32_t)((T.start[b] + T.len[b]) % ring_tokens(T));
    }
  } else {
    // quantize into workspace records laid out [entry][touched block], then copy rows out
    for (int b = b0; b < b1; ++b) {
      const int64_t o0 = T.start[b] + T.len[b];
      max_touched = std::max<int>(max_touched, (int)((o0 + n_tokens - 1) / L.bt - o0 / L.bt + 1));
    }
    if (!workspace || ws_bytes < (size_t)a.n_seq * max_touched * L.rec_bytes) return TTKV_ERR_WORKSPACE;
    if (T.ring_blocks < max_touched) return TTKV_ERR_CAPACITY;
    a.dst = make_slot_view(T, L, workspace, max_touched);
    for (int b = b0; b < b1; ++b) {
      const int j = b - b0;
      a.seq_id[j] = b;
      a.dst_rec_base[j] = j * max_touched;
      a.dst_first_tok[j] = (int32_t)((T.start[b] + T.len[b]) % L.bt);
    }
  }
  int nk = 0;
  TTKV_HIP(h, launch_convert(a, stream, &nk));
  TTKV_HIP(h, run_summary(a, c, tier, stream, &nk));
  h->stats.kernels += nk;
  if (direct) h->stats.d2h_bytes += (uint64_t)a.n_seq * (uint64_t)n_tokens * (L.kc + L.km + L.vc + L.vm) * c->n_kv_heads;
  if (host_variant && !direct) {
    for (int b = b0; b < b1; ++b) {
      const int j = b - b0;
      const int64_t o0 = T.start[b] + T.len[b];
      for (int64_t id = o0 / L.bt; id <= (o0 + n_tokens - 1) / L.bt; ++id) {
        const int lo = (int)std::max<int64_t>(o0 - id * L.bt, 0);
        const int hi = (int)std::min<int64_t>(o0 + n_tokens - id * L.bt, L.bt);
        uint8_t *host_rec = (uint8_t *)T.data + record_of(T, b, id % T.ring_blocks) * L.rec_bytes;
        const uint8_t *dev_rec = (const uint8_t *)workspace + ((int64_t)j * max_touched + (id - o0 / L.bt)) * L.rec_bytes;
        st = copy_rows_to_host(h, L, c->n_kv_heads, host_rec, dev_rec, lo, hi, stream);
        if (st != TTKV_OK) return st;
      }
    }
  }
  for (int b = b0; b < b1; ++b) T.len[b] += n_tokens;
  return TTKV_OK;
}

// Events are created on the first call that chains streams (on the device
// current at that time), so that a handle can exist without a device.
ttkv_status ensure_events(Handle *h) {
  if (h->have_events) return TTKV_OK;
  TTKV_HIP(h, hipGetDevice(&h->device));
  for (int i = 0; i < TTKV_MAX_SLOTS; ++i) {
    TTKV_HIP(h, hipEventCreateWithFlags(&h->ready[i], hipEventDisableTiming));
    TTKV_HIP(h, hipEventCreateWithFlags(&h->freed[i], hipEventDisableTiming));
  }
  TTKV_HIP(h, hipEventCreateWithFlags(&h->fence, hipEventDisableTiming));
  TTKV_HIP(h, hipEventCreateWithFlags(&h->fence2, hipEventDisableTiming));
  h->have_events = true;
  return TTKV_OK;
}

}  // namespace

extern "C" {

ttkv_status ttkv_create(ttkv_handle *out) {
  if (!out) return TTKV_ERR_INVALID_ARG;
  Handle *h = new (std::nothrow) Handle();
  if (!h) return TTKV_ERR_INVALID_ARG;
  try {
    h->plan.runs.reserve(TTKV_PLAN_RESERVE);
    h->plan.fetch.reserve(TTKV_PLAN_RESERVE);
    h->plan.order.reserve(TTKV_PLAN_RESERVE);
  } catch (...) {
    delete h;
    return TTKV_ERR_INVALID_ARG;
  }
  h->have_events = false;
  h->plan.memo.valid = false;
  h->target_items = 0;
  h->check_tables = true;
  h->time_on = false;
  h->time_max = h->time_n = 0;
  h->time_ev = nullptr;
  h->time_reps = nullptr;
  h->time_repeat = 1;
  *out = reinterpret_cast<ttkv_handle>(h);
  return TTKV_OK;
}

ttkv_status ttkv_destroy(ttkv_handle hh) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h) return TTKV_ERR_INVALID_ARG;
  if (h->have_events) {
    for (int i = 0; i < TTKV_MAX_SLOTS; ++i) {
      (void)hipEventDestroy(h->ready[i]);
      (void)hipEventDestroy(h->freed[i]);
    }
    (void)hipEventDestroy(h->fence);
    (void)hipEventDestroy(h->fence2);
  }
  for (int i = 0; i < 2 * h->time_max; ++i) (void)hipEventDestroy(h->time_ev[i]);
  free(h->time_ev);
  free(h->time_reps);
  delete h;
  return TTKV_OK;
}

void ttkv_get_stats(ttkv_handle hh, ttkv_stats *out) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (h && out) *out = h->stats;
}
void ttkv_reset_stats(ttkv_handle hh) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (h) h->stats = ttkv_stats{};
}

const char *ttkv_status_string(ttkv_status s) {
  switch (s) {
    case TTKV_OK: return "ok";
    case TTKV_ERR_INVALID_ARG: return "invalid argument";
    case TTKV_ERR_CAPACITY: return "tier capacity";
    case TTKV_ERR_UNSUPPORTED: return "unsupported";
    case TTKV_ERR_WORKSPACE: return "workspace too small";
    case TTKV_ERR_HIP: return "HIP error";
  }
  return "unknown status";
}

size_t ttkv_record_bytes(const ttkv_cache *c, int32_t tier) {
  if (!c || tier < 0 || tier >= c->n_tiers || tier >= TTKV_MAX_TIERS) return 0;
  const ttkv_tier &T = c->tier[tier];
  if (!is_tier_fmt(T.k_fmt) || !is_tier_fmt(T.v_fmt) || T.block_tokens <= 0 || c->n_kv_heads <= 0) return 0;
  return (size_t)make_layout(T, c->n_kv_heads).rec_bytes;
}

ttkv_status ttkv_locate(const ttkv_cache *c, int32_t b, int64_t pos, int32_t *tier, int64_t *block_id, int32_t *row,
                        int64_t *record) {
  ttkv_status st = validate_cache(c);
  if (st != TTKV_OK) return st;
  if (b < 0 || b >= c->batch || pos < 0) return TTKV_ERR_INVALID_ARG;
  // tiers hold adjacent ranges, oldest tokens in the last tier
  int64_t base = 0;
  for (int t = c->n_tiers - 1; t >= 0; --t) {
    const ttkv_tier &T = c->tier[t];
    if (pos < base + T.len[b]) {
      const int64_t o = T.start[b] + (pos - base);
      if (tier) *tier = t;
      if (block_id) *block_id = o / T.block_tokens;
      if (row) *row = (int32_t)(o % T.block_tokens);
      if (record) *record = record_of(T, b, (o / T.block_tokens) % T.ring_blocks);
      return TTKV_OK;
    }
    base += T.len[b];
  }
  return TTKV_ERR_INVALID_ARG;
}

size_t ttkv_workspace_bytes(const ttkv_cache *c, int32_t max_parts, int32_t n_slots) {
  if (validate_cache(c) != TTKV_OK || max_parts < 1 || n_slots < 0 || n_slots > TTKV_MAX_SLOTS) return 0;
  size_t slot = 0;
  for (int t = 0; t < c->n_tiers; ++t)
    if (c->tier[t].mem == TTKV_MEM_HOST_PINNED) {
      const Layout L = make_layout(c->tier[t], c->n_kv_heads);
      slot = std::max(slot, align256((size_t)copy_granule(L.rec_bytes) * L.rec_bytes));
    }
  const size_t rows = (size_t)c->batch * c->n_q_heads;
  return (size_t)n_slots * slot + align256(rows * max_parts * 130 * sizeof(float)) + 256;
}

size_t ttkv_demote_workspace_bytes(const ttkv_cache *c, int32_t src_tier) {
  if (validate_cache(c) != TTKV_OK || src_tier < 0 || src_tier + 1 >= c->n_tiers) return 0;
  const ttkv_tier &D = c->tier[src_tier + 1];
  if (D.mem != TTKV_MEM_HOST_PINNED) return 0;
  const Layout L = make_layout(D, c->n_kv_heads);
  const int touched = c->tier[src_tier].block_tokens / D.block_tokens + 2;
  return (size_t)c->batch * touched * L.rec_bytes;
}

size_t ttkv_append_host_workspace_bytes(const ttkv_cache *c, int32_t tier, int32_t seq, int64_t n_tokens) {
  if (validate_cache(c) != TTKV_OK || tier < 0 || tier >= c->n_tiers || n_tokens < 0) return 0;
  const Layout L = make_layout(c->tier[tier], c->n_kv_heads);
  const int64_t touched = n_tokens / L.bt + 2;
  return (size_t)(seq < 0 ? c->batch : 1) * touched * L.rec_bytes;
}

int32_t ttkv_count_parts(ttkv_handle hh, const ttkv_cache *c, const int32_t *sel_blocks, const int32_t *sel_count,
                         int32_t sel_stride, int32_t n_slots) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h || validate_cache(c, h->check_tables) != TTKV_OK || check_sel(c, sel_blocks, sel_count, sel_stride) != TTKV_OK) return -1;
  Plan &P = h->plan;
  build_plan(c, sel_blocks, sel_count, sel_stride, n_slots > 0, h->target_items, &P);
  return P.status == TTKV_OK ? P.max_parts : -1;
}

ttkv_status ttkv_quantize_append(ttkv_handle hh, ttkv_cache *c, int32_t tier, int32_t seq, const void *k_src,
                                 const void *v_src, int32_t src_fmt, int64_t n_tokens, int32_t through_tiers,
                                 void *stream) {
  return append_impl(reinterpret_cast<Handle *>(hh), c, tier, seq, k_src, v_src, src_fmt, n_tokens, through_tiers, nullptr,
                     0, (hipStream_t)stream, false);
}

ttkv_status ttkv_quantize_append_host(ttkv_handle hh, ttkv_cache *c, int32_t tier, int32_t seq, const void *k_src,
                                      const void *v_src, int32_t src_fmt, int64_t n_tokens, int32_t through_tiers,
                                      void *workspace, size_t ws_bytes, void *stream) {
  return append_impl(reinterpret_cast<Handle *>(hh), c, tier, seq, k_src, v_src, src_fmt, n_tokens, through_tiers,
                     workspace, ws_bytes, (hipStream_t)stream, true);
}

ttkv_status ttkv_tier_demote(ttkv_handle hh, ttkv_cache *c, int32_t src_tier, int32_t max_blocks, void *workspace,
                             size_t ws_bytes, void *compute_, void *copy_) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h) return TTKV_ERR_INVALID_ARG;
  ttkv_status st = validate_cache(c, h->check_tables);
  if (st != TTKV_OK) return st;
  if (src_tier < 0 || src_tier + 1 >= c->n_tiers) return TTKV_ERR_INVALID_ARG;
  ttkv_tier &S = c->tier[src_tier];
  ttkv_tier &D = c->tier[src_tier + 1];
  if (S.mem != TTKV_MEM_DEVICE) return TTKV_ERR_UNSUPPORTED;
  if (is_fp(D.k_fmt) && D.k_fmt != S.k_fmt) return TTKV_ERR_UNSUPPORTED;
  if (is_fp(D.v_fmt) && D.v_fmt != S.v_fmt) return TTKV_ERR_UNSUPPORTED;
  if (D.k_fmt == TTKV_I4_ASYM_T128 && S.block_tokens % 128) return TTKV_ERR_UNSUPPORTED;   // whole token groups arrive
  hipStream_t compute = (hipStream_t)compute_, copy = (hipStream_t)copy_;
  const Layout LS = make_layout(S, c->n_kv_heads), LD = make_layout(D, c->n_kv_heads);
  // host destination with a workspace: staging records + copies; without one the kernels store into the pinned
  // records themselves (ordered on `compute` like a device destination)
  const bool to_host = D.mem == TTKV_MEM_HOST_PINNED && workspace != nullptr;
  const bool host_direct = D.mem == TTKV_MEM_HOST_PINNED && workspace == nullptr;
  if (host_direct && D.block_table && !D.block_table_dev) return TTKV_ERR_INVALID_ARG;   // the kernels look the records up

  // how many blocks each sequence moves; check every ring before touching anything
  int nmove[TTKV_MAX_BATCH], rounds = 0;
  for (int b = 0; b < c->batch; ++b) {
    int64_t len = S.len[b];
    int n = 0;
    while (len >= S.capacity_tokens && (max_blocks <= 0 || n < max_blocks)) {
      if (len < LS.bt) return TTKV_ERR_CAPACITY;
      len -= LS.bt;
      ++n;
    }
    nmove[b] = n;
    rounds = std::max(rounds, n);
    if (D.len[b] + (int64_t)n * LS.bt > ring_tokens(D)) return TTKV_ERR_CAPACITY;
  }
  if (rounds == 0) return TTKV_OK;
  const int touched = LS.bt / LD.bt + 2;
  if (to_host && ws_bytes < (size_t)c->batch * touched * LD.rec_bytes) return TTKV_ERR_WORKSPACE;
  if (to_host && (st = ensure_events(h)) != TTKV_OK) return st;

  for (int round = 0; round < rounds; ++round) {
    ConvArgs a{};
    a.s.from_tier = 1;
    a.s.src = make_view(S, LS);
    a.Hkv = c->n_kv_heads;
    a.n_tokens = LS.bt;
    a.n_via = 0;
    a.dst = to_host ? make_slot_view(D, LD, workspace, touched) : make_view(D, LD);
    for (int b = 0; b < c->batch; ++b) {
      if (round >= nmove[b]) continue;
      const int j = a.n_seq++;
      a.seq_id[j] = b;
      a.s.src_first_tok[j] = (int32_t)(S.start[b] % ring_tokens(S));
      a.s.src_rec_base[j] = (int32_t)((int64_t)b * S.ring_blocks);
      const int64_t o = D.start[b] + D.len[b];  // ordinal of the first row written
      if (to_host) {
        a.dst_rec_base[j] = j * touched;
        a.dst_first_tok[j] = (int32_t)(o % LD.bt);
      } else {
        a.dst_rec_base[j] = (int32_t)((int64_t)b * D.ring_blocks);
        a.dst_first_tok[j] = (int32_t)(o % ring_tokens(D));
      }
    }
    int nk = 0;
    TTKV_HIP(h, launch_convert(a, compute, &nk));
    TTKV_HIP(h, run_summary(a, c, src_tier + 1, compute, &nk));
    h->stats.kernels += nk;

    if (to_host) {
      TTKV_HIP(h, hipEventRecord(h->fence2, compute));
      TTKV_HIP(h, hipStreamWaitEvent(copy, h->fence2, 0));
    }
    for (int j = 0; j < a.n_seq; ++j) {
      const int b = a.seq_id[j];
      if (to_host) {
        const int64_t o0 = D.start[b] + D.len[b];
        for (int64_t id = o0 / LD.bt; id <= (o0 + LS.bt - 1) / LD.bt; ++id) {
          const int lo = (int)std::max<int64_t>(o0 - id * LD.bt, 0);
          const int hi = (int)std::min<int64_t>(o0 + LS.bt - id * LD.bt, LD.bt);
          uint8_t *host_rec = (uint8_t *)D.data + record_of(D, b, id % D.ring_blocks) * LD.rec_bytes;
          const uint8_t *dev_rec = (const uint8_t *)workspace + ((int64_t)j * touched + (id - o0 / LD.bt)) * LD.rec_bytes;
          st = copy_rows_to_host(h, LD, c->n_kv_heads, host_rec, dev_rec, lo, hi, copy);
          if (st != TTKV_OK) return st;
        }
      }
      if (host_direct) h->stats.d2h_bytes += (uint64_t)LS.bt * (LD.kc + LD.km + LD.vc + LD.vm) * c->n_kv_heads;
      S.start[b] += LS.bt;
      S.len[b] -= LS.bt;
      D.len[b] += LS.bt;
      h->stats.demotions += 1;
    }
    if (to_host && round + 1 < rounds) {
      // the staging records are reused by the next round: wait for the copies
      TTKV_HIP(h, hipEventRecord(h->fence2, copy));
      TTKV_HIP(h, hipStreamWaitEvent(compute, h->fence2, 0));
    }
  }
  if (to_host) {
    // later compute work (and the next step's fetches on `copy`) must see the host records complete;
    // `copy` is ordered by itself, `compute` is released by this event
    TTKV_HIP(h, hipEventRecord(h->fence2, copy));
    TTKV_HIP(h, hipStreamWaitEvent(compute, h->fence2, 0));
  }
  return TTKV_OK;
}

// The stream operations of one attention call -- the copy/compute chain of streaming attention (Sec. 4.3) -- behind
// one interface, so that the code that issues them drives HIP or, for ttkv_staged_schedule, a recorder: the order
// checked on the CPU is then the order the GPU gets.
enum { EV_FENCE = 0, EV_READY = 1, EV_FREED = 1 + TTKV_MAX_SLOTS };   // event ids: fence, ready[slot], freed[slot]
struct Chain {
  virtual hipError_t record(int event, int on_copy_stream) = 0;
  virtual hipError_t wait(int on_copy_stream, int event) = 0;
  virtual hipError_t copy(int fetch, int slot, void *dst, const void *src, size_t bytes) = 0;
  virtual hipError_t attend(int fetch, int slot, const FusedArgs &a, int *nk, int *nm) = 0;   // fetch -1: the tiers read in place
  virtual hipError_t merge(const MergeArgs &m) = 0;
  virtual ~Chain() {}
};
struct HipChain : Chain {
  Handle *h;
  hipStream_t compute, copy_s;
  HipChain(Handle *h_, hipStream_t c, hipStream_t y) : h(h_), compute(c), copy_s(y) {}
  hipEvent_t ev(int e) { return e == EV_FENCE ? h->fence : e < EV_FREED ? h->ready[e - EV_READY] : h->freed[e - EV_FREED]; }
  hipError_t record(int e, int on_copy) override { return hipEventRecord(ev(e), on_copy ? copy_s : compute); }
  hipError_t wait(int on_copy, int e) override { return hipStreamWaitEvent(on_copy ? copy_s : compute, ev(e), 0); }
  hipError_t copy(int, int, void *dst, const void *src, size_t bytes) override {
    return hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, copy_s);
  }
  hipError_t attend(int, int, const FusedArgs &a, int *nk, int *nm) override { return launch_attn(a, compute, nk, nm); }
  hipError_t merge(const MergeArgs &m) override { return launch_merge(m, compute); }
};
struct TraceChain : Chain {
  ttkv_chain_op *ops;
  int32_t capacity, n;
  bool same_stream;
  TraceChain(ttkv_chain_op *o, int32_t cap, bool same) : ops(o), capacity(cap), n(0), same_stream(same) {}
  void put(int32_t kind, int on_copy, int32_t event, int32_t slot, int32_t fetch, uint64_t bytes) {
    if (n < capacity) ops[n] = ttkv_chain_op{kind, (on_copy && !same_stream) ? 1 : 0, event, slot, fetch, bytes};
    ++n;
  }
  hipError_t record(int e, int on_copy) override { put(TTKV_OP_RECORD, on_copy, e, -1, -1, 0); return hipSuccess; }
  hipError_t wait(int on_copy, int e) override { put(TTKV_OP_WAIT, on_copy, e, -1, -1, 0); return hipSuccess; }
  hipError_t copy(int fetch, int slot, void *, const void *, size_t bytes) override {
    put(TTKV_OP_COPY, 1, -1, slot, fetch, bytes);
    return hipSuccess;
  }
  hipError_t attend(int fetch, int slot, const FusedArgs &, int *nk, int *) override {
    put(TTKV_OP_ATTEND, 0, -1, slot, fetch, 0);
    *nk += 1;
    return hipSuccess;
  }
  hipError_t merge(const MergeArgs &) override { put(TTKV_OP_MERGE, 0, -1, -1, -1, 0); return hipSuccess; }
};

// Attention over the cached tokens and the merge.  k_new non-null: the step's new token as well, which the merge
// kernel adds and stores at the tail of tier 0 (an fp device tier of format new_fmt with room for it: the caller
// has checked); len[] of tier 0 then grows by one.
static ttkv_status decode_impl(Handle *h, const ttkv_cache *c, const void *q, int32_t q_fmt, float *out, float *lse,
                               const int32_t *sel_blocks, const int32_t *sel_count, int32_t sel_stride, void *workspace,
                               size_t ws_bytes, int32_t n_slots, void *compute_, void *copy_, const void *k_new,
                               const void *v_new, int32_t new_fmt, bool check_only = false, const DevSel *ds = nullptr,
                               Chain *trace = nullptr) {
  ttkv_status st = validate_cache(c, h ? h->check_tables : true);
  if (st != TTKV_OK) return st;
  if (!q || !out || (q_fmt != TTKV_F16 && q_fmt != TTKV_BF16)) return TTKV_ERR_INVALID_ARG;
  st = check_sel(c, sel_blocks, sel_count, sel_stride);
  if (st != TTKV_OK) return st;
  if (n_slots < 0 || n_slots > TTKV_MAX_SLOTS) return TTKV_ERR_INVALID_ARG;
  for (int t = 0; t < c->n_tiers; ++t) {
    const ttkv_tier &T = c->tier[t];
    if (T.k_fmt == TTKV_BF16 && q_fmt != TTKV_BF16) return TTKV_ERR_UNSUPPORTED;   // a bf16 tier takes bf16 queries
    if (n_slots == 0 && T.block_table && !T.block_table_dev) return TTKV_ERR_INVALID_ARG;
  }
  hipStream_t compute = (hipStream_t)compute_, copy = (hipStream_t)copy_;
  const bool staged = n_slots > 0;

  Plan &P = h->plan;
  build_plan(c, sel_blocks, sel_count, sel_stride, staged, h->target_items, &P, ds);
  if (P.status != TTKV_OK) return P.status;
  if (!workspace) return TTKV_ERR_WORKSPACE;
  // workspace = [n_slots staging slots][m][l][acc]
  const size_t slots_bytes = (size_t)n_slots * P.slot_bytes;
  const size_t rows = (size_t)c->batch * c->n_q_heads;
  const size_t mis = (256 - ((uintptr_t)workspace & 255)) & 255;
  if (ws_bytes < mis + slots_bytes) return TTKV_ERR_WORKSPACE;
  const int64_t stride = (int64_t)((ws_bytes - mis - slots_bytes) / (rows * 130 * sizeof(float)));
  if (stride < std::max(1, P.max_parts)) return TTKV_ERR_WORKSPACE;
  const int32_t part_stride = (int32_t)std::min<int64_t>(stride, 1 << 20);
  if (check_only) return TTKV_OK;   // nothing enqueued so far
  if (!trace && !P.fetch.empty() && copy != compute && (st = ensure_events(h)) != TTKV_OK) return st;
  HipChain hip_chain(h, compute, copy);
  Chain &ch = trace ? *trace : static_cast<Chain &>(hip_chain);
  uint8_t *ws = (uint8_t *)workspace + mis;
  float *pm = (float *)(ws + slots_bytes);
  float *pl = pm + rows * part_stride;
  float *pacc = pl + rows * part_stride;

  int nk = 0, nm = 0;
  FusedArgs a{};
  a.q = q;
  a.q_fmt = q_fmt;
  a.pm = pm; a.pl = pl; a.pacc = pacc;
  a.part_stride = part_stride;
  a.Hq = c->n_q_heads;
  a.Hkv = c->n_kv_heads;
  a.scale = c->softmax_scale;

  if (!P.fetch.empty() && copy != compute) {
    // staging slots may still be read by earlier work on `compute`
    TTKV_HIP(h, ch.record(EV_FENCE, 0));
    TTKV_HIP(h, ch.wait(1, EV_FENCE));
  }
  // every run that is attended in place goes into one launch (split only when the entry table is full)
  for (int t = 0; t < c->n_tiers; ++t) {
    const ttkv_tier &T = c->tier[t];
    a.tv[t] = make_view(T, make_layout(T, c->n_kv_heads));
    a.chunk[t] = P.chunk[t];
  }
  if (ds) {
    const ttkv_tier &T = c->tier[c->n_tiers - 1];
    a.sel_ids = ds->ids;
    for (int b = 0; b < c->batch; ++b) {
      const int64_t live_end = T.start[b] + T.len[b];
      a.sel_last_ntok[b] = T.len[b] ? (int32_t)(live_end - (live_end - 1) / T.block_tokens * T.block_tokens) : 0;
    }
  }
  const bool timed = !trace && h->time_on && h->time_n < h->time_max && !P.runs.empty();
  if (timed) TTKV_HIP(h, hipEventRecord(h->time_ev[2 * h->time_n], compute));
  // launch order: runs of host tiers first, so that the PCIe stream starts with the first workgroups
  // and the device-tier items fill the remaining slots while it runs
  std::vector<const Run *> &order = P.order;
  order.clear();
  for (int pass = 0; pass < 2; ++pass)
    for (const Run &r : P.runs)
      if ((c->tier[r.tier].mem == TTKV_MEM_HOST_PINNED) == (pass == 0)) order.push_back(&r);
  // a timed call may issue its launch(es) several times back to back (same arguments, same partials): the event
  // pair's own cost is then spread over them
  const int reps = timed ? std::max(1, h->time_repeat) : 1;
  if (timed) h->time_reps[h->time_n] = reps;
  for (int rep = 0; rep < reps; ++rep)
  for (size_t r0 = 0; r0 < order.size(); r0 += TTKV_MAX_ENTRIES) {
    const size_t r1 = std::min(order.size(), r0 + TTKV_MAX_ENTRIES);
    a.n_entries = (int32_t)(r1 - r0);
    int items = 0;
    for (size_t i = r0; i < r1; ++i) {
      const Run &r = *order[i];
      Entry &e = a.e[i - r0];
      e.tier_seq = (r.no_table ? (1 << 24) : 0) | (r.selected ? (1 << 25) : 0) | (r.tier << 16) | r.b;
      e.rec_base = r.rec_base;
      e.first_tok = r.first_tok;
      e.len = r.len;
      e.item_start = items;
      e.part_base = r.part_base;
      items += r.n_chunks;
    }
    a.n_items = items;
    TTKV_HIP(h, ch.attend(-1, -1, a, &nk, &nm));
  }
  if (timed) {
    TTKV_HIP(h, hipEventRecord(h->time_ev[2 * h->time_n + 1], compute));
    h->time_n += 1;
  }
  // staged host-tier blocks: copy i+1 overlaps compute on i
  int issued = 0;
  for (const Fetch &f : P.fetch) {
    const ttkv_tier &T = c->tier[f.tier];
    const Layout L = make_layout(T, c->n_kv_heads);
    const int slot = issued % n_slots;
    uint8_t *dst = ws + (size_t)slot * P.slot_bytes;
    // a slot is written again only after the kernel that read it has finished
    if (issued >= n_slots && copy != compute) TTKV_HIP(h, ch.wait(1, EV_FREED + slot));
    const size_t bytes = (size_t)f.nrec * L.rec_bytes;
    TTKV_HIP(h, ch.copy(issued, slot, dst, (const uint8_t *)T.data + f.rec * L.rec_bytes, bytes));
    if (copy != compute) {
      TTKV_HIP(h, ch.record(EV_READY + slot, 1));
      TTKV_HIP(h, ch.wait(0, EV_READY + slot));
    }
    a.tv[0] = make_slot_view(T, L, dst, f.nrec);
    a.chunk[0] = f.chunk;
    a.n_entries = 1;
    a.e[0].tier_seq = (1 << 24) | f.b;
    a.e[0].rec_base = 0;
    a.e[0].first_tok = 0;
    a.e[0].len = f.ntok;
    a.e[0].item_start = 0;
    a.e[0].part_base = f.part_base;
    a.n_items = (f.ntok + f.chunk - 1) / f.chunk;
    TTKV_HIP(h, ch.attend(issued, slot, a, &nk, &nm));
    if (copy != compute) TTKV_HIP(h, ch.record(EV_FREED + slot, 0));
    ++issued;
  }
  if (trace) {
    MergeArgs none{};
    TTKV_HIP(h, ch.merge(none));
    return TTKV_OK;                   // a recorded schedule: no statistics, no lengths
  }
  // host-tier traffic (Sec. 5.1 item 5): whole records, whether copied or read in place
  for (const Fetch &f : P.fetch) {
    h->stats.h2d_bytes += (uint64_t)f.nrec * make_layout(c->tier[f.tier], c->n_kv_heads).rec_bytes;
    h->stats.blocks_fetched += f.nrec;
  }
  for (const Run &r : P.runs) {
    const ttkv_tier &T = c->tier[r.tier];
    if (T.mem != TTKV_MEM_HOST_PINNED) continue;
    const int nrec = r.selected ? r.len : (r.len + T.block_tokens - 1) / T.block_tokens;
    h->stats.h2d_bytes += (uint64_t)nrec * make_layout(T, c->n_kv_heads).rec_bytes;
    h->stats.blocks_fetched += nrec;
  }
  MergeArgs m{};
  m.m = pm; m.l = pl; m.acc = pacc;
  m.n_parts = P.max_parts;
  m.part_stride = part_stride;
  m.rows = (int32_t)rows;
  m.n_parts_row = nullptr;
  m.rows_per_seq = c->n_q_heads;
  for (int b = 0; b < c->batch; ++b) m.cnt[b] = P.parts[b];
  m.out = out;
  m.lse = lse;
  if (k_new) {
    const ttkv_tier &T0 = c->tier[0];
    m.q = q; m.k_new = k_new; m.v_new = v_new;
    m.q_fmt = q_fmt; m.new_fmt = new_fmt;
    m.Hq = c->n_q_heads; m.Hkv = c->n_kv_heads;
    m.scale = c->softmax_scale;
    m.dst = make_view(T0, make_layout(T0, c->n_kv_heads));
    for (int b = 0; b < c->batch; ++b) m.new_tok[b] = (int32_t)((T0.start[b] + T0.len[b]) % ring_tokens(T0));
  }
  TTKV_HIP(h, ch.merge(m));
  if (k_new)
    for (int b = 0; b < c->batch; ++b) c->tier[0].len[b] += 1;
  h->stats.mfma_launches += nm;
  h->stats.kernels += nk + 1;
  return TTKV_OK;
}

ttkv_status ttkv_decode_attn(ttkv_handle hh, const ttkv_cache *c, const void *q, int32_t q_fmt, float *out, float *lse,
                             const int32_t *sel_blocks, const int32_t *sel_count, int32_t sel_stride, void *workspace,
                             size_t ws_bytes, int32_t n_slots, void *compute, void *copy) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h) return TTKV_ERR_INVALID_ARG;
  return decode_impl(h, c, q, q_fmt, out, lse, sel_blocks, sel_count, sel_stride, workspace, ws_bytes, n_slots, compute,
                     copy, nullptr, nullptr, 0);
}

ttkv_status ttkv_staged_schedule(ttkv_handle hh, const ttkv_cache *c, const int32_t *sel_blocks, const int32_t *sel_count,
                                 int32_t sel_stride, int32_t n_slots, int32_t same_stream, ttkv_chain_op *ops,
                                 int32_t capacity, int32_t *n_out) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h || !n_out || capacity < 0 || (capacity > 0 && !ops)) return TTKV_ERR_INVALID_ARG;
  TraceChain tc(ops, capacity, same_stream != 0);
  // no memory is touched: any non-null pointers do, and a workspace that is always large enough
  void *const fake = reinterpret_cast<void *>(256);
  void *const compute = reinterpret_cast<void *>(8), *const copy = same_stream ? compute : reinterpret_cast<void *>(16);
  const ttkv_status st = decode_impl(h, c, fake, TTKV_BF16, reinterpret_cast<float *>(fake), nullptr, sel_blocks, sel_count,
                                     sel_stride, fake, (size_t)1 << 46, n_slots, compute, copy, nullptr, nullptr, 0, false,
                                     nullptr, &tc);
  *n_out = tc.n;
  return st;
}

// Split partials of ttkv_decode_attn_noalloc: one array per GPU (every device that loads this code object holds
// its own copy at its own address), held until the process ends.  The name is a host-side stand-in: host code
// uses the address hipGetSymbolAddress returns for the current device, never the name.
static __device__ __align__(256) unsigned char scratch[TTKV_NOALLOC_SCRATCH_BYTES];
#define TTKV_MAX_DEVICES 64
static void *g_scratch_ptr[TTKV_MAX_DEVICES];
static std::mutex g_scratch_mutex;

// Address of the current device's `scratch`, looked up once per device.
static ttkv_status scratch_of_current_device(Handle *h, void **out) {
  int dev = -1;
  TTKV_HIP(h, hipGetDevice(&dev));
  if (dev < 0 || dev >= TTKV_MAX_DEVICES) return TTKV_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    TTKV_HIP(h, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return TTKV_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return TTKV_OK;
}

ttkv_status ttkv_decode_attn_noalloc(ttkv_handle hh, const ttkv_cache *c, const void *q, int32_t q_fmt, float *out,
                                     float *lse, const int32_t *sel_blocks, const int32_t *sel_count, int32_t sel_stride,
                                     void *stream) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h) return TTKV_ERR_INVALID_ARG;
  void *ws = nullptr;
  ttkv_status st = scratch_of_current_device(h, &ws);   // a lookup; enqueues nothing
  if (st != TTKV_OK) return st;
  // the partials need no clearing: every part the merge reads is written by this call's attention launch first
  return decode_impl(h, c, q, q_fmt, out, lse, sel_blocks, sel_count, sel_stride, ws, TTKV_NOALLOC_SCRATCH_BYTES, 0, stream,
                     stream, nullptr, nullptr, 0);
}

ttkv_status ttkv_decode_step(ttkv_handle hh, ttkv_cache *c, const void *q, int32_t q_fmt, const void *k_new,
                             const void *v_new, int32_t new_fmt, float *out, float *lse, const int32_t *sel_blocks,
                             const int32_t *sel_count, int32_t sel_stride, void *workspace, size_t ws_bytes,
                             int32_t n_slots, void *compute, void *copy) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h) return TTKV_ERR_INVALID_ARG;
  ttkv_status st = validate_cache(c, h->check_tables);
  if (st != TTKV_OK) return st;
  if (!k_new || !v_new || (new_fmt != TTKV_F16 && new_fmt != TTKV_BF16)) return TTKV_ERR_INVALID_ARG;
  ttkv_tier &T0 = c->tier[0];
  for (int b = 0; b < c->batch; ++b)
    if (T0.len[b] + 1 > ring_tokens(T0)) return TTKV_ERR_CAPACITY;
  const bool in_merge = T0.mem == TTKV_MEM_DEVICE && is_fp(T0.k_fmt) && T0.k_fmt == T0.v_fmt && !T0.k_sum;
  if (in_merge) {
    if (T0.k_fmt != new_fmt) return TTKV_ERR_UNSUPPORTED;   // an fp tier takes only its own format
    return decode_impl(h, c, q, q_fmt, out, lse, sel_blocks, sel_count, sel_stride, workspace, ws_bytes, n_slots, compute,
                       copy, k_new, v_new, new_fmt);
  }
  // any other first tier: the two calls.  What the second one checks before it enqueues is checked first, on the
  // lengths it will see, so that a refusal leaves the cache as it was.
  for (int b = 0; b < c->batch; ++b) T0.len[b] += 1;
  st = decode_impl(h, c, q, q_fmt, out, lse, sel_blocks, sel_count, sel_stride, workspace, ws_bytes, n_slots, compute, copy,
                   nullptr, nullptr, 0, true);
  for (int b = 0; b < c->batch; ++b) T0.len[b] -= 1;
  if (st != TTKV_OK) return st;
  st = append_impl(h, c, 0, -1, k_new, v_new, new_fmt, 1, 0, nullptr, 0, (hipStream_t)compute,
                   T0.mem == TTKV_MEM_HOST_PINNED);
  if (st != TTKV_OK) return st;
  return decode_impl(h, c, q, q_fmt, out, lse, sel_blocks, sel_count, sel_stride, workspace, ws_bytes, n_slots, compute,
                     copy, nullptr, nullptr, 0);
}

ttkv_status ttkv_merge_partials(ttkv_handle hh, const float *m, const float *l, const float *acc, int32_t n_parts,
                                int32_t part_stride, const int32_t *n_parts_row, int32_t rows, float *out, float *lse,
                                void *stream) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h || !m || !l || !acc || !out || n_parts < 0 || part_stride < n_parts || rows < 0) return TTKV_ERR_INVALID_ARG;
  MergeArgs a{};
  a.m = m; a.l = l; a.acc = acc;
  a.n_parts = n_parts;
  a.part_stride = part_stride;
  a.rows = rows;
  a.n_parts_row = n_parts_row;
  a.rows_per_seq = 0;
  a.out = out;
  a.lse = lse;
  TTKV_HIP(h, launch_merge(a, (hipStream_t)stream));
  h->stats.kernels += rows > 0;
  return TTKV_OK;
}

// Scores and top-k of the last tier's live blocks, enqueued on `stream`; the result stays on the device:
// counts at sel_out[0 .. batch), ids of sequence b at sel_out[batch + b * sel_stride ...].
static ttkv_status enqueue_select(Handle *h, const ttkv_cache *c, const void *q, int32_t q_fmt, int32_t k, int32_t sel_stride,
                                  void *scratch, size_t scratch_bytes, hipStream_t stream, int32_t **sel_out) {
  if (!q || (q_fmt != TTKV_F16 && q_fmt != TTKV_BF16) || k < 0 || sel_stride < 1) return TTKV_ERR_INVALID_ARG;
  const ttkv_tier &T = c->tier[c->n_tiers - 1];
  if (!T.k_summary) return TTKV_ERR_UNSUPPORTED;
  SelectArgs a{};
  a.q = q;
  a.q_fmt = q_fmt;
  a.k_summary = (const uint16_t *)T.k_summary;
  a.table = T.block_table_dev;
  a.ring_blocks = (int32_t)T.ring_blocks;
  a.Hq = c->n_q_heads;
  a.Hkv = c->n_kv_heads;
  a.k = std::min(k, sel_stride);
  a.sel_stride = sel_stride;
  a.n_seq = c->batch;
  a.max_blocks = 1;
  for (int b = 0; b < c->batch; ++b) {
    const int64_t first_id = T.start[b] / T.block_tokens;
    const int64_t end_id = (T.start[b] + T.len[b] + T.block_tokens - 1) / T.block_tokens;
    a.rec_base[b] = (int32_t)((int64_t)b * T.ring_blocks);
    a.first_block[b] = (int32_t)(first_id % T.ring_blocks);
    a.first_block_id[b] = first_id;
    a.n_blocks[b] = (int32_t)(end_id - first_id);
    a.max_blocks = std::max(a.max_blocks, a.n_blocks[b]);
  }
  if (a.max_blocks > 1024) return TTKV_ERR_UNSUPPORTED;
  const size_t need = align256((size_t)c->batch * a.max_blocks * sizeof(float)) + (size_t)c->batch * (sel_stride + 1) * sizeof(int32_t);
  if (!scratch || scratch_bytes < need) return TTKV_ERR_WORKSPACE;
  a.scores = (float *)scratch;
  a.sel_out = (int32_t *)((uint8_t *)scratch + align256((size_t)c->batch * a.max_blocks * sizeof(float)));
  TTKV_HIP(h, launch_select(a, stream));
  h->stats.kernels += 2;
  *sel_out = a.sel_out;
  return TTKV_OK;
}

ttkv_status ttkv_select_blocks(ttkv_handle hh, const ttkv_cache *c, const void *q, int32_t q_fmt, int32_t k,
                               int32_t *sel_blocks, int32_t *sel_count, int32_t sel_stride, void *scratch,
                               size_t scratch_bytes, void *stream_) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h) return TTKV_ERR_INVALID_ARG;
  ttkv_status st = validate_cache(c, h->check_tables);
  if (st != TTKV_OK) return st;
  if (!sel_blocks || !sel_count) return TTKV_ERR_INVALID_ARG;
  hipStream_t stream = (hipStream_t)stream_;
  int32_t *sel_out = nullptr;
  st = enqueue_select(h, c, q, q_fmt, k, sel_stride, scratch, scratch_bytes, stream, &sel_out);
  if (st != TTKV_OK) return st;
  // sel_out = [batch counts][batch][sel_stride ids]
  TTKV_HIP(h, hipMemcpyAsync(sel_count, sel_out, (size_t)c->batch * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
  TTKV_HIP(h, hipMemcpyAsync(sel_blocks, sel_out + c->batch, (size_t)c->batch * sel_stride * sizeof(int32_t),
                             hipMemcpyDeviceToHost, stream));
  TTKV_HIP(h, hipStreamSynchronize(stream));
  return TTKV_OK;
}

ttkv_status ttkv_decode_step_topk(ttkv_handle hh, ttkv_cache *c, const void *q, int32_t q_fmt, const void *k_new,
                                  const void *v_new, int32_t new_fmt, float *out, float *lse, int32_t k,
                                  int32_t *sel_blocks_out, int32_t *sel_count_out, int32_t sel_stride, void *sel_scratch,
                                  size_t sel_scratch_bytes, void *workspace, size_t ws_bytes, void *stream_) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h) return TTKV_ERR_INVALID_ARG;
  ttkv_status st = validate_cache(c, h->check_tables);
  if (st != TTKV_OK) return st;
  if ((k_new == nullptr) != (v_new == nullptr) || (sel_blocks_out == nullptr) != (sel_count_out == nullptr))
    return TTKV_ERR_INVALID_ARG;
  if (k < 0 || sel_stride < 1) return TTKV_ERR_INVALID_ARG;
  const ttkv_tier &TL = c->tier[c->n_tiers - 1];
  if (!TL.k_summary) return TTKV_ERR_UNSUPPORTED;
  if (TL.block_table && !TL.block_table_dev) return TTKV_ERR_INVALID_ARG;   // the kernels look the records up
  ttkv_tier &T0 = c->tier[0];
  if (k_new) {
    if (new_fmt != TTKV_F16 && new_fmt != TTKV_BF16) return TTKV_ERR_INVALID_ARG;
    // the new token goes through the merge kernel: an fp device tier of its format (ttkv_decode_step's other
    // first tiers would need their own append call first)
    if (!(T0.mem == TTKV_MEM_DEVICE && is_fp(T0.k_fmt) && T0.k_fmt == T0.v_fmt && !T0.k_sum) || T0.k_fmt != new_fmt)
      return TTKV_ERR_UNSUPPORTED;
    for (int b = 0; b < c->batch; ++b)
      if (T0.len[b] + 1 > ring_tokens(T0)) return TTKV_ERR_CAPACITY;
  }
  hipStream_t stream = (hipStream_t)stream_;
  // everything the attention call checks before it enqueues, first: nothing is enqueued on a refusal
  DevSel probe{nullptr, k, sel_stride};
  st = decode_impl(h, c, q, q_fmt, out, lse, nullptr, nullptr, 0, workspace, ws_bytes, 0, stream_, stream_, k_new, v_new, new_fmt,
                   true, &probe);
  if (st != TTKV_OK) return st;
  int32_t *sel_out = nullptr;
  st = enqueue_select(h, c, q, q_fmt, k, sel_stride, sel_scratch, sel_scratch_bytes, stream, &sel_out);
  if (st != TTKV_OK) return st;
  const DevSel ds{sel_out + c->batch, k, sel_stride};
  st = decode_impl(h, c, q, q_fmt, out, lse, nullptr, nullptr, 0, workspace, ws_bytes, 0, stream_, stream_, k_new, v_new,
                   new_fmt, false, &ds);
  if (st != TTKV_OK) return st;
  if (sel_blocks_out) {   // for the caller's information, behind the attention; valid once `stream` has drained
    TTKV_HIP(h, hipMemcpyAsync(sel_count_out, sel_out, (size_t)c->batch * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
    TTKV_HIP(h, hipMemcpyAsync(sel_blocks_out, sel_out + c->batch, (size_t)c->batch * sel_stride * sizeof(int32_t),
                               hipMemcpyDeviceToHost, stream));
  }
  return TTKV_OK;
}

ttkv_status ttkv_set_table_check(ttkv_handle hh, int32_t on) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h || (on != 0 && on != 1)) return TTKV_ERR_INVALID_ARG;
  h->check_tables = on != 0;
  return TTKV_OK;
}

ttkv_status ttkv_set_split(ttkv_handle hh, int32_t target_items) {
  Handle *h = reinterpret_cast<Handle *>(hh);
  if (!h || target_items < 0 || target_items > (1 << 20)) return TTKV_ERR_INVALID_ARG;
  h->target_items = target_items;
  return TTKV_OK;
}

}  // extern "C"
