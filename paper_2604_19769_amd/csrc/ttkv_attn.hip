// Split-K decode attention partials over every tier in ONE launch (Alg. 1: Attn on
// the fast tier, Decompress + Attn per slow-tier block) and the log-sum-exp merge
// of the partials (the "+" of Alg. 1, normalised once at the end).
//
// Work item = (tier, sequence, chunk of tokens, KV head[, pair of query heads]); one
// workgroup of four wave64 per item, each wave streaming 1/4 of the chunk's tiles.
// This is the kernel for one query head per KV head; launches with two or more go to
// the matrix-core kernel where its cases take the formats, else here in head pairs.
//
// Lane mapping: a K or V row of one token-head is ROWB bytes = LPT lanes x 16 B, so
// one 128-bit load per lane brings TPL = 64/LPT whole rows per wave, fully
// coalesced.  Lane L holds elements [slice*EPL, +EPL) of token L/LPT.  The lane
// that owns a token's K slice also owns its V slice, so softmax weights never
// leave their lane (K 8-bit + V 4-bit needs one lane shuffle per V row).
//
// Arithmetic: codes are never expanded to fp32.  int4 nibbles and int8 bytes are
// spliced into the mantissa of an fp16 constant (1024+n, 64+n, 1152+c), giving
// packed half pairs for v_dot2_f32_f16 (q.k) and v_fma_mix_f32 (p.v); the known
// offsets and the per-group scale/zero are factored out of the inner loops:
//   q.k  = s_g * (sum_i q_i (c_i + o_i) - sum_i q_i o_i) + z_g * sum_i q_i
//   sum_t p_t v_t = sum_t (p_t s_t)(c_t + o) - o * sum_t p_t s_t + sum_t p_t z_t
// Accumulation is fp32 throughout.  Query values are held as fp16 for the fp16 and
// quantized tiers (bf16 queries are converted; |q| must stay below 65504) and as
// bf16 pairs for the bf16 tier.  Keys grouped over 128 tokens per channel fold the
// token group's scales into the queries per tile (see process).
//
// K/V bytes are read once per launch: the tile loads carry the non-temporal hint.
//
// The host tier needs no separate path: pinned host memory is read by the same
// loads (PCIe reads in flight while other waves compute), or from a staging slot
// in HBM when the caller asks for explicit block copies.
#include "ttkv_attn_dev.h"

#include <type_traits>

namespace ttkv {

namespace {

using namespace dev;

// Everything one wave accumulates for one item.
template <int KF, int VF, int G>
__device__ __forceinline__ void process(const FusedArgs &a, const TierView &tv, const Entry &en, const int32_t *sel,
                                        int chunk_tokens, int chunk, int seq, int hkv, int hq0, float (*s_acc)[4][G][128],
                                        float (*s_m)[G], float (*s_l)[G]) {
  // sel: null, or the block ids behind a run made of selected blocks (ring block of token i: sel[i / bt])
  using FK = Fmt<KF>;
  using FV = Fmt<VF>;
  static_assert(FV::TPL % FK::TPL == 0, "V rows must not be wider than K rows");
  constexpr int TT = 4 * FK::TPL;          // tokens per wave tile
  constexpr int NLK = 4;                   // K loads per lane per tile
  constexpr int NLV = TT / FV::TPL;        // V loads per lane per tile
  constexpr int R = FV::TPL / FK::TPL;     // K loads covered by one V load
  constexpr int QN = FK::EPL / 2;          // packed q registers per head
  constexpr bool KT = KF == TTKV_I4_ASYM_T128;   // keys grouped over 128 tokens per channel: scale folds into q
  constexpr bool KQ = (KF == TTKV_I8_SYM_G32 || KF == TTKV_I4_ASYM_G64 || KT);
  constexpr bool VQ = (VF == TTKV_I8_SYM_G32 || VF == TTKV_I4_ASYM_G64);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c0 = chunk * chunk_tokens;
  const int c1 = min(en.len, c0 + chunk_tokens);
  const int ring_tokens = tv.ring_blocks * tv.bt;
  const int kslice = lane % FK::LPT, ktok = lane / FK::LPT;
  const int vslice = lane % FV::LPT, vtok = lane / FV::LPT;
  const float cs = a.scale * kLog2e;       // scores are kept in the log2 domain

  // ---- q slice of this lane, packed to match unpack16<KF>; offset and plain sums for the factored terms
  uint32_t qp[G][QN];
  float qoff[G], qsum[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    // EPL 16-bit values = EPL/8 aligned 128-bit loads; one wave-uniform branch on the query type
    const uint4 *qsrc = (const uint4 *)((const uint16_t *)a.q + ((int64_t)seq * a.Hq + hq0 + g) * 128 + kslice * FK::EPL);
    uint32_t qw[FK::EPL / 2];
#pragma unroll
    for (int i = 0; i < FK::EPL / 8; ++i) {
      const uint4 w = qsrc[i];
      qw[4 * i] = w.x; qw[4 * i + 1] = w.y; qw[4 * i + 2] = w.z; qw[4 * i + 3] = w.w;
    }
    if constexpr (KF != TTKV_BF16) {
      if (a.q_fmt == TTKV_BF16) {   // bf16 -> fp16 (exact inside the fp16 normal range, clamped outside)
#pragma unroll
        for (int i = 0; i < FK::EPL / 2; ++i) {
          const float lo = fminf(fmaxf(__uint_as_float(qw[i] << 16), -65504.0f), 65504.0f);
          const float hi = fminf(fmaxf(__uint_as_float(qw[i] & 0xffff0000u), -65504.0f), 65504.0f);
          qw[i] = (uint32_t)__half_as_ushort(__float2half_rn(lo)) | ((uint32_t)__half_as_ushort(__float2half_rn(hi)) << 16);
        }
      }
    }
    uint16_t qb[FK::EPL];
    float so = 0.0f, ss = 0.0f;
#pragma unroll
    for (int e = 0; e < FK::EPL; ++e) {
      qb[e] = (uint16_t)(qw[e / 2] >> (16 * (e % 2)));
      const float v = KF == TTKV_BF16 ? __uint_as_float((uint32_t)qb[e] << 16) : h2f(qb[e]);
      ss += v;
      so = fmaf(v, elem_offset<KF>(e), so);
    }
#pragma unroll
    for (int r = 0; r < QN; ++r) qp[g][r] = 0;
#pragma unroll
    for (int e = 0; e < FK::EPL; ++e) qp[g][pair_reg<KF>(e)] |= (uint32_t)qb[e] << (16 * pair_half<KF>(e));
    qoff[g] = so;
    qsum[g] = ss * cs;
  }

  float m[G], l[G], zacc[G], psum[G];
  float acc[G][FV::EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = zacc[g] = psum[g] = 0.0f;
#pragma unroll
    for (int e = 0; e < FV::EPL; ++e) acc[g][e] = 0.0f;
  }

  Splice sp;
  sp.init();
  // per-lane byte offsets of its row slice inside a tile's sections (loop invariant)
  const uint32_t kvoff = ktok * FK::ROWB + kslice * 16, vvoff = vtok * FV::ROWB + vslice * 16;
  const uint32_t kmoff = ktok * 8 + (kslice >> 1) * (KF == TTKV_I8_SYM_G32 ? 2 : 4);
  const uint32_t vmoff = vtok * 8 + (vslice >> 1) * (VF == TTKV_I8_SYM_G32 ? 2 : 4);

  // Registers of one tile of TT tokens in flight.
  struct TileRegs {
    uint4 kw[NLK], vw[NLV];
    uint32_t kmeta[NLK], vmeta[NLV];
    uint4 gm[KT ? 8 : 1];   // KT: {scale, zero} of the lane's 32 channels for the tile's token group
  };

  // Issue every load of the tile at i0.  FULL: every row is live (no clamping).
  auto load_tile = [&](TileRegs &t, int i0, int nv, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    int tok0 = en.first_tok + i0;
    if (tok0 >= ring_tokens) tok0 -= ring_tokens;
    int rb = tok0 / tv.bt;
    const int row0 = tok0 - rb * tv.bt;
    if (sel) rb = sel[rb] % tv.ring_blocks;
    const int64_t rec = tv.table ? (int64_t)tv.table[(int64_t)seq * tv.ring_blocks + rb] : (int64_t)en.rec_base + rb;
    const uint8_t *head = tv.base + rec * tv.rec_bytes + (int64_t)hkv * tv.head_bytes;
    // wave-uniform section bases of the tile + per-lane 32-bit offsets: the loads below can
    // use the scalar-base + vector-offset + immediate addressing form
    const uint8_t *kb = head + row0 * FK::ROWB, *kmb = head + tv.k_meta_off + row0 * 8;
    const uint8_t *vb = head + tv.v_off + row0 * FV::ROWB, *vmb = head + tv.v_meta_off + row0 * 8;
    constexpr uint32_t KMW = KF == TTKV_I8_SYM_G32 ? 2 : 4, VMW = VF == TTKV_I8_SYM_G32 ? 2 : 4;
    if constexpr (KT) {   // a tile of 64 tokens lies inside one aligned group of 128: its 128 meta rows x 4 B
      const uint4 *g = (const uint4 *)(head + tv.k_meta_off + (row0 & ~127) * 4 + kslice * 128);
#pragma unroll
      for (int i = 0; i < 8; ++i) t.gm[i] = g[i];
    }
#pragma unroll
    for (int n = 0; n < NLK; ++n) {
      const uint32_t r = FULL ? n * FK::TPL + ktok : min(n * FK::TPL + ktok, nv - 1);
      const uint32_t co = FULL ? kvoff + n * FK::TPL * FK::ROWB : r * FK::ROWB + kslice * 16;
      const uint32_t mo = FULL ? kmoff + n * FK::TPL * 8 : r * 8 + (kslice >> 1) * KMW;
      t.kw[n] = ld_stream((const uint4 *)(kb + co));
      if constexpr (KF == TTKV_I8_SYM_G32)
        t.kmeta[n] = ld_stream((const uint16_t *)(kmb + mo));
      else if constexpr (KF == TTKV_I4_ASYM_G64)
        t.kmeta[n] = ld_stream((const uint32_t *)(kmb + mo));
    }
#pragma unroll
    for (int n = 0; n < NLV; ++n) {
      const uint32_t r = FULL ? n * FV::TPL + vtok : min(n * FV::TPL + vtok, nv - 1);
      const uint32_t co = FULL ? vvoff + n * FV::TPL * FV::ROWB : r * FV::ROWB + vslice * 16;
      const uint32_t mo = FULL ? vmoff + n * FV::TPL * 8 : r * 8 + (vslice >> 1) * VMW;
      t.vw[n] = ld_stream((const uint4 *)(vb + co));
      if constexpr (VF == TTKV_I8_SYM_G32)
        t.vmeta[n] = ld_stream((const uint16_t *)(vmb + mo));
      else if constexpr (VF == TTKV_I4_ASYM_G64)
        t.vmeta[n] = ld_stream((const uint32_t *)(vmb + mo));
    }
  };

  // Scores, online softmax and weighted V of one loaded tile.
  auto compute_tile = [&](const TileRegs &t, int nv, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    const uint4 *kw = t.kw, *vw = t.vw;
    const uint32_t *kmeta = t.kmeta, *vmeta = t.vmeta;
    (void)kmeta; (void)vmeta;

    // ---- KT: q . k = sum_d (q_d s_d) (c_d - 8) + sum_d q_d (z_d + 8 s_d) with s, z of the tile's token group.
    // q_d s_d (22 significant bits) is carried as two fp16 values, the rounded product and its exact remainder
    // (one fused multiply-add), so the scores keep fp32 accuracy; the sums over q s and q z are exact products
    // accumulated in fp32.
    uint32_t qsh_[KT ? G : 1][KT ? QN : 1], qsl_[KT ? G : 1][KT ? QN : 1];
    float qoff_t[KT ? G : 1];
    if constexpr (KT) {
      uint32_t sp2[QN], zp2[QN];
#pragma unroll
      for (int dd = 0; dd < 4; ++dd) {
        const uint32_t m8[8] = {t.gm[2 * dd].x, t.gm[2 * dd].y, t.gm[2 * dd].z, t.gm[2 * dd].w,
                                t.gm[2 * dd + 1].x, t.gm[2 * dd + 1].y, t.gm[2 * dd + 1].z, t.gm[2 * dd + 1].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {   // pair register 4 dd + j holds channels (8 dd + j, 8 dd + j + 4)
          sp2[4 * dd + j] = __builtin_amdgcn_perm(m8[j + 4], m8[j], 0x05040100u);
          zp2[4 * dd + j] = __builtin_amdgcn_perm(m8[j + 4], m8[j], 0x07060302u);
        }
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float se = 0.0f, so = 0.0f, qz = 0.0f;   // sum q s over the registers with splice offset 1024 / 64, sum q z
#pragma unroll
        for (int r = 0; r < QN; ++r) {
          const h2 q2 = as_h2(qp[g][r]), s2 = as_h2(sp2[r]);
          const h2 hi = q2 * s2;
          const h2 lo = __builtin_elementwise_fma(q2, s2, -hi);
          qsh_[g][r] = __builtin_bit_cast(uint32_t, hi);
          qsl_[g][r] = __builtin_bit_cast(uint32_t, lo);
          if (r & 1) so = __builtin_amdgcn_fdot2(q2, s2, so, false);
          else se = __builtin_amdgcn_fdot2(q2, s2, se, false);
          qz = __builtin_amdgcn_fdot2(q2, as_h2(zp2[r]), qz, false);
        }
        // what leaves with the initial value: splice offsets 1024 / 64 plus the centre 8, minus the zero-point sum
        qoff_t[g] = fmaf(1032.0f, se, 72.0f * so) - fmaf(8.0f, se + so, qz);
      }
    }

    // ---- scores (log2 domain)
    float s[G][NLK];
#pragma unroll
    for (int n = 0; n < NLK; ++n) {
      uint32_t kr[QN];
      unpack16<KF>(kw[n], kr, sp);
      float ks = cs, kz = 0.0f;
      if constexpr (KF == TTKV_I8_SYM_G32) ks = h2f((uint16_t)kmeta[n]) * cs;
      if constexpr (KF == TTKV_I4_ASYM_G64) {
        ks = h2f((uint16_t)(kmeta[n] & 0xffff)) * cs;
        kz = h2f((uint16_t)(kmeta[n] >> 16));
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d0 = KT ? -qoff_t[g] : (KQ ? -qoff[g] : 0.0f), d1 = 0.0f;   // the splice offsets leave with the initial value
#pragma unroll
        for (int r = 0; r < QN; r += 2) {
          if constexpr (KF == TTKV_BF16) {
            d0 = __builtin_amdgcn_fdot2_f32_bf16(as_b2(kr[r]), as_b2(qp[g][r]), d0, false);
            d1 = __builtin_amdgcn_fdot2_f32_bf16(as_b2(kr[r + 1]), as_b2(qp[g][r + 1]), d1, false);
          } else {
            d0 = __builtin_amdgcn_fdot2(as_h2(kr[r]), as_h2(KT ? qsh_[g][r] : qp[g][r]), d0, false);
            d1 = __builtin_amdgcn_fdot2(as_h2(kr[r + 1]), as_h2(KT ? qsh_[g][r + 1] : qp[g][r + 1]), d1, false);
            if constexpr (KT) {
              d0 = __builtin_amdgcn_fdot2(as_h2(kr[r]), as_h2(qsl_[g][r]), d0, false);
              d1 = __builtin_amdgcn_fdot2(as_h2(kr[r + 1]), as_h2(qsl_[g][r + 1]), d1, false);
            }
          }
        }
        float d = (d0 + d1) * ks;
        if constexpr (KF == TTKV_I4_ASYM_G64) d = fmaf(kz, qsum[g], d);
        d = group_sum<FK::LPT>(d);
        s[g][n] = (FULL || n * FK::TPL + ktok < nv) ? d : -INFINITY;
      }
    }

    // ---- online softmax (base 2)
    float p[G][NLK];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mt = fmaxf(fmaxf(s[g][0], s[g][1]), fmaxf(s[g][2], s[g][3]));
      mt = wave_max(mt);
      if (mt > m[g]) {  // wave-uniform
        const float alpha = __builtin_amdgcn_exp2f(m[g] - mt);
        l[g] *= alpha;
        zacc[g] *= alpha;
        psum[g] *= alpha;
#pragma unroll
        for (int e = 0; e < FV::EPL; ++e) acc[g][e] *= alpha;
        m[g] = mt;
      }
      float ps = 0.0f;
#pragma unroll
      for (int n = 0; n < NLK; ++n) {
        p[g][n] = __builtin_amdgcn_exp2f(s[g][n] - m[g]);
        ps += p[g][n];
      }
      if (kslice == 0) l[g] += ps;
    }

    // ---- weighted V
#pragma unroll
    for (int n = 0; n < NLV; ++n) {
      uint32_t vr[FV::EPL / 2];
      unpack16<VF>(vw[n], vr, sp);
      float vs = 1.0f, vz = 0.0f;
      if constexpr (VF == TTKV_I8_SYM_G32) vs = h2f((uint16_t)vmeta[n]);
      if constexpr (VF == TTKV_I4_ASYM_G64) {
        vs = h2f((uint16_t)(vmeta[n] & 0xffff));
        vz = h2f((uint16_t)(vmeta[n] >> 16));
      }
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float pv;   // 0 for rows past the end of the chunk: their score is -inf
        if constexpr (R == 1) {
          pv = p[g][n];
        } else {
          // token n*TPL_V + vtok sits in K load n*R + vtok / TPL_K, lane group vtok % TPL_K
          const int src = (vtok % FK::TPL) * FK::LPT;
          pv = 0.0f;
#pragma unroll
          for (int rr = 0; rr < R; ++rr) {
            const float cand = __shfl(p[g][n * R + rr], src);
            if (vtok / FK::TPL == rr) pv = cand;
          }
        }
        if constexpr (VF == TTKV_I4_ASYM_G64) zacc[g] = fmaf(pv, vz, zacc[g]);
        if constexpr (VQ) {
          pv *= vs;
          psum[g] += pv;
        }
#pragma unroll
        for (int e = 0; e < FV::EPL; ++e) {
          const uint32_t reg = vr[pair_reg<VF>(e)];
          float x;
          if constexpr (VF == TTKV_BF16)
            x = pair_half<VF>(e) ? __uint_as_float(reg & 0xffff0000u) : __uint_as_float(reg << 16);
          else
            x = pair_half<VF>(e) ? (float)as_h2(reg).y : (float)as_h2(reg).x;
          acc[g][e] = fmaf(x, pv, acc[g][e]);
        }
      }
    }
  };

  {
    TileRegs ra;
    int i0 = c0 + wave * TT;
    for (; i0 + TT <= c1; i0 += 4 * TT) {
      load_tile(ra, i0, TT, std::true_type{});
      compute_tile(ra, TT, std::true_type{});
    }
    if (i0 < c1) {
      load_tile(ra, i0, c1 - i0, std::false_type{});
      compute_tile(ra, c1 - i0, std::false_type{});
    }
  }

  // ---- reduce: lanes with the same V slice hold sums over different tokens.  Within a
  // row of 16 lanes by DPP rotations, across the 4 rows and 4 waves through LDS.
#pragma unroll
  for (int g = 0; g < G; ++g) {
    l[g] = wave_sum(l[g]);
#pragma unroll
    for (int e = 0; e < FV::EPL; ++e) {
      float v = acc[g][e] + zacc[g];
      if constexpr (VQ) v = fmaf(-elem_offset<VF>(e), psum[g], v);
      if constexpr (FV::LPT <= 4) v += dpp<0x124>(v);   // row_ror:4
      if constexpr (FV::LPT <= 8) v += dpp<0x128>(v);   // row_ror:8  (after ror:4 this completes the 4-lane stride sum)
      acc[g][e] = v;
    }
    if ((lane & 15) < FV::LPT) {
#pragma unroll
      for (int e = 0; e < FV::EPL; ++e) s_acc[wave][lane >> 4][g][vslice * FV::EPL + e] = acc[g][e];
    }
    if (lane == 0) {
      s_m[wave][g] = m[g];
      s_l[wave][g] = l[g];
    }
  }
}

// T128: the launch contains a tier whose keys are grouped over 128 tokens per channel.  That case holds 32 more
// registers per tile (the group's scales and zeros), so it is compiled into an instantiation of its own and the
// other formats keep their occupancy.
template <int G, bool T128>
__global__ __launch_bounds__(256) void attn_fused_kernel(const FusedArgs a) {
  __shared__ float s_acc[4][4][G][128];   // [wave][row of 16 lanes][head][channel]
  __shared__ float s_m[4][G], s_l[4][G];

  // Linear workgroup id -> (item, KV head, query-head group).  Workgroups are dealt round-robin
  // to the 8 XCDs (id % 8), each with its own L2: the groups of one (item, KV head), which read
  // the same K/V bytes, get ids 8 apart so that they land on the same XCD at the same time and
  // the second reader is served from that L2.
  const int Gtot = a.Hq / a.Hkv;
  const uint32_t n_hz = Gtot / G;
  const uint32_t id = blockIdx.x;
  const uint32_t base = ((id >> 3) / n_hz) * 8 + (id & 7);
  if (base >= (uint32_t)a.n_items * a.Hkv) return;
  const int item = base / a.Hkv;
  const int hkv = base % a.Hkv;
  const int hq0 = hkv * Gtot + ((id >> 3) % n_hz) * G;

  int lo = 0, hi = a.n_entries - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (a.e[mid].item_start <= item) lo = mid; else hi = mid - 1;
  }
  Entry en = a.e[lo];
  const int tier = (en.tier_seq >> 16) & 0xff, seq = en.tier_seq & 0xffff;
  TierView tv = a.tv[tier];
  if (en.tier_seq & (1 << 24)) tv.table = nullptr;   // the run names pool records directly
  int chunk_tokens = a.chunk[tier];
  const bool equal_items = chunk_tokens == 0;
  if (equal_items) chunk_tokens = even_chunk(en.len, (lo + 1 < a.n_entries ? a.e[lo + 1].item_start : a.n_items) - en.item_start);
  const int part = en.part_base + item - en.item_start;   // this item's partial
  int chunk = item - en.item_start;
  const int32_t *sel = resolve_selected(a, tv, en, seq, equal_items, chunk_tokens, chunk);

  const int combo = tv.k_fmt * 8 + tv.v_fmt;
  switch (combo) {
    case TTKV_F16 * 8 + TTKV_F16:
      process<TTKV_F16, TTKV_F16, G>(a, tv, en, sel, chunk_tokens, chunk, seq, hkv, hq0, s_acc, s_m, s_l);
      break;
    case TTKV_BF16 * 8 + TTKV_BF16:
      process<TTKV_BF16, TTKV_BF16, G>(a, tv, en, sel, chunk_tokens, chunk, seq, hkv, hq0, s_acc, s_m, s_l);
      break;
    case TTKV_I8_SYM_G32 * 8 + TTKV_I8_SYM_G32:
      process<TTKV_I8_SYM_G32, TTKV_I8_SYM_G32, G>(a, tv, en, sel, chunk_tokens, chunk, seq, hkv, hq0, s_acc, s_m, s_l);
      break;
    case TTKV_I4_ASYM_G64 * 8 + TTKV_I4_ASYM_G64:
      process<TTKV_I4_ASYM_G64, TTKV_I4_ASYM_G64, G>(a, tv, en, sel, chunk_tokens, chunk, seq, hkv, hq0, s_acc, s_m, s_l);
      break;
    case TTKV_I4_ASYM_T128 * 8 + TTKV_I4_ASYM_G64:
      if constexpr (T128)
        process<TTKV_I4_ASYM_T128, TTKV_I4_ASYM_G64, G>(a, tv, en, sel, chunk_tokens, chunk, seq, hkv, hq0, s_acc, s_m, s_l);
      break;
    default:
      process<TTKV_I8_SYM_G32, TTKV_I4_ASYM_G64, G>(a, tv, en, sel, chunk_tokens, chunk, seq, hkv, hq0, s_acc, s_m, s_l);
      break;
  }
  __syncthreads();

  // ---- merge the four waves (each with its own running max) and write the item's partial
  for (int idx = threadIdx.x; idx < G * 128; idx += 256) {
    const int g = idx >> 7, dch = idx & 127;
    const float M = fmaxf(fmaxf(s_m[0][g], s_m[1][g]), fmaxf(s_m[2][g], s_m[3][g]));
    float o = 0.0f, ll = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = s_m[w][g] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(s_m[w][g] - M);
      const float rows = (s_acc[w][0][g][dch] + s_acc[w][1][g][dch]) + (s_acc[w][2][g][dch] + s_acc[w][3][g][dch]);
      o = fmaf(rows, wgt, o);
      ll = fmaf(s_l[w][g], wgt, ll);
    }
    const int64_t prow = ((int64_t)seq * a.Hq + hq0 + g) * a.part_stride + part;
    a.pacc[prow * 128 + dch] = o;
    if (dch == 0) {
      a.pm[prow] = M * kLn2;  // natural-log units outside the kernel
      a.pl[prow] = ll;
    }
  }
}

// One workgroup of 256 threads per row: thread = channel, the parts split over the two halves of the workgroup.
// The kernel is a chain of memory latencies, so each part's (m, l) is loaded once, by thread p of its half; the
// half's maximum and the weights e^(m_p - M) go through LDS, and the acc loads (independent of them) are issued
// eight at a time, the first eight before anything else.
// With a new token (Alg. 1 appends it before attending) the row's own term is formed here from q, k_new and
// v_new, and the first query head of each KV head stores the token's row at the tail of tier 0: the attention
// kernels then run over the tokens already cached and a step needs no launch of its own for the append.
__global__ __launch_bounds__(256) void merge_kernel(const MergeArgs a) {
  __shared__ float s_o[128], s_w[2][128], s_hm[4], s_hl[4], s_dot[4];
  const int row = blockIdx.x, dch = threadIdx.x & 127, half = threadIdx.x >> 7, wave = threadIdx.x >> 6;
  int n = a.n_parts;
  if (a.n_parts_row)
    n = a.n_parts_row[row];
  else if (a.rows_per_seq > 0)
    n = a.cnt[row / a.rows_per_seq];
  const float *pm = a.m + (int64_t)row * a.part_stride;
  const float *pl = a.l + (int64_t)row * a.part_stride;
  const float *pa = a.acc + (int64_t)row * a.part_stride * 128 + dch;
  const int p0 = half ? (n + 1) / 2 : 0, p1 = half ? n : (n + 1) / 2;
  const int nb = ((n + 1) / 2 + 127) / 128;   // batches of 128 parts: the same count in both halves (barriers inside)
  constexpr int U = 8;
  float av[U];
#pragma unroll
  for (int u = 0; u < U; ++u) av[u] = p0 + u < p1 ? pa[(int64_t)(p0 + u) * 128] : 0.0f;

  float v_new = 0.0f;
  if (a.k_new) {   // launch-uniform
    const int seq = row / a.Hq, hq = row - seq * a.Hq, G = a.Hq / a.Hkv, hkv = hq / G;
    const int64_t src = ((int64_t)seq * a.Hkv + hkv) * 128 + dch;
    const uint16_t kb = ((const uint16_t *)a.k_new)[src], vb = ((const uint16_t *)a.v_new)[src];
    const uint16_t qb = ((const uint16_t *)a.q)[(int64_t)row * 128 + dch];
    const float kf = a.new_fmt == TTKV_F16 ? h2f(kb) : __uint_as_float((uint32_t)kb << 16);
    const float qf = a.q_fmt == TTKV_F16 ? h2f(qb) : __uint_as_float((uint32_t)qb << 16);
    v_new = a.new_fmt == TTKV_F16 ? h2f(vb) : __uint_as_float((uint32_t)vb << 16);
    const float part = wave_sum(qf * kf);   // both halves form the same two wave sums
    if ((threadIdx.x & 63) == 0) s_dot[wave] = part;
    if (hq == hkv * G) {   // half 0 stores the key row, half 1 the value row
      const int tok = a.new_tok[seq];
      const int rb = tok / a.dst.bt, r = tok - rb * a.dst.bt;
      const int64_t rec = a.dst.table ? (int64_t)a.dst.table[(int64_t)seq * a.dst.ring_blocks + rb]
                                      : (int64_t)seq * a.dst.ring_blocks + rb;
      uint8_t *head = a.dst.base + rec * a.dst.rec_bytes + (int64_t)hkv * a.dst.head_bytes;
      ((uint16_t *)(head + (half ? a.dst.v_off : 0) + r * 256))[dch] = half ? vb : kb;
    }
  }

  // the half's maximum
  float mp0 = -INFINITY, pl0 = 0.0f, M = -INFINITY;   // mp0, pl0: (m, l) of this thread's part in the first batch
  for (int b = 0; b < nb; ++b) {
    const int p = p0 + b * 128 + dch;
    const float mp = p < p1 ? pm[p] : -INFINITY;
    if (b == 0) {
      mp0 = mp;
      pl0 = p < p1 ? pl[p] : 0.0f;
    }
    M = fmaxf(M, mp);
  }
  M = wave_max(M);
  if ((threadIdx.x & 63) == 0) s_hm[wave] = M;
  __syncthreads();
  M = fmaxf(s_hm[2 * half], s_hm[2 * half + 1]);

  float o = 0.0f, l = 0.0f;
  for (int b = 0; b < nb; ++b) {
    const int pb = p0 + b * 128, p = pb + dch;
    float w = 0.0f;
    if (p < p1) {
      const float mp = b == 0 ? mp0 : pm[p];
      w = mp == -INFINITY ? 0.0f : __expf(mp - M);
      l = fmaf(b == 0 ? pl0 : pl[p], w, l);
    }
    if (b) __syncthreads();   // the weights of the batch before have been used
    s_w[half][dch] = w;
    __syncthreads();
    const int cnt = min(128, p1 - pb);   // <= 0 when the other half has one batch more
    int u = 0;
    if (b == 0) {
#pragma unroll
      for (; u < U; ++u)
        if (u < cnt) o = fmaf(av[u], s_w[half][u], o);
    }
#pragma unroll 8
    for (; u < cnt; ++u) o = fmaf(pa[(int64_t)(pb + u) * 128], s_w[half][u], o);
  }
  l = wave_sum(l);
  if ((threadIdx.x & 63) == 0) s_hl[wave] = l;
  if (half) s_o[dch] = o;
  __syncthreads();
  if (!half) {
    const float Mn = a.k_new ? (s_dot[0] + s_dot[1]) * a.scale : -INFINITY;   // the new token: (m, l, acc) = (score, 1, v)
    const float M2 = fmaxf(s_hm[2], s_hm[3]), Mt = fmaxf(fmaxf(M, M2), Mn);
    const float w1 = M == -INFINITY ? 0.0f : __expf(M - Mt), w2 = M2 == -INFINITY ? 0.0f : __expf(M2 - Mt);
    const float wn = Mn == -INFINITY ? 0.0f : __expf(Mn - Mt);
    o = o * w1 + s_o[dch] * w2 + v_new * wn;
    l = (s_hl[0] + s_hl[1]) * w1 + (s_hl[2] + s_hl[3]) * w2 + wn;
    a.out[(int64_t)row * 128 + dch] = l > 0.0f ? o / l : 0.0f;
    if (a.lse && dch == 0) a.lse[row] = l > 0.0f ? Mt + __logf(l) : -INFINITY;
  }
}

}  // namespace

// Query heads of one KV head handled together by one workgroup (register budget: 2).
int attn_group_width(int Gtot) { return Gtot % 2 == 0 ? 2 : 1; }

bool attn_supported(int k_fmt, int v_fmt, int G) {
  // values stored channel-major per 32 tokens exist for the matrix-core kernel only (two or more heads per KV head)
  if (v_fmt == TTKV_I4_ASYM_G64_T32) return G >= 2 && (k_fmt == TTKV_I8_SYM_G32 || k_fmt == TTKV_I4_ASYM_G64);
  if (k_fmt == TTKV_I4_ASYM_G64_T32) return false;
  if (k_fmt == TTKV_I4_ASYM_T128 || v_fmt == TTKV_I4_ASYM_T128) return k_fmt == TTKV_I4_ASYM_T128 && v_fmt == TTKV_I4_ASYM_G64;
  if (k_fmt == v_fmt) return is_tier_fmt(k_fmt);
  return k_fmt == TTKV_I8_SYM_G32 && v_fmt == TTKV_I4_ASYM_G64;
}

hipError_t launch_attn(const FusedArgs &a, hipStream_t s, int *n_kernels, int *n_mfma) {
  if (a.n_items <= 0) return hipSuccess;
  const int Gtot = a.Hq / a.Hkv;
  ++*n_kernels;
  if (attn_mfma_eligible(a)) {
    ++*n_mfma;
    return launch_attn_mfma(a, s);
  }
  const int G = attn_group_width(Gtot);
  const uint32_t bases = ((uint32_t)a.n_items * a.Hkv + 7) / 8 * 8;
  dim3 grid(bases * (Gtot / G));
  bool t128 = false;
  for (int j = 0; j < a.n_entries; ++j) t128 |= a.tv[(a.e[j].tier_seq >> 16) & 0xff].k_fmt == TTKV_I4_ASYM_T128;
  if (G == 1) {
    if (t128) hipLaunchKernelGGL((attn_fused_kernel<1, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((attn_fused_kernel<1, false>), grid, dim3(256), 0, s, a);
  } else {
    if (t128) hipLaunchKernelGGL((attn_fused_kernel<2, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((attn_fused_kernel<2, false>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_merge(const MergeArgs &a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(merge_kernel, dim3(a.rows), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ttkv
