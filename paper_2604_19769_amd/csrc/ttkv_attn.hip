// Split-K decode attention partials over one tier (Alg. 1: Attn on the fast
// tier, Decompress + Attn per slow-tier block) and the log-sum-exp merge of the
// partials (the "+" of Alg. 1, normalised once at the end).
//
// Mapping (wave64): a K or V row of one token-head is ROWB bytes = LPT lanes x
// 16 B, so one 128-bit load per lane brings TPL = 64/LPT whole rows per wave,
// fully coalesced.  Lane L holds elements [slice*EPL, slice*EPL+EPL) of token
// L/LPT; codes are decompressed in registers; the q.k dot is finished with
// log2(LPT) lane shuffles; the lane that owns a token's K slice also owns its
// V slice, so softmax weights never leave their lane (K 8-bit + V 4-bit needs
// one shuffle per V row).  Scale/zero are factored out of the inner loops:
//   q.k  = s_g * sum_i q_i c_i + z_g * sum_i q_i         (per group g)
//   sum_t p_t v_t = sum_t (p_t s_t) c_t + sum_t p_t z_t
#include "ttkv_internal.h"

#include <hip/hip_fp16.h>

namespace ttkv {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int F> struct Fmt;
template <> struct Fmt<TTKV_F16> { static constexpr int ROWB = 256, LPT = 16, TPL = 4, EPL = 8; };
template <> struct Fmt<TTKV_BF16> { static constexpr int ROWB = 256, LPT = 16, TPL = 4, EPL = 8; };
template <> struct Fmt<TTKV_I8_SYM_G32> { static constexpr int ROWB = 128, LPT = 8, TPL = 8, EPL = 16; };
template <> struct Fmt<TTKV_I4_ASYM_G64> { static constexpr int ROWB = 64, LPT = 4, TPL = 16, EPL = 32; };

__device__ __forceinline__ float h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// 16 bytes of one row -> EPL raw element values (codes as floats; fp formats: the value).
template <int F>
__device__ __forceinline__ void decode16(const uint4 &w, float *x) {
  const uint32_t u[4] = {w.x, w.y, w.z, w.w};
  if constexpr (F == TTKV_F16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = h2f((uint16_t)(u[i] & 0xffff));
      x[2 * i + 1] = h2f((uint16_t)(u[i] >> 16));
    }
  } else if constexpr (F == TTKV_BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(u[i] << 16);
      x[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
    }
  } else if constexpr (F == TTKV_I8_SYM_G32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[4 * i + 0] = (float)((int)(u[i] << 24) >> 24);
      x[4 * i + 1] = (float)((int)(u[i] << 16) >> 24);
      x[4 * i + 2] = (float)((int)(u[i] << 8) >> 24);
      x[4 * i + 3] = (float)((int)u[i] >> 24);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int n = 0; n < 8; ++n) x[8 * i + n] = (float)((u[i] >> (4 * n)) & 0xf);
  }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v = fmaxf(v, __shfl_xor(v, m));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
  return v;
}

template <int KF, int VF, int G>
__global__ __launch_bounds__(256) void attn_partial_kernel(const AttnArgs a) {
  using FK = Fmt<KF>;
  using FV = Fmt<VF>;
  static_assert(FV::TPL % FK::TPL == 0, "V rows must not be wider than K rows");
  constexpr int TT = 4 * FK::TPL;          // tokens per wave tile (K is the wider or equal row)
  constexpr int NLK = 4;                   // K loads per lane per tile
  constexpr int NLV = TT / FV::TPL;        // V loads per lane per tile
  constexpr int R = FV::TPL / FK::TPL;     // K loads covered by one V load
  constexpr bool KQ = (KF == TTKV_I8_SYM_G32 || KF == TTKV_I4_ASYM_G64);
  constexpr bool VQ = (VF == TTKV_I8_SYM_G32 || VF == TTKV_I4_ASYM_G64);

  __shared__ float s_acc[4][G][128];
  __shared__ float s_m[4][G], s_l[4][G];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int item = blockIdx.x;
  const int hkv = blockIdx.y;
  const int Gtot = a.Hq / a.Hkv;
  const int hq0 = hkv * Gtot + blockIdx.z * G;

  int j = 0;
  while (j + 1 < a.st.n_seq && item >= a.st.item_start[j + 1]) ++j;
  const int chunk = item - a.st.item_start[j];
  const int seq = a.st.seq_id[j];
  const int len = a.st.len[j];
  const int c0 = chunk * a.chunk_tokens;
  const int c1 = min(len, c0 + a.chunk_tokens);
  const int ring_tokens = a.tv.ring_blocks * a.tv.bt;

  const int kslice = lane % FK::LPT, ktok = lane / FK::LPT;
  const int vslice = lane % FV::LPT, vtok = lane / FV::LPT;

  // q slice of this lane for every head of the group, pre-multiplied by
  // softmax_scale * log2(e) so that the softmax runs on exp2.
  float q[G][FK::EPL];
  float qsum[G];
  {
    const float qs = a.scale * kLog2e;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const uint16_t *qp = (const uint16_t *)a.q + ((int64_t)seq * a.Hq + hq0 + g) * 128 + kslice * FK::EPL;
      qsum[g] = 0.0f;
#pragma unroll
      for (int e = 0; e < FK::EPL; ++e) {
        float v = a.q_fmt == TTKV_F16 ? h2f(qp[e]) : __uint_as_float((uint32_t)qp[e] << 16);
        q[g][e] = v * qs;
        qsum[g] += q[g][e];
      }
    }
  }

  float m[G], l[G], zacc[G];
  float acc[G][FV::EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = -INFINITY;
    l[g] = 0.0f;
    zacc[g] = 0.0f;
#pragma unroll
    for (int e = 0; e < FV::EPL; ++e) acc[g][e] = 0.0f;
  }

  for (int i0 = c0 + wave * TT; i0 < c1; i0 += 4 * TT) {
    const int nv = min(TT, c1 - i0);
    int tok0 = a.st.first_tok[j] + i0;
    if (tok0 >= ring_tokens) tok0 -= ring_tokens;
    const int r = tok0 / a.tv.bt;
    const int row0 = tok0 - r * a.tv.bt;
    const int64_t rec = a.tv.table ? (int64_t)a.tv.table[(int64_t)seq * a.tv.ring_blocks + r] : (int64_t)a.st.rec_base[j] + r;
    const uint8_t *head = a.tv.base + rec * a.tv.rec_bytes + (int64_t)hkv * a.tv.head_bytes;

    // ---- issue all loads of the tile
    uint4 kw[NLK], vw[NLV];
    uint32_t kmeta[NLK], vmeta[NLV];
#pragma unroll
    for (int n = 0; n < NLK; ++n) {
      const int t = min(n * FK::TPL + ktok, nv - 1);
      kw[n] = *(const uint4 *)(head + (row0 + t) * FK::ROWB + kslice * 16);
      if constexpr (KF == TTKV_I8_SYM_G32)
        kmeta[n] = *(const uint16_t *)(head + a.tv.k_meta_off + (row0 + t) * 8 + (kslice >> 1) * 2);
      else if constexpr (KF == TTKV_I4_ASYM_G64)
        kmeta[n] = *(const uint32_t *)(head + a.tv.k_meta_off + (row0 + t) * 8 + (kslice >> 1) * 4);
    }
#pragma unroll
    for (int n = 0; n < NLV; ++n) {
      const int t = min(n * FV::TPL + vtok, nv - 1);
      vw[n] = *(const uint4 *)(head + a.tv.v_off + (row0 + t) * FV::ROWB + vslice * 16);
      if constexpr (VF == TTKV_I8_SYM_G32)
        vmeta[n] = *(const uint16_t *)(head + a.tv.v_meta_off + (row0 + t) * 8 + (vslice >> 1) * 2);
      else if constexpr (VF == TTKV_I4_ASYM_G64)
        vmeta[n] = *(const uint32_t *)(head + a.tv.v_meta_off + (row0 + t) * 8 + (vslice >> 1) * 4);
    }

    // ---- scores (log2 domain)
    float s[G][NLK];
#pragma unroll
    for (int n = 0; n < NLK; ++n) {
      float x[FK::EPL];
      decode16<KF>(kw[n], x);
      float ks = 1.0f, kz = 0.0f;
      if constexpr (KF == TTKV_I8_SYM_G32) ks = h2f((uint16_t)kmeta[n]);
      if constexpr (KF == TTKV_I4_ASYM_G64) {
        ks = h2f((uint16_t)(kmeta[n] & 0xffff));
        kz = h2f((uint16_t)(kmeta[n] >> 16));
      }
      const bool valid = n * FK::TPL + ktok < nv;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float d = 0.0f;
#pragma unroll
        for (int e = 0; e < FK::EPL; ++e) d = fmaf(x[e], q[g][e], d);
        if constexpr (KQ) d = d * ks + kz * qsum[g];
#pragma unroll
        for (int msk = 1; msk < FK::LPT; msk <<= 1) d += __shfl_xor(d, msk);
        s[g][n] = valid ? d : -INFINITY;
      }
    }

    // ---- online softmax
    float p[G][NLK];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mt = s[g][0];
#pragma unroll
      for (int n = 1; n < NLK; ++n) mt = fmaxf(mt, s[g][n]);
      mt = wave_max(mt);
      if (mt > m[g]) {  // wave-uniform
        const float alpha = exp2f(m[g] - mt);
        l[g] *= alpha;
        zacc[g] *= alpha;
#pragma unroll
        for (int e = 0; e < FV::EPL; ++e) acc[g][e] *= alpha;
        m[g] = mt;
      }
      float ps = 0.0f;
#pragma unroll
      for (int n = 0; n < NLK; ++n) {
        p[g][n] = exp2f(s[g][n] - m[g]);
        ps += p[g][n];
      }
      if (kslice == 0) l[g] += ps;
    }

    // ---- weighted V
#pragma unroll
    for (int n = 0; n < NLV; ++n) {
      float x[FV::EPL];
      decode16<VF>(vw[n], x);
      float vs = 1.0f, vz = 0.0f;
      if constexpr (VF == TTKV_I8_SYM_G32) vs = h2f((uint16_t)vmeta[n]);
      if constexpr (VF == TTKV_I4_ASYM_G64) {
        vs = h2f((uint16_t)(vmeta[n] & 0xffff));
        vz = h2f((uint16_t)(vmeta[n] >> 16));
      }
      const bool valid = n * FV::TPL + vtok < nv;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float pv;
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
        if (!valid) pv = 0.0f;
        if constexpr (VF == TTKV_I4_ASYM_G64) zacc[g] = fmaf(pv, vz, zacc[g]);
        if constexpr (VQ) pv *= vs;
#pragma unroll
        for (int e = 0; e < FV::EPL; ++e) acc[g][e] = fmaf(pv, x[e], acc[g][e]);
      }
    }
  }

  // ---- reduce the wave: lanes with the same V slice hold partial sums over different tokens
#pragma unroll
  for (int g = 0; g < G; ++g) {
    l[g] = wave_sum(l[g]);
#pragma unroll
    for (int e = 0; e < FV::EPL; ++e) {
      float v = acc[g][e] + zacc[g];
#pragma unroll
      for (int msk = FV::LPT; msk < 64; msk <<= 1) v += __shfl_xor(v, msk);
      acc[g][e] = v;
    }
    if (vtok == 0) {
#pragma unroll
      for (int e = 0; e < FV::EPL; ++e) s_acc[wave][g][vslice * FV::EPL + e] = acc[g][e];
    }
    if (lane == 0) {
      s_m[wave][g] = m[g];
      s_l[wave][g] = l[g];
    }
  }
  __syncthreads();

  // ---- merge the four waves and write the workgroup's partial
  const int part = a.st.part_base[j] + chunk;
  for (int idx = threadIdx.x; idx < G * 128; idx += 256) {
    const int g = idx >> 7, dch = idx & 127;
    float M = fmaxf(fmaxf(s_m[0][g], s_m[1][g]), fmaxf(s_m[2][g], s_m[3][g]));
    float o = 0.0f, ll = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = s_m[w][g] == -INFINITY ? 0.0f : exp2f(s_m[w][g] - M);
      o = fmaf(s_acc[w][g][dch], wgt, o);
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

// One workgroup of 128 threads per row: thread = channel.
__global__ __launch_bounds__(128) void merge_kernel(const MergeArgs a) {
  const int row = blockIdx.x, dch = threadIdx.x;
  int n = a.n_parts;
  if (a.n_parts_row)
    n = a.n_parts_row[row];
  else if (a.rows_per_seq > 0)
    n = a.cnt[row / a.rows_per_seq];
  const float *pm = a.m + (int64_t)row * a.part_stride;
  const float *pl = a.l + (int64_t)row * a.part_stride;
  const float *pa = a.acc + (int64_t)row * a.part_stride * 128;
  float M = -INFINITY;
  for (int p = 0; p < n; ++p) M = fmaxf(M, pm[p]);
  float o = 0.0f, l = 0.0f;
  for (int p = 0; p < n; ++p) {
    const float mp = pm[p];
    if (mp == -INFINITY) continue;
    const float w = __expf(mp - M);
    o = fmaf(pa[(int64_t)p * 128 + dch], w, o);
    l = fmaf(pl[p], w, l);
  }
  a.out[(int64_t)row * 128 + dch] = l > 0.0f ? o / l : 0.0f;
  if (a.lse && dch == 0) a.lse[row] = l > 0.0f ? M + __logf(l) : -INFINITY;
}

template <int KF, int VF>
hipError_t launch_g(const AttnArgs &a, hipStream_t s, int G, dim3 grid) {
  switch (G) {
    case 1: hipLaunchKernelGGL((attn_partial_kernel<KF, VF, 1>), grid, dim3(256), 0, s, a); break;
    case 2: hipLaunchKernelGGL((attn_partial_kernel<KF, VF, 2>), grid, dim3(256), 0, s, a); break;
    default: hipLaunchKernelGGL((attn_partial_kernel<KF, VF, 4>), grid, dim3(256), 0, s, a); break;
  }
  return hipGetLastError();
}

int group_width(int Gtot) { return Gtot % 4 == 0 ? 4 : (Gtot % 2 == 0 ? 2 : 1); }

}  // namespace

bool attn_supported(int k_fmt, int v_fmt, int G) {
  (void)G;
  if (k_fmt == v_fmt) return is_tier_fmt(k_fmt);
  return k_fmt == TTKV_I8_SYM_G32 && v_fmt == TTKV_I4_ASYM_G64;
}

hipError_t launch_attn_partial(const AttnArgs &a, hipStream_t s, int *n_kernels) {
  const int items = a.st.item_start[a.st.n_seq];
  if (items <= 0) return hipSuccess;
  const int Gtot = a.Hq / a.Hkv;
  const int G = group_width(Gtot);
  dim3 grid(items, a.Hkv, Gtot / G);
  ++*n_kernels;
  const int kf = a.tv.k_fmt, vf = a.tv.v_fmt;
  if (kf == TTKV_F16 && vf == TTKV_F16) return launch_g<TTKV_F16, TTKV_F16>(a, s, G, grid);
  if (kf == TTKV_BF16 && vf == TTKV_BF16) return launch_g<TTKV_BF16, TTKV_BF16>(a, s, G, grid);
  if (kf == TTKV_I8_SYM_G32 && vf == TTKV_I8_SYM_G32) return launch_g<TTKV_I8_SYM_G32, TTKV_I8_SYM_G32>(a, s, G, grid);
  if (kf == TTKV_I4_ASYM_G64 && vf == TTKV_I4_ASYM_G64) return launch_g<TTKV_I4_ASYM_G64, TTKV_I4_ASYM_G64>(a, s, G, grid);
  if (kf == TTKV_I8_SYM_G32 && vf == TTKV_I4_ASYM_G64) return launch_g<TTKV_I8_SYM_G32, TTKV_I4_ASYM_G64>(a, s, G, grid);
  --*n_kernels;
  return hipErrorInvalidValue;
}

hipError_t launch_merge(const MergeArgs &a, hipStream_t s) {
  if (a.rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(merge_kernel, dim3(a.rows), dim3(128), 0, s, a);
  return hipGetLastError();
}

}  // namespace ttkv
