// Block identification (Alg. 1: score every slow-tier block with phi, keep the
// top k).  phi(q, B_j) = sum over query heads h of q_h . mean_key_j[h/G]: each
// head's dot product is a chain of fused multiply-adds over the channels in
// ascending order (fp32), the per-head results are added in ascending head
// order, so the score is one well-defined number and the selection (ties to
// the lower block id) is reproducible exactly -- while the heads' chains are
// independent and run one per lane.
#include "ttkv_internal.h"

#include <hip/hip_fp16.h>

#include <algorithm>

namespace ttkv {

namespace {

constexpr int SCORE_WAVES = 4;   // score_kernel: one wave64 per live block, four blocks per workgroup

template <bool BF16>
__device__ __forceinline__ float q2f(uint32_t bits16) {
  if (BF16) return __uint_as_float(bits16 << 16);
  return __half2float(__ushort_as_half((uint16_t)bits16));
}
__device__ __forceinline__ float h2f(uint32_t bits16) { return __half2float(__ushort_as_half((uint16_t)bits16)); }

// One head's chain over 8 channels held in a 16-byte piece of q and of the mean key.
template <bool BF16>
__device__ __forceinline__ float chain8(const uint4 qq, const uint4 mm, float s) {
  const uint32_t qw[4] = {qq.x, qq.y, qq.z, qq.w}, mw[4] = {mm.x, mm.y, mm.z, mm.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    s = __fmaf_rn(q2f<BF16>(qw[e] & 0xffffu), h2f(mw[e] & 0xffffu), s);
    s = __fmaf_rn(q2f<BF16>(qw[e] >> 16), h2f(mw[e] >> 16), s);
  }
  return s;
}

// One wave per (sequence, live block): lane = query head (passes of 64 heads), 128 fused multiply-adds per lane,
// then the lanes' results are added in head order (every lane forms the same sum).  Blocks are independent, so the
// launch spreads over the chip and its latency is one block's: the loads of 2 KiB of mean keys and a 128-deep chain.
template <bool BF16>
__global__ __launch_bounds__(SCORE_WAVES * 64) void score_kernel(const SelectArgs a) {
  const int b = blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * SCORE_WAVES + (threadIdx.x >> 6);
  if (i >= a.n_blocks[b]) return;                     // whole waves leave together
  const int G = a.Hq / a.Hkv;
  const uint16_t *q = (const uint16_t *)a.q + (int64_t)b * a.Hq * 128;
  int r = a.first_block[b] + i;
  if (r >= a.ring_blocks) r -= a.ring_blocks;
  const int64_t rec = a.table ? (int64_t)a.table[(int64_t)b * a.ring_blocks + r] : (int64_t)a.rec_base[b] + r;
  const uint16_t *mu = a.k_summary + rec * a.Hkv * 128;
  float phi = 0.0f;
  for (int h0 = 0; h0 < a.Hq; h0 += 64) {
    const int h = h0 + lane;
    float s = 0.0f;
    if (h < a.Hq) {
      const uint4 *qp = (const uint4 *)(q + h * 128);
      const uint4 *mp = (const uint4 *)(mu + (h / G) * 128);
      uint4 qv[16], mv[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        qv[j] = qp[j];
        mv[j] = mp[j];
      }
#pragma unroll
      for (int j = 0; j < 16; ++j) s = chain8<BF16>(qv[j], mv[j], s);
    }
    const int cnt = min(64, a.Hq - h0);
    for (int l = 0; l < cnt; ++l) phi = phi + __shfl(s, l, 64);
  }
  if (lane == 0) a.scores[(int64_t)b * a.max_blocks + i] = phi;
}

// One workgroup per sequence, a thread per block where the launch can afford it (256 to 1024 threads, chosen from the
// largest live block count: the ranking is n^2 comparisons -- at 768 blocks 86 us with 256 threads, a quarter of
// that with 1024).  rank(j) = #{i : s_i > s_j or (s_i == s_j and i < j)} with NaN read as -inf, so the ranks are a
// permutation; block j is kept iff rank(j) < k; ids are written ascending, never more than min(k, sel_stride).
__global__ __launch_bounds__(1024) void topk_kernel(const SelectArgs a) {
  __shared__ __align__(16) float score[1024];
  __shared__ int wave_kept[16];
  const int b = blockIdx.x;
  const int n = a.n_blocks[b];
  const int threads = blockDim.x, n_waves = threads >> 6;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n4 = (n + 3) & ~3;
  for (int j = threadIdx.x; j < n4; j += threads) {
    const float s = j < n ? a.scores[(int64_t)b * a.max_blocks + j] : -INFINITY;   // padding: never ahead of a live block with a lower index
    score[j] = s != s ? -INFINITY : s;
  }
  __syncthreads();
  const int limit = min(a.k, a.sel_stride);
  int32_t *ids = a.sel_out + a.n_seq + (int64_t)b * a.sel_stride;
  int written = 0;                                     // ids written by earlier rounds (same in every thread)
  for (int base = 0; base < n; base += threads) {
    const int j = base + threadIdx.x;
    bool kept = false;
    if (j < n) {
      const float sj = score[j];
      int rank = 0;
      for (int i = 0; i < n4; i += 4) {
        const float4 si = *(const float4 *)&score[i];
        rank += (si.x > sj) || (si.x == sj && i < j);
        rank += (si.y > sj) || (si.y == sj && i + 1 < j);
        rank += (si.z > sj) || (si.z == sj && i + 2 < j);
        rank += (si.w > sj) || (si.w == sj && i + 3 < j);
      }
      kept = rank < a.k;
    }
    // ascending ids: a kept block's place is the number of kept blocks before it
    const unsigned long long mask = __ballot(kept);
    if (lane == 0) wave_kept[wave] = __popcll(mask);
    __syncthreads();
    int before = written, all = 0;
    for (int w = 0; w < n_waves; ++w) {
      const int kw = wave_kept[w];
      before += w < wave ? kw : 0;
      all += kw;
    }
    const int pos = before + __popcll(mask & ((1ull << lane) - 1ull));
    if (kept && pos < limit) ids[pos] = (int32_t)(a.first_block_id[b] + j);
    written += all;
    __syncthreads();
  }
  if (threadIdx.x == 0) a.sel_out[b] = min(written, limit);
}

}  // namespace

hipError_t launch_select(const SelectArgs &a, hipStream_t s) {
  const dim3 grid((a.max_blocks + SCORE_WAVES - 1) / SCORE_WAVES, a.n_seq);
  if (a.q_fmt == TTKV_BF16)
    hipLaunchKernelGGL(score_kernel<true>, grid, dim3(SCORE_WAVES * 64), 0, s, a);
  else
    hipLaunchKernelGGL(score_kernel<false>, grid, dim3(SCORE_WAVES * 64), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int threads = std::min(1024, std::max(256, (a.max_blocks + 63) / 64 * 64));
  hipLaunchKernelGGL(topk_kernel, dim3(a.n_seq), dim3(threads), 0, s, a);
  return hipGetLastError();
}

}  // namespace ttkv
