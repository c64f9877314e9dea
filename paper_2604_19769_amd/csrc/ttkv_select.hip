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

// One workgroup per sequence, one thread per live block (at most 1024).  The k blocks to keep are those with
// rank(j) = #{i : s_i > s_j or (s_i == s_j and i < j)} < k, NaN read as -inf.  Instead of counting ranks (n^2
// comparisons: 86 us at 768 blocks) the k-th largest score is found by a radix select over the scores' order-
// preserving 32-bit keys, one byte per pass (a 256-bin histogram in LDS, its crossing bin found by one wave), which
// is exact; among the blocks whose score equals it the lowest ids fill the remaining places.  Ids are written
// ascending by a ballot / popcount prefix, never more than min(k, sel_stride) of them.
__global__ __launch_bounds__(1024) void topk_kernel(const SelectArgs a) {
  __shared__ __align__(16) uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_remaining;
  __shared__ int wave_eq[16], wave_kept[16];
  const int b = blockIdx.x;
  const int n = a.n_blocks[b];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_waves = blockDim.x >> 6;
  const bool valid = tid < n;                       // the launch has at least as many threads as live blocks
  float s = valid ? a.scores[(int64_t)b * a.max_blocks + tid] : -INFINITY;
  if (s != s) s = -INFINITY;
  if (s == 0.0f) s = 0.0f;                          // -0 and +0 compare equal: one key for both
  const uint32_t u = __float_as_uint(s);
  const uint32_t key = (u >> 31) ? ~u : (u | 0x80000000u);   // a larger score is a larger key; equal scores, equal keys
  const int limit = min(a.k, a.sel_stride);
  const int keep = min(a.k, n);
  int32_t *ids = a.sel_out + a.n_seq + (int64_t)b * a.sel_stride;
  bool kept = valid && keep >= n;
  if (keep > 0 && keep < n) {                       // workgroup-uniform
    uint32_t prefix = 0, remaining = (uint32_t)keep;   // high bytes of the k-th largest key found so far; places left among the keys that share them
    for (int pass = 3; pass >= 0; --pass) {
      for (int i = tid; i < 256; i += blockDim.x) hist[i] = 0;
      __syncthreads();
      if (valid && (pass == 3 || (key >> (8 * (pass + 1))) == prefix)) atomicAdd(&hist[(key >> (8 * pass)) & 255u], 1u);
      __syncthreads();
      if (wave == 0) {
        // lane l holds bins 4 l .. 4 l + 3; suffix sums over the lanes find the bin in which the count from the top
        // reaches `remaining`
        const uint4 h4 = ((const uint4 *)hist)[lane];
        const uint32_t mine = h4.x + h4.y + h4.z + h4.w;
        uint32_t suf = mine;
        for (int d = 1; d < 64; d <<= 1) {
          const uint32_t o = __shfl_down(suf, d, 64);
          if (lane + d < 64) suf += o;
        }
        const uint32_t above = suf - mine;          // keys in the bins of the lanes above this one
        if (suf >= remaining && above < remaining) {   // exactly one lane
          uint32_t r = remaining - above;
          uint32_t bin;
          if (h4.w >= r) bin = 3;
          else if (h4.w + h4.z >= r) { bin = 2; r -= h4.w; }
          else if (h4.w + h4.z + h4.y >= r) { bin = 1; r -= h4.w + h4.z; }
          else { bin = 0; r -= h4.w + h4.z + h4.y; }
          s_prefix = (prefix << 8) | (4u * lane + bin);
          s_remaining = r;
        }
      }
      __syncthreads();
      prefix = s_prefix;
      remaining = s_remaining;
    }
    // prefix is the k-th largest key; `remaining` of the blocks that have it are kept, lowest ids first
    const bool eq = valid && key == prefix;
    const unsigned long long eq_mask = __ballot(eq);
    if (lane == 0) wave_eq[wave] = __popcll(eq_mask);
    __syncthreads();
    int eq_before = __popcll(eq_mask & ((1ull << lane) - 1ull));
    for (int w = 0; w < wave; ++w) eq_before += wave_eq[w];
    kept = valid && (key > prefix || (eq && (uint32_t)eq_before < remaining));
  }
  // ascending ids: a kept block's place is the number of kept blocks before it
  const unsigned long long mask = __ballot(kept);
  if (lane == 0) wave_kept[wave] = __popcll(mask);
  __syncthreads();
  int pos = __popcll(mask & ((1ull << lane) - 1ull)), all = 0;
  for (int w = 0; w < n_waves; ++w) {
    const int kw = wave_kept[w];
    pos += w < wave ? kw : 0;
    all += kw;
  }
  if (kept && pos < limit) ids[pos] = (int32_t)(a.first_block_id[b] + tid);
  if (tid == 0) a.sel_out[b] = min(all, limit);
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
  const int threads = std::min(1024, std::max(64, (a.max_blocks + 63) / 64 * 64));   // one thread per live block
  hipLaunchKernelGGL(topk_kernel, dim3(a.n_seq), dim3(threads), 0, s, a);
  return hipGetLastError();
}

}  // namespace ttkv
