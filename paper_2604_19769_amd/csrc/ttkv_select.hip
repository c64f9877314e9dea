// Block identification (Alg. 1: score every slow-tier block with phi, keep the
// top k).  phi(q, B_j) = sum over query heads h and channels i of
// q[h][i] * mean_key_j[h/G][i], accumulated in that fixed order with fused
// multiply-adds in fp32, so the score is one well-defined number and the
// selection (ties to the lower block id) is reproducible exactly.
#include "ttkv_internal.h"

#include <hip/hip_fp16.h>

namespace ttkv {

namespace {

__device__ __forceinline__ float h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }

// One thread per (sequence, live block): the sum is sequential by definition.
__global__ __launch_bounds__(64) void score_kernel(const SelectArgs a) {
  const int b = blockIdx.y;
  const int i = blockIdx.x * 64 + threadIdx.x;
  if (i >= a.n_blocks[b]) return;
  int r = a.first_block[b] + i;
  if (r >= a.ring_blocks) r -= a.ring_blocks;
  const int64_t rec = a.table ? (int64_t)a.table[(int64_t)b * a.ring_blocks + r] : (int64_t)a.rec_base[b] + r;
  const uint16_t *mu = a.k_summary + rec * a.Hkv * 128;
  const uint16_t *q = (const uint16_t *)a.q + (int64_t)b * a.Hq * 128;
  const int G = a.Hq / a.Hkv;
  float s = 0.0f;
  for (int h = 0; h < a.Hq; ++h) {
    const uint16_t *m = mu + (h / G) * 128;
    for (int ch = 0; ch < 128; ++ch) {
      const uint16_t qb = q[h * 128 + ch];
      const float qv = a.q_fmt == TTKV_F16 ? h2f(qb) : __uint_as_float((uint32_t)qb << 16);
      s = __fmaf_rn(qv, h2f(m[ch]), s);
    }
  }
  a.scores[(int64_t)b * a.max_blocks + i] = s;
}

// One workgroup per sequence.  rank(j) = #{i : s_i > s_j or (s_i == s_j and i < j)};
// block j is kept iff rank(j) < k.  Ids are written ascending.
__global__ __launch_bounds__(256) void topk_kernel(const SelectArgs a) {
  __shared__ int keep[1024];
  const int b = blockIdx.x;
  const int n = a.n_blocks[b];
  const float *s = a.scores + (int64_t)b * a.max_blocks;
  for (int j = threadIdx.x; j < n; j += 256) {
    const float sj = s[j];
    int rank = 0;
    for (int i = 0; i < n; ++i) {
      const float si = s[i];
      rank += (si > sj) || (si == sj && i < j);
    }
    keep[j] = rank < a.k;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int cnt = 0;
    int32_t *ids = a.sel_out + a.n_seq + (int64_t)b * a.sel_stride;
    for (int j = 0; j < n; ++j)
      if (keep[j]) ids[cnt++] = (int32_t)(a.first_block_id[b] + j);
    a.sel_out[b] = cnt;
  }
}

}  // namespace

hipError_t launch_select(const SelectArgs &a, hipStream_t s) {
  hipLaunchKernelGGL(score_kernel, dim3((a.max_blocks + 63) / 64, a.n_seq), dim3(64), 0, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topk_kernel, dim3(a.n_seq), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ttkv
