// Row conversion kernels: append (Sec. 4.1), Q_8bit / Q_4bit (Sec. 4.2) and the
// eviction path's decompress -> re-quantize.  Compiled with -ffp-contract=off:
// every fp32 step below is one IEEE operation (divide and fp16 conversion
// round to nearest even), so codes, scales and zeros are reproducible bit for bit.
#include "ttkv_internal.h"

#include <hip/hip_fp16.h>

namespace ttkv {

namespace {

__device__ __forceinline__ float h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }
__device__ __forceinline__ uint16_t f2h(float f) { return __half_as_ushort(__float2half_rn(f)); }
__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Record index and row of ring token `tok` of sequence `seq`.
__device__ __forceinline__ uint8_t *head_ptr(const TierView &v, int seq, int rec_base, int tok, int h, int *row) {
  int r = tok / v.bt;
  *row = tok - r * v.bt;
  int64_t rec = v.table ? (int64_t)v.table[(int64_t)seq * v.ring_blocks + r] : (int64_t)rec_base + r;
  return v.base + rec * v.rec_bytes + (int64_t)h * v.head_bytes;
}

__device__ __forceinline__ int wrap(int tok, const TierView &v) {
  int ring = v.ring_blocks * v.bt;
  return tok >= ring ? tok - ring : tok;
}

// rint(x / s) as the IEEE division followed by round-to-nearest-even gives it (the recipe of Sec. 4.2's quantizers,
// one IEEE operation per step), wherever the caller's clamp to [-127, 127] or [0, 15] lets the difference show, for
// a group's many x against one s: r = 1 / s is divided once; x * r is within 2^-22 |x / s| of the true quotient,
// i.e. within 5e-5 for |x / s| < 200, so the two rounded integers agree unless the quotient lies within that
// distance of a half-integer -- ties included -- and there the exact division decides (about one element in a
// thousand takes it).  Beyond 200 either rounding is clamped to the same bound.
__device__ __forceinline__ float quot_rint(float x, float s, float r) {
  const float t = x * r;
  float q = rintf(t);
  if (fabsf(t - q) > 0.4995f) q = rintf(x / s);
  return q;
}

// ---- in-register quantize / decompress over a group spread across `LANES`
// consecutive lanes holding N values each.

// Q1 on a 32-element group: returns the fp16 scale bits, codes as ints.
template <int N, int LANES>
__device__ __forceinline__ uint16_t q1_group(const float (&x)[N], int (&c)[N]) {
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < N; ++i) amax = fmaxf(amax, fabsf(x[i]));
#pragma unroll
  for (int m = 1; m < LANES; m <<= 1) amax = fmaxf(amax, __shfl_xor(amax, m));
  float s32 = amax / 127.0f;
  uint16_t sh = f2h(s32);
  float s = h2f(sh);
  const float r = s != 0.0f ? 1.0f / s : 0.0f;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    float q = 0.0f;
    if (s != 0.0f) q = fminf(fmaxf(quot_rint(x[i], s, r), -127.0f), 127.0f);
    c[i] = (int)q;
  }
  return sh;
}

// Q2 on a 64-element group: fp16 scale and zero bits, codes 0..15.
template <int N, int LANES>
__device__ __forceinline__ void q2_group(const float (&x)[N], int (&c)[N], uint16_t *sh_out, uint16_t *zh_out) {
  float lo = x[0], hi = x[0];
#pragma unroll
  for (int i = 1; i < N; ++i) {
    lo = fminf(lo, x[i]);
    hi = fmaxf(hi, x[i]);
  }
#pragma unroll
  for (int m = 1; m < LANES; m <<= 1) {
    lo = fminf(lo, __shfl_xor(lo, m));
    hi = fmaxf(hi, __shfl_xor(hi, m));
  }
  if (lo == 0.0f) lo = 0.0f;  // a zero minimum is stored as +0 whatever its sign
  float s32 = (hi - lo) / 15.0f;
  uint16_t sh = f2h(s32), zh = f2h(lo);
  float s = h2f(sh), z = h2f(zh);
  const float r = s != 0.0f ? 1.0f / s : 0.0f;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    float q = 0.0f;
    if (s != 0.0f) q = fminf(fmaxf(quot_rint(x[i] - z, s, r), 0.0f), 15.0f);
    c[i] = (int)q;
  }
  *sh_out = sh;
  *zh_out = zh;
}

// The values a format decompresses to (a token that passed through a tier).
template <int N, int L8, int L4>
__device__ __forceinline__ void roundtrip(int fmt, float (&x)[N]) {
  int c[N];
  if (fmt == TTKV_I8_SYM_G32) {
    uint16_t sh = q1_group<N, L8>(x, c);
    float s = h2f(sh);
#pragma unroll
    for (int i = 0; i < N; ++i) x[i] = (float)c[i] * s;
  } else if (fmt == TTKV_I4_ASYM_G64) {
    uint16_t sh, zh;
    q2_group<N, L4>(x, c, &sh, &zh);
    float s = h2f(sh), z = h2f(zh);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      float p = (float)c[i] * s;
      x[i] = p + z;
    }
  }
}

// ---- loading 8 consecutive elements [8*l16, 8*l16+8) of one row as fp32.
__device__ __forceinline__ void load8_flat(const void *flat, int fmt, int64_t row, int l16, float (&x)[8]) {
  if (fmt == TTKV_F32) {
    const float4 *p = (const float4 *)((const float *)flat + row * 128 + l16 * 8);
    float4 a = p[0], b = p[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  } else {
    uint4 w = *(const uint4 *)((const uint16_t *)flat + row * 128 + l16 * 8);
    uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint16_t a = (uint16_t)(u[i] & 0xffff), b = (uint16_t)(u[i] >> 16);
      x[2 * i] = fmt == TTKV_F16 ? h2f(a) : bf2f(a);
      x[2 * i + 1] = fmt == TTKV_F16 ? h2f(b) : bf2f(b);
    }
  }
}

__device__ __forceinline__ void load8_tier(const uint8_t *head, int fmt, int code_off, int meta_off, int row, int l16,
                                           float (&x)[8]) {
  if (fmt == TTKV_F16 || fmt == TTKV_BF16) {
    uint4 w = *(const uint4 *)(head + code_off + row * 256 + l16 * 16);
    uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint16_t a = (uint16_t)(u[i] & 0xffff), b = (uint16_t)(u[i] >> 16);
      x[2 * i] = fmt == TTKV_F16 ? h2f(a) : bf2f(a);
      x[2 * i + 1] = fmt == TTKV_F16 ? h2f(b) : bf2f(b);
    }
  } else if (fmt == TTKV_I8_SYM_G32) {
    uint2 w = *(const uint2 *)(head + code_off + row * 128 + l16 * 8);
    float s = h2f(*(const uint16_t *)(head + meta_off + row * 8 + (l16 >> 2) * 2));
    uint32_t u[2] = {w.x, w.y};
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (float)(int)(int8_t)((u[i >> 2] >> (8 * (i & 3))) & 0xff) * s;
  } else {
    uint32_t w = *(const uint32_t *)(head + code_off + row * 64 + l16 * 4);
    uint32_t sz = *(const uint32_t *)(head + meta_off + row * 8 + (l16 >> 3) * 4);
    float s = h2f((uint16_t)(sz & 0xffff)), z = h2f((uint16_t)(sz >> 16));
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float p = (float)(int)((w >> (4 * i)) & 0xf) * s;
      x[i] = p + z;
    }
  }
}

__device__ __forceinline__ void store8_tier(uint8_t *head, int fmt, int code_off, int meta_off, int row, int l16,
                                            float (&x)[8], bool live) {
  if (fmt == TTKV_F16 || fmt == TTKV_BF16) {
    uint32_t u[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t a, b;
      if (fmt == TTKV_F16) {
        a = f2h(x[2 * i]);
        b = f2h(x[2 * i + 1]);
      } else {  // source values are bf16 already: the upper half is exact
        a = __float_as_uint(x[2 * i]) >> 16;
        b = __float_as_uint(x[2 * i + 1]) >> 16;
      }
      u[i] = a | (b << 16);
    }
    if (live) *(uint4 *)(head + code_off + row * 256 + l16 * 16) = make_uint4(u[0], u[1], u[2], u[3]);
  } else if (fmt == TTKV_I8_SYM_G32) {
    int c[8];
    uint16_t sh = q1_group<8, 4>(x, c);
    uint32_t u[2] = {0, 0};
#pragma unroll
    for (int i = 0; i < 8; ++i) u[i >> 2] |= ((uint32_t)c[i] & 0xffu) << (8 * (i & 3));
    if (live) {
      *(uint2 *)(head + code_off + row * 128 + l16 * 8) = make_uint2(u[0], u[1]);
      if ((l16 & 3) == 0) *(uint16_t *)(head + meta_off + row * 8 + (l16 >> 2) * 2) = sh;
    }
  } else {
    int c[8];
    uint16_t sh, zh;
    q2_group<8, 8>(x, c, &sh, &zh);
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) w |= ((uint32_t)c[i] & 0xfu) << (4 * i);
    if (live) {
      *(uint32_t *)(head + code_off + row * 64 + l16 * 4) = w;
      if ((l16 & 7) == 0) *(uint32_t *)(head + meta_off + row * 8 + (l16 >> 3) * 4) = (uint32_t)sh | ((uint32_t)zh << 16);
    }
  }
}

// One 16-lane group converts one row (one token of one KV head); blockIdx.y
// picks K (0) or V (1), blockIdx.z the (entry, KV head).
__global__ __launch_bounds__(256) void convert_rows_kernel(const ConvArgs a) {
  // grid: (16 tokens per workgroup, K / V, entry x KV head) -- no per-thread division of a 64-bit row number
  const int which = blockIdx.y + a.which0;
  const int l16 = threadIdx.x & 15;
  int t = blockIdx.x * 16 + (threadIdx.x >> 4);
  const bool live = t < a.n_tokens;
  if (!live) t = a.n_tokens - 1;
  const int j = blockIdx.z / a.Hkv, h = blockIdx.z - j * a.Hkv;
  const int seq = a.seq_id[j];

  float x[8];
  if (!a.s.from_tier) {
    load8_flat(which ? a.s.v_flat : a.s.k_flat, a.s.flat_fmt, ((int64_t)j * a.Hkv + h) * a.n_tokens + t, l16, x);
  } else {
    int row;
    const uint8_t *head = head_ptr(a.s.src, seq, a.s.src_rec_base[j], wrap(a.s.src_first_tok[j] + t, a.s.src), h, &row);
    if (which)
      load8_tier(head, a.s.src.v_fmt, a.s.src.v_off, a.s.src.v_meta_off, row, l16, x);
    else
      load8_tier(head, a.s.src.k_fmt, 0, a.s.src.k_meta_off, row, l16, x);
  }
  for (int u = 0; u < a.n_via; ++u) roundtrip<8, 4, 8>(which ? a.via_v[u] : a.via_k[u], x);

  int row;
  uint8_t *head = head_ptr(a.dst, seq, a.dst_rec_base[j], wrap(a.dst_first_tok[j] + t, a.dst), h, &row);
  if (which)
    store8_tier(head, a.dst.v_fmt, a.dst.v_off, a.dst.v_meta_off, row, l16, x, live);
  else
    store8_tier(head, a.dst.k_fmt, 0, a.dst.k_meta_off, row, l16, x, live);
}

// Key value of token t (of this call) of entry j, KV head h, channel i, as it arrives at the destination tier:
// read from the flat source or from the source tier, then through the formats of the tiers in between.
// Called by all 128 channel-threads of a head together (the round trips reduce over 32 / 64 lanes).
__device__ __forceinline__ float arriving_key(const ConvArgs &a, int j, int seq, int h, int t, int i) {
  float x[1];
  if (!a.s.from_tier) {
    int64_t row = ((int64_t)j * a.Hkv + h) * a.n_tokens + t;
    if (a.s.flat_fmt == TTKV_F32)
      x[0] = ((const float *)a.s.k_flat)[row * 128 + i];
    else {
      uint16_t w = ((const uint16_t *)a.s.k_flat)[row * 128 + i];
      x[0] = a.s.flat_fmt == TTKV_F16 ? h2f(w) : bf2f(w);
    }
  } else {
    int row;
    const uint8_t *head = head_ptr(a.s.src, seq, a.s.src_rec_base[j], wrap(a.s.src_first_tok[j] + t, a.s.src), h, &row);
    const int f = a.s.src.k_fmt;
    if (f == TTKV_F16 || f == TTKV_BF16) {
      uint16_t w = *(const uint16_t *)(head + row * 256 + i * 2);
      x[0] = f == TTKV_F16 ? h2f(w) : bf2f(w);
    } else if (f == TTKV_I8_SYM_G32) {
      float s = h2f(*(const uint16_t *)(head + a.s.src.k_meta_off + row * 8 + (i >> 5) * 2));
      x[0] = (float)(int)(int8_t)head[row * 128 + i] * s;
    } else {
      uint32_t sz = *(const uint32_t *)(head + a.s.src.k_meta_off + row * 8 + (i >> 6) * 4);
      uint8_t byte = head[row * 64 + (i >> 1)];
      float p = (float)(int)((i & 1) ? (byte >> 4) : (byte & 0xf)) * h2f((uint16_t)(sz & 0xffff));
      x[0] = p + h2f((uint16_t)(sz >> 16));
    }
  }
  for (int u = 0; u < a.n_via; ++u) roundtrip<1, 32, 64>(a.via_k[u], x);
  return x[0];
}

// Running key sums per destination block, token order, and the fp16 mean key: one thread per channel, one
// workgroup per (sequence entry, KV head, destination block touched by this call).  A block that was partly
// filled before continues from its stored sum.
__global__ __launch_bounds__(128) void summary_kernel(const ConvArgs a) {
  const int j = blockIdx.x, h = blockIdx.y, z = blockIdx.z, i = threadIdx.x;
  const int seq = a.seq_id[j];
  const int r0 = a.dst_first_tok[j] % a.dst.bt;                 // row of the call's first token in its block
  const int t_lo = max(0, z * a.dst.bt - r0), t_hi = min(a.n_tokens, (z + 1) * a.dst.bt - r0);
  float sum = 0.0f;
  for (int t = t_lo; t < t_hi; ++t) {
    const float x = arriving_key(a, j, seq, h, t, i);
    const int tok = wrap(a.dst_first_tok[j] + t, a.dst);
    const int r = tok / a.dst.bt, row = tok - r * a.dst.bt;
    const int64_t rec = a.sum_table ? (int64_t)a.sum_table[(int64_t)seq * a.sum_ring_blocks + r] : (int64_t)a.sum_rec_base[j] + r;
    const int64_t o = (rec * a.Hkv + h) * 128 + i;
    if (row == 0)
      sum = 0.0f;
    else if (t == t_lo)
      sum = a.k_sum[o];
    sum = sum + x;
    if (row == a.dst.bt - 1 || t == a.n_tokens - 1) {
      a.k_sum[o] = sum;
      a.k_summary[o] = f2h(sum * a.inv_bt);
    }
  }
}

// Keys of a tier whose int4 groups run over 128 consecutive tokens of one channel (Q_4bit's arithmetic with the
// group turned by 90 degrees): one workgroup per (token group, KV head, entry), thread = channel.  Two passes
// over the group's 128 arriving rows: range, then codes; the two channels of a byte meet by a lane exchange.
__global__ __launch_bounds__(128) void convert_keys_t128_kernel(const ConvArgs a) {
  const int g = blockIdx.x, h = blockIdx.y, j = blockIdx.z, i = threadIdx.x;
  const int seq = a.seq_id[j];
  float lo = 0.0f, hi = 0.0f;
  for (int t = 0; t < 128; ++t) {
    const float x = arriving_key(a, j, seq, h, g * 128 + t, i);
    lo = t ? fminf(lo, x) : x;
    hi = t ? fmaxf(hi, x) : x;
  }
  if (lo == 0.0f) lo = 0.0f;  // a zero minimum is stored as +0 whatever its sign
  const float s32 = (hi - lo) / 15.0f;
  const uint16_t sh = f2h(s32), zh = f2h(lo);
  const float s = h2f(sh), z = h2f(zh);
  const float r = s != 0.0f ? 1.0f / s : 0.0f;
  int row0;
  uint8_t *head = head_ptr(a.dst, seq, a.dst_rec_base[j], wrap(a.dst_first_tok[j] + g * 128, a.dst), h, &row0);
  // the group's 128 meta rows of 4 bytes hold {scale, zero} of the 128 channels
  *(uint32_t *)(head + a.dst.k_meta_off + row0 * 4 + i * 4) = (uint32_t)sh | ((uint32_t)zh << 16);
  for (int t = 0; t < 128; ++t) {
    const float x = arriving_key(a, j, seq, h, g * 128 + t, i);
    float q = 0.0f;
    if (s != 0.0f) q = fminf(fmaxf(quot_rint(x - z, s, r), 0.0f), 15.0f);
    const int c = (int)q;
    const int other = __shfl_xor(c, 1);
    if (!(i & 1)) head[(row0 + t) * 64 + (i >> 1)] = (uint8_t)(c | (other << 4));
  }
}

// Values of a tier that stores Q_4bit codes channel-major per 32 tokens (TTKV_I4_ASYM_G64_T32): one workgroup per
// (group of 32 arriving tokens, KV head, entry).  Rows are quantized exactly as convert_rows_kernel does (a 16-lane
// group per row, 8 channels per lane); the meta rows go to their token-major section as usual, the codes meet in LDS
// and leave as the group's 2 KiB in the operand order of the matrix-core kernel: piece p = 64 hh + 16 kg + c, word w:
// channel 16 (4 hh + w) + c, nibble j: token kTok[j] + 4 kg.
__global__ __launch_bounds__(256) void convert_values_t32_kernel(const ConvArgs a) {
  __shared__ uint8_t s_code[32][128];
  const int g = blockIdx.x, h = blockIdx.y, j = blockIdx.z;
  const int seq = a.seq_id[j];
  const int l16 = threadIdx.x & 15;
  int row0;
  uint8_t *head = head_ptr(a.dst, seq, a.dst_rec_base[j], wrap(a.dst_first_tok[j] + g * 32, a.dst), h, &row0);   // row0 % 32 == 0
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = pass * 16 + (threadIdx.x >> 4), t = g * 32 + r;
    float x[8];
    if (!a.s.from_tier) {
      load8_flat(a.s.v_flat, a.s.flat_fmt, ((int64_t)j * a.Hkv + h) * a.n_tokens + t, l16, x);
    } else {
      int row;
      const uint8_t *src = head_ptr(a.s.src, seq, a.s.src_rec_base[j], wrap(a.s.src_first_tok[j] + t, a.s.src), h, &row);
      load8_tier(src, a.s.src.v_fmt, a.s.src.v_off, a.s.src.v_meta_off, row, l16, x);
    }
    for (int u = 0; u < a.n_via; ++u) roundtrip<8, 4, 8>(a.via_v[u], x);
    int c[8];
    uint16_t sh, zh;
    q2_group<8, 8>(x, c, &sh, &zh);
    if ((l16 & 7) == 0) *(uint32_t *)(head + a.dst.v_meta_off + (row0 + r) * 8 + (l16 >> 3) * 4) = (uint32_t)sh | ((uint32_t)zh << 16);
#pragma unroll
    for (int i = 0; i < 8; ++i) s_code[r][l16 * 8 + i] = (uint8_t)c[i];
  }
  __syncthreads();
  const int kTok[8] = {0, 2, 16, 18, 1, 3, 17, 19};
  uint32_t *out = (uint32_t *)(head + a.dst.v_off + row0 * 64);     // the group's 2 KiB: 512 words, two per thread
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int d = threadIdx.x + 256 * k;          // word index: piece d / 4, word d % 4
    const int p = d >> 2, w = d & 3;
    const int hh = p >> 6, kg = (p >> 4) & 3, c = p & 15;
    const int ch = 16 * (4 * hh + w) + c;
    uint32_t v = 0;
#pragma unroll
    for (int jn = 0; jn < 8; ++jn) v |= (uint32_t)s_code[kTok[jn] + 4 * kg][ch] << (4 * jn);
    out[d] = v;
  }
}

}  // namespace

hipError_t launch_convert(const ConvArgs &a, hipStream_t s, int *n_kernels) {
  const int64_t total = (int64_t)a.n_seq * a.Hkv * a.n_tokens;
  if (total <= 0) return hipSuccess;
  if (a.dst.k_fmt == TTKV_I4_ASYM_T128) {
    // values row by row, keys by groups of 128 tokens per channel (the caller has checked alignment)
    ConvArgs v = a;
    v.which0 = 1;
    hipLaunchKernelGGL(convert_rows_kernel, dim3((a.n_tokens + 15) / 16, 1, a.n_seq * a.Hkv), dim3(256), 0, s, v);
    hipLaunchKernelGGL(convert_keys_t128_kernel, dim3(a.n_tokens / 128, a.Hkv, a.n_seq), dim3(128), 0, s, a);
    *n_kernels += 2;
    return hipGetLastError();
  }
  if (a.dst.v_fmt == TTKV_I4_ASYM_G64_T32) {
    // keys row by row, values by groups of 32 tokens (the caller has checked alignment)
    hipLaunchKernelGGL(convert_rows_kernel, dim3((a.n_tokens + 15) / 16, 1, a.n_seq * a.Hkv), dim3(256), 0, s, a);   // which0 = 0: K only
    hipLaunchKernelGGL(convert_values_t32_kernel, dim3(a.n_tokens / 32, a.Hkv, a.n_seq), dim3(256), 0, s, a);
    *n_kernels += 2;
    return hipGetLastError();
  }
  dim3 grid((a.n_tokens + 15) / 16, 2, a.n_seq * a.Hkv);
  hipLaunchKernelGGL(convert_rows_kernel, grid, dim3(256), 0, s, a);
  ++*n_kernels;
  return hipGetLastError();
}

// `a.dst` gives the destination ring geometry only (block_tokens, ring_blocks);
// the kernel writes k_sum / k_summary, never dst.
hipError_t launch_summary(const ConvArgs &a, hipStream_t s, int *n_kernels) {
  if (a.n_seq <= 0 || a.n_tokens <= 0 || !a.k_sum) return hipSuccess;
  hipLaunchKernelGGL(summary_kernel, dim3(a.n_seq, a.Hkv, a.n_tokens / a.dst.bt + 2), dim3(128), 0, s, a);
  ++*n_kernels;
  return hipGetLastError();
}

}  // namespace ttkv
