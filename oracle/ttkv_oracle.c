/*
 * TTKV oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar CPU statement of what the tiered decode-attention path
 * computes.  It shares no code with the HIP library and is never called by it:
 * only tests, the smoke check and the benchmark's cpu_baseline leg load this.
 *
 * What each function follows (paper: "TTKV: Temporal-Tiered KV Cache"):
 *   - quantizers Q_8bit / Q_4bit and Decompress: Sec. 4.2 (differential
 *     quantization) and Alg. 1 "Decompress".  The paper fixes only the bit
 *     widths; scale / zero / group / rounding are this build's reading:
 *       Q1  symmetric int8,  32 consecutive elements of one token-head per group,
 *           one fp16 scale  = fp16(amax / 127)
 *       Q2  asymmetric int4, 64 consecutive elements per group,
 *           fp16 scale = fp16((hi - lo) / 15), fp16 zero = fp16(lo)
 *     every step is a single IEEE fp32 operation, rounding to nearest even.
 *   - attention partials and their merge: Alg. 1 (Attn on the fast tier, then
 *     "o <- o + Attn(q, K_j, V_j)" per slow-tier block), read as accumulation
 *     of un-normalised partials (m, l, acc) merged by log-sum-exp and
 *     normalised once at the end, so the result is softmax attention over the
 *     union of all attended tokens (Sec. 4.3).  All attention arithmetic is
 *     fp64.
 *   - block scoring phi and TopK: Alg. 1 "Block Identification"; phi is this
 *     build's reading (query . mean key summed over query heads).
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py
 * against closed forms, brute force, invariants or an independent library
 * routine, except nothing the paper prints (it prints no worked example).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

/* ------------------------------------------------------------------ fp16 */

/* fp32 -> fp16 bit pattern, round to nearest even, overflow to infinity. */
uint16_t o_f32_to_f16(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t sign = (u >> 16) & 0x8000u;
  uint32_t mag = u & 0x7fffffffu;
  if (mag >= 0x7f800000u) /* inf / nan */
    return (uint16_t)(sign | 0x7c00u | ((mag > 0x7f800000u) ? 0x200u : 0u));
  int32_t e = (int32_t)(mag >> 23) - 127; /* unbiased exponent */
  uint32_t man = mag & 0x7fffffu;
  if (e > 15) return (uint16_t)(sign | 0x7c00u);
  if (e >= -14) { /* normal half: keep 10 mantissa bits */
    uint32_t h = ((uint32_t)(e + 15) << 10) | (man >> 13);
    uint32_t rest = man & 0x1fffu; /* 13 dropped bits */
    if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) h += 1; /* may carry into exponent: correct */
    return (uint16_t)(sign | h);
  }
  if (e < -25) return (uint16_t)sign; /* below half of the smallest subnormal */
  /* subnormal half: value = m * 2^-24, m in [0, 1023] */
  man |= 0x800000u;                     /* 24-bit significand, value = man * 2^(e-23) */
  int shift = -e - 1;                   /* m = man >> shift, shift in [14, 24] */
  uint32_t h = man >> shift;
  uint32_t rest = man & ((1u << shift) - 1u);
  uint32_t half = 1u << (shift - 1);
  if (rest > half || (rest == half && (h & 1u))) h += 1;
  return (uint16_t)(sign | h);
}

float o_f16_to_f32(uint16_t h) {
  uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
  uint32_t e = (h >> 10) & 0x1fu;
  uint32_t m = h & 0x3ffu;
  float out;
  if (e == 0) { /* zero / subnormal: m * 2^-24 */
    out = (float)m * 5.9604644775390625e-08f;
    uint32_t u;
    memcpy(&u, &out, 4);
    u |= sign;
    memcpy(&out, &u, 4);
    return out;
  }
  uint32_t u = (e == 31) ? (sign | 0x7f800000u | (m << 13)) : (sign | ((e + 112u) << 23) | (m << 13));
  memcpy(&out, &u, 4);
  return out;
}

void o_f32_to_f16_array(const float *x, int64_t n, uint16_t *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = o_f32_to_f16(x[i]);
}
void o_f16_to_f32_array(const uint16_t *h, int64_t n, float *out) {
  for (int64_t i = 0; i < n; ++i) out[i] = o_f16_to_f32(h[i]);
}

/* ------------------------------------------------------------ quantizers */

/* Q1: symmetric int8, group of 32 along d.  x [rows][d] fp32 (d % 32 == 0),
 * codes [rows][d] int8, scale [rows][d/32] fp16 bits. */
void o_quant_i8_sym_g32(const float *x, int64_t rows, int32_t d, int8_t *codes, uint16_t *scale) {
  const int32_t ng = d / 32;
  for (int64_t r = 0; r < rows; ++r)
    for (int32_t g = 0; g < ng; ++g) {
      const float *xg = x + r * d + g * 32;
      float amax = 0.0f;
      for (int i = 0; i < 32; ++i) {
        float a = fabsf(xg[i]);
        if (a > amax) amax = a;
      }
      float s32 = amax / 127.0f;
      uint16_t sh = o_f32_to_f16(s32);
      float s = o_f16_to_f32(sh);
      scale[r * ng + g] = sh;
      for (int i = 0; i < 32; ++i) {
        float c = 0.0f;
        if (s != 0.0f) {
          c = rintf(xg[i] / s);
          if (c > 127.0f) c = 127.0f;
          if (c < -127.0f) c = -127.0f;
        }
        codes[r * d + g * 32 + i] = (int8_t)c;
      }
    }
}

/* Decompress for Q1: xhat = float(code) * float(scale), one fp32 multiply. */
void o_dequant_i8_sym_g32(const int8_t *codes, const uint16_t *scale, int64_t rows, int32_t d, float *xhat) {
  const int32_t ng = d / 32;
  for (int64_t r = 0; r < rows; ++r)
    for (int32_t j = 0; j < d; ++j)
      xhat[r * d + j] = (float)codes[r * d + j] * o_f16_to_f32(scale[r * ng + j / 32]);
}

/* Q2: asymmetric int4, group of 64 along d.  packed [rows][d/2]: element 2i in
 * the low nibble and 2i+1 in the high nibble of byte i.  scale, zero
 * [rows][d/64] fp16 bits. */
void o_quant_i4_asym_g64(const float *x, int64_t rows, int32_t d, uint8_t *packed, uint16_t *scale,
                         uint16_t *zero) {
  const int32_t ng = d / 64;
  for (int64_t r = 0; r < rows; ++r)
    for (int32_t g = 0; g < ng; ++g) {
      const float *xg = x + r * d + g * 64;
      float lo = xg[0], hi = xg[0];
      for (int i = 1; i < 64; ++i) {
        if (xg[i] < lo) lo = xg[i];
        if (xg[i] > hi) hi = xg[i];
      }
      if (lo == 0.0f) lo = 0.0f; /* a zero minimum is stored as +0 whatever its sign */
      float s32 = (hi - lo) / 15.0f;
      uint16_t sh = o_f32_to_f16(s32);
      uint16_t zh = o_f32_to_f16(lo);
      float s = o_f16_to_f32(sh);
      float z = o_f16_to_f32(zh);
      scale[r * ng + g] = sh;
      zero[r * ng + g] = zh;
      uint8_t c[64];
      for (int i = 0; i < 64; ++i) {
        float q = 0.0f;
        if (s != 0.0f) {
          q = rintf((xg[i] - z) / s);
          if (q > 15.0f) q = 15.0f;
          if (q < 0.0f) q = 0.0f;
        }
        c[i] = (uint8_t)q;
      }
      for (int i = 0; i < 32; ++i)
        packed[r * (d / 2) + g * 32 + i] = (uint8_t)(c[2 * i] | (c[2 * i + 1] << 4));
    }
}

/* Decompress for Q2: xhat = float(code) * float(scale) + float(zero); a
 * multiply then an add, each rounded to fp32 (no fused multiply-add). */
void o_dequant_i4_asym_g64(const uint8_t *packed, const uint16_t *scale, const uint16_t *zero,
                           int64_t rows, int32_t d, float *xhat) {
  const int32_t ng = d / 64;
  for (int64_t r = 0; r < rows; ++r)
    for (int32_t j = 0; j < d; ++j) {
      uint8_t byte = packed[r * (d / 2) + j / 2];
      float c = (float)((j & 1) ? (byte >> 4) : (byte & 0xf));
      volatile float prod = c * o_f16_to_f32(scale[r * ng + j / 64]);
      xhat[r * d + j] = prod + o_f16_to_f32(zero[r * ng + j / 64]);
    }
}

/* Q2 with the group turned by 90 degrees: asymmetric int4 where a group is the
 * 128 values one channel takes over 128 consecutive tokens (keys have the larger
 * variance and dynamic range, Sec. 3 "Tier Content" and Sec. 4.2, and it sits in a few
 * channels; a group along the tokens keeps such a channel from setting the
 * scale of its 63 neighbours).  Same arithmetic as o_quant_i4_asym_g64, same
 * nibble packing of a token's row.  x [tokens][d], tokens a multiple of 128;
 * packed [tokens][d/2]; scale, zero [tokens/128][d] fp16 bits. */
void o_quant_i4_asym_t128(const float *x, int64_t tokens, int32_t d, uint8_t *packed, uint16_t *scale,
                          uint16_t *zero) {
  for (int64_t g = 0; g < tokens / 128; ++g)
    for (int32_t j = 0; j < d; ++j) {
      const float *xg = x + g * 128 * d + j; /* stride d */
      float lo = xg[0], hi = xg[0];
      for (int t = 1; t < 128; ++t) {
        float v = xg[(int64_t)t * d];
        if (v < lo) lo = v;
        if (v > hi) hi = v;
      }
      if (lo == 0.0f) lo = 0.0f; /* a zero minimum is stored as +0 whatever its sign */
      float s32 = (hi - lo) / 15.0f;
      uint16_t sh = o_f32_to_f16(s32);
      uint16_t zh = o_f32_to_f16(lo);
      float s = o_f16_to_f32(sh);
      float z = o_f16_to_f32(zh);
      scale[g * d + j] = sh;
      zero[g * d + j] = zh;
      for (int t = 0; t < 128; ++t) {
        float q = 0.0f;
        if (s != 0.0f) {
          q = rintf((xg[(int64_t)t * d] - z) / s);
          if (q > 15.0f) q = 15.0f;
          if (q < 0.0f) q = 0.0f;
        }
        uint8_t *byte = packed + (g * 128 + t) * (d / 2) + j / 2;
        if (j & 1)
          *byte = (uint8_t)((*byte & 0x0f) | ((uint8_t)q << 4));
        else
          *byte = (uint8_t)((*byte & 0xf0) | (uint8_t)q);
      }
    }
}

/* Decompress for the above: xhat = float(code) * float(scale) + float(zero),
 * a multiply then an add, each rounded to fp32. */
void o_dequant_i4_asym_t128(const uint8_t *packed, const uint16_t *scale, const uint16_t *zero,
                            int64_t tokens, int32_t d, float *xhat) {
  for (int64_t t = 0; t < tokens; ++t)
    for (int32_t j = 0; j < d; ++j) {
      uint8_t byte = packed[t * (d / 2) + j / 2];
      float c = (float)((j & 1) ? (byte >> 4) : (byte & 0xf));
      volatile float prod = c * o_f16_to_f32(scale[(t / 128) * d + j]);
      xhat[t * d + j] = prod + o_f16_to_f32(zero[(t / 128) * d + j]);
    }
}

/* ------------------------------------------------------------- attention */

/* One un-normalised partial of Alg. 1's Attn(q, K, V) for every query head of
 * one sequence over tokens [t0, t0+n):
 *   s_j = softmax_scale * sum_i q[h][i] * K[h/G][j][i]
 *   m = max_j s_j,  l = sum_j exp(s_j - m),  acc[i] = sum_j exp(s_j - m) * V[h/G][j][i]
 * q [Hq][d]; K, V [Hkv][stride][d] (fp32 holding the stored or decompressed
 * values).  An empty range gives (m, l, acc) = (-inf, 0, 0).  fp64 throughout. */
void o_attn_partial(const float *q, int32_t Hq, int32_t Hkv, int32_t d, const float *K, const float *V,
                    int64_t stride, int64_t t0, int64_t n, double softmax_scale, double *m, double *l,
                    double *acc) {
  const int32_t G = Hq / Hkv;
#pragma omp parallel for schedule(static)
  for (int32_t h = 0; h < Hq; ++h) {
    const float *Kh = K + (int64_t)(h / G) * stride * d;
    const float *Vh = V + (int64_t)(h / G) * stride * d;
    double mm = -INFINITY;
    for (int64_t j = t0; j < t0 + n; ++j) {
      double s = 0.0;
      for (int32_t i = 0; i < d; ++i) s += (double)q[h * d + i] * (double)Kh[j * d + i];
      s *= softmax_scale;
      if (s > mm) mm = s;
    }
    double ll = 0.0;
    for (int32_t i = 0; i < d; ++i) acc[h * d + i] = 0.0;
    for (int64_t j = t0; j < t0 + n; ++j) {
      double s = 0.0;
      for (int32_t i = 0; i < d; ++i) s += (double)q[h * d + i] * (double)Kh[j * d + i];
      s *= softmax_scale;
      double p = exp(s - mm);
      ll += p;
      for (int32_t i = 0; i < d; ++i) acc[h * d + i] += p * (double)Vh[j * d + i];
    }
    m[h] = mm;
    l[h] = ll;
  }
}

/* Log-sum-exp merge of partial b into partial a, per row (rows = query heads):
 *   m* = max(ma, mb); l* = la e^(ma-m*) + lb e^(mb-m*); acc* likewise.
 * (-inf, 0, 0) is the identity. */
void o_merge_into(double *ma, double *la, double *acca, const double *mb, const double *lb,
                  const double *accb, int32_t rows, int32_t d) {
  for (int32_t r = 0; r < rows; ++r) {
    double mn = ma[r] > mb[r] ? ma[r] : mb[r];
    double wa = (ma[r] == -INFINITY) ? 0.0 : exp(ma[r] - mn);
    double wb = (mb[r] == -INFINITY) ? 0.0 : exp(mb[r] - mn);
    la[r] = la[r] * wa + lb[r] * wb;
    for (int32_t i = 0; i < d; ++i) acca[r * d + i] = acca[r * d + i] * wa + accb[r * d + i] * wb;
    ma[r] = mn;
  }
}

/* out = acc / l, lse = m + ln l.  Rows with no attended token give 0 and -inf. */
void o_finalize(const double *m, const double *l, const double *acc, int32_t rows, int32_t d,
                double *out, double *lse) {
  for (int32_t r = 0; r < rows; ++r) {
    if (l[r] == 0.0) {
      for (int32_t i = 0; i < d; ++i) out[r * d + i] = 0.0;
      lse[r] = -INFINITY;
    } else {
      for (int32_t i = 0; i < d; ++i) out[r * d + i] = acc[r * d + i] / l[r];
      lse[r] = m[r] + log(l[r]);
    }
  }
}

/* -------------------------------------------------- block summary, scoring */

/* Running per-block key sum, token order, fp32:  sum[h][i] += x[h][t][i] for
 * t = 0..n-1 in order.  x [Hkv][stride][d] starting at token t0. */
void o_summary_accumulate(float *sum, const float *x, int32_t Hkv, int32_t d, int64_t stride,
                          int64_t t0, int64_t n) {
  for (int32_t h = 0; h < Hkv; ++h)
    for (int32_t i = 0; i < d; ++i) {
      float s = sum[h * d + i];
      for (int64_t t = t0; t < t0 + n; ++t) s = s + x[((int64_t)h * stride + t) * d + i];
      sum[h * d + i] = s;
    }
}

/* mean-key summary: fp16( sum * (1 / block_tokens) ), one fp32 multiply. */
void o_summary_finish(const float *sum, int32_t n, int32_t block_tokens, uint16_t *mu) {
  const float inv = 1.0f / (float)block_tokens;
  for (int32_t i = 0; i < n; ++i) mu[i] = o_f32_to_f16(sum[i] * inv);
}

/* phi(q, B_j) = sum over query heads h of (q_h . mu_{h/G}): each head's dot
 * product is accumulated over the channels in ascending order with fused
 * multiply-add in fp32, and the per-head dot products are then added in
 * ascending head order in fp32, so that the value is one well-defined number
 * (and every head's chain can run on its own lane). */
float o_block_score(const float *q, const uint16_t *mu, int32_t Hq, int32_t Hkv, int32_t d) {
  const int32_t G = Hq / Hkv;
  float phi = 0.0f;
  for (int32_t h = 0; h < Hq; ++h) {
    float s = 0.0f;
    for (int32_t i = 0; i < d; ++i) s = fmaf(q[h * d + i], o_f16_to_f32(mu[(h / G) * d + i]), s);
    phi = phi + s;
  }
  return phi;
}

/* TopK: the k largest scores, ties to the lower block index; indices returned
 * ascending.  A NaN score (possible only with non-finite inputs, which are
 * outside the method's contract) ranks as -infinity, so that the ranks stay a
 * permutation and exactly min(k, n) blocks are chosen whatever the scores.
 * Returns the count written (min(k, n)). */
int32_t o_topk(const float *score, int32_t n, int32_t k, int32_t *sel) {
  if (k > n) k = n;
  if (k < 0) k = 0;
  uint8_t taken[65536];
  if (n > 65536) return -1;
  memset(taken, 0, (size_t)n);
  for (int32_t r = 0; r < k; ++r) {
    int32_t best = -1;
    float best_s = 0.0f;
    for (int32_t j = 0; j < n; ++j) {
      const float sj = score[j] != score[j] ? -INFINITY : score[j];
      if (!taken[j] && (best < 0 || sj > best_s)) {
        best = j;
        best_s = sj;
      }
    }
    taken[best] = 1;
  }
  int32_t c = 0;
  for (int32_t j = 0; j < n; ++j)
    if (taken[j]) sel[c++] = j;
  return c;
}
