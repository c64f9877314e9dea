// Grouped-query variant of the split-K decode attention partials (Alg. 1: Attn on the
// fast tier, Decompress + Attn per slow-tier block): all query heads that share a KV
// head are served by ONE pass over that head's K/V bytes, with the two contractions on
// the matrix cores (v_mfma_f32_16x16x32 f16 / bf16 for q.k and p.v, v_mfma_f32_16x16x16 for
// the layout changes).  Same work items, same partials and same record layout as the vector
// kernel; only the lane mapping differs.
//
// One 16-token tile, lane = (c = lane % 16, kg = lane / 16):
//   K rows are loaded in the MFMA A layout: lane (c, kg) holds 32 channels of token c, the 16-byte
//   pieces kg, kg + 4, ... of the row (one piece for int4, two for int8, four for fp16 / bf16), spliced
//   into packed 16-bit pairs as in the vector kernel.  Four 32-deep steps give
//       S[token][column] = sum_d K[token][d] * Q[d][column]
//   where a column is (quantization group, query head): the q operand is zero outside the
//   column's group, so every column is a per-group dot product.  The splice offsets leave
//   through the initial accumulator value.  In the MFMA result layout lane (c, kg) holds
//   column c of tokens 4 kg .. 4 kg + 3.  The token's four fp16 meta values (scale / zero per
//   group) reach that layout by one more product: meta words as A operand against a 0/1
//   selector of the column's group, which is exact.  The groups of one head are then summed
//   by DPP row rotations, which also leaves every column with its head's score.
//   The softmax is per column (lane-local over 4 tokens, two lane exchanges over kg); its scale
//   is applied inside the exponent.
//   V rows are loaded like K rows and dequantized in packed fp16 while the lane still owns
//   one token and one group: the centred code (int8: signed code, int4: code - 8) is taken out of the
//   splice exactly and multiplied by the scale, one rounding to nearest even.  A product with the identity matrix brings
//   the tile from [token][channel] to [channel][token]: the fp32 result (exact) has lane (c, kg)
//   holding channel-row c for tokens 4 kg .. 4 kg + 3, exactly the A layout of
//       O[channel][column] += sum_token V^T[channel][token] * P[token][column].
//   Two 16-token tiles feed one 32-deep product.  The int4 zero points and scales ride along as a
//   4-channel V (the meta words transposed the same way), giving sum_t p_t z_t and sum_t p_t s_t per group in fp32
//   (zero point + 8 x scale is what the centred codes leave out).  P is rounded to
//   fp16 once and that rounded value is used for the row sum as well, so the normalisation is consistent.
//   Values stored channel-major per 32 tokens (TTKV_I4_ASYM_G64_T32) need neither the dequantization nor the
//   transposition: a lane's 32-bit word IS eight tokens of one channel, i.e. after the splice the A operand of a
//   32-deep product, and the token's scale goes into the other operand instead: B_g = fp16(p_t * s_{t,g}), one per
//   channel group g (the four meta values of a token reach the score layout through the selector product that the
//   key meta uses).  The splice offsets (1024 / 64 per nibble position) and the centre 8 are removed by one more
//   product of B_g with a constant operand of "code 8" words; the zero points and the centre come back as
//   sum_t p_t (z_{t,g} + 8 s_{t,g}) in fp32 on the vector units.
//   Keys grouped over 128 tokens per channel have no channel groups (one column per head); the token
//   group's scales fold into the q operand, carried as fp16 rounded product + exact remainder
//   (two products per step), rebuilt for every 64 tokens in flight.
//
// Column budget: (group, head) columns come 16 to a pass of the score product, heads padded to 4, 8 or 16 where
// the keys have channel groups (idle columns cost nothing).  One pass serves int4 keys (2 groups) with up to 8
// heads per KV head and int8 keys (4 groups) with up to 4; two passes (a second q operand and selector, summed
// before the softmax) int8 keys with up to 8 heads and int4 keys with up to 16; four passes (one per group, the
// instantiation for 16 heads runs two waves per SIMD and has the registers for four q operands) int8 keys with up
// to 16.  fp16 / bf16 and keys grouped over tokens take any count up to 16.  More heads per KV head are cut into
// blocks of 16, one workgroup and one pass over the bytes per block (measured, 64 q / 4 kv heads, int8 keys: one
// block of 16 heads 5.8 TB/s of stored bytes against 4.0 as two blocks of 8).  Launches where the vector kernel is
// as fast or faster (two heads per KV head of one format) stay on the vector kernel.
#include "ttkv_attn_dev.h"

#include <algorithm>
#include <type_traits>

namespace ttkv {

namespace {

using namespace dev;

typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef short s4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));

template <bool BF>
__device__ __forceinline__ f4 mma(uint32_t a0, uint32_t a1, uint32_t b0, uint32_t b1, f4 c) {
  const uint2 A = {a0, a1}, B = {b0, b1};
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s4, A), __builtin_bit_cast(s4, B), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(h4, A), __builtin_bit_cast(h4, B), c, 0, 0, 0);
}

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
// 32-deep step (v_mfma_f32_16x16x32): lane (c, kg) supplies eight k-values; which eight is free as long as
// the A and the B lane of the same kg agree, so two 16-deep steps simply concatenate.
template <bool BF>
__device__ __forceinline__ f4 mma32(const uint32_t *a, const uint32_t *b, f4 c) {
  const uint4 A = {a[0], a[1], a[2], a[3]}, B = {b[0], b[1], b[2], b[3]};
  if constexpr (BF)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, A), __builtin_bit_cast(b8, B), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, A), __builtin_bit_cast(h8, B), c, 0, 0, 0);
}

// two fp32 values -> packed fp16, round to nearest even (v_cvt_pk_f16_f32)
typedef float f2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk(float x, float y) {
  const f2 v = {x, y};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, h2));
}

template <int F>
constexpr int n_groups() {
  return (F == TTKV_I4_ASYM_G64 || F == TTKV_I4_ASYM_G64_T32) ? 2 : (F == TTKV_I8_SYM_G32 ? 4 : 1);
}
// Channel, relative to the lane's 32-channel slice, of k-value i of step s: step s takes
// the packed registers 2s and 2s+1 that unpack16 produced (int4 pairs are (0,4) (1,5) | (2,6) (3,7)).
template <int F>
constexpr int chan(int s, int i) {
  if (is_i4<F>())
    return 8 * (s / 2) + ((s % 2) ? (i < 2 ? 2 + 4 * i : 3 + 4 * (i - 2)) : (i < 2 ? 4 * i : 1 + 4 * (i - 2)));
  return 4 * s + i;
}
// A lane's 32 channels of a row are the 16-byte pieces kg, kg + 4, ... of it (piece x of the lane = bytes
// [64 x + 16 kg, + 16) of the row), so that every load instruction of a tile reads 64 contiguous bytes per row
// (measured on a load-only kernel: 6.3 TB/s, against 5.3 TB/s when a lane's pieces are adjacent).  Element j
// of the lane's slice (j = 4 s + i in unpack order for fp16 / bf16 / int8) is therefore row channel:
template <int F>
__device__ __forceinline__ constexpr int slice_channel(int kg, int j) {
  if (is_i4<F>()) return 32 * kg + j;                                     // one piece of 32 channels
  if (F == TTKV_I8_SYM_G32) return 64 * (j / 16) + 16 * kg + j % 16;      // two pieces of 16
  return 32 * (j / 8) + 8 * kg + j % 8;                                   // four pieces of 8
}
// Splice offset carried by k-value i of a step.
template <int F>
constexpr float k_offset(int i) {
  return is_i4<F>() ? (i < 2 ? 1024.0f : 64.0f) : (F == TTKV_I8_SYM_G32 ? 1152.0f : 0.0f);
}

// ---- tiles of quantized rows prefetched through LDS
// The rows of a batch of tiles are copied global -> LDS asynchronously (no registers in between), the K half and
// the V half separately, while the batch before is being computed; the copy instructions read whole rows (whole
// 128-byte lines, so they carry the streaming hint), and the lanes then read their 16-byte pieces from LDS in the
// operand layout.  Inside LDS row r keeps its pieces in the order p ^ swz(r), which makes the 16 rows that the
// lanes of one piece read at a time fall into 16 different bank groups; the copy realises the order by choosing
// which piece each lane fetches.
constexpr int kTileRowsLds = 8 * 1024, kTileLds = kTileRowsLds + 4 * 256;   // per wave: K rows, V rows, 4 planes of meta words
typedef const __attribute__((address_space(1))) void *gas_ptr;
typedef __attribute__((address_space(3))) void *las_ptr;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// lane L's 16 (4) bytes land at dst + 16 L (4 L); dst is wave-uniform; OFF is added to both addresses.
template <int OFF = 0>
__device__ __forceinline__ void dma16(const uint8_t *src, char *dst) {
  __builtin_amdgcn_global_load_lds((gas_ptr)src, (las_ptr)dst, 16, OFF, 2);   // 2: non-temporal
}
__device__ __forceinline__ void dma4(const uint8_t *src, char *dst) {
  __builtin_amdgcn_global_load_lds((gas_ptr)src, (las_ptr)dst, 4, 0, 2);
}
// At most N of the wave's vector-memory loads are still outstanding (they complete in order).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// LDS reads of a landed half and the wait for them as one block (no use of a result can be scheduled in between;
// the reads are opaque to the compiler, which would otherwise wait for every copy in flight before an LDS read).
// A batch is 32 tokens = two tiles.  Rows: int8 w[0..3] = tile 0 piece x = 0, 1 (a0, a1), tile 1 likewise, 2 KiB
// further; int4 w[0..1] = the lane's one piece of tile 0, 1 (a0, 1 KiB further).  Meta: tile tt's two words from
// m0 + 64 tt and m0 + 256 + 64 tt.
__device__ __forceinline__ void lds_half_i4x2(uint32_t a0, uint32_t m0, u32x4 *w, uint32_t *m) {
  asm volatile("ds_read_b128 %0, %6\n\tds_read_b128 %1, %6 offset:1024\n\t"
               "ds_read_b32 %2, %7\n\tds_read_b32 %3, %7 offset:256\n\tds_read_b32 %4, %7 offset:64\n\t"
               "ds_read_b32 %5, %7 offset:320\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(w[0]), "=&v"(w[1]), "=&v"(m[0]), "=&v"(m[1]), "=&v"(m[2]), "=&v"(m[3])
               : "v"(a0), "v"(m0) : "memory");
}
// a batch of 64 tokens = four tiles: w[tt] = the lane's one piece of tile tt (a0, 1 KiB apart); meta: tile tt's two
// words from m0 + 64 tt and m0 + 256 + 64 tt
__device__ __forceinline__ void lds_half_i4x4(uint32_t a0, uint32_t m0, u32x4 *w, uint32_t *m) {
  asm volatile("ds_read_b128 %0, %12\n\tds_read_b128 %1, %12 offset:1024\n\tds_read_b128 %2, %12 offset:2048\n\t"
               "ds_read_b128 %3, %12 offset:3072\n\t"
               "ds_read_b32 %4, %13\n\tds_read_b32 %5, %13 offset:256\n\tds_read_b32 %6, %13 offset:64\n\t"
               "ds_read_b32 %7, %13 offset:320\n\tds_read_b32 %8, %13 offset:128\n\tds_read_b32 %9, %13 offset:384\n\t"
               "ds_read_b32 %10, %13 offset:192\n\tds_read_b32 %11, %13 offset:448\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(w[0]), "=&v"(w[1]), "=&v"(w[2]), "=&v"(w[3]), "=&v"(m[0]), "=&v"(m[1]), "=&v"(m[2]), "=&v"(m[3]),
                 "=&v"(m[4]), "=&v"(m[5]), "=&v"(m[6]), "=&v"(m[7])
               : "v"(a0), "v"(m0) : "memory");
}
// fp16 / bf16: w[4 tt + x] = piece x of the lane of tile tt, from ax (tile 1: 4 KiB further); no meta words.
__device__ __forceinline__ void lds_half_fp(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3, u32x4 *w) {
  asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\tds_read_b128 %3, %11\n\t"
               "ds_read_b128 %4, %8 offset:4096\n\tds_read_b128 %5, %9 offset:4096\n\t"
               "ds_read_b128 %6, %10 offset:4096\n\tds_read_b128 %7, %11 offset:4096\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(w[0]), "=&v"(w[1]), "=&v"(w[2]), "=&v"(w[3]), "=&v"(w[4]), "=&v"(w[5]), "=&v"(w[6]), "=&v"(w[7])
               : "v"(a0), "v"(a1), "v"(a2), "v"(a3) : "memory");
}
__device__ __forceinline__ void lds_half_i8(uint32_t a0, uint32_t a1, uint32_t m0, u32x4 *w, uint32_t *m) {
  asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %8 offset:2048\n\t"
               "ds_read_b128 %3, %9 offset:2048\n\t"
               "ds_read_b32 %4, %10\n\tds_read_b32 %5, %10 offset:256\n\tds_read_b32 %6, %10 offset:64\n\t"
               "ds_read_b32 %7, %10 offset:320\n\ts_waitcnt lgkmcnt(0)"
               : "=&v"(w[0]), "=&v"(w[1]), "=&v"(w[2]), "=&v"(w[3]), "=&v"(m[0]), "=&v"(m[1]), "=&v"(m[2]), "=&v"(m[3])
               : "v"(a0), "v"(a1), "v"(m0) : "memory");
}

// GT: query heads per KV head, padded to 4, 8 or 16, as a compile-time constant (quantized K: the column layout
// and the group sum below depend on it; columns of heads beyond the real count stay zero), or 0 to take the real
// count from the arguments (fp16 / bf16 / keys grouped over tokens: any count up to 16).
template <int KF, int VF, int GT>
__device__ __forceinline__ void process_mfma(const FusedArgs &a, const TierView &tv, const Entry &en, const int32_t *sel,
                                             int chunk_tokens, int chunk, int seq, int hq0, int Gr, int hkv, char *s_buf,
                                             float (*s_m)[16], float (*s_l)[16]) {
  // sel: null, or the block ids behind a run made of selected blocks (ring block of token i: sel[i / bt])
  // hq0, Gr: first query head and number of heads of this workgroup's block of heads (all heads of the KV head,
  // or a block of up to 8 / 16 of them)
  const int G = GT ? GT : Gr;              // heads per group block of columns
  using FK = Fmt<KF>;
  using FV = Fmt<VF>;
  constexpr int NLK = FK::ROWB / 64, NLV = FV::ROWB / 64;   // 16-byte loads per lane per 16-token tile
  // Quantized keys: rows prefetched through LDS (asynchronous global -> LDS copies with the streaming hint, the batch
  // after next in flight while one is computed).  Measured per format against register loads: K8/V8 5.2 -> 6.0-6.2
  // TB/s, K8/V4 4.9-5.1 -> 5.7-5.8 (batches of 32 tokens); int4 keys in batches of 64 tokens: with channel-major
  // values 5.2 -> 5.97 (of which 32 -> 64 tokens per batch 5.85 -> 5.97), with token-major values 5.09 -> 5.27 (in
  // batches of 32 they gained nothing: their unpack / dequantize / transpose arithmetic fills the issue slots).
  // fp16 / bf16 rows take the one-region variant further down.
  constexpr bool PF = (KF == TTKV_I8_SYM_G32 && (VF == TTKV_I8_SYM_G32 || VF == TTKV_I4_ASYM_G64 || VF == TTKV_I4_ASYM_G64_T32)) ||
                      (KF == TTKV_I4_ASYM_G64 && (VF == TTKV_I4_ASYM_G64_T32 || VF == TTKV_I4_ASYM_G64));
  // tiles in flight per wave (int4 on register loads: 4; with 2 that kernel is 10 % slower)
  constexpr bool PF64 = KF == TTKV_I4_ASYM_G64 && (VF == TTKV_I4_ASYM_G64_T32 || VF == TTKV_I4_ASYM_G64);   // prefetched in batches of 64 tokens
  constexpr int NT = PF64 ? 4 : (NLK == 4 || PF) ? 2 : 4 / NLK;
  constexpr int TT = 16 * NT;
  constexpr int NGK = n_groups<KF>(), NGV = n_groups<VF>();
  constexpr bool KQ = NGK > 1, VQ = NGV > 1;
  constexpr bool KT = KF == TTKV_I4_ASYM_T128;   // keys grouped over 128 tokens per channel: the scales fold into q
  constexpr bool KBF = KF == TTKV_BF16, VBF = VF == TTKV_BF16;
  constexpr bool VT = VF == TTKV_I4_ASYM_G64_T32;   // values channel-major per 32 tokens: no dequantization, no transposition
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, kg = lane >> 4;
  char *const wbuf = s_buf + wave * kTileLds;   // the wave's LDS: a batch of tiles in flight, at the end its result
  const int c0 = chunk * chunk_tokens;
  const int c1 = min(en.len, c0 + chunk_tokens);
  const int ring_tokens = tv.ring_blocks * tv.bt;
  const float cs = a.scale * kLog2e;       // scores are kept in the log2 domain

  // (group, head) columns: groups x heads of them, 16 per pass of the score product (NP = 2 when they exceed
  // one tile: int8 keys with 8 heads, int4 keys with 16; NP = 4: int8 keys with 16 heads).  Column n of pass pp is group (16 pp + n) / G of head n % G.
  constexpr int NP = KQ ? (NGK * GT + 15) / 16 : 1;
  const int g = n % G;                                   // head of this column
  int gam[NP];                                           // K group of this column, per pass
  bool col_on[NP];
#pragma unroll
  for (int pp = 0; pp < NP; ++pp) {
    gam[pp] = KQ ? min((16 * pp + n) / G, NGK - 1) : 0;
    col_on[pp] = 16 * pp + n < NGK * G && g < Gr;
  }

  // ---- q operand: 16 packed registers (step s: 2s, 2s+1), offset sum and plain sum of the column.  Element j
  // of the lane's slice enters only if its channel lies in the column's group.
  uint32_t qB[NP][16];
  float off[NP], qs[NP];
  {
    const uint4 *qrow = (const uint4 *)((const uint16_t *)a.q + ((int64_t)seq * a.Hq + hq0 + min(g, Gr - 1)) * 128);
    uint32_t qw[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {     // 8 channels per 16-byte load
      const uint4 w = qrow[slice_channel<KF>(kg, 8 * i) / 8];
      qw[4 * i] = w.x; qw[4 * i + 1] = w.y; qw[4 * i + 2] = w.z; qw[4 * i + 3] = w.w;
    }
    if constexpr (!KBF) {
      if (a.q_fmt == TTKV_BF16) {   // bf16 -> fp16 (exact inside the fp16 normal range, clamped outside)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float lo = fminf(fmaxf(__uint_as_float(qw[i] << 16), -65504.0f), 65504.0f);
          const float hi = fminf(fmaxf(__uint_as_float(qw[i] & 0xffff0000u), -65504.0f), 65504.0f);
          qw[i] = (uint32_t)__half_as_ushort(__float2half_rn(lo)) | ((uint32_t)__half_as_ushort(__float2half_rn(hi)) << 16);
        }
      }
    }
    // Register r of the operand pairs with register r of unpack16: elements (2r, 2r+1) of the slice, or for int4
    // (r = 4d + e) elements (8d + e, 8d + e + 4).  Both elements of a register lie in the same group.
    const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
    for (int pp = 0; pp < NP; ++pp) {
      float se = 0.0f, so = 0.0f;   // sums over the registers that carry splice offset 1024 / 64 (int4: even / odd)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        uint32_t w;
        int j0;   // first element of the register
        if constexpr (is_i4<KF>()) {
          const int dd = r / 4, e = r % 4;
          j0 = 8 * dd + e;
          w = __builtin_amdgcn_perm(qw[4 * dd + 2 + e / 2], qw[4 * dd + e / 2], (e & 1) ? 0x07060302u : 0x05040100u);
        } else {
          j0 = 2 * r;
          w = qw[r];
        }
        const bool on = col_on[pp] && slice_channel<KF>(kg, j0) / (128 / NGK) == gam[pp];
        qB[pp][r] = on ? w : 0u;
        if constexpr (KQ) {   // quantized keys are dotted with fp16 queries
          if ((r & 1) && KF == TTKV_I4_ASYM_G64) so = __builtin_amdgcn_fdot2(as_h2(qB[pp][r]), ones, so, false);
          else se = __builtin_amdgcn_fdot2(as_h2(qB[pp][r]), ones, se, false);
        }
      }
      qs[pp] = se + so;
      off[pp] = KF == TTKV_I4_ASYM_G64 ? fmaf(1024.0f, se, 64.0f * so) : k_offset<KF>(0) * se;
      // the column's group is spread over the channel slices of several lanes; the others contributed zero
      off[pp] += __shfl_xor(off[pp], 16); off[pp] += __shfl_xor(off[pp], 32);
      qs[pp] += __shfl_xor(qs[pp], 16);   qs[pp] += __shfl_xor(qs[pp], 32);
    }
  }

  // identity operand of the transposing product: k-value i of this lane is row 4 kg + i
  const uint32_t one = VBF ? 0x3F80u : 0x3C00u;
  const uint32_t id0 = (n == 4 * kg ? one : 0u) | (n == 4 * kg + 1 ? one << 16 : 0u);
  const uint32_t id1 = (n == 4 * kg + 2 ? one : 0u) | (n == 4 * kg + 3 ? one << 16 : 0u);
  // Selection operands that bring a token's four fp16 meta values (scale, zero per group) into the
  // score layout: with the meta words as A operand, k-values 0..3 of the kg = 0 lanes, the product
  // with a 0/1 column selector is exactly the scale (or zero) of the column's group, per token.
  uint32_t bs0[NP], bs1[NP], bz0[NP], bz1[NP];
#pragma unroll
  for (int pp = 0; pp < NP; ++pp) {
    bs0[pp] = bs1[pp] = bz0[pp] = bz1[pp] = 0;
    if (KQ && kg == 0) {
      const int ss = KF == TTKV_I4_ASYM_G64 ? 2 * gam[pp] : gam[pp];
      bs0[pp] = ss == 0 ? 0x3C00u : (ss == 1 ? 0x3C000000u : 0u);
      bs1[pp] = ss == 2 ? 0x3C00u : (ss == 3 ? 0x3C000000u : 0u);
      if (KF == TTKV_I4_ASYM_G64) {
        bz0[pp] = gam[pp] == 0 ? 0x3C000000u : 0u;
        bz1[pp] = gam[pp] == 1 ? 0x3C000000u : 0u;
      }
    }
  }
  // VT: 0/1 selectors of the token's V meta value number v = 0..3 (s0, z0, s1, z1) for every column at once
  uint32_t vm_sel[4][2];
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    vm_sel[v][0] = (VT && kg == 0 && v < 2) ? (v == 0 ? 0x3C00u : 0x3C000000u) : 0u;
    vm_sel[v][1] = (VT && kg == 0 && v >= 2) ? (v == 2 ? 0x3C00u : 0x3C000000u) : 0u;
  }
  // byte selectors that duplicate the fp16 scale of the group of this lane's piece x out of the V meta words:
  // int4 (s0, z0, s1, z1): one piece, group kg / 2; int8 (s0, s1, s2, s3): piece x lies in group 2 x + kg / 2
  uint32_t vsel[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const uint32_t vh = VF == TTKV_I4_ASYM_G64 ? (kg >> 1) * 2 : 2 * x + (kg >> 1);
    vsel[x] = (2 * vh) | ((2 * vh + 1) << 8) | ((2 * vh) << 16) | ((2 * vh + 1) << 24);
  }
  // minus (splice offset + centre) as packed fp16 pairs: int4 -(1024 + 8), -(64 + 8); int8 -(1024 + 128)
  uint32_t no_a = 0xE408E408u, no_b = 0xD480D480u, no_c = 0xE480E480u;
  asm volatile("" : "+s"(no_a), "+s"(no_b), "+s"(no_c));

  const f4 zero4 = f4{0.0f, 0.0f, 0.0f, 0.0f};
  f4 acc[8], accz = zero4;
  f4 accoff[VT ? 2 : 1];          // VT: sum_t B_g[t] * (splice offset of t's nibble position + 8), per channel group
  float zs[2] = {0.0f, 0.0f};     // VT: sum_t p_t (z_{t,g} + 8 s_{t,g})
#pragma unroll
  for (int s = 0; s < 8; ++s) acc[s] = zero4;
#pragma unroll
  for (int g2 = 0; g2 < (VT ? 2 : 1); ++g2) accoff[g2] = zero4;
  float m = -INFINITY, l = 0.0f;

  Splice sp;
  sp.init();

  struct TileRegs {
    uint4 kw[NT][NLK], vw[NT][NLV];
    uint2 kmeta[NT], vmeta[NT];
    uint4 gm[KT ? 8 : 1];   // KT: {scale, zero} of the lane's 32 channels for the token group of these tiles
  };
  const uint32_t kdoff = n * FK::ROWB + kg * 16, vdoff = n * FV::ROWB + kg * 16;

  // Plain loads here, not the non-temporal ones of the vector kernel: the load instructions of a tile share
  // cache lines (each reads 64 of a line's 128 bytes), and lines fetched with the streaming hint do not
  // survive until the next instruction.
  // Head section and row inside it of the chunk's token i.  The block table does not change during the launch and
  // the index is wave-uniform: it is read through the constant address space (a scalar load).
  auto locate = [&](int i, int &row0) -> const uint8_t * {
    int tok0 = en.first_tok + i;
    if (tok0 >= ring_tokens) tok0 -= ring_tokens;
    int rb = tok0 / tv.bt;
    row0 = tok0 - rb * tv.bt;
    typedef const __attribute__((address_space(4))) int32_t *const_i32;
    if (sel) rb = ((const_i32)(uintptr_t)sel)[rb] % tv.ring_blocks;   // written by the launch before this one: a scalar load
    const int64_t rec = tv.table ? (int64_t)((const_i32)(uintptr_t)tv.table)[(int64_t)seq * tv.ring_blocks + rb]
                                 : (int64_t)en.rec_base + rb;
    return tv.base + rec * tv.rec_bytes + (int64_t)hkv * tv.head_bytes;
  };
  auto load_tiles = [&](TileRegs &t, int i0, int nv, auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    int row0;
    const uint8_t *head = locate(i0, row0);
    const uint8_t *kb = head + row0 * FK::ROWB, *kmb = head + tv.k_meta_off + row0 * 8;
    const uint8_t *vb = head + tv.v_off + row0 * FV::ROWB, *vmb = head + tv.v_meta_off + row0 * 8;
    if constexpr (KT) {   // the 64 tokens in flight lie inside one aligned group of 128: its 128 meta rows x 4 B
      const uint4 *gp = (const uint4 *)(head + tv.k_meta_off + (row0 & ~127) * 4 + kg * 128);
#pragma unroll
      for (int i = 0; i < 8; ++i) t.gm[i] = gp[i];
    }
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
      const uint32_t row = FULL ? tt * 16 + n : min(tt * 16 + n, nv - 1);   // rows past the end re-read the last live row
      const uint32_t ko = FULL ? kdoff + tt * 16 * FK::ROWB : row * FK::ROWB + kg * 16;
      const uint32_t vo = FULL ? vdoff + tt * 16 * FV::ROWB : row * FV::ROWB + kg * 16;
#pragma unroll
      for (int x = 0; x < NLK; ++x) t.kw[tt][x] = *(const uint4 *)(kb + ko + 64 * x);
      if constexpr (VT) {
        // piece hh = tt % 2 of the 32-token group tt / 2 (a group past the end re-reads the last live one):
        // lane L's piece is number 64 hh + L of the group's 2 KiB
        const uint32_t grp = FULL ? tt / 2 : min(tt / 2, (nv - 1) / 32);
        t.vw[tt][0] = *(const uint4 *)(vb + grp * 2048 + (tt & 1) * 1024 + lane * 16);
      } else {
#pragma unroll
        for (int x = 0; x < NLV; ++x) t.vw[tt][x] = *(const uint4 *)(vb + vo + 64 * x);
      }
      if constexpr (KQ) t.kmeta[tt] = *(const uint2 *)(kmb + row * 8);
      if constexpr (VQ) t.vmeta[tt] = *(const uint2 *)(vmb + row * 8);
    }
  };

  // ---- PF: the same rows as asynchronous copies into the wave's LDS and reads from there.
  // LDS of the wave: K rows at 0, V rows at 4 KiB (row r at r ROWB, its piece p at 16 (p ^ swz(r))), then four
  // planes of 64 meta words: K words 0 and 1 of the batch's tokens, V words 0 and 1.
  constexpr int PK = FK::ROWB / 16, PV = FV::ROWB / 16;              // pieces per row
  constexpr int NDK = TT * FK::ROWB / 1024, NDV = TT * FV::ROWB / 1024;   // copy instructions of 1 KiB per half
  constexpr int N_K = NDK + 2, N_V = NDV + 2;                          // with the two meta planes
  static_assert(!PF || PF64 || (NT == 2 && ((PK == 8 && NDK == 4) || (PK == 4 && NDK == 2)) && (NDV == 4 || NDV == 2)),
                "the batch the LDS readers cover");
  auto swz = [](int pieces, int r) { return pieces == 4 ? (r >> 2) & 3 : (r >> 1) & 7; };
  // per-lane byte offset of copy instruction j inside a full batch, minus j KiB (even and odd j differ for 8 pieces)
  uint32_t dko[2], dvo[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int rk = j * (64 / PK) + lane / PK, rv = j * (64 / PV) + lane / PV;
    dko[j] = rk * FK::ROWB + ((lane % PK) ^ swz(PK, rk)) * 16 - j * 1024;
    dvo[j] = rv * FV::ROWB + ((lane % PV) ^ swz(PV, rv)) * 16 - j * 1024;
  }
  const uint32_t lds0 = (uint32_t)(uintptr_t)(las_ptr)wbuf;
  // where lane (n, kg) finds its piece kg (and kg + 4) of row n of tile 0
  auto piece_addr = [&](int pieces, int rowb, int x) -> uint32_t {
    return n * rowb + (((kg + 4 * x) ^ swz(pieces, n)) * 16);
  };
  const uint32_t lka0 = lds0 + piece_addr(PK, FK::ROWB, 0), lka1 = lds0 + piece_addr(PK, FK::ROWB, PK == 8 ? 1 : 0);
  const uint32_t lva0 = VT ? lds0 + 4096 + lane * 16 : lds0 + 4096 + piece_addr(PV, FV::ROWB, 0);
  const uint32_t lva1 = lds0 + 4096 + piece_addr(PV, FV::ROWB, PV == 8 ? 1 : 0);
  const uint32_t lkm = lds0 + kTileRowsLds + n * 4, lvm = lkm + 512;
  const uint8_t *nx_head = nullptr;   // batch whose K half was issued last
  int nx_row0 = 0, nx_nv = 0;
  auto issue_k = [&](int i0) {
    nx_head = locate(i0, nx_row0);
    nx_nv = min(TT, c1 - i0);
    const uint8_t *kb = nx_head + nx_row0 * FK::ROWB, *kmb = nx_head + tv.k_meta_off + nx_row0 * 8;
    if (nx_nv == TT) {
      dma16<0>(kb + dko[0], wbuf); dma16<1024>(kb + dko[1], wbuf);
      if constexpr (NDK == 4) {
        dma16<2048>(kb + dko[0], wbuf); dma16<3072>(kb + dko[1], wbuf);
      }
    } else {
#pragma unroll
      for (int j = 0; j < NDK; ++j) {
        const int r = j * (64 / PK) + lane / PK;   // LDS row; rows past the end repeat the last live row
        dma16(kb + min(r, nx_nv - 1) * FK::ROWB + ((lane % PK) ^ swz(PK, r)) * 16, wbuf + j * 1024);
      }
    }
    const uint32_t mo = min(lane, nx_nv - 1) * 8;   // one lane per token (TT = 32: the upper lanes repeat the last row)
    dma4(kmb + mo, wbuf + kTileRowsLds);
    dma4(kmb + mo + 4, wbuf + kTileRowsLds + 256);
  };
  auto issue_v = [&]() {
    const uint8_t *vb = nx_head + tv.v_off + nx_row0 * FV::ROWB, *vmb = nx_head + tv.v_meta_off + nx_row0 * 8;
    if constexpr (VT) {   // whole 2 KiB groups (lengths are multiples of 32), copied as they lie
      dma16<0>(vb + lane * 16, wbuf + 4096); dma16<1024>(vb + lane * 16, wbuf + 4096);
      if constexpr (PF64) {   // the second group: inside the record even when the run ends before it (its weights are 0)
        dma16<2048>(vb + lane * 16, wbuf + 4096); dma16<3072>(vb + lane * 16, wbuf + 4096);
      }
    } else if (nx_nv == TT) {
      dma16<0>(vb + dvo[0], wbuf + 4096); dma16<1024>(vb + dvo[1], wbuf + 4096);
      if constexpr (NDV == 4) {
        dma16<2048>(vb + dvo[0], wbuf + 4096); dma16<3072>(vb + dvo[1], wbuf + 4096);
      }
    } else {
#pragma unroll
      for (int j = 0; j < NDV; ++j) {
        const int r = j * (64 / PV) + lane / PV;
        dma16(vb + min(r, nx_nv - 1) * FV::ROWB + ((lane % PV) ^ swz(PV, r)) * 16, wbuf + 4096 + j * 1024);
      }
    }
    const uint32_t mo = min(lane, nx_nv - 1) * 8;
    dma4(vmb + mo, wbuf + kTileRowsLds + 512);
    dma4(vmb + mo + 4, wbuf + kTileRowsLds + 768);
  };
  auto fetch_k = [&](auto &t) {   // generic: compiled only where it is called, i.e. for the formats of PF
    u32x4 w[4];
    uint32_t mw[8];
    if constexpr (PK == 8) lds_half_i8(lka0, lka1, lkm, w, mw);
    else if constexpr (PF64) lds_half_i4x4(lka0, lkm, w, mw);
    else lds_half_i4x2(lka0, lkm, w, mw);
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
#pragma unroll
      for (int x = 0; x < NLK; ++x) {
        const u32x4 v = w[tt * NLK + x];
        t.kw[tt][x] = uint4{v.x, v.y, v.z, v.w};
      }
      t.kmeta[tt] = uint2{mw[2 * tt], mw[2 * tt + 1]};
    }
  };
  auto fetch_v = [&](auto &t) {
    u32x4 w[4];
    uint32_t mw[8];
    if constexpr (PV == 8) lds_half_i8(lva0, lva1, lvm, w, mw);
    else if constexpr (PF64) lds_half_i4x4(lva0, lvm, w, mw);
    else lds_half_i4x2(lva0, lvm, w, mw);
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
#pragma unroll
      for (int x = 0; x < NLV; ++x) {
        const u32x4 v = w[tt * NLV + x];
        t.vw[tt][x] = uint4{v.x, v.y, v.z, v.w};
      }
      t.vmeta[tt] = uint2{mw[2 * tt], mw[2 * tt + 1]};
    }
  };

  // before_v runs between the softmax and the first use of the batch's V half.
  auto compute_tiles = [&](TileRegs &t, int nv, auto full_tag, auto before_v) {
    constexpr bool FULL = decltype(full_tag)::value;
    // ---- KT: q . k = sum_d (q_d s_d) (c_d - 8) + sum_d q_d (z_d + 8 s_d) with s, z of the token group.  q_d s_d
    // is carried as two fp16 operands (rounded product and exact remainder), both multiplied with the codes;
    // the sums over q s and q z are exact products accumulated in fp32 and leave with the initial value.
    uint32_t qh[KT ? 16 : 1], ql[KT ? 16 : 1];
    float off_t = 0.0f;
    if constexpr (KT) {
      float se = 0.0f, so = 0.0f, qz = 0.0f;
#pragma unroll
      for (int dd = 0; dd < 4; ++dd) {
        const uint32_t m8[8] = {t.gm[2 * dd].x, t.gm[2 * dd].y, t.gm[2 * dd].z, t.gm[2 * dd].w,
                                t.gm[2 * dd + 1].x, t.gm[2 * dd + 1].y, t.gm[2 * dd + 1].z, t.gm[2 * dd + 1].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {   // operand register 4 dd + j holds channels (8 dd + j, 8 dd + j + 4) of the slice
          const int r = 4 * dd + j;
          const h2 s2 = as_h2(__builtin_amdgcn_perm(m8[j + 4], m8[j], 0x05040100u));
          const h2 z2 = as_h2(__builtin_amdgcn_perm(m8[j + 4], m8[j], 0x07060302u));
          const h2 q2 = as_h2(qB[0][r]);
          const h2 hi = q2 * s2;
          qh[r] = __builtin_bit_cast(uint32_t, hi);
          ql[r] = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(q2, s2, -hi));
          if (r & 1) so = __builtin_amdgcn_fdot2(q2, s2, so, false);
          else se = __builtin_amdgcn_fdot2(q2, s2, se, false);
          qz = __builtin_amdgcn_fdot2(q2, z2, qz, false);
        }
      }
      // splice offsets 1024 / 64 plus the centre 8, minus the zero-point sum; summed over the four channel slices
      off_t = fmaf(1032.0f, se, 72.0f * so) - fmaf(8.0f, se + so, qz);
      off_t += __shfl_xor(off_t, 16);
      off_t += __shfl_xor(off_t, 32);
    }

    // ---- scores (log2 domain), column n of tokens 4 kg + i
    f4 S[NT];
    float mt = -INFINITY;
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
      uint32_t kr[16];
#pragma unroll
      for (int x = 0; x < NLK; ++x) unpack16<KF>(t.kw[tt][x], kr + x * (16 / NLK), sp);
      f4 sv[NP], ksv[NP], kzv[NP];
#pragma unroll
      for (int pp = 0; pp < NP; ++pp) {
        if constexpr (KT) {
          sv[pp] = f4{-off_t, -off_t, -off_t, -off_t};
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            sv[pp] = mma32<false>(kr + 4 * s, qh + 4 * s, sv[pp]);
            sv[pp] = mma32<false>(kr + 4 * s, ql + 4 * s, sv[pp]);
          }
        } else {
          sv[pp] = f4{-off[pp], -off[pp], -off[pp], -off[pp]};
#pragma unroll
          for (int s = 0; s < 4; ++s) sv[pp] = mma32<KBF>(kr + 4 * s, qB[pp] + 4 * s, sv[pp]);
        }
        ksv[pp] = kzv[pp] = zero4;
        if constexpr (KQ) ksv[pp] = mma<false>(t.kmeta[tt].x, t.kmeta[tt].y, bs0[pp], bs1[pp], zero4);
        if constexpr (KF == TTKV_I4_ASYM_G64) kzv[pp] = mma<false>(t.kmeta[tt].x, t.kmeta[tt].y, bz0[pp], bz1[pp], zero4);
      }
      f4 sc;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float x = 0.0f;
#pragma unroll
        for (int pp = 0; pp < NP; ++pp) {
          if constexpr (KF == TTKV_I8_SYM_G32) x = fmaf(sv[pp][i], ksv[pp][i], x);
          else if constexpr (KF == TTKV_I4_ASYM_G64) x += fmaf(kzv[pp][i], qs[pp], sv[pp][i] * ksv[pp][i]);
          else x = sv[pp][i];
        }
        if constexpr (KQ) {   // sum the groups of a head: cyclic over the columns with the same n % G
          if constexpr (GT <= 8) x += dpp<0x128>(x);
          if constexpr (GT <= 4) x += dpp<0x124>(x);
          if constexpr (GT <= 2) x += dpp<0x122>(x);
        }
        if (!FULL && tt * 16 + 4 * kg + i >= nv) x = -INFINITY;
        sc[i] = x;
        mt = fmaxf(mt, x);
      }
      S[tt] = sc;
    }

    // ---- online softmax (base 2) per column; m is kept in raw score units, the scale enters the exponent
    mt = fmaxf(mt, __shfl_xor(mt, 16));
    mt = fmaxf(mt, __shfl_xor(mt, 32));
    if (__any(mt > m)) {
      const float mn = fmaxf(m, mt);
      const float alpha = __builtin_amdgcn_exp2f((m - mn) * cs);
      l *= alpha;
      accz *= alpha;
      if constexpr (VT) {
        accoff[0] *= alpha; accoff[1] *= alpha;
        zs[0] *= alpha; zs[1] *= alpha;
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) acc[s] *= alpha;
      m = mn;
    }
    const float mcs = -m * cs;
    const h2 ones = {(_Float16)1.0f, (_Float16)1.0f};

    // ---- weighted V, two 16-token tiles per 32-deep product
    before_v();
    if constexpr (VT) {
      // Values channel-major per 32 tokens: tiles tp, tp + 1 are one group; its two pieces are the A operands of the
      // eight channel blocks as they lie (after the splice), the scales ride on the weights.  What is removed with
      // the offsets is the spliced word of eight codes 8, so that a weight's rounding error multiplies code - 8.
      const uint32_t code8[4] = {sp.c0 | 0x00080008u, sp.c1 | 0x00800080u, sp.c0 | 0x00080008u, sp.c1 | 0x00800080u};
#pragma unroll
      for (int tp = 0; tp < NT; tp += 2) {
        uint32_t Bg[2][4];       // fp16(p_t * s_{t,g}) of the pair's 8 tokens per lane, per channel group g
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int tt = tp + u;
          // the token's meta values (s0, z0, s1, z1) in the score layout: tokens 4 kg + i of the tile, any column
          f4 mv[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) mv[v] = mma<false>(t.vmeta[tt].x, t.vmeta[tt].y, vm_sel[v][0], vm_sel[v][1], zero4);
          float p[4];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            p[i] = __builtin_amdgcn_exp2f(fmaf(S[tt][i], cs, mcs));
            l += p[i];
            zs[0] = fmaf(p[i], fmaf(8.0f, mv[0][i], mv[1][i]), zs[0]);   // zero point + the centre 8 * scale
            zs[1] = fmaf(p[i], fmaf(8.0f, mv[2][i], mv[3][i]), zs[1]);
          }
          Bg[0][2 * u] = pk(p[0] * mv[0][0], p[1] * mv[0][1]);
          Bg[0][2 * u + 1] = pk(p[2] * mv[0][2], p[3] * mv[0][3]);
          Bg[1][2 * u] = pk(p[0] * mv[2][0], p[1] * mv[2][1]);
          Bg[1][2 * u + 1] = pk(p[2] * mv[2][2], p[3] * mv[2][3]);
        }
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          uint32_t vr[16];       // word w of piece hh -> registers 4 w .. 4 w + 3: channel 16 (4 hh + w) + (lane % 16)
          unpack16<TTKV_I4_ASYM_G64>(t.vw[tp + hh][0], vr, sp);
#pragma unroll
          for (int w = 0; w < 4; ++w) acc[4 * hh + w] = mma32<false>(vr + 4 * w, Bg[hh], acc[4 * hh + w]);
          accoff[hh] = mma32<false>(code8, Bg[hh], accoff[hh]);
        }
      }
    } else {
#pragma unroll
    for (int tp = 0; tp < NT; tp += 2) {
      uint32_t pB[4];          // softmax weights of the pair, rounded to fp16: the B operand
      uint32_t vr[2][16];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int tt = tp + u;
        float p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) p[i] = __builtin_amdgcn_exp2f(fmaf(S[tt][i], cs, mcs));
        pB[2 * u] = pk(p[0], p[1]);
        pB[2 * u + 1] = pk(p[2], p[3]);
        l = __builtin_amdgcn_fdot2(as_h2(pB[2 * u]), ones, l, false);       // the row sum uses the rounded weights
        l = __builtin_amdgcn_fdot2(as_h2(pB[2 * u + 1]), ones, l, false);

#pragma unroll
        for (int x = 0; x < NLV; ++x) unpack16<VF>(t.vw[tt][x], vr[u] + x * (16 / NLV), sp);
        if constexpr (VQ) {
          // codes -> code * scale in fp16 with one rounding (to nearest even), while the lane still owns one token
          // and one group.  The splice holds offset + code; the centred code (int8: the signed code, int4: code - 8)
          // is taken out first, which is exact, and then scaled, so that the one rounding is relative to a value of
          // the size of the element itself (scaling offset + code in one fused step and removing offset * scale
          // afterwards would round a value up to the row's whole range: an error of range x 2^-11 on its smallest
          // elements).  The int4 centre 8 * scale rejoins with the zero points at the end.
          const uint32_t vsb0 = __builtin_amdgcn_perm(t.vmeta[tt].y, t.vmeta[tt].x, vsel[0]);
          const uint32_t vsb1 = VF == TTKV_I8_SYM_G32 ? __builtin_amdgcn_perm(t.vmeta[tt].y, t.vmeta[tt].x, vsel[1]) : vsb0;
          const h2 vs2[2] = {as_h2(vsb0), as_h2(vsb1)};
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const uint32_t no = VF == TTKV_I8_SYM_G32 ? no_c : ((r & 1) ? no_b : no_a);
            vr[u][r] = __builtin_bit_cast(uint32_t, (as_h2(vr[u][r]) + as_h2(no)) * vs2[r / 8]);
          }
        }
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const f4 d0 = mma<VBF>(vr[0][2 * s], vr[0][2 * s + 1], id0, id1, zero4);
        const f4 d1 = mma<VBF>(vr[1][2 * s], vr[1][2 * s + 1], id0, id1, zero4);
        const uint32_t A[4] = {pk(d0[0], d0[1]), pk(d0[2], d0[3]), pk(d1[0], d1[1]), pk(d1[2], d1[3])};
        acc[s] = mma32<false>(A, pB, acc[s]);
      }
      if constexpr (VF == TTKV_I4_ASYM_G64) {
        // the meta words transposed like a 4-channel V: every row group of four then accumulates
        // sum_t p_t * (s0, z0, s1, z1)
        const f4 d0 = mma<false>(t.vmeta[tp].x, t.vmeta[tp].y, id0, id1, zero4);
        const f4 d1 = mma<false>(t.vmeta[tp + 1].x, t.vmeta[tp + 1].y, id0, id1, zero4);
        const uint32_t A[4] = {pk(d0[0], d0[1]), pk(d0[2], d0[3]), pk(d1[0], d1[1]), pk(d1[2], d1[3])};
        accz = mma32<false>(A, pB, accz);
      }
    }
    }
  };

  // ---- fp16 / bf16 rows through LDS: a half (K or V rows of a batch of 32 tokens) is 8 KiB, so the wave's LDS
  // takes one half at a time: K of batch i is read out, V of batch i is copied in while the scores are computed,
  // read out, K of batch i + 1 copied in while the weighted values are computed.  Row r keeps its 16 pieces in the
  // order p ^ (r & 15).
  constexpr bool PF2 = (KF == TTKV_F16 || KF == TTKV_BF16) && KF == VF;
  const uint8_t *cur_head = nullptr;
  int cur_row0 = 0, cur_nv = 0;
  auto issue_fp = [&](const uint8_t *rows, int nv) {   // rows: the half's first row
    if (nv == 32) {
      const uint32_t r0 = lane >> 4, s0 = (lane & 15) ^ r0;   // copy j: row 4 j + r0, piece s0 ^ 4 (j & 3)
      const uint8_t *a0 = rows + r0 * 256 + s0 * 16, *a1 = rows + r0 * 256 + (s0 ^ 4) * 16;
      const uint8_t *a2 = rows + r0 * 256 + (s0 ^ 8) * 16, *a3 = rows + r0 * 256 + (s0 ^ 12) * 16;
      dma16<0>(a0, wbuf); dma16<1024>(a1, wbuf); dma16<2048>(a2, wbuf); dma16<3072>(a3, wbuf);
      dma16<0>(a0 + 4096, wbuf + 4096); dma16<1024>(a1 + 4096, wbuf + 4096);
      dma16<2048>(a2 + 4096, wbuf + 4096); dma16<3072>(a3 + 4096, wbuf + 4096);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = 4 * j + (lane >> 4);   // LDS row; rows past the end repeat the last live row
        dma16(rows + min(r, nv - 1) * 256 + (((lane & 15) ^ (r & 15)) * 16), wbuf + j * 1024);
      }
    }
  };
  auto fetch_fp = [&](auto *dst) {   // dst: kw or vw of the tile registers
    const uint32_t base = (uint32_t)(uintptr_t)(las_ptr)wbuf + n * 256 + ((kg ^ (n & 3)) * 16);
    const uint32_t hi = n >> 2;   // piece kg + 4 x sits at slot (kg ^ (n & 3)) + 4 (x ^ hi)
    u32x4 w[8];
    lds_half_fp(base + ((0 ^ hi) << 6), base + ((1 ^ hi) << 6), base + ((2 ^ hi) << 6), base + ((3 ^ hi) << 6), w);
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const u32x4 v = w[4 * tt + x];
        dst[tt][x] = uint4{v.x, v.y, v.z, v.w};
      }
  };
  auto fp_loop = [&](auto &ra) {   // generic: compiled only for the formats of PF2
    int i0 = c0 + wave * TT;
    if (i0 < c1) {
      cur_head = locate(i0, cur_row0);
      cur_nv = min(TT, c1 - i0);
      issue_fp(cur_head + cur_row0 * 256, cur_nv);
    }
    auto step = [&](int nv, auto full_tag) {
      wait_vmcnt<0>();
      fetch_fp(ra.kw);
      issue_fp(cur_head + tv.v_off + cur_row0 * 256, cur_nv);
      compute_tiles(ra, nv, full_tag, [&]() {
        wait_vmcnt<0>();
        fetch_fp(ra.vw);
        if (i0 + 4 * TT < c1) {   // wave-uniform
          cur_head = locate(i0 + 4 * TT, cur_row0);
          cur_nv = min(TT, c1 - i0 - 4 * TT);
          issue_fp(cur_head + cur_row0 * 256, cur_nv);
        }
      });
    };
    for (; i0 + TT <= c1; i0 += 4 * TT) step(TT, std::true_type{});
    if (i0 < c1) step(c1 - i0, std::false_type{});
  };

  auto register_loop = [&]() {
    TileRegs ra;
    int i0 = c0 + wave * TT;
    for (; i0 + TT <= c1; i0 += 4 * TT) {
      load_tiles(ra, i0, TT, std::true_type{});
      compute_tiles(ra, TT, std::true_type{}, []() {});
    }
    if (i0 < c1) {
      load_tiles(ra, i0, c1 - i0, std::false_type{});
      compute_tiles(ra, c1 - i0, std::false_type{}, []() {});
    }
  };
  // int8-key records in pinned host memory keep the register loads: over PCIe the copies through LDS are 3-4 %
  // slower for them (measured), and the streaming hint has nothing to gain there.
  if constexpr (PF) {
    if (!tv.in_host) {
      // While batch i is computed the copies of batch i + 1 are in flight: its K half is issued once batch i's K
      // rows are in registers, its V half once batch i's V rows are.  Loads complete in order, so "at most as
      // many outstanding as were issued after it" means a half has landed.
      TileRegs ra;
      int i0 = c0 + wave * TT;
      if (i0 < c1) {
        issue_k(i0);
        issue_v();
      }
      auto step = [&](int nv, auto full_tag) {
        const bool more = i0 + 4 * TT < c1;   // wave-uniform
        wait_vmcnt<N_V>();
        fetch_k(ra);
        if (more) issue_k(i0 + 4 * TT);
        compute_tiles(ra, nv, full_tag, [&]() {
          if (more) wait_vmcnt<N_K>();
          else wait_vmcnt<0>();
          fetch_v(ra);
          if (more) issue_v();
        });
      };
      for (; i0 + TT <= c1; i0 += 4 * TT) step(TT, std::true_type{});
      if (i0 < c1) step(c1 - i0, std::false_type{});
    } else {
      register_loop();
    }
  } else if constexpr (PF2) {
    static_assert(!PF2 || (TT == 32 && NT == 2 && NLK == 4 && NLV == 4), "the batch the LDS readers cover");
    // also for a tier in pinned host memory: the copies read whole 256-byte rows, where the register loads ask
    // for 64 bytes of a row per instruction -- over PCIe 55.7 against 42.8 GB/s (measured)
    TileRegs ra;
    fp_loop(ra);
  } else {
    register_loop();
  }

  // ---- the wave's result: column n < G of lane (n, kg) holds, in acc[s][i], the row channel of slice element
  // chan(s, i); the zero-point sums of that channel's group are added here
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
  float z[2] = {0.0f, 0.0f};   // zero-point sum of the channels' group
  if constexpr (VF == TTKV_I4_ASYM_G64)   // sum_t p_t * (zero + 8 * scale)
    z[0] = z[1] = (kg >> 1) ? fmaf(8.0f, accz[2], accz[3]) : fmaf(8.0f, accz[0], accz[1]);
  if constexpr (VT) {   // per channel group: the lanes' zero-point sums over their tokens, minus the splice offsets
#pragma unroll
    for (int g2 = 0; g2 < 2; ++g2) {
      zs[g2] += __shfl_xor(zs[g2], 16);
      zs[g2] += __shfl_xor(zs[g2], 32);
      z[g2] = zs[g2] - accoff[g2][0];   // every row of accoff holds the column's sum
    }
  }
  float (*w_acc)[128] = (float (*)[128])wbuf;   // [head][channel]; the wave's last batch has been consumed
  if (n < Gr) {
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (VT) w_acc[n][16 * s + 4 * kg + i] = acc[s][i] + z[s / 4];   // block s row 4 kg + i, as the product leaves it
        else w_acc[n][slice_channel<VF>(kg, chan<VF>(s, i))] = acc[s][i] + z[s / 4];
      }
    if (kg == 0) {
      s_m[wave][n] = m * cs;   // log2 domain
      s_l[wave][n] = l;
    }
  }
}

// GQ: query heads per KV head the quantized-key cases are compiled for (4, 8 or 16; fp16 / bf16 tiers take any
// count).  WIDE: the launch has a tier whose (group, head) columns need more than one pass of the score product
// (int8 keys with 8 or 16 heads, int4 keys with 16); those cases hold further q operands, so they get
// instantiations of their own and the one-pass cases keep their registers.
// T128: the launch has a tier whose keys are grouped over 128 tokens per channel (its own instantiations as well).
template <int GQ, bool WIDE, bool T128>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(GQ == 16 ? 2 : 3, GQ == 16 ? 2 : 3))) void attn_mfma_kernel(const FusedArgs a) {
  static_assert(kTileLds >= 16 * 128 * 4, "the wave's result fits its tile buffer");
  __shared__ __attribute__((aligned(256))) char s_buf[4 * kTileLds];   // per wave: batch in flight, then [head][channel] floats
  __shared__ float s_m[4][16], s_l[4][16];

  // Linear workgroup id -> (item, KV head, block of heads).  More heads per KV head than one tile takes are cut
  // into blocks of mfma_heads; the blocks of one (item, KV head) read the same bytes and get ids 8 apart, so that
  // they run on the same XCD at the same time and the later readers are served from its L2.
  const int Gtot = a.Hq / a.Hkv;
  const uint32_t n_hb = (Gtot + a.mfma_heads - 1) / a.mfma_heads;
  const uint32_t id = blockIdx.x;
  const uint32_t base = ((id >> 3) / n_hb) * 8 + (id & 7);
  if (base >= (uint32_t)a.n_items * a.Hkv) return;
  const int item = base / a.Hkv;
  const int hkv = base % a.Hkv;
  const int hb0 = ((id >> 3) % n_hb) * a.mfma_heads;          // first head of the block within the KV head's heads
  const int hq0 = hkv * Gtot + hb0;
  const int G = min(a.mfma_heads, Gtot - hb0);                // heads in this block

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
#define TTKV_MFMA_CASE(KF, VF, GT) process_mfma<KF, VF, GT>(a, tv, en, sel, chunk_tokens, chunk, seq, hq0, G, hkv, s_buf, s_m, s_l)
  switch (combo) {
    case TTKV_F16 * 8 + TTKV_F16: TTKV_MFMA_CASE(TTKV_F16, TTKV_F16, 0); break;
    case TTKV_BF16 * 8 + TTKV_BF16: TTKV_MFMA_CASE(TTKV_BF16, TTKV_BF16, 0); break;
    case TTKV_I8_SYM_G32 * 8 + TTKV_I8_SYM_G32:
      if constexpr (GQ == 4 || ((GQ == 8 || GQ == 16) && WIDE)) TTKV_MFMA_CASE(TTKV_I8_SYM_G32, TTKV_I8_SYM_G32, GQ);
      break;
    case TTKV_I8_SYM_G32 * 8 + TTKV_I4_ASYM_G64:
      if constexpr (GQ == 4 || ((GQ == 8 || GQ == 16) && WIDE)) TTKV_MFMA_CASE(TTKV_I8_SYM_G32, TTKV_I4_ASYM_G64, GQ);
      break;
    case TTKV_I4_ASYM_T128 * 8 + TTKV_I4_ASYM_G64:
      if constexpr (T128) TTKV_MFMA_CASE(TTKV_I4_ASYM_T128, TTKV_I4_ASYM_G64, 0);
      break;
    case TTKV_I8_SYM_G32 * 8 + TTKV_I4_ASYM_G64_T32:
      if constexpr (GQ == 4 || ((GQ == 8 || GQ == 16) && WIDE)) TTKV_MFMA_CASE(TTKV_I8_SYM_G32, TTKV_I4_ASYM_G64_T32, GQ);
      break;
    case TTKV_I4_ASYM_G64 * 8 + TTKV_I4_ASYM_G64_T32:
      if constexpr (GQ <= 8 || WIDE) TTKV_MFMA_CASE(TTKV_I4_ASYM_G64, TTKV_I4_ASYM_G64_T32, GQ);
      break;
    default:
      if constexpr (GQ <= 8 || WIDE) TTKV_MFMA_CASE(TTKV_I4_ASYM_G64, TTKV_I4_ASYM_G64, GQ);
      break;
  }
#undef TTKV_MFMA_CASE
  __syncthreads();

  // ---- merge the four waves (each with its own running max) and write the item's partials
  for (int idx = threadIdx.x; idx < G * 128; idx += 256) {
    const int g = idx >> 7, dch = idx & 127;
    const float M = fmaxf(fmaxf(s_m[0][g], s_m[1][g]), fmaxf(s_m[2][g], s_m[3][g]));
    float o = 0.0f, ll = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float wgt = s_m[w][g] == -INFINITY ? 0.0f : __builtin_amdgcn_exp2f(s_m[w][g] - M);
      o = fmaf(((const float *)(s_buf + w * kTileLds))[g * 128 + dch], wgt, o);
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

}  // namespace

// Can one 16-column tile hold every (group, head) column of these formats, and does the
// single pass pay off (from four query heads per KV head on, measured)?
// Heads one workgroup serves in a single pass over the bytes: the 16 columns of the second product, whatever the
// stored format.  More heads per KV head are cut into blocks of this many.
int mfma_block_heads(int k_fmt) { (void)k_fmt; return 16; }

// Do the kernel's cases take these formats?
bool attn_mfma_fits(int k_fmt, int v_fmt, int G) {
  if (G < 2) return false;
  if (v_fmt == TTKV_I4_ASYM_G64_T32) return k_fmt == TTKV_I8_SYM_G32 || k_fmt == TTKV_I4_ASYM_G64;
  if (k_fmt == TTKV_I4_ASYM_G64) return v_fmt == k_fmt;
  return true;
}

// Does the single pass over the bytes pay off?  From two query heads per KV head on (measured against the vector
// kernel's head pair at two heads: fp16 6.4 against 6.2 TB/s, int8 6.2 against 5.3, int4 5.2 against 4.5, K 8-bit /
// V 4-bit 6.0 against 4.3, keys grouped over tokens 4.4 against 3.5).
bool attn_mfma_pays(int G, bool has_mixed_or_t128) {
  (void)has_mixed_or_t128;
  return G >= 2;
}

namespace {
int padded_heads(int G) { return G <= 4 ? 4 : (G <= 8 ? 8 : 16); }
bool quantized_per_token(int k_fmt) { return k_fmt == TTKV_I8_SYM_G32 || k_fmt == TTKV_I4_ASYM_G64; }

// What one launch needs: heads per block (the smallest any of its tiers takes), the padded count the
// quantized-key cases are compiled for, two-pass cases, keys grouped over tokens.
struct MfmaShape {
  int heads, padded;
  bool wide, t128, mixed, ok;
};
MfmaShape mfma_shape(const FusedArgs &a) {
  const int G = a.Hq / a.Hkv;
  MfmaShape m{16, 4, false, false, false, true};
  bool quant = false;
  for (int j = 0; j < a.n_entries; ++j) {
    const TierView &tv = a.tv[(a.e[j].tier_seq >> 16) & 0xff];
    m.ok &= attn_mfma_fits(tv.k_fmt, tv.v_fmt, G);
    m.heads = std::min(m.heads, mfma_block_heads(tv.k_fmt));
    m.t128 |= tv.k_fmt == TTKV_I4_ASYM_T128;
    m.mixed |= tv.k_fmt == TTKV_I8_SYM_G32 && tv.v_fmt != tv.k_fmt;
    quant |= quantized_per_token(tv.k_fmt);
  }
  m.heads = std::min(m.heads, G);
  if (quant) m.padded = padded_heads(m.heads);
  for (int j = 0; j < a.n_entries; ++j) {
    const int kf = a.tv[(a.e[j].tier_seq >> 16) & 0xff].k_fmt;
    m.wide |= (kf == TTKV_I8_SYM_G32 && m.padded >= 8) || (kf == TTKV_I4_ASYM_G64 && m.padded == 16);
  }
  return m;
}
}  // namespace

bool attn_mfma_eligible(const FusedArgs &a) {
  const MfmaShape m = mfma_shape(a);
  // two-pass cases together with keys grouped over tokens have no instantiation: vector kernel
  return m.ok && attn_mfma_pays(a.Hq / a.Hkv, m.t128 || m.mixed) && !(m.wide && m.t128);
}

hipError_t launch_attn_mfma(const FusedArgs &a0, hipStream_t s) {
  const MfmaShape m = mfma_shape(a0);
  FusedArgs a = a0;
  a.mfma_heads = m.heads;
  const int G = a.Hq / a.Hkv;
  const uint32_t n_hb = (G + m.heads - 1) / m.heads;
  const dim3 grid(((uint32_t)a.n_items * a.Hkv + 7) / 8 * 8 * n_hb);
  if (m.t128 && m.padded == 8) hipLaunchKernelGGL((attn_mfma_kernel<8, false, true>), grid, dim3(256), 0, s, a);
  else if (m.t128) hipLaunchKernelGGL((attn_mfma_kernel<4, false, true>), grid, dim3(256), 0, s, a);
  else if (m.padded == 16) hipLaunchKernelGGL((attn_mfma_kernel<16, true, false>), grid, dim3(256), 0, s, a);
  else if (m.padded == 8 && m.wide) hipLaunchKernelGGL((attn_mfma_kernel<8, true, false>), grid, dim3(256), 0, s, a);
  else if (m.padded == 8) hipLaunchKernelGGL((attn_mfma_kernel<8, false, false>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((attn_mfma_kernel<4, false, false>), grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace ttkv
