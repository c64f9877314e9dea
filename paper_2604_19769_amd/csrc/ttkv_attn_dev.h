// Device helpers shared by the attention kernels: row geometry per format, the
// splice of int4 / int8 codes into fp16 mantissas, DPP lane exchanges.
#pragma once
#include "ttkv_internal.h"

#include <hip/hip_fp16.h>

namespace ttkv {
namespace dev {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef __bf16 b2 __attribute__((ext_vector_type(2)));

template <int F> struct Fmt;
template <> struct Fmt<TTKV_F16> { static constexpr int ROWB = 256, LPT = 16, TPL = 4, EPL = 8; };
template <> struct Fmt<TTKV_BF16> { static constexpr int ROWB = 256, LPT = 16, TPL = 4, EPL = 8; };
template <> struct Fmt<TTKV_I8_SYM_G32> { static constexpr int ROWB = 128, LPT = 8, TPL = 8, EPL = 16; };
template <> struct Fmt<TTKV_I4_ASYM_G64> { static constexpr int ROWB = 64, LPT = 4, TPL = 16, EPL = 32; };
template <> struct Fmt<TTKV_I4_ASYM_T128> { static constexpr int ROWB = 64, LPT = 4, TPL = 16, EPL = 32; };   // rows as int4
template <> struct Fmt<TTKV_I4_ASYM_G64_T32> { static constexpr int ROWB = 64, LPT = 4, TPL = 16, EPL = 32; };   // bytes per token as int4
template <int F> constexpr bool is_i4() { return F == TTKV_I4_ASYM_G64 || F == TTKV_I4_ASYM_T128 || F == TTKV_I4_ASYM_G64_T32; }

// Streaming loads: K/V bytes are read exactly once per launch, so they are fetched with the
// non-temporal hint (no reuse expected).  On MI355X a load-only kernel moves 6.5-7.0 TB/s this way
// against 5.7-6.1 TB/s with plain loads (measured, 2 GiB, same access pattern).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ld_stream(const uint4 *p) {
  const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
  return uint4{v.x, v.y, v.z, v.w};
}
__device__ __forceinline__ uint2 ld_stream(const uint2 *p) {
  const u32x2 v = __builtin_nontemporal_load((const u32x2 *)p);
  return uint2{v.x, v.y};
}
__device__ __forceinline__ uint32_t ld_stream(const uint32_t *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ uint16_t ld_stream(const uint16_t *p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ float h2f(uint16_t h) { return __half2float(__ushort_as_half(h)); }
__device__ __forceinline__ h2 as_h2(uint32_t u) { return __builtin_bit_cast(h2, u); }
__device__ __forceinline__ b2 as_b2(uint32_t u) { return __builtin_bit_cast(b2, u); }

// Position of element e of a lane's 16-byte slice inside the packed pair registers:
// register e/2-ish and half, per format (see unpack16).
//   F16 / BF16 / I8 : pair r = e/2 holds (e, e+1)                      -> natural
//   I4              : dword d = e/8, pairs (0,4) (1,5) (2,6) (3,7)     -> r = 4d + e%4, half = (e%8)/4
template <int F>
__device__ __forceinline__ constexpr int pair_reg(int e) {
  return is_i4<F>() ? 4 * (e / 8) + (e % 4) : e / 2;
}
template <int F>
__device__ __forceinline__ constexpr int pair_half(int e) {
  return is_i4<F>() ? (e % 8) / 4 : e % 2;
}
// Offset o_e that unpack16 leaves on element e.
template <int F>
__device__ __forceinline__ constexpr float elem_offset(int e) {
  return is_i4<F>() ? ((e % 2) ? 64.0f : 1024.0f) : (F == TTKV_I8_SYM_G32 ? 1152.0f : 0.0f);
}

// Bit patterns used to splice int4 codes into fp16 mantissas.  They are kept in
// registers the compiler cannot see through (two SGPR masks, two VGPR constants):
// gfx9 VOP3 encodings take no literals, and with literals the compiler falls back
// to v_and + v_or instead of one v_and_or_b32 per pair.
struct Splice {
  uint32_t m0, m1, c0, c1;
  __device__ __forceinline__ void init() {
    m0 = 0x000F000Fu; m1 = 0x00F000F0u; c0 = 0x64006400u; c1 = 0x54005400u;
    asm volatile("" : "+s"(m0), "+s"(m1), "+v"(c0), "+v"(c1));
  }
};

// 16 bytes of a row -> EPL/2 registers of packed 16-bit pairs (fp16, or bf16 for the bf16 tier).
template <int F>
__device__ __forceinline__ void unpack16(const uint4 &w, uint32_t *r, const Splice &k) {
  const uint32_t u[4] = {w.x, w.y, w.z, w.w};
  if constexpr (F == TTKV_F16 || F == TTKV_BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = u[i];
  } else if constexpr (F == TTKV_I8_SYM_G32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t x = u[i] ^ 0x80808080u;                       // byte -> code + 128 in [1, 255]
      r[2 * i] = __builtin_amdgcn_perm(0x64646464u, x, 0x04010400u);      // (1024 + b0, 1024 + b1)
      r[2 * i + 1] = __builtin_amdgcn_perm(0x64646464u, x, 0x04030402u);  // (1024 + b2, 1024 + b3)
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t x = u[i], y = u[i] >> 8;
      r[4 * i + 0] = (x & k.m0) | k.c0;   // (1024 + n0, 1024 + n4)
      r[4 * i + 1] = (x & k.m1) | k.c1;   // (  64 + n1,   64 + n5)
      r[4 * i + 2] = (y & k.m0) | k.c0;   // (1024 + n2, 1024 + n6)
      r[4 * i + 3] = (y & k.m1) | k.c1;   // (  64 + n3,   64 + n7)
    }
  }
}

template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// sum / max over groups of LPT consecutive lanes (LPT = 4, 8, 16) -- every lane gets the result
template <int LPT>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp<0xB1>(v);                       // quad_perm [1,0,3,2]
  v += dpp<0x4E>(v);                       // quad_perm [2,3,0,1]: every lane holds its quad's sum
  if constexpr (LPT >= 8) v += dpp<0x141>(v);   // row_half_mirror: lane i <- lane 7-i = the other quad's sum
  if constexpr (LPT >= 16) v += dpp<0x140>(v);  // row_mirror: lane i <- lane 15-i = the other half's sum
  return v;
}
// A run whose blocks are named by the device-side selection (ids ascending, so only the last can be the tier's
// partly filled newest block).  Two forms, told apart by the tier's item size in the launch arguments:
//   fixed items (host tiers): item `chunk` of the run is sub-chunk chunk % ipb of the run's (chunk / ipb)-th
//     selected block; the entry is rewritten into a run over that one block;
//   equal items (tiers in HBM): the tokens of all selected blocks form ONE run of len tokens, cut like any other
//     run; token i of it lies in block ids[i / bt], which the tile address look-up follows (`sel`), so an item may
//     span several blocks and small blocks cost no more than large ones.
// Either way everything after this sees an ordinary run.  Returns the run's id list for the second form.
__device__ __forceinline__ const int32_t *resolve_selected(const FusedArgs &a, const TierView &tv, Entry &en, int seq,
                                                           bool equal_items, int chunk_tokens, int &chunk) {
  if (!(en.tier_seq & (1 << 25))) return nullptr;
  if (equal_items) {
    const int32_t *ids = a.sel_ids + en.rec_base;
    if (ids[en.len / tv.bt - 1] == en.first_tok) en.len -= tv.bt - a.sel_last_ntok[seq];
    en.first_tok = 0;
    en.rec_base = seq * tv.ring_blocks;
    return ids;
  }
  const int ipb = (tv.bt + chunk_tokens - 1) / chunk_tokens;
  const int blk = chunk / ipb;
  chunk -= blk * ipb;
  const int32_t id = a.sel_ids[en.rec_base + blk];
  en.len = id == en.first_tok ? a.sel_last_ntok[seq] : tv.bt;
  en.first_tok = (id % tv.ring_blocks) * tv.bt;
  en.rec_base = seq * tv.ring_blocks;
  return nullptr;
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp<0xB1>(v));
  v = fmaxf(v, dpp<0x4E>(v));
  v = fmaxf(v, dpp<0x124>(v));             // row_ror:4
  v = fmaxf(v, dpp<0x128>(v));             // row_ror:8
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m);
  return v;
}

}  // namespace dev
}  // namespace ttkv
