// 8-bit weight codes (FP8 E4M3, INT8) -> bf16 MFMA fragments in registers (device code shared by the LM-head kernels).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "jd_kernels.hpp"

namespace jd {

// Two FP8 E4M3 codes (the low or the high 16 bits of `src`) to two packed bf16 values: gfx950 does it in
// one instruction (the scale operand is 1; every E4M3 value is a bf16 value, so the result is exact -
// checked on the device for all code pairs against the float conversion).  Inline assembly because the
// instruction has to stay behind the MFMA it is written behind: between two MFMAs of a lone wavefront
// exactly one vector, LDS or memory instruction issues for free, every further one delays the next MFMA by
// about 7 cycles (measured); scalar instructions ride along.  Left to the compiler, all conversions of a
// K step end up in one block.
__device__ __forceinline__ uint32_t fp8x2_to_bf16x2(uint32_t src, bool high_half) {
  uint32_t o;
  if (high_half)
    asm volatile("v_cvt_scalef32_pk_bf16_fp8 %0, %1, 1.0 op_sel:[1,0,0]" : "=v"(o) : "v"(src));
  else
    asm volatile("v_cvt_scalef32_pk_bf16_fp8 %0, %1, 1.0" : "=v"(o) : "v"(src));
  return o;
}

// Dword j (0..3) of the bf16 fragment of the eight codes (lo, hi), ascending hidden index.
__device__ __forceinline__ uint32_t fp8_frag_dword(uint32_t lo, uint32_t hi, int j) {
  return fp8x2_to_bf16x2(j < 2 ? lo : hi, (j & 1) != 0);
}

// The same for either one-byte code type.  INT8 (two's complement): two sign-extending byte -> float conversions;
// an integer of magnitude <= 128 has at most 8 significant bits, so the upper half of its float is exactly its bf16,
// and a byte permute packs the two halves - three instructions where FP8 needs one.
template <int WK>
__device__ __forceinline__ uint32_t w8_frag_dword(uint32_t lo, uint32_t hi, int j) {
  if constexpr (WK == kWFp8) {
    return fp8_frag_dword(lo, hi, j);
  } else {
    static_assert(WK == kWInt8, "8-bit code");
    const uint32_t w = j < 2 ? lo : hi;
    const int sh = (j & 1) * 16;
    const float a = (float)(int)(int8_t)(w >> sh), b = (float)(int)(int8_t)(w >> (sh + 8));
    return __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);  // b.hi16 : a.hi16
  }
}

__device__ __forceinline__ void set_dword(uint4& v, int j, uint32_t x) {
  if (j == 0) v.x = x; else if (j == 1) v.y = x; else if (j == 2) v.z = x; else v.w = x;
}

// Eight codes (two dwords, ascending hidden index) to eight bf16 values, left to the compiler's scheduler
// (the small-row kernel is bound by HBM, not by issue slots).  FP8: one instruction per two codes.
// INT8 (two's complement): sign-extending byte -> float conversions; an integer of magnitude <= 128 has at
// most 8 significant bits, so the upper half of its float is exactly its bf16 and a byte permute packs two.
template <int WK>
__device__ __forceinline__ uint4 w8x8_to_bf16x8(uint32_t lo, uint32_t hi) {
  if constexpr (WK == kWFp8) {
    auto cv = [](uint32_t w, bool high) {
      return __builtin_bit_cast(uint32_t, high ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true)
                                               : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false));
    };
    return make_uint4(cv(lo, false), cv(lo, true), cv(hi, false), cv(hi, true));
  } else {
    static_assert(WK == kWInt8, "8-bit code");
    auto pair = [](uint32_t w, int i) {
      const float a = (float)(int)(int8_t)(w >> (8 * i)), b = (float)(int)(int8_t)(w >> (8 * i + 8));
      return __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);  // b.hi16 : a.hi16
    };
    return make_uint4(pair(lo, 0), pair(lo, 2), pair(hi, 0), pair(hi, 2));
  }
}

}  // namespace jd
