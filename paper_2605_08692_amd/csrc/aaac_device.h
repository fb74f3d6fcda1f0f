// Device-side helpers shared by the gfx950 kernels: bf16 / FP8-E4M3 bit
// conversions and DPP cross-lane moves for 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aaac {

constexpr int kWave = 64;

// ---- bf16 <-> fp32 ----------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// ---- OCP FP8 E4M3 (bias 7, subnormal step 2^-9, max 448, no inf) -------
// q >= 0 -> 7-bit code, round to nearest even, saturating at 448.
__device__ __forceinline__ uint32_t e4m3_rne_sat(float q) {
  if (!(q < 448.0f)) return 0x7Eu;
  if (q < 0.015625f) return (uint32_t)__float2int_rn(q * 512.0f);  // multiples of 2^-9, 8 = first normal
  uint32_t u = __float_as_uint(q);
  u += 0x7FFFFu + ((u >> 20) & 1u);
  return (u >> 20) - (120u << 3);
}

__device__ __forceinline__ float e4m3_value(uint32_t c) {  // c in 0..0x7E
  float sub = (float)c * 0.001953125f;
  float nrm = __uint_as_float((((c >> 3) + 120u) << 23) | ((c & 7u) << 20));
  return c < 8u ? sub : nrm;
}

// Correctly rounded fp32 quotient via fp64 (the fp64 quotient of two fp32
// values rounds to fp32 the same way the exact quotient does).
__device__ __forceinline__ float div_rn(float a, float b) { return (float)((double)a / (double)b); }

// Scale of a group from its absmax (FMT 0: FP8 E4M3 of absmax / 6; FMT 1: bf16 of absmax / 7; a
// scale that would be zero, or a subnormal bf16, becomes the smallest positive value); returns the
// unsigned stored code and the scale's value in *s.
template <int FMT>
__device__ __forceinline__ uint32_t scale_code(float absmax, float* s) {
  if (FMT == 0) {
    uint32_t c = e4m3_rne_sat(div_rn(absmax, 6.0f));
    c = c == 0u ? 1u : c;
    *s = e4m3_value(c);
    return c;
  }
  uint32_t c = bf16_rne(div_rn(absmax, 7.0f));
  c = c < 0x80u ? 0x80u : c;
  *s = __uint_as_float(c << 16);
  return c;
}

// ---- DPP lane exchanges -------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside each 16 lanes

// Sum (or max) of `v` over aligned blocks of LANES lanes, result in every lane
// of the block.  Level by level each lane combines its value with the one held
// by the neighbouring sub-block, so the association is that of a balanced tree
// of adjacent pairs; after the quad levels all lanes of a quad are equal, which
// is what makes the mirror moves act as xor-4 and xor-8.
template <int LANES>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(LANES == 1 || LANES == 2 || LANES == 4 || LANES == 8 || LANES == 16, "lanes per group");
  if (LANES >= 2) v = v + dpp<kDppXor1>(v);
  if (LANES >= 4) v = v + dpp<kDppXor2>(v);
  if (LANES >= 8) v = v + dpp<kDppHalfMirror>(v);
  if (LANES >= 16) v = v + dpp<kDppMirror>(v);
  return v;
}
template <int LANES>
__device__ __forceinline__ float group_max(float v) {
  if (LANES >= 2) v = fmaxf(v, dpp<kDppXor1>(v));
  if (LANES >= 4) v = fmaxf(v, dpp<kDppXor2>(v));
  if (LANES >= 8) v = fmaxf(v, dpp<kDppHalfMirror>(v));
  if (LANES >= 16) v = fmaxf(v, dpp<kDppMirror>(v));
  return v;
}
// The same with the group width known only at run time (2, 4, 8 or 16 lanes, wavefront-uniform).
__device__ __forceinline__ float group_max_lanes(float v, int lanes) {
  v = fmaxf(v, dpp<kDppXor1>(v));
  if (lanes >= 4) v = fmaxf(v, dpp<kDppXor2>(v));
  if (lanes >= 8) v = fmaxf(v, dpp<kDppHalfMirror>(v));
  if (lanes >= 16) v = fmaxf(v, dpp<kDppMirror>(v));
  return v;
}


// Eight bf16 weights held by one lane.
struct W8 {
  float w[8];
};
__device__ __forceinline__ W8 unpack8(uint4 v) {
  W8 r;
  r.w[0] = bf16_lo(v.x); r.w[1] = bf16_hi(v.x);
  r.w[2] = bf16_lo(v.y); r.w[3] = bf16_hi(v.y);
  r.w[4] = bf16_lo(v.z); r.w[5] = bf16_hi(v.z);
  r.w[6] = bf16_lo(v.w); r.w[7] = bf16_hi(v.w);
  return r;
}
__device__ __forceinline__ float absmax8(const W8& x) {
  float a = fmaxf(fmaxf(fabsf(x.w[0]), fabsf(x.w[1])), fmaxf(fabsf(x.w[2]), fabsf(x.w[3])));
  float b = fmaxf(fmaxf(fabsf(x.w[4]), fabsf(x.w[5])), fmaxf(fabsf(x.w[6]), fabsf(x.w[7])));
  return fmaxf(a, b);
}

}  // namespace aaac
