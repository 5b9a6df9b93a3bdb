// Small device helpers: dtype-tagged loads/stores, bf16 conversion, activation
// functions, wave/block reductions for 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace gpp {

typedef __bf16 bf16_t;

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t u) {
  return __uint_as_float(((uint32_t)u) << 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  bf16_t b = (bf16_t)f;  // round to nearest even
  return __builtin_bit_cast(uint16_t, b);
}

__device__ __forceinline__ float load_as_f32(const void *p, int32_t dtype, int64_t i) {
  if (dtype == DT_BF16) return bf16_bits_to_f32(((const uint16_t *)p)[i]);
  return ((const float *)p)[i];
}
__device__ __forceinline__ void store_from_f32(void *p, int32_t dtype, int64_t i, float v) {
  if (dtype == DT_BF16)
    ((uint16_t *)p)[i] = f32_to_bf16_bits(v);
  else
    ((float *)p)[i] = v;
}

template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) {
  return v;
}
template <>
__device__ __forceinline__ float to_f32<uint16_t>(uint16_t v) {
  return bf16_bits_to_f32(v);
}

// GELU in its erf form, y = z * Phi(z), and its derivative Phi(z) + z * phi(z), from ONE exponential:
// erf(z / sqrt 2) = sign(z) * (1 - P(t) * exp(-z^2 / 2)), t = 1 / (1 + c |z| / sqrt 2), with the five-term
// polynomial P of Abramowitz & Stegun 7.1.26 (absolute error of erf below 1.5e-7), and phi(z) is that
// same exponential over sqrt(2 pi).
__device__ __forceinline__ void gelu_both(float z, float &y, float &dy) {
  const float az = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * az);     // v_rcp_f32 (1 ulp); the exact reciprocal is ten instructions
  const float e = __expf(-az * az);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float erf_abs = 1.0f - poly * e;
  const float cdf = 0.5f * (1.0f + copysignf(erf_abs, z));
  y = z * cdf;
  dy = cdf + z * (0.3989422804014327f * e);
}
__device__ __forceinline__ float gelu_f(float z) {
  float y, dy;
  gelu_both(z, y, dy);
  return y;
}
__device__ __forceinline__ float gelu_grad_f(float z) {
  float y, dy;
  gelu_both(z, y, dy);
  return dy;
}
__device__ __forceinline__ float act_apply(float z, int32_t act) {
  if (act == ACT_RELU) return z > 0.0f ? z : 0.0f;
  if (act == ACT_GELU) return gelu_f(z);
  return z;
}
// What a forward epilogue stashes for the backward pass of an activation that needs more than the
// sign of its output: for GELU the DERIVATIVE at the pre-activation (the forward pass has the
// exponential at hand), so that the backward epilogue is one multiplication.
__device__ __forceinline__ float act_stash(float z, int32_t act) { return act == ACT_GELU ? gelu_grad_f(z) : z; }
// derivative factor from the mask source: ReLU uses the stored output (y > 0 <=> z > 0), GELU the
// stashed derivative
__device__ __forceinline__ float act_grad(float src, int32_t act) {
  if (act == ACT_RELU) return src > 0.0f ? 1.0f : 0.0f;
  return src;
}

// Wave-wide sum / maximum, the same value in every lane, in a fixed order.  Inside a row of 16 lanes the partner
// values come through the DPP operand path (quad permutations, then the half-row and row mirrors: after each step
// the lanes of a growing group hold that group's total); the four row totals are read out as scalars and combined.
// Six cross-lane LDS permutations (ds_bpermute, ~100 cycles each, and on the LDS wait counter) were 0.5 us per
// reduction: most of a LayerNorm row's critical path.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_f32(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<0xB1>(v);      // quad_perm [1, 0, 3, 2]
  v += dpp_f32<0x4E>(v);      // quad_perm [2, 3, 0, 1]
  v += dpp_f32<0x141>(v);     // row_half_mirror
  v += dpp_f32<0x140>(v);     // row_mirror
  return (lane_f32(v, 0) + lane_f32(v, 16)) + (lane_f32(v, 32) + lane_f32(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<0xB1>(v));
  v = fmaxf(v, dpp_f32<0x4E>(v));
  v = fmaxf(v, dpp_f32<0x141>(v));
  v = fmaxf(v, dpp_f32<0x140>(v));
  return fmaxf(fmaxf(lane_f32(v, 0), lane_f32(v, 16)), fmaxf(lane_f32(v, 32), lane_f32(v, 48)));
}

// Finds the record whose [blk_begin, next blk_begin) range holds `blk`.
template <typename P>
__device__ __forceinline__ int find_prob(const P *probs, int n, int blk) {
  int lo = 0, hi = n - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (probs[mid].blk_begin <= blk)
      lo = mid;
    else
      hi = mid - 1;
  }
  return lo;
}

}  // namespace gpp
