// Arithmetic of the rotary embedding shared by the stand-alone kernel (rope.hip) and the chunk-attention
// kernel, which rotates its query rows while they are staged in LDS: both produce the same bits.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace citrus {

typedef __attribute__((ext_vector_type(2))) __bf16 rope_bf16x2;
typedef __attribute__((ext_vector_type(2))) float rope_f32x2;

// Sine and cosine of rotary pair i (frequency base^(-2 i / d)) at an integer position, for the bf16
// paths: the hardware sine / cosine take their argument in revolutions; it is reduced to [0, 1) first.
// At positions in the thousands the reduction leaves an absolute error of a few 1e-4 rad, well below
// bf16's resolution of the rotated values.
__device__ inline void rope_sincos_bf16(int pos, int i, int d, float log2_base, float& sn, float& cs) {
  const float inv_freq = __builtin_amdgcn_exp2f(-static_cast<float>(2 * i) / static_cast<float>(d) * log2_base);
  const float rev = __builtin_amdgcn_fractf(static_cast<float>(pos) * inv_freq * 0.15915494309189535f);
  sn = __builtin_amdgcn_sinf(rev);
  cs = __builtin_amdgcn_cosf(rev);
}

// One 32-bit word of the low half (elements i, i + 1) and the word of their partners (i + d/2, ...).
__device__ inline void rope_rotate_words(uint32_t lo_w, uint32_t hi_w, float cs0, float sn0, float cs1, float sn1,
                                         uint32_t& lo_out, uint32_t& hi_out) {
  const float a0 = __uint_as_float(lo_w << 16), a1 = __uint_as_float(lo_w & 0xffff0000u);
  const float b0 = __uint_as_float(hi_w << 16), b1 = __uint_as_float(hi_w & 0xffff0000u);
  // one rounded product, then one fused multiply-add: the same two operations wherever this is inlined
  const rope_f32x2 lo = {fmaf(a0, cs0, -(b0 * sn0)), fmaf(a1, cs1, -(b1 * sn1))};
  const rope_f32x2 hi = {fmaf(b0, cs0, a0 * sn0), fmaf(b1, cs1, a1 * sn1)};
  lo_out = __builtin_bit_cast(uint32_t, __builtin_convertvector(lo, rope_bf16x2));  // round to nearest even
  hi_out = __builtin_bit_cast(uint32_t, __builtin_convertvector(hi, rope_bf16x2));
}

}  // namespace citrus
