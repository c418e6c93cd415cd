// Shared device-side types and small helpers for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define DEV __device__ __forceinline__

// two floats -> packed bf16 pair, round-to-nearest-even (lo in bits 0..15)
DEV uint32_t pack_bf16(float lo, float hi) {
  bf16x2 p;
  p[0] = (__bf16)lo;
  p[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, p);
}
DEV float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
DEV float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }
DEV float bf16_to_f32(bf16_t v) { return (float)v; }

// Logistic function on the hardware's 2^x and reciprocal units (1 ulp each; the results are rounded to bf16).
// 2^x overflowing to +inf gives 1/inf = 0 and underflowing to 0 gives 1: the correct limits.
DEV float sigmoid_f(float x) { return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x)); }

// GeLU and its derivative (fp32); tanh form by default, erf form selectable.  With u = sqrt(2/pi) (x + 0.044715 x^3)
// the tanh form 0.5 x (1 + tanh u) equals x * sigmoid(2 u), which costs one 2^x and one reciprocal; its derivative is
// s + x s (1 - s) 2 u' with s = sigmoid(2 u).
DEV float gelu_f(float x, bool tanh_form) {
  if (tanh_form) {
    const float x2 = x * x;
    const float two_u = x * (1.5957691216057308f + 0.07135481627267621f * x2);     // 2 sqrt(2/pi) (1, 0.044715)
    return x * sigmoid_f(two_u);
  }
  return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f));
}
DEV float gelu_grad_f(float x, bool tanh_form) {
  if (tanh_form) {
    const float x2 = x * x;
    const float two_u = x * (1.5957691216057308f + 0.07135481627267621f * x2);
    const float s = sigmoid_f(two_u);
    const float two_du = 1.5957691216057308f + 0.21406444881802863f * x2;          // d(2u)/dx
    return s + x * s * (1.0f - s) * two_du;
  }
  float cdf = 0.5f * (1.0f + erff(x * 0.7071067811865476f));
  float pdf = __expf(-0.5f * x * x) * 0.3989422804014327f;
  return cdf + x * pdf;
}

// Rotary embedding (Sec. 5.4 names it for Llama-2): the pair (i, i + d/2) of a head at sequence position pos turns by
// the angle pos * base^(-2 i / d).
DEV float rope_freq(int i, int d, float log2_base) { return exp2f(-2.0f * (float)i / (float)d * log2_base); }
// sin and cos of pos * freq on the hardware's sine / cosine units, which take their argument in revolutions: the angle
// is reduced to its fractional number of turns first (at 4096 positions fp32 leaves about 5e-4 rad of it, a sixteenth
// of what rounding the rotated value to bf16 costs).
DEV void rope_sincos(float pos, float freq, float* sn, float* cs) {
  const float turns = __builtin_amdgcn_fractf(pos * freq * 0.15915494309189535f);
  *sn = __builtin_amdgcn_sinf(turns);
  *cs = __builtin_amdgcn_cosf(turns);
}

// wave64 reductions over all lanes, on the VALU's data-parallel primitives (no LDS traffic): swaps inside quads,
// rotations inside the rows of 16 lanes, then the two row broadcasts leave the total in lane 63, which is read
// back as a wave-uniform value.  The order of the additions is fixed.
template <int CTRL, int ROW_MASK>
DEV float dpp_take(float v) {    // lanes of the rows in ROW_MASK get the CTRL-selected lane's v, all others 0
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
DEV float wave_sum(float v) {
  v += dpp_take<0xB1, 0xF>(v);     // quad_perm [1,0,3,2]
  v += dpp_take<0x4E, 0xF>(v);     // quad_perm [2,3,0,1]
  v += dpp_take<0x124, 0xF>(v);    // row_ror:4
  v += dpp_take<0x128, 0xF>(v);    // row_ror:8: every lane holds its row's sum
  v += dpp_take<0x142, 0xA>(v);    // row_bcast:15 into rows 1 and 3
  v += dpp_take<0x143, 0xC>(v);    // row_bcast:31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// value of the lane 32 away (the other half of the wave) through the gfx950 half-swap instruction: no LDS
// permute and no wait on the LDS counter
DEV float other_half(float v) {
  const unsigned u = __builtin_bit_cast(unsigned, v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // r[0] = [lo, lo], r[1] = [hi, hi]
  return __builtin_bit_cast(float, (threadIdx.x & 32) ? r[0] : r[1]);
}
DEV float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
