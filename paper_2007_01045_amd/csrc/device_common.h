// Device-side helpers shared by the gfx950 kernels.
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dapple {

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short short4v;

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // round to nearest even

// GELU u*Phi(u) and its derivative Phi(u) + u*phi(u), Phi the normal CDF.
// erfc(x) for x >= 0 is evaluated with the rational approximation 7.1.26 of Abramowitz
// and Stegun, erfc(x) = (a1 t + ... + a5 t^5) exp(-x^2), t = 1/(1 + p x), absolute
// error below 1.5e-7 -- far inside the fp32 and bf16 parity tolerances, and a fifth of
// the instructions of the library erff.  The same exponential gives phi(u).
__device__ __forceinline__ void gelu_both(float u, float& g, float& gp) {
  float x = fabsf(u) * 0.70710678118654752f;
  float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
  // = exp(-u^2 / 2), as the bare v_exp_f32 (the argument is never positive; a result below 2^-126 may be zero)
  float e = __builtin_amdgcn_exp2f(-x * x * 1.4426950408889634f);
  float poly = t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f),
                        0.254829592f);
  float half_erfc = 0.5f * poly * e;                 // Phi(-|u|)
  float Phi = u >= 0.f ? 1.0f - half_erfc : half_erfc;
  g = u * Phi;
  gp = fmaf(u * 0.39894228040143268f, e, Phi);
}
__device__ __forceinline__ float gelu_f(float u) {
  float g, gp;
  gelu_both(u, g, gp);
  return g;
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  float g, gp;
  gelu_both(u, g, gp);
  return gp;
}

// LDS transpose read (gfx950): the 16 lanes of a group each point at 4
// consecutive 16-bit elements; lanes 4e..4e+3 together supply "row e" (16
// elements), and lane i of the group receives element i of rows 0..3.
__device__ __forceinline__ bf16x4 lds_read_tr16(const bf16* p) {
  short4v r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((short4v __attribute__((address_space(3)))*)(p));
  return __builtin_bit_cast(bf16x4, r);
}

__device__ __forceinline__ bf16x8 join8(bf16x4 lo, bf16x4 hi) {
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// wave-wide sum (64 lanes), result in every lane, in a fixed order: inside each row of 16 lanes a tree of four
// steps whose cross-lane operand is part of the add itself (lane pairs, pairs of pairs, the two quads of a half
// row by its mirror image, the two half rows by the row's mirror image), then the four row totals in ascending
// order through scalar registers.  No trip through the LDS crossbar: six dependent ds_bpermute round trips took
// longer than the rest of a LayerNorm row's arithmetic.
__device__ __forceinline__ float wave_sum(float v) {
  auto step = [](float x, auto CTRL) {
    return x + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(CTRL)::value,
                                                                     0xF, 0xF, true));
  };
  v = step(v, std::integral_constant<int, 0xB1>{});   // quad_perm [1,0,3,2]
  v = step(v, std::integral_constant<int, 0x4E>{});   // quad_perm [2,3,0,1]
  v = step(v, std::integral_constant<int, 0x141>{});  // row_half_mirror
  v = step(v, std::integral_constant<int, 0x140>{});  // row_mirror
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return ((r0 + r1) + r2) + r3;
}

}  // namespace dapple
