// Shared device-side helpers for the gfx950 kernels: bf16 conversion, MFMA fragment types,
// LDS transposing reads, wavefront reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mllm {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef uint16_t bf16_t;  // raw storage type in global memory

#define MLLM_LDS __attribute__((address_space(3)))

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// fp32 -> bf16, round to nearest even, through the hardware conversion (v_cvt_pk_bf16_f32).
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2_t;
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2_t v = {lo, hi};
  const bf16x2_t b = __builtin_convertvector(v, bf16x2_t);
  return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

union Frag8 {  // eight bf16 = one MFMA A/B operand of the k=16 (32x32) or k=32 (16x16) shapes
  bf16x8 v;
  uint4 u;
  uint32_t w[4];
  s16x4 h[2];
};

// LDS transposing read.  Within each group of 16 lanes, lane i returns
// tile[k0 + e][n0 + i] for e = 0..3 when the lane passes the address of
// tile[k0 + i/4][n0 + 4*(i%4)] (tile rows are `stride` elements apart).
__device__ __forceinline__ s16x4 lds_read_tr4(const bf16_t* tile, int stride, int k0, int n0,
                                              int lane16) {
  const bf16_t* p = tile + (k0 + (lane16 >> 2)) * stride + n0 + 4 * (lane16 & 3);
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((MLLM_LDS s16x4*)p);
}

// erf to 1.5e-7 absolute (Abramowitz and Stegun 7.1.26: 1 - (a1 t + ... + a5 t^5) exp(-x^2) with
// t = 1 / (1 + p |x|), odd in x), with the hardware reciprocal and exp2: a dozen instructions where
// the library routine takes several times as many, which made the GELU kernels ALU-bound.  The
// results are rounded to bf16 (2^-9 relative), far above this error.
__device__ __forceinline__ float fast_erf(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * ax * ax);
  return copysignf(fmaf(-p * t, e, 1.f), x);
}
// GELU (act 0: exact erf form, 1: tanh form) and its derivative.
// tanh through the hardware exp2 and reciprocal: 1 - 2 / (1 + e^(2u)); exact at both ends (e = inf or 0).
__device__ __forceinline__ float fast_tanh(float u) {
  return fmaf(-2.f, __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(2.8853900817779268f * u)), 1.f);
}
__device__ __forceinline__ float gelu_f(int act, float z) {
  if (act == 1) {
    float u = 0.7978845608028654f * (z + 0.044715f * z * z * z);
    return 0.5f * z * (1.f + fast_tanh(u));
  }
  return 0.5f * z * (1.f + fast_erf(z * 0.7071067811865476f));
}
__device__ __forceinline__ float gelu_grad_f(int act, float z) {
  if (act == 1) {
    float u = 0.7978845608028654f * (z + 0.044715f * z * z * z);
    float t = fast_tanh(u);
    return 0.5f * (1.f + t) +
           0.5f * z * (1.f - t * t) * 0.7978845608028654f * (1.f + 3.f * 0.044715f * z * z);
  }
  return 0.5f * (1.f + fast_erf(z * 0.7071067811865476f)) +
         z * __builtin_amdgcn_exp2f(-0.7213475204444817f * z * z) * 0.3989422804014327f;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace mllm
