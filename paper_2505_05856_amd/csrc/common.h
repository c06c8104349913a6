// Shared device/host helpers for the dpstage kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace dp {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int kDtype = 0; };
template <> struct Elem<bf16> { static constexpr int kDtype = 1; };

// ---- 8-element vector load/store (16 B for bf16, 32 B for fp32) -------------
__device__ __forceinline__ void load8(const float *p, float (&v)[8]) {
  const float4 a = reinterpret_cast<const float4 *>(p)[0];
  const float4 b = reinterpret_cast<const float4 *>(p)[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16 *p, float (&v)[8]) {
  const bf16x8 a = *reinterpret_cast<const bf16x8 *>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = (float)a[i];
}
__device__ __forceinline__ void store8(float *p, const float (&v)[8]) {
  reinterpret_cast<float4 *>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
  reinterpret_cast<float4 *>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16 *p, const float (&v)[8]) {
  bf16x8 a;
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = (bf16)v[i];
  *reinterpret_cast<bf16x8 *>(p) = a;
}
// Eight elements as they lie in memory, for loads that wait in registers before they are used.
template <typename T> struct Raw8;
template <> struct Raw8<float> {
  float v[8];
  __device__ __forceinline__ void load(const float *p) { load8(p, v); }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = v[i];
  }
};
template <> struct Raw8<bf16> {
  bf16x8 v;
  __device__ __forceinline__ void load(const bf16 *p) { v = *reinterpret_cast<const bf16x8 *>(p); }
  __device__ __forceinline__ void unpack(float (&o)[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (float)v[i];
  }
};
__device__ __forceinline__ float ldf(const float *p) { return *p; }
__device__ __forceinline__ float ldf(const bf16 *p) { return (float)*p; }
__device__ __forceinline__ void stf(float *p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16 *p, float v) { *p = (bf16)v; }

// ---- wavefront reductions (all 64 lanes take part, result in every lane) ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

// ---- GELU ----------------------------------------------------------------------------
// One definition for every kernel that applies it (the standalone kernels and the GEMM
// epilogue must agree to the bit, so that a recomputed GELU_OUT equals the fused one);
// contraction is off and every fused multiply-add is written out, so that no
// context-dependent fma formation can change a result.
//
// The normal distribution function comes from the rational approximation of erf by
// Abramowitz & Stegun (formula 7.1.26, |error| <= 1.5e-7): with z = |x|/sqrt(2),
// t = 1/(1 + p z), 1 - erf(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2).
// The lower tail q = Phi(-|x|) is formed directly (no cancellation) and Phi(x) is q or
// 1 - q; exp(-x^2/2) is shared with the density in the derivative.  About a third of the
// instructions of erff, which matters where the activation rides a GEMM epilogue.
__device__ __forceinline__ float normal_cdf_parts(float x, float *density_exp) {
#pragma clang fp contract(off)
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, z, 1.0f));
  float p = __builtin_fmaf(t, 1.061405429f, -1.453152027f);
  p = __builtin_fmaf(t, p, 1.421413741f);
  p = __builtin_fmaf(t, p, -0.284496736f);
  p = __builtin_fmaf(t, p, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(x * x * -0.72134752044448170f);   // exp(-x^2/2)
  *density_exp = e;
  const float q = 0.5f * (p * t) * e;
  return x < 0.f ? q : 1.0f - q;
}
__device__ __forceinline__ float gelu_f(float x, int kind) {
#pragma clang fp contract(off)
  if (kind == 0) { float e; return x * normal_cdf_parts(x, &e); }
  if (kind == 2) return fmaxf(x, 0.f);   // ReLU
  const float u = 0.79788456080286536f * (x + 0.044715f * x * x * x);
  return 0.5f * x * (1.0f + tanhf(u));
}
__device__ __forceinline__ float gelu_df(float x, int kind) {
#pragma clang fp contract(off)
  if (kind == 0) {
    float e;
    const float cdf = normal_cdf_parts(x, &e);
    return cdf + x * (0.39894228040143268f * e);
  }
  if (kind == 2) return x > 0.f ? 1.0f : 0.f;   // ReLU: the derivative at 0 is taken as 0
  const float u = 0.79788456080286536f * (x + 0.044715f * x * x * x);
  const float t = tanhf(u);
  const float du = 0.79788456080286536f * (1.0f + 0.134145f * x * x);
  return 0.5f * (1.0f + t) + 0.5f * x * (1.0f - t * t) * du;
}

// ---- dropout masks ----------------------------------------------------------------------
// Whether an element is kept is a pure function of where it sits (counter-based), so that a
// recomputed tensor and the backward pass get the mask of the forward pass without any state:
//   mix(x): the 32-bit integer mixer x^=x>>16, x*=0x7feb352d, x^=x>>15, x*=0x846ca68b, x^=x>>16
//   base  = mix chain over (seed, micro-batch counter, 8*layer + site)   [host, per launch]
//   k0    = mix(base ^ unit*0x9e3779b1), k1 = mix(k0 ^ 0x85ebca6b)       [per batch*head / tensor]
//   bits(i) = the mixer on i ^ k0 with k1 xored in between its two multiplications
//   keep(i) = bits(i) >= floor(p * 2^32); kept values are scaled by 1/(1-p).
__host__ __device__ __forceinline__ uint32_t drop_mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
__host__ __device__ __forceinline__ uint32_t drop_bits(uint32_t idx, uint32_t k0, uint32_t k1) {
  uint32_t x = idx ^ k0;
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x ^= k1; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
struct DropKeys { uint32_t k0, k1; };
__host__ __device__ __forceinline__ DropKeys drop_keys(uint32_t base, uint32_t unit) {
  DropKeys k;
  k.k0 = drop_mix(base ^ (unit * 0x9e3779b1u));
  k.k1 = drop_mix(k.k0 ^ 0x85ebca6bu);
  return k;
}

}  // namespace dp
