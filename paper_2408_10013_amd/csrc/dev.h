// Internal device-side helpers: bf16 storage type, element load/store in fp32, the
// activation functions and wavefront (64-lane) reductions.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

namespace ssdt {

struct bf16 {
  uint16_t v;
};

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
// fp32 -> bf16, round to nearest, ties to even: the hardware conversion (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2_hw_t __attribute__((ext_vector_type(2)));
typedef float f32x2_hw_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf2(float lo, float hi) {
  f32x2_hw_t v = {lo, hi};
  union { bf16x2_hw_t b; uint32_t u; } c;
  c.b = __builtin_convertvector(v, bf16x2_hw_t);
  return c.u;
}
__device__ __forceinline__ uint16_t f2bf(float f) { return (uint16_t)(pack_bf2(f, 0.f) & 0xffffu); }

__device__ __forceinline__ float ld(const float *p) { return *p; }
__device__ __forceinline__ float ld(const bf16 *p) { return bf2f(p->v); }
__device__ __forceinline__ void st(float *p, float x) { *p = x; }
__device__ __forceinline__ void st(bf16 *p, float x) { p->v = f2bf(x); }

// erf by the rational approximation 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7):
// a handful of FMAs, one hardware reciprocal (v_rcp_f32, 1 ulp; a correctly rounded division would cost ten
// instructions more per element of a GEMM epilogue) and one hardware exponential.
// erf_core(x, e) returns erf(x) given e = exp(-x*x), so that callers that need the exponential too share it.
__device__ __forceinline__ float erf_core(float x, float e) {
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, fabsf(x), 1.f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  return copysignf(fmaf(-poly * t, e, 1.f), x);
}
// exp(-u*u/2) = 2^(-u*u * log2(e)/2)
__device__ __forceinline__ float exp_mhalf_sq(float u) { return __builtin_amdgcn_exp2f(u * u * -0.72134752044448170f); }
// GELU in its erf form and its derivative: cdf(u) = (1 + erf(u / sqrt 2)) / 2, pdf(u) = exp(-u*u/2) / sqrt(2 pi).
__device__ __forceinline__ float gelu_f(float u) {
  return 0.5f * u * (1.f + erf_core(u * 0.70710678118654752f, exp_mhalf_sq(u)));
}
__device__ __forceinline__ float gelu_grad_f(float u) {
  const float e = exp_mhalf_sq(u);
  const float cdf = 0.5f * (1.f + erf_core(u * 0.70710678118654752f, e));
  return fmaf(u * 0.39894228040143268f, e, cdf);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace ssdt
