// Small device helpers shared by the kernel files (conversions, activations,
// wavefront reductions).  gfx950 only: wavefronts are 64 lanes wide.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "abs_internal.h"

namespace absk {

__device__ __forceinline__ float bf2f(bf16_t h) {
  return __uint_as_float(static_cast<uint32_t>(h) << 16);
}
// float -> bfloat16, round to nearest even (the hardware conversion of gfx950)
__device__ __forceinline__ bf16_t f2bf(float f) {
  __bf16 b = static_cast<__bf16>(f);
  return __builtin_bit_cast(uint16_t, b);
}
// two floats -> packed bfloat16 pair (lo in bits 0..15), one v_cvt_pk_bf16_f32
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <class T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float ld(const float *p) { return *p; }
  static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
  static __device__ __forceinline__ float rnd(float v) { return v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t *p) { return bf2f(*p); }
  static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f2bf(v); }
  static __device__ __forceinline__ float rnd(float v) { return bf2f(f2bf(v)); }
};

// Exact-form GELU phi(z) = z Phi(z) and its derivative Phi(z) + z pdf(z).
// Phi comes from the rational-times-exponential erfc approximation of Abramowitz & Stegun
// 7.1.26 (absolute error of erf below 1.5e-7, i.e. fp32 rounding level); it shares its single
// exponential with the density, so value and derivative cost one v_exp and one v_rcp.
__device__ __forceinline__ void gelu_fwd(float z, float &a, float &d) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));         // v_rcp_f32, 1 ulp
  const float e = __builtin_amdgcn_exp2f(z * z * -0.72134752044448170f);    // exp(-z^2/2) = 2^(-z^2 log2(e)/2)
  float poly = fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);          // coefficients carry the 1/2 of erfc/2
  poly = fmaf(poly, t, 0.5f * 1.421413741f);
  poly = fmaf(poly, t, 0.5f * -0.284496736f);
  poly = fmaf(poly, t, 0.5f * 0.254829592f);
  const float half_erfc = poly * t * e;                 // 0.5 erfc(|z|/sqrt 2)
  const float cdf = z >= 0.0f ? 1.0f - half_erfc : half_erfc;
  a = z * cdf;
  d = fmaf(z * 0.39894228040143268f, e, cdf);
}

template <int ACT>
__device__ __forceinline__ void act_fwd(float z, float &a, float &d) {
  if (ACT == ACT_RELU) { a = z > 0.0f ? z : 0.0f; d = z > 0.0f ? 1.0f : 0.0f; }
  else if (ACT == ACT_GELU) { gelu_fwd(z, a, d); }
  else { a = z; d = 1.0f; }
}

// One parameter's optimizer step (the inner optimizers named in Sec. 4.2; formulas: SGD x - lr g; heavy ball
// v <- mu v + g, x <- x - lr v; AdaGrad v <- v + g^2, x <- x - lr g / (sqrt v + eps); AdamW with bias
// corrections c1 = 1/(1 - beta1^t), c2 = 1/(1 - beta2^t) and decoupled decay).  Used by the update kernel and by
// the weight-gradient epilogue that applies the step in place; the same expression order in both.
struct OptHyper { float lr, momentum, beta1, beta2, eps, wd, c1, c2; };
template <int OPT>
__device__ __forceinline__ void opt_step_elem(float &x, float g, float &v, float &m, const OptHyper &h) {
  if (OPT == OPT_SGD) {
    x = fmaf(-h.lr, g, x);
  } else if (OPT == OPT_SHB) {
    v = fmaf(h.momentum, v, g);
    x = fmaf(-h.lr, v, x);
  } else if (OPT == OPT_ADAGRAD) {
    v = fmaf(g, g, v);
    const float den = sqrtf(v) + h.eps;          // den == 0 only where no gradient has ever arrived
    if (den > 0.f) x = x - h.lr * g / den;
  } else {
    m = fmaf(h.beta1, m, (1.0f - h.beta1) * g);
    v = fmaf(h.beta2, v, (1.0f - h.beta2) * g * g);
    const float mhat = m * h.c1, vhat = v * h.c2;
    x = x * (1.0f - h.lr * h.wd) - h.lr * mhat / (sqrtf(vhat) + h.eps);
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Sum over a block of NW wavefronts in a fixed order; result valid in thread 0.
template <int NW>
__device__ __forceinline__ double block_sum(double v, double *smem /*NW doubles*/) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) smem[w] = v;
  __syncthreads();
  double r = 0.0;
  if (threadIdx.x == 0) {
#pragma unroll
    for (int i = 0; i < NW; ++i) r += smem[i];
  }
  __syncthreads();
  return r;
}

}  // namespace absk
