// Shared device helpers for the gfx950 kernels: element types, bf16
// conversion, wavefront (64-lane) and workgroup reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pt {

typedef __bf16 bf16;

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return static_cast<float>(x); }

template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
// gfx950 converts fp32 -> bf16 in hardware with round-to-nearest-even.
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return static_cast<bf16>(x); }

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

// Sum over a workgroup of NW waves; every thread gets the result.  `red` is
// LDS scratch of at least NW floats.  Fixed order, so deterministic.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) s += red[i];
  return s;
}
template <int NW>
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int i = 1; i < NW; ++i) s = fmaxf(s, red[i]);
  return s;
}

// GELU in its erf form, h*Phi(h), and its derivative Phi(h) + h*phi(h).  Phi comes from the rational
// approximation of erfc (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7, 4e-7 with fp32 rounding), evaluated
// on the side without cancellation: Phi(h) = q for h < 0 and 1 - q otherwise, q = 0.5 * poly(t) * exp(-h^2/2),
// t = 1 / (1 + p |h| / sqrt 2).  The exponential is the one phi(h) needs, so the derivative costs two more
// operations; the whole thing is about a third of the instructions of erff() + expf().
__device__ __forceinline__ float gelu_cdf(float h, float* e_out) {
  const float z = fabsf(h) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  const float poly =
      t * fmaf(t, fmaf(t, fmaf(t, fmaf(t, 1.061405429f, -1.453152027f), 1.421413741f), -0.284496736f), 0.254829592f);
  const float e = __expf(-(z * z));   // = exp(-h*h/2)
  const float q = 0.5f * poly * e;
  *e_out = e;
  return h < 0.f ? q : 1.0f - q;
}
__device__ __forceinline__ float gelu_f(float h) {
  float e;
  return h * gelu_cdf(h, &e);
}
// GELU(h) and its derivative from one evaluation of Phi and of the exponential
__device__ __forceinline__ float gelu_both(float h, float* d_out) {
  float e;
  const float cdf = gelu_cdf(h, &e);
  *d_out = fmaf(h * 0.39894228040143268f, e, cdf);
  return h * cdf;
}
__device__ __forceinline__ float dgelu_f(float h) {
  float e;
  const float cdf = gelu_cdf(h, &e);
  return fmaf(h * 0.39894228040143268f, e, cdf);
}

inline int cdiv(int a, int b) { return (a + b - 1) / b; }
inline int64_t cdiv64(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace pt
