// LayerNorm backward over rows, as device code shared by the stand-alone kernel (rowops.hip) and by the
// grouped weight-gradient launch, whose spare workgroups run one such pass beside the matrix work
// (gemm_dma.hip).
#pragma once
#include "common.h"

namespace pt {

// ---- 4-element vector access ------------------------------------------------
__device__ __forceinline__ void load4(const float* p, float (&v)[4]) {
  const float4 t = *reinterpret_cast<const float4*>(p);
  v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
__device__ __forceinline__ void load4(const bf16* p, float (&v)[4]) {
  const uint2 t = *reinterpret_cast<const uint2*>(p);
  v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
  v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}
__device__ __forceinline__ void store4(float* p, const float (&v)[4]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void store4(bf16* p, const float (&v)[4]) {
  union { bf16 h[4]; uint2 u; } t;
#pragma unroll
  for (int i = 0; i < 4; ++i) t.h[i] = from_f32<bf16>(v[i]);
  *reinterpret_cast<uint2*>(p) = t.u;
}

// four elements as loaded (converted to fp32 only when used, so a prefetched row costs few registers)
template <typename T> struct Raw4;
template <> struct Raw4<float> {
  float4 r;
  __device__ __forceinline__ void ld(const float* p) { r = *reinterpret_cast<const float4*>(p); }
  __device__ __forceinline__ void zero() { r = make_float4(0.f, 0.f, 0.f, 0.f); }
  __device__ __forceinline__ void get(float (&v)[4]) const { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
};
template <> struct Raw4<bf16> {
  uint2 r;
  __device__ __forceinline__ void ld(const bf16* p) { r = *reinterpret_cast<const uint2*>(p); }
  __device__ __forceinline__ void zero() { r = make_uint2(0u, 0u); }
  __device__ __forceinline__ void get(float (&v)[4]) const {
    v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
    v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
  }
};

// One LayerNorm backward pass (the arguments of layernorm_bwd, see kernels.h).
template <typename T, typename TDY, typename TX>
struct LnBwdArgs {
  const TDY* dy; int64_t lddy;
  const TX* x; int64_t ldx;
  const float* mean; const float* rstd;
  const T* gamma;
  const float* dres; int64_t lddres;
  float* dx_s; T* dx_o; int64_t lddx;
  float* partial;   // [number of workgroups][3 D]: d(gamma), d(beta) and the output's column sums per workgroup
  int rows, D;
};

// Workgroup `wg` of `nwg`, NWAVES waves of 64 lanes, one row per wave at a time; red = 3 D floats of LDS.
// dy may be the fp32 gradient stream or a T tensor; the result goes to an fp32 stream buffer (dx_s), a T copy
// for the matrix-core operands (dx_o), or both (either may be null).
template <typename T, typename TDY, typename TX, int VPL, int NWAVES>
__device__ __forceinline__ void ln_bwd_rows(const LnBwdArgs<T, TDY, TX>& a, float* __restrict__ red, int wg, int nwg) {
  const TDY* __restrict__ dy = a.dy; const TX* __restrict__ x = a.x;
  const float* __restrict__ mean = a.mean; const float* __restrict__ rstd = a.rstd;
  const float* __restrict__ dres = a.dres;
  float* __restrict__ dx_s = a.dx_s; T* __restrict__ dx_o = a.dx_o;
  const int64_t lddy = a.lddy, ldx = a.ldx, lddres = a.lddres, lddx = a.lddx;
  const int rows = a.rows, D = a.D;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nvec = D >> 2;
  float g[VPL][4], ag[VPL][4], ab[VPL][4], as[VPL][4];
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int c = lane + 64 * j;
#pragma unroll
    for (int e = 0; e < 4; ++e) { ag[j][e] = 0.f; ab[j][e] = 0.f; as[j][e] = 0.f; g[j][e] = 0.f; }
    if (c < nvec) load4(a.gamma + 4 * c, g[j]);
  }
  // The loads of a wave's next row go out before the current row is worked on: a wave handles only a few
  // rows, one after the other, and without this it has nothing in flight while it reduces and stores.
  struct RowIn {
    Raw4<TX> x[VPL];
    Raw4<TDY> d[VPL];
    Raw4<float> r[VPL];
    float mu, rs;
  };
  auto fetch = [&](int row, RowIn& in) {
    in.mu = mean[row];
    in.rs = rstd[row];
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c = lane + 64 * j;
      in.x[j].zero(); in.d[j].zero(); in.r[j].zero();
      if (c < nvec) {
        in.x[j].ld(x + (int64_t)row * ldx + 4 * c);
        in.d[j].ld(dy + (int64_t)row * lddy + 4 * c);
        if (dres) in.r[j].ld(dres + (int64_t)row * lddres + 4 * c);
      }
    }
  };
  const int stride = nwg * NWAVES;
  int row = wg * NWAVES + wave;
  RowIn cur, nxt;
  if (row < rows) fetch(row, cur);
  for (; row < rows; row += stride) {
    const bool more = row + stride < rows;
    if (more) fetch(row + stride, nxt);
    const float mu = cur.mu, rs = cur.rs;
    float xh[VPL][4], dh[VPL][4];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c = lane + 64 * j;
      if (c < nvec) {
        float xv[4], dv[4];
        cur.x[j].get(xv);
        cur.d[j].get(dv);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          xh[j][e] = (xv[e] - mu) * rs;
          ag[j][e] += dv[e] * xh[j][e];
          ab[j][e] += dv[e];
          dh[j][e] = dv[e] * g[j][e];
          s1 += dh[j][e];
          s2 += dh[j][e] * xh[j][e];
        }
      }
    }
    if (dx_s || dx_o) {   // else only the parameter gradients are wanted
      const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        const int c = lane + 64 * j;
        if (c < nvec) {
          float o[4], res[4];
          cur.r[j].get(res);
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (dh[j][e] - m1 - xh[j][e] * m2) * rs + res[e];
#pragma unroll
          for (int e = 0; e < 4; ++e) as[j][e] += o[e];
          if (dx_s) store4(dx_s + (int64_t)row * lddx + 4 * c, o);
          if (dx_o) store4(dx_o + (int64_t)row * lddx + 4 * c, o);
        }
      }
    }
    if (more) cur = nxt;
  }
  // combine the waves of the workgroup in wave order (fixed, so reproducible)
  for (int w = 0; w < NWAVES; ++w) {
    if (wave == w) {
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        const int c = lane + 64 * j;
        if (c < nvec) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * c + e;
            red[i] = (w ? red[i] : 0.f) + ag[j][e];
            red[D + i] = (w ? red[D + i] : 0.f) + ab[j][e];
            red[2 * D + i] = (w ? red[2 * D + i] : 0.f) + as[j][e];
          }
        }
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < 3 * D; i += 64 * NWAVES) a.partial[(size_t)wg * 3 * D + i] = red[i];
}

}  // namespace pt
