// Memory-bound passes of the step: LayerNorm forward/backward, bias-gradient
// column sums, front ends (ViT patch embedding plumbing, BERT embedding lookup
// and its scatter-add), losses, and row copies for the activation cache.
// Row reductions are wavefront shuffles (one 64-lane wave per row); reductions
// across rows are two-stage with a fixed summation order, so every result is
// reproducible run to run.
#include "common.h"
#include "kernels.h"
#include "ln_bwd_rows.h"

namespace pt {

// ---------------------------------------------------------------------------
// LayerNorm forward: one wave per row, row held in registers (D <= 256*VPL)
// ---------------------------------------------------------------------------
constexpr int kLnFwdBlocks = 768;   // persistent workgroups (three per CU), four waves each
template <typename T, typename TX, int VPL>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const TX* __restrict__ x, int64_t ldx, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ y, int64_t ldy,
                                                     float* __restrict__ mean, float* __restrict__ rstd, int rows, int D,
                                                     float eps) {
  const int lane = threadIdx.x & 63;
  const int nvec = D >> 2;
  Raw4<T> gr[VPL], br[VPL];
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int c = lane + 64 * j;
    gr[j].zero(); br[j].zero();
    if (c < nvec) { gr[j].ld(gamma + 4 * c); br[j].ld(beta + 4 * c); }
  }
  // a wave walks over its rows with the next row's loads in flight while it reduces and stores the current one
  auto fetch = [&](int row, Raw4<TX> (&in)[VPL]) {
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c = lane + 64 * j;
      in[j].zero();
      if (c < nvec) in[j].ld(x + (int64_t)row * ldx + 4 * c);
    }
  };
  const int stride = gridDim.x * 4;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  Raw4<TX> cur[VPL], nxt[VPL];
  if (row < rows) fetch(row, cur);
  for (; row < rows; row += stride) {
    const bool more = row + stride < rows;
    if (more) fetch(row + stride, nxt);
    float v[VPL][4];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      cur[j].get(v[j]);
      s += (v[j][0] + v[j][1]) + (v[j][2] + v[j][3]);
    }
    const float mu = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c = lane + 64 * j;
      if (c < nvec) {
#pragma unroll
        for (int e = 0; e < 4; ++e) { const float d = v[j][e] - mu; q += d * d; }
      }
    }
    const float rs = rsqrtf(wave_sum(q) / (float)D + eps);
    if (lane == 0 && mean) { mean[row] = mu; rstd[row] = rs; }
    T* yr = y + (int64_t)row * ldy;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c = lane + 64 * j;
      if (c < nvec) {
        float g[4], b[4], o[4];
        gr[j].get(g);
        br[j].get(b);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (v[j][e] - mu) * rs * g[e] + b[e];
        store4(yr + 4 * c, o);
      }
    }
    if (more) {
#pragma unroll
      for (int j = 0; j < VPL; ++j) cur[j] = nxt[j];
    }
  }
}

// bf16 rows whose length is a multiple of 256: half a wave per row, so that a lane moves 16 bytes per access
// (8-byte accesses, which the one-wave-per-row kernel makes on bf16 rows, reach 4.4 TB/s on this pass)
template <int VPL>
__global__ __launch_bounds__(256) void ln_fwd_half_kernel(const bf16* __restrict__ x, int64_t ldx, const bf16* __restrict__ gamma,
                                                          const bf16* __restrict__ beta, bf16* __restrict__ y, int64_t ldy,
                                                          float* __restrict__ mean, float* __restrict__ rstd, int rows, int D,
                                                          float eps) {
  const int lane = threadIdx.x & 31;
  auto cvt = [](const uint4& r, float (&v)[8]) {
    v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
    v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
    v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
    v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
  };
  auto half_sum = [](float v) {
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
  };
  uint4 gr[VPL], br[VPL];
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    gr[j] = *reinterpret_cast<const uint4*>(gamma + 8 * (lane + 32 * j));
    br[j] = *reinterpret_cast<const uint4*>(beta + 8 * (lane + 32 * j));
  }
  const int stride = gridDim.x * 16;   // eight half-waves per workgroup, two rows per half-wave in flight
  int row = blockIdx.x * 8 + (threadIdx.x >> 5);
  const int step = gridDim.x * 8;
  uint4 cur[VPL], nxt[VPL];
  (void)stride;
  auto fetch = [&](int r, uint4 (&in)[VPL]) {
    const int rc = r < rows ? r : rows - 1;
#pragma unroll
    for (int j = 0; j < VPL; ++j) in[j] = *reinterpret_cast<const uint4*>(x + (int64_t)rc * ldx + 8 * (lane + 32 * j));
  };
  fetch(row, cur);
  // both half-waves of a wave run the same number of iterations (the shuffles need all lanes present)
  const int base_row = blockIdx.x * 8 + ((threadIdx.x >> 6) << 1);
  for (int r0 = base_row; r0 < rows; r0 += step, row += step) {
    fetch(row + step, nxt);
    float v[VPL][8];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      cvt(cur[j], v[j]);
      s += ((v[j][0] + v[j][1]) + (v[j][2] + v[j][3])) + ((v[j][4] + v[j][5]) + (v[j][6] + v[j][7]));
    }
    const float mu = half_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < VPL; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = v[j][e] - mu; q += d * d; }
    const float rs = rsqrtf(half_sum(q) / (float)D + eps);
    if (row < rows) {
      if (lane == 0 && mean) { mean[row] = mu; rstd[row] = rs; }
      bf16* yr = y + (int64_t)row * ldy;
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        float g[8], b[8];
        cvt(gr[j], g);
        cvt(br[j], b);
        union { bf16 h[8]; uint4 u; } t;
#pragma unroll
        for (int e = 0; e < 8; ++e) t.h[e] = from_f32<bf16>((v[j][e] - mu) * rs * g[e] + b[e]);
        *reinterpret_cast<uint4*>(yr + 8 * (lane + 32 * j)) = t.u;
      }
    }
#pragma unroll
    for (int j = 0; j < VPL; ++j) cur[j] = nxt[j];
  }
}

void layernorm_fwd(int dt, bool x_f32, const void* x, int64_t ldx, const void* gamma, const void* beta, void* y,
                   int64_t ldy, float* mean, float* rstd, int rows, int D, float eps, hipStream_t st) {
  if (rows <= 0) return;
  if (dt != 0 && !x_f32 && (D == 768 || D == 1024) && ldx % 8 == 0 && ldy % 8 == 0 &&
      ((uintptr_t)x | (uintptr_t)y | (uintptr_t)gamma | (uintptr_t)beta) % 16 == 0) {
    const dim3 g(cdiv(rows, 8) < kLnFwdBlocks ? cdiv(rows, 8) : kLnFwdBlocks), b(256);
    if (D == 768)
      hipLaunchKernelGGL((ln_fwd_half_kernel<3>), g, b, 0, st, (const bf16*)x, ldx, (const bf16*)gamma, (const bf16*)beta,
                         (bf16*)y, ldy, mean, rstd, rows, D, eps);
    else
      hipLaunchKernelGGL((ln_fwd_half_kernel<4>), g, b, 0, st, (const bf16*)x, ldx, (const bf16*)gamma, (const bf16*)beta,
                         (bf16*)y, ldy, mean, rstd, rows, D, eps);
    return;
  }
  dim3 grid(cdiv(rows, 4) < kLnFwdBlocks ? cdiv(rows, 4) : kLnFwdBlocks), blk(256);
#define LN_FWD(T, TX, V)                                                                                  \
  hipLaunchKernelGGL((ln_fwd_kernel<T, TX, V>), grid, blk, 0, st, (const TX*)x, ldx, (const T*)gamma, \
                     (const T*)beta, (T*)y, ldy, mean, rstd, rows, D, eps)
#define LN_FWD_V(T, TX)                               \
  do {                                                \
    if (D <= 768) LN_FWD(T, TX, 3);                   \
    else if (D <= 1024) LN_FWD(T, TX, 4);             \
    else LN_FWD(T, TX, 8);                            \
  } while (0)
  if (dt == 0) LN_FWD_V(float, float);
  else if (x_f32) LN_FWD_V(bf16, float);
  else LN_FWD_V(bf16, bf16);
#undef LN_FWD_V
#undef LN_FWD
}

// ---------------------------------------------------------------------------
// LayerNorm backward
// ---------------------------------------------------------------------------
constexpr int kLnBwdBlocks = 512;   // workgroups (partial rows) at most: two per CU, each wave with two rows in flight
constexpr int kLnBwdWaves = 4;      // waves per workgroup, one row per wave at a time
size_t ln_partial_floats(int D) { return (size_t)kLnBwdBlocks * 3 * D; }
constexpr int g_ln_bwd_blocks = 0;   // workgroups of the backward kernel (0 = default)

// dy may be the fp32 gradient stream or a T tensor; the result goes to an fp32 stream
// buffer (dx_s), a T copy for the matrix-core operands (dx_o), or both (either may be null).
template <typename T, typename TDY, typename TX, int VPL>
__global__ __launch_bounds__(64 * kLnBwdWaves) void ln_bwd_kernel(LnBwdArgs<T, TDY, TX> a) {
  extern __shared__ float red[];  // [3][D]: d(gamma), d(beta), column sums of the output
  ln_bwd_rows<T, TDY, TX, VPL, kLnBwdWaves>(a, red, blockIdx.x, gridDim.x);
}

// out[i] = sum over p of partial[p][i] in a fixed order: 32 columns per workgroup (one 128-byte line per
// partial row), 32 interleaved row groups, each with eight independent running sums so that many loads are
// in flight (the kernel is latency-bound: 9 MB over 72 workgroups); the sums are combined in a fixed order.
// Column i goes to out0[i] for i < n0, to out1[i - n0] for i < 2 n0, else to out2[i - 2 n0]; a null
// destination drops the column.
__device__ __forceinline__ void reduce_partials_body(const float* __restrict__ partial, int np, int n,
                                                     float* __restrict__ out0, int n0, float* __restrict__ out1,
                                                     float* __restrict__ out2, float (&red)[32][33]) {
  const int c = threadIdx.x & 31, rg = threadIdx.x >> 5;
  const int i = blockIdx.x * 32 + c;
  float s[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) s[u] = 0.f;
  if (i < n) {
    int p = rg;
    for (; p + 7 * 32 < np; p += 8 * 32) {
#pragma unroll
      for (int u = 0; u < 8; ++u) s[u] += partial[(size_t)(p + 32 * u) * n + i];
    }
    for (; p < np; p += 32) s[0] += partial[(size_t)p * n + i];
  }
  red[rg][c] = ((s[0] + s[1]) + (s[2] + s[3])) + ((s[4] + s[5]) + (s[6] + s[7]));
  __syncthreads();
  if (rg == 0 && i < n) {
    float t = red[0][c];
#pragma unroll
    for (int k = 1; k < 32; ++k) t += red[k][c];
    float* dst = i < n0 ? out0 : (i < 2 * n0 ? out1 : out2);
    if (dst) dst[i % n0] = t;
  }
}
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const float* __restrict__ partial, int np, int n,
                                                               float* __restrict__ out0, int n0,
                                                               float* __restrict__ out1, float* __restrict__ out2) {
  __shared__ float red[32][33];
  reduce_partials_body(partial, np, n, out0, n0, out1, out2, red);
}
// the same for several LayerNorm backward passes at once (blockIdx.y = pass): their parameter gradients are
// read by nothing before the end of the backward pass, so one launch there replaces one launch per pass
struct LnReduceBatch {
  const float* partial[kLnReduceBatch];
  float* dgamma[kLnReduceBatch];
  float* dbeta[kLnReduceBatch];
  float* dxsum[kLnReduceBatch];
  int np[kLnReduceBatch];
};
__global__ __launch_bounds__(1024) void reduce_partials_batch_kernel(LnReduceBatch b, int D) {
  __shared__ float red[32][33];
  const int j = blockIdx.y;
  reduce_partials_body(b.partial[j], b.np[j], 3 * D, b.dgamma[j], D, b.dbeta[j], b.dxsum[j], red);
}

void layernorm_bwd_reduce(const LnReduceJob* jobs, int n, int D, hipStream_t st) {
  for (int j0 = 0; j0 < n; j0 += kLnReduceBatch) {
    LnReduceBatch b;
    const int m = n - j0 < kLnReduceBatch ? n - j0 : kLnReduceBatch;
    for (int j = 0; j < m; ++j) {
      b.partial[j] = jobs[j0 + j].partial; b.np[j] = jobs[j0 + j].np;
      b.dgamma[j] = jobs[j0 + j].dgamma; b.dbeta[j] = jobs[j0 + j].dbeta; b.dxsum[j] = jobs[j0 + j].dxsum;
    }
    hipLaunchKernelGGL(reduce_partials_batch_kernel, dim3(cdiv(3 * D, 32), m), dim3(1024), 0, st, b, D);
  }
}

void layernorm_bwd(int dt, bool dy_f32, bool x_f32, const void* dy, int64_t lddy, const void* x, int64_t ldx,
                   const float* mean, const float* rstd, const void* gamma, const float* dres, int64_t lddres,
                   float* dx_s, void* dx_o, int64_t lddx, float* dgamma, float* dbeta, float* dxsum, float* partial,
                   int rows, int D, hipStream_t st, LnReduceJob* deferred) {
  if (deferred) *deferred = LnReduceJob{partial, 0, dgamma, dbeta, dxsum};
  if (rows <= 0) return;
  const int cap = g_ln_bwd_blocks > 0 && g_ln_bwd_blocks < kLnBwdBlocks ? g_ln_bwd_blocks : kLnBwdBlocks;
  const int nb = cdiv(rows, kLnBwdWaves) < cap ? cdiv(rows, kLnBwdWaves) : cap;
  const size_t shm = (size_t)3 * D * sizeof(float);
#define LN_BWD(T, TDY, TX, V)                                                                                      \
  do {                                                                                                             \
    const LnBwdArgs<T, TDY, TX> a_{(const TDY*)dy, lddy, (const TX*)x, ldx, mean, rstd, (const T*)gamma, dres, lddres, \
                                   dx_s, (T*)dx_o, lddx, partial, rows, D};                                        \
    hipLaunchKernelGGL((ln_bwd_kernel<T, TDY, TX, V>), dim3(nb), dim3(64 * kLnBwdWaves), shm, st, a_);             \
  } while (0)
#define LN_BWD_V(T, TDY, TX)                                             \
  do {                                                                   \
    if (D <= 256) LN_BWD(T, TDY, TX, 1);                                 \
    else if (D <= 768) LN_BWD(T, TDY, TX, 3);                            \
    else if (D <= 1024) LN_BWD(T, TDY, TX, 4);                           \
    else LN_BWD(T, TDY, TX, 8);                                          \
  } while (0)
  if (dt == 0) LN_BWD_V(float, float, float);
  else if (dy_f32 && x_f32) LN_BWD_V(bf16, float, float);
  else if (dy_f32) LN_BWD_V(bf16, float, bf16);
  else if (x_f32) LN_BWD_V(bf16, bf16, float);
  else LN_BWD_V(bf16, bf16, bf16);
#undef LN_BWD_V
#undef LN_BWD
  // the sums over the workgroups' partial rows: now, or later in one launch with those of other passes
  if (deferred) deferred->np = nb;
  else hipLaunchKernelGGL(reduce_partials_kernel, dim3(cdiv(3 * D, 32)), dim3(1024), 0, st, partial, nb, 3 * D, dgamma, D,
                          dbeta, dxsum);
}

// ---------------------------------------------------------------------------
// column sums (bias gradients)
// ---------------------------------------------------------------------------
constexpr int kColsumRowBlocks = 128;
size_t colsum_partial_floats(int N) { return (size_t)kColsumRowBlocks * N; }

template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ X, int64_t ld, int M, int N,
                                                     float* __restrict__ partial) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= N) return;
  float s = 0.f;
  for (int r = blockIdx.y; r < M; r += gridDim.y) s += to_f32(X[(int64_t)r * ld + col]);
  partial[(size_t)blockIdx.y * N + col] = s;
}

void colsum(int dt, const void* X, int64_t ld, int M, int N, float* out, float* partial, hipStream_t st) {
  const int nby = M < kColsumRowBlocks ? M : kColsumRowBlocks;
  dim3 grid(cdiv(N, 256), nby);
  if (dt == 0) hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, st, (const float*)X, ld, M, N, partial);
  else hipLaunchKernelGGL(colsum_kernel<bf16>, grid, dim3(256), 0, st, (const bf16*)X, ld, M, N, partial);
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(cdiv(N, 32)), dim3(1024), 0, st, partial, nby, N, out, N,
                     (float*)nullptr, (float*)nullptr);
}

// ---------------------------------------------------------------------------
// ViT front end plumbing
// ---------------------------------------------------------------------------
template <typename T>
__global__ void patchify_kernel(const float* __restrict__ img, const int64_t* __restrict__ map, T* __restrict__ out,
                                int nb, int chans, int side, int p) {
  const int g = side / p, pd = chans * p * p;
  const int64_t total = (int64_t)nb * g * g * pd;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int j = (int)(i % pd);
    const int64_t pi = i / pd;
    const int gx = (int)(pi % g), gy = (int)((pi / g) % g);
    const int64_t bo = pi / ((int64_t)g * g);
    const int64_t b = map ? map[bo] : bo;
    const int px = j % p, py = (j / p) % p, c = j / (p * p);
    out[i] = from_f32<T>(img[((b * chans + c) * side + gy * p + py) * side + gx * p + px]);
  }
}
// four consecutive pixels of a patch row per thread (patch side and image side multiples of 4)
template <typename T>
__global__ void patchify4_kernel(const float* __restrict__ img, const int64_t* __restrict__ map, T* __restrict__ out,
                                 int nb, int chans, int side, int p) {
  const int g = side / p, pd4 = chans * p * p / 4, p4 = p / 4;
  const int64_t total = (int64_t)nb * g * g * pd4;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int j = (int)(i % pd4);
    const int64_t pi = i / pd4;
    const int gx = (int)(pi % g), gy = (int)((pi / g) % g);
    const int64_t bo = pi / ((int64_t)g * g);
    const int64_t b = map ? map[bo] : bo;
    const int px = (j % p4) * 4, py = (j / p4) % p, c = j / (p4 * p);
    const float4 v = *reinterpret_cast<const float4*>(img + ((b * chans + c) * side + gy * p + py) * side + gx * p + px);
    const float a[4] = {v.x, v.y, v.z, v.w};
    store4(out + i * 4, a);
  }
}
void vit_patchify(int dt, const float* images, const int64_t* map, void* patches, int nb, int chans, int img, int patch,
                  hipStream_t st) {
  if (patch % 4 == 0 && img % 4 == 0 && (reinterpret_cast<uintptr_t>(images) & 15) == 0 &&
      (reinterpret_cast<uintptr_t>(patches) & 15) == 0) {
    const int64_t total4 = (int64_t)nb * chans * img * img / 4;
    const int blocks4 = (int)(cdiv64(total4, 256) < 65536 ? cdiv64(total4, 256) : 65536);
    if (blocks4 <= 0) return;
    if (dt == 0) hipLaunchKernelGGL(patchify4_kernel<float>, dim3(blocks4), dim3(256), 0, st, images, map, (float*)patches, nb, chans, img, patch);
    else hipLaunchKernelGGL(patchify4_kernel<bf16>, dim3(blocks4), dim3(256), 0, st, images, map, (bf16*)patches, nb, chans, img, patch);
    return;
  }
  const int64_t total = (int64_t)nb * chans * img * img;
  const int blocks = (int)(cdiv64(total, 256) < 65536 ? cdiv64(total, 256) : 65536);
  if (blocks <= 0) return;
  if (dt == 0) hipLaunchKernelGGL(patchify_kernel<float>, dim3(blocks), dim3(256), 0, st, images, map, (float*)patches, nb, chans, img, patch);
  else hipLaunchKernelGGL(patchify_kernel<bf16>, dim3(blocks), dim3(256), 0, st, images, map, (bf16*)patches, nb, chans, img, patch);
}

template <typename T>
__global__ void vit_assemble_kernel(const T* __restrict__ E, const T* __restrict__ cls, const T* __restrict__ pos,
                                    T* __restrict__ X, int nb, int S, int D) {
  const int nv = D >> 2;
  const int64_t total = (int64_t)nb * S * nv;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % nv);
    const int64_t r = i / nv;
    const int s = (int)(r % S), b = (int)(r / S);
    float a[4], pz[4], o[4];
    if (s == 0) load4(cls + 4 * c, a); else load4(E + ((int64_t)b * (S - 1) + (s - 1)) * D + 4 * c, a);
    load4(pos + (int64_t)s * D + 4 * c, pz);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = a[e] + pz[e];
    store4(X + r * D + 4 * c, o);
  }
}
void vit_assemble(int dt, const void* E, const void* cls, const void* pos, void* X, int nb, int S, int D,
                  hipStream_t st) {
  const int64_t total = (int64_t)nb * S * (D / 4);
  const int blocks = (int)(cdiv64(total, 256) < 65536 ? cdiv64(total, 256) : 65536);
  if (blocks <= 0) return;
  if (dt == 0) hipLaunchKernelGGL(vit_assemble_kernel<float>, dim3(blocks), dim3(256), 0, st, (const float*)E, (const float*)cls, (const float*)pos, (float*)X, nb, S, D);
  else hipLaunchKernelGGL(vit_assemble_kernel<bf16>, dim3(blocks), dim3(256), 0, st, (const bf16*)E, (const bf16*)cls, (const bf16*)pos, (bf16*)X, nb, S, D);
}

template <typename T>
__global__ void vit_front_bwd_kernel(const float* __restrict__ dX, T* __restrict__ dE, float* __restrict__ dpos,
                                     float* __restrict__ dcls, int nb, int S, int D) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * D) return;
  const int s = i / D, d = i % D;
  float acc = 0.f;
  for (int b = 0; b < nb; ++b) {
    const float v = dX[((int64_t)b * S + s) * D + d];
    acc += v;
    if (s > 0) dE[((int64_t)b * (S - 1) + (s - 1)) * D + d] = from_f32<T>(v);
  }
  dpos[i] = acc;
  if (s == 0) dcls[d] = acc;
}
// the same with four columns per thread and eight samples' loads in flight (D a multiple of 4)
template <typename T>
__global__ __launch_bounds__(256) void vit_front_bwd4_kernel(const float* __restrict__ dX, T* __restrict__ dE,
                                                             float* __restrict__ dpos, float* __restrict__ dcls, int nb,
                                                             int S, int D) {
  const int nv = D >> 2;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * nv) return;
  const int s = i / nv, d = 4 * (i % nv);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int b0 = 0; b0 < nb; b0 += 8) {
    float v[8][4];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      v[u][0] = v[u][1] = v[u][2] = v[u][3] = 0.f;
      if (b0 + u < nb) load4(dX + ((int64_t)(b0 + u) * S + s) * D + d, v[u]);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (b0 + u >= nb) break;
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] += v[u][e];   // sample order, as in the scalar kernel
      if (s > 0) store4(dE + ((int64_t)(b0 + u) * (S - 1) + (s - 1)) * D + d, v[u]);
    }
  }
  store4(dpos + (int64_t)s * D + d, acc);
  if (s == 0) store4(dcls + d, acc);
}
void vit_front_bwd(int dt, const float* dX, void* dE, float* dpos, float* dcls, int nb, int S, int D, hipStream_t st) {
  if (D % 4 == 0) {
    dim3 grid4(cdiv(S * (D / 4), 256));
    if (dt == 0) hipLaunchKernelGGL(vit_front_bwd4_kernel<float>, grid4, dim3(256), 0, st, dX, (float*)dE, dpos, dcls, nb, S, D);
    else hipLaunchKernelGGL(vit_front_bwd4_kernel<bf16>, grid4, dim3(256), 0, st, dX, (bf16*)dE, dpos, dcls, nb, S, D);
    return;
  }
  dim3 grid(cdiv(S * D, 256));
  if (dt == 0) hipLaunchKernelGGL(vit_front_bwd_kernel<float>, grid, dim3(256), 0, st, dX, (float*)dE, dpos, dcls, nb, S, D);
  else hipLaunchKernelGGL(vit_front_bwd_kernel<bf16>, grid, dim3(256), 0, st, dX, (bf16*)dE, dpos, dcls, nb, S, D);
}

// ---------------------------------------------------------------------------
// BERT front end
// ---------------------------------------------------------------------------
// ids and labels come from the caller; an out-of-range value is clamped so that no
// access leaves its table
__device__ __forceinline__ int clamp_id(int v, int n) { return v < 0 ? 0 : (v >= n ? n - 1 : v); }

template <typename T>
__global__ void bert_embed_kernel(const int32_t* __restrict__ ids, const int64_t* __restrict__ map,
                                  const T* __restrict__ Ew, const T* __restrict__ Ep, float* __restrict__ emb, int nb,
                                  int S, int D, int vocab) {
  const int nv = D >> 2;
  const int64_t total = (int64_t)nb * S * nv;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(i % nv);
    const int64_t t = i / nv;
    const int s = (int)(t % S);
    const int64_t bo = t / S;
    const int64_t tin = (map ? map[bo] : bo) * S + s;
    float a[4], b[4], o[4];
    load4(Ew + (int64_t)clamp_id(ids[tin], vocab) * D + 4 * c, a);
    load4(Ep + (int64_t)s * D + 4 * c, b);
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = a[e] + b[e];
    store4(emb + t * D + 4 * c, o);
  }
}
void bert_embed(int dt, const int32_t* ids, const int64_t* map, const void* Ew, const void* Ep, float* emb, int nb, int S,
                int D, int vocab, hipStream_t st) {
  const int64_t total = (int64_t)nb * S * (D / 4);
  const int blocks = (int)(cdiv64(total, 256) < 65536 ? cdiv64(total, 256) : 65536);
  if (blocks <= 0) return;
  if (dt == 0) hipLaunchKernelGGL(bert_embed_kernel<float>, dim3(blocks), dim3(256), 0, st, ids, map, (const float*)Ew, (const float*)Ep, emb, nb, S, D, vocab);
  else hipLaunchKernelGGL(bert_embed_kernel<bf16>, dim3(blocks), dim3(256), 0, st, ids, map, (const bf16*)Ew, (const bf16*)Ep, emb, nb, S, D, vocab);
}

// Token-table gradient, reproducibly: tokens are grouped by id with a counting sort whose buckets are then put
// in token order by rank (integer atomics only decide where a token waits inside its bucket, never a
// floating-point order), and one workgroup per distinct id sums that id's rows in token order.
//   ws layout (int32): count[vocab] | cursor[vocab] | offset[vocab] | bucket[ntok] | sorted[ntok] | rank[ntok]
__global__ void token_count_kernel(const int32_t* __restrict__ ids, int32_t* __restrict__ count, int ntok, int vocab) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < ntok) atomicAdd(&count[clamp_id(ids[t], vocab)], 1);
}
// offset = exclusive prefix sum of count, one workgroup: each of its 16 waves owns a contiguous range of ids,
// sums it (pass 1), and after the wave totals are known scans it 64 ids at a time (pass 2); loads go out
// eight at a time
__global__ __launch_bounds__(1024) void token_offsets_kernel(const int32_t* __restrict__ count,
                                                              int32_t* __restrict__ offset, int vocab) {
  __shared__ int32_t wsum[16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = ((vocab + 1023) / 1024) * 64;   // ids per wave, a multiple of 64
  const int lo = wave * chunk, hi = lo + chunk < vocab ? lo + chunk : vocab;
  int32_t s = 0;
  for (int v0 = lo; v0 < hi; v0 += 512) {
    int32_t c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { const int v = v0 + 64 * u + lane; c[u] = count[v < hi ? v : lo]; }
#pragma unroll
    for (int u = 0; u < 8; ++u) { const int v = v0 + 64 * u + lane; s += v < hi ? c[u] : 0; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (lane == 0) wsum[wave] = s;
  __syncthreads();
  int32_t run = 0;
  for (int w = 0; w < wave; ++w) run += wsum[w];
  for (int v0 = lo; v0 < hi; v0 += 512) {
    int32_t c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { const int v = v0 + 64 * u + lane; c[u] = count[v < hi ? v : lo]; }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int v = v0 + 64 * u + lane;
      const int32_t x = v < hi ? c[u] : 0;
      int32_t inc = x;   // inclusive scan over the wave's 64 ids
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int32_t t = __shfl_up(inc, o, 64);
        if (lane >= o) inc += t;
      }
      if (v < hi) offset[v] = run + inc - x;
      run += __shfl(inc, 63, 64);
    }
  }
}
__global__ void token_bucket_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ offset,
                                    int32_t* __restrict__ cursor, int32_t* __restrict__ bucket, int ntok, int vocab) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= ntok) return;
  const int id = clamp_id(ids[t], vocab);
  bucket[offset[id] + atomicAdd(&cursor[id], 1)] = t;
}
// rank[t] = number of smaller token indices in t's bucket; sorted[offset + rank] = t
__global__ void token_rank_kernel(const int32_t* __restrict__ ids, const int32_t* __restrict__ count,
                                  const int32_t* __restrict__ offset, const int32_t* __restrict__ bucket,
                                  int32_t* __restrict__ sorted, int32_t* __restrict__ rank, int ntok, int vocab) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= ntok) return;
  const int id = clamp_id(ids[t], vocab);
  const int n = count[id], base = offset[id];
  int r = 0;
  for (int j = 0; j < n; ++j) r += bucket[base + j] < t;
  rank[t] = r;
  sorted[base + r] = t;
}
// One workgroup per first occurrence of an id: sums the rows of its bucket in token order.
__global__ __launch_bounds__(256) void embed_scatter_kernel(const int32_t* __restrict__ ids,
                                                            const int32_t* __restrict__ count,
                                                            const int32_t* __restrict__ offset,
                                                            const int32_t* __restrict__ sorted,
                                                            const int32_t* __restrict__ rank,
                                                            const float* __restrict__ demb, float* __restrict__ dEw,
                                                            int D, int vocab) {
  const int t0 = blockIdx.x;
  if (rank[t0] != 0) return;
  const int id = clamp_id(ids[t0], vocab);
  const int n = count[id], base = offset[id];
  for (int d = threadIdx.x; d < D; d += 256) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) acc += demb[(int64_t)sorted[base + j] * D + d];
    dEw[(int64_t)id * D + d] = acc;
  }
}
__global__ void pos_sum_kernel(const float* __restrict__ demb, float* __restrict__ dEp, int nb, int S, int D) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S * D) return;
  float acc = 0.f;
  for (int b = 0; b < nb; ++b) acc += demb[(int64_t)b * S * D + i];
  dEp[i] = acc;
}
size_t bert_embed_ws_ints(int ntok, int vocab) { return (size_t)3 * ((vocab + 3) & ~3) + (size_t)3 * ((ntok + 3) & ~3); }
void bert_embed_bwd(const int32_t* ids, const float* demb, float* dEw, float* dEp, int32_t* ws, int nb, int S, int D,
                    int vocab, hipStream_t st) {
  const int ntok = nb * S;
  const size_t va = (size_t)((vocab + 3) & ~3), ta = (size_t)((ntok + 3) & ~3);   // 16-byte aligned sub-arrays
  int32_t* count = ws;
  int32_t* cursor = ws + va;
  int32_t* offset = ws + 2 * va;
  int32_t* bucket = ws + 3 * va;
  int32_t* sorted = bucket + ta;
  int32_t* rank = sorted + ta;
  fill_zero(count, 2 * va * 4, st);   // count and cursor
  const int tb = cdiv(ntok, 256);
  hipLaunchKernelGGL(token_count_kernel, dim3(tb), dim3(256), 0, st, ids, count, ntok, vocab);
  hipLaunchKernelGGL(token_offsets_kernel, dim3(1), dim3(1024), 0, st, count, offset, vocab);
  hipLaunchKernelGGL(token_bucket_kernel, dim3(tb), dim3(256), 0, st, ids, offset, cursor, bucket, ntok, vocab);
  hipLaunchKernelGGL(token_rank_kernel, dim3(tb), dim3(256), 0, st, ids, count, offset, bucket, sorted, rank, ntok, vocab);
  hipLaunchKernelGGL(embed_scatter_kernel, dim3(ntok), dim3(256), 0, st, ids, count, offset, sorted, rank, demb, dEw, D,
                     vocab);
  hipLaunchKernelGGL(pos_sum_kernel, dim3(cdiv(S * D, 256)), dim3(256), 0, st, demb, dEp, nb, S, D);
}

// ---------------------------------------------------------------------------
// losses
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void ce_rows_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels,
                                                      float* __restrict__ loss_rows, T* __restrict__ dz, int nb, int C) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  const float* zr = z + (int64_t)b * C;
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < C; c += 256) mx = fmaxf(mx, zr[c]);
  mx = block_max<4>(mx, red);
  float s = 0.f;
  for (int c = threadIdx.x; c < C; c += 256) s += expf(zr[c] - mx);
  s = block_sum<4>(s, red);
  const float lse = mx + logf(s);
  const int lab = clamp_id(labels[b], C);
  if (threadIdx.x == 0) loss_rows[b] = lse - zr[lab];
  const float inv = 1.0f / (float)nb;
  for (int c = threadIdx.x; c < C; c += 256) {
    const float p = expf(zr[c] - lse);
    dz[(int64_t)b * C + c] = from_f32<T>((p - (c == lab ? 1.f : 0.f)) * inv);
  }
}
void ce_rows(int dt, const float* z, const int32_t* labels, float* loss_rows, void* dz, int nb, int C, hipStream_t st) {
  if (dt == 0) hipLaunchKernelGGL(ce_rows_kernel<float>, dim3(nb), dim3(256), 0, st, z, labels, loss_rows, (float*)dz, nb, C);
  else hipLaunchKernelGGL(ce_rows_kernel<bf16>, dim3(nb), dim3(256), 0, st, z, labels, loss_rows, (bf16*)dz, nb, C);
}

// z[t,c] = x[t,:] . W[:,c] + b[c], one wave per token
template <typename T>
__global__ __launch_bounds__(256) void qa_logits_kernel(const T* __restrict__ x, const T* __restrict__ W,
                                                        const T* __restrict__ b, float* __restrict__ z, int rows, int D) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= rows) return;
  float s0 = 0.f, s1 = 0.f;
  for (int d = lane; d < D; d += 64) {
    const float xv = to_f32(x[(int64_t)t * D + d]);
    s0 += xv * to_f32(W[2 * d]);
    s1 += xv * to_f32(W[2 * d + 1]);
  }
  s0 = wave_sum(s0);
  s1 = wave_sum(s1);
  if (lane == 0) { z[2 * (int64_t)t] = s0 + to_f32(b[0]); z[2 * (int64_t)t + 1] = s1 + to_f32(b[1]); }
}
void qa_logits(int dt, const void* x, const void* W, const void* b, float* z, int rows, int D, hipStream_t st) {
  dim3 grid(cdiv(rows, 4));
  if (dt == 0) hipLaunchKernelGGL(qa_logits_kernel<float>, grid, dim3(256), 0, st, (const float*)x, (const float*)W, (const float*)b, z, rows, D);
  else hipLaunchKernelGGL(qa_logits_kernel<bf16>, grid, dim3(256), 0, st, (const bf16*)x, (const bf16*)W, (const bf16*)b, z, rows, D);
}

// one workgroup per sample; cross-entropy over the sequence axis for each of the two logit columns
__global__ __launch_bounds__(256) void qa_ce_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels,
                                                    float* __restrict__ loss_rows, float* __restrict__ dz, int nb, int S) {
  __shared__ float red[4];
  const int b = blockIdx.x;
  float loss = 0.f;
  for (int c = 0; c < 2; ++c) {
    const float* zc = z + (int64_t)b * S * 2 + c;
    float mx = -INFINITY;
    for (int s = threadIdx.x; s < S; s += 256) mx = fmaxf(mx, zc[2 * s]);
    mx = block_max<4>(mx, red);
    float sum = 0.f;
    for (int s = threadIdx.x; s < S; s += 256) sum += expf(zc[2 * s] - mx);
    sum = block_sum<4>(sum, red);
    const float lse = mx + logf(sum);
    const int lab = clamp_id(labels[2 * b + c], S);
    loss += 0.5f * (lse - zc[2 * lab]);
    const float sc = 0.5f / (float)nb;
    for (int s = threadIdx.x; s < S; s += 256)
      dz[((int64_t)b * S + s) * 2 + c] = (expf(zc[2 * s] - lse) - (s == lab ? 1.f : 0.f)) * sc;
  }
  if (threadIdx.x == 0) loss_rows[b] = loss;
}
void qa_ce(int dt, const float* z, const int32_t* labels, float* loss_rows, float* dz, int nb, int S, hipStream_t st) {
  (void)dt;
  hipLaunchKernelGGL(qa_ce_kernel, dim3(nb), dim3(256), 0, st, z, labels, loss_rows, dz, nb, S);
}

constexpr int kQaBlocks = 512;   // workgroups (partial rows) at most; four waves each, one row per wave at a time
size_t qa_partial_floats(int D) { return (size_t)kQaBlocks * (2 * D + 2); }

// dx = dz W^T, and per workgroup the partial sums of dW = x^T dz and db = column sums of dz.  One wave per row,
// four columns per lane and slot, the next row's loads in flight while the current one is used.
template <typename T, int VPL>
__global__ __launch_bounds__(256) void qa_head_bwd_kernel(const T* __restrict__ x, const T* __restrict__ W,
                                                          const float* __restrict__ dz, float* __restrict__ dx,
                                                          float* __restrict__ partial, int rows, int D) {
  extern __shared__ float red[];   // [2*D + 2], laid out like W and b
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nvec = D >> 2;
  float w0[VPL][4], w1[VPL][4], a0[VPL][4], a1[VPL][4];
#pragma unroll
  for (int j = 0; j < VPL; ++j) {
    const int c = lane + 64 * j;
    float t0[4] = {0.f, 0.f, 0.f, 0.f}, t1[4] = {0.f, 0.f, 0.f, 0.f};
    if (c < nvec) { load4(W + 8 * c, t0); load4(W + 8 * c + 4, t1); }   // W is [D, 2]
    w0[j][0] = t0[0]; w1[j][0] = t0[1]; w0[j][1] = t0[2]; w1[j][1] = t0[3];
    w0[j][2] = t1[0]; w1[j][2] = t1[1]; w0[j][3] = t1[2]; w1[j][3] = t1[3];
#pragma unroll
    for (int e = 0; e < 4; ++e) { a0[j][e] = 0.f; a1[j][e] = 0.f; }
  }
  struct RowIn {
    Raw4<T> x[VPL];
    float g0, g1;
  };
  auto fetch = [&](int row, RowIn& in) {
    in.g0 = dz[2 * (int64_t)row];
    in.g1 = dz[2 * (int64_t)row + 1];
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c = lane + 64 * j;
      in.x[j].zero();
      if (c < nvec) in.x[j].ld(x + (int64_t)row * D + 4 * c);
    }
  };
  float b0 = 0.f, b1 = 0.f;
  const int stride = gridDim.x * 4;
  int row = blockIdx.x * 4 + wave;
  RowIn cur, nxt;
  if (row < rows) fetch(row, cur);
  for (; row < rows; row += stride) {
    const bool more = row + stride < rows;
    if (more) fetch(row + stride, nxt);
    const float g0 = cur.g0, g1 = cur.g1;
    b0 += g0; b1 += g1;
#pragma unroll
    for (int j = 0; j < VPL; ++j) {
      const int c = lane + 64 * j;
      if (c < nvec) {
        float xv[4], o[4];
        cur.x[j].get(xv);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a0[j][e] += xv[e] * g0;
          a1[j][e] += xv[e] * g1;
          o[e] = g0 * w0[j][e] + g1 * w1[j][e];
        }
        store4(dx + (int64_t)row * D + 4 * c, o);
      }
    }
    if (more) cur = nxt;
  }
  // combine the waves of the workgroup in wave order (fixed, so reproducible)
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int j = 0; j < VPL; ++j) {
        const int c = lane + 64 * j;
        if (c < nvec) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 2 * (4 * c + e);
            red[i] = (w ? red[i] : 0.f) + a0[j][e];
            red[i + 1] = (w ? red[i + 1] : 0.f) + a1[j][e];
          }
        }
      }
      if (lane == 0) {
        red[2 * D] = (w ? red[2 * D] : 0.f) + b0;
        red[2 * D + 1] = (w ? red[2 * D + 1] : 0.f) + b1;
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < 2 * D + 2; i += 256) partial[(size_t)blockIdx.x * (2 * D + 2) + i] = red[i];
}
void qa_head_bwd(int dt, const void* x, const void* W, const float* dz, float* dx, float* dW, float* db, float* partial,
                 int rows, int D, hipStream_t st) {
  if (rows <= 0) return;
  const int nb = cdiv(rows, 4) < kQaBlocks ? cdiv(rows, 4) : kQaBlocks;
  const size_t shm = (size_t)(2 * D + 2) * sizeof(float);
#define QA_BWD(T, V)                                                                                              \
  hipLaunchKernelGGL((qa_head_bwd_kernel<T, V>), dim3(nb), dim3(256), shm, st, (const T*)x, (const T*)W, dz, dx, \
                     partial, rows, D)
#define QA_BWD_V(T)                       \
  do {                                    \
    if (D <= 768) QA_BWD(T, 3);           \
    else if (D <= 1024) QA_BWD(T, 4);     \
    else QA_BWD(T, 8);                    \
  } while (0)
  if (dt == 0) QA_BWD_V(float);
  else QA_BWD_V(bf16);
#undef QA_BWD_V
#undef QA_BWD
  hipLaunchKernelGGL(reduce_partials_kernel, dim3(cdiv(2 * D + 2, 32)), dim3(1024), 0, st, partial, nb, 2 * D + 2, dW,
                     2 * D, db, (float*)nullptr);
}

__global__ __launch_bounds__(256) void mean_reduce_kernel(const float* __restrict__ rows, int n, float* __restrict__ out) {
  __shared__ float red[4];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += rows[i];
  s = block_sum<4>(s, red);
  if (threadIdx.x == 0) out[0] = s / (float)n;
}
void mean_reduce(const float* rows, int n, float* out, hipStream_t st) {
  hipLaunchKernelGGL(mean_reduce_kernel, dim3(1), dim3(256), 0, st, rows, n, out);
}

// blockIdx.y < n: row blockIdx.y; blockIdx.y == n: the column sums
template <typename T>
__global__ __launch_bounds__(256) void add_rows_kernel(const float* __restrict__ r, float* __restrict__ x_s, T* __restrict__ x_o,
                                                       int64_t row_stride, float* __restrict__ colsum, int n, int D) {
  const int d = blockIdx.x * 256 + threadIdx.x, i = blockIdx.y;
  if (d >= D) return;
  if (i < n) {
    const float t = x_s[i * row_stride + d] + r[(int64_t)i * D + d];
    x_s[i * row_stride + d] = t;
    if (x_o) x_o[i * row_stride + d] = from_f32<T>(t);
  } else if (colsum) {
    float s = 0.f;
    for (int j0 = 0; j0 < n; j0 += 8) {   // eight loads in flight, added in row order
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = j0 + u < n ? r[(int64_t)(j0 + u) * D + d] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) s += t[u];
    }
    colsum[d] += s;
  }
}
void add_rows(int dt, const float* r, float* x_s, void* x_o, int64_t row_stride, float* colsum, int n, int D,
              hipStream_t st) {
  if (n <= 0 || D <= 0) return;
  if (dt == 0) hipLaunchKernelGGL(add_rows_kernel<float>, dim3(cdiv(D, 256), n + 1), dim3(256), 0, st, r, x_s, (float*)x_o, row_stride, colsum, n, D);
  else hipLaunchKernelGGL(add_rows_kernel<bf16>, dim3(cdiv(D, 256), n + 1), dim3(256), 0, st, r, x_s, (bf16*)x_o, row_stride, colsum, n, D);
}

// ---------------------------------------------------------------------------
// plumbing
// ---------------------------------------------------------------------------
__global__ void fill_zero_kernel(uint32_t* __restrict__ p, size_t n32) {
  const size_t nv = n32 >> 2;
  uint4* pv = reinterpret_cast<uint4*>(p);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nv; i += (size_t)gridDim.x * blockDim.x)
    pv[i] = make_uint4(0, 0, 0, 0);
  if (blockIdx.x == 0 && threadIdx.x < (n32 & 3)) p[(nv << 2) + threadIdx.x] = 0u;
}
// p must be 16-byte aligned, bytes a multiple of 4
void fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return;
  const size_t n32 = bytes / 4;
  size_t blocks = (n32 / 4 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks == 0) blocks = 1;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t*)p, n32);
}

__global__ __launch_bounds__(256) void copy_rows_kernel(uint4* __restrict__ dst, const int64_t* __restrict__ dst_idx,
                                                        const uint4* __restrict__ src,
                                                        const int64_t* __restrict__ src_idx, size_t row_vecs) {
  const int r = blockIdx.y;
  const int64_t dr = dst_idx ? dst_idx[r] : r, sr = src_idx ? src_idx[r] : r;
  uint4* d = dst + dr * row_vecs;
  const uint4* s = src + sr * row_vecs;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < row_vecs; i += (size_t)gridDim.x * 256) d[i] = s[i];
}
void copy_rows(void* dst, const int64_t* dst_idx, const void* src, const int64_t* src_idx, int nrows,
               size_t row_bytes, hipStream_t st) {
  if (nrows <= 0) return;
  const size_t rv = row_bytes / 16;
  size_t bx = (rv + 1023) / 1024;
  if (bx == 0) bx = 1;
  hipLaunchKernelGGL(copy_rows_kernel, dim3((unsigned)bx, nrows), dim3(256), 0, st, (uint4*)dst, dst_idx,
                     (const uint4*)src, src_idx, rv);
}

// several strided row copies in one launch: blockIdx.y picks the copy, blockIdx.x the row
struct RowCopyBatch {
  RowCopy d[kMaxRowCopies];
  int n;
};
__global__ __launch_bounds__(256) void strided_rows_kernel(RowCopyBatch b) {
  const RowCopy c = b.d[blockIdx.y];
  const char* s = (const char*)c.src + (int64_t)blockIdx.x * c.src_stride;
  char* d = (char*)c.dst + (int64_t)blockIdx.x * c.dst_stride;
  if (((c.row_bytes | c.src_stride | c.dst_stride | (int64_t)(uintptr_t)c.src | (int64_t)(uintptr_t)c.dst) & 3) == 0) {
    for (int i = threadIdx.x; i < c.row_bytes / 4; i += 256)
      reinterpret_cast<uint32_t*>(d)[i] = reinterpret_cast<const uint32_t*>(s)[i];
  } else {
    for (int i = threadIdx.x; i < c.row_bytes; i += 256) d[i] = s[i];
  }
}
void strided_rows_copy(const RowCopy* d, int n, int nrows, hipStream_t st) {
  if (n <= 0 || nrows <= 0) return;
  RowCopyBatch b{};
  b.n = n < kMaxRowCopies ? n : kMaxRowCopies;
  for (int i = 0; i < b.n; ++i) b.d[i] = d[i];
  hipLaunchKernelGGL(strided_rows_kernel, dim3(nrows, b.n), dim3(256), 0, st, b);
  if (n > kMaxRowCopies) strided_rows_copy(d + kMaxRowCopies, n - kMaxRowCopies, nrows, st);
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ s, bf16* __restrict__ d, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    d[i] = from_f32<bf16>(s[i]);
}
__global__ void bf16_to_f32_kernel(const bf16* __restrict__ s, float* __restrict__ d, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    d[i] = to_f32(s[i]);
}
static unsigned grid_for(size_t n) {
  size_t b = (n + 255) / 256;
  if (b > 65536) b = 65536;
  return b ? (unsigned)b : 1u;
}
void f32_to_bf16(const float* src, void* dst, size_t n, hipStream_t st) {
  if (n) hipLaunchKernelGGL(f32_to_bf16_kernel, dim3(grid_for(n)), dim3(256), 0, st, src, (bf16*)dst, n);
}
void bf16_to_f32(const void* src, float* dst, size_t n, hipStream_t st) {
  if (n) hipLaunchKernelGGL(bf16_to_f32_kernel, dim3(grid_for(n)), dim3(256), 0, st, (const bf16*)src, dst, n);
}

}  // namespace pt
