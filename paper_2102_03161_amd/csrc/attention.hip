// Multi-head softmax attention over a packed qkv tensor [nb, S, 3D]
// (columns [Q|K|V], head h = columns h*dh..(h+1)*dh-1 of each third), no mask.
//
// Generic fp32-FMA kernels for any element type, sequence length and head
// size (dh a multiple of 8, dh <= 128).  One workgroup owns a (sample, head,
// 32-row tile); keys/values stream through LDS in tiles.  The backward pass
// recomputes the probabilities from the saved row log-sum-exp and is split in
// a dq kernel (per query tile) and a dk/dv kernel (per key tile) so that no
// atomics are needed and results are reproducible.
#include <algorithm>

#include "common.h"
#include "kernels.h"

namespace pt {

constexpr int TQ = 32;   // rows owned by a workgroup
constexpr int TK = 64;   // streamed tile (forward, dq)

// ---------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const T* __restrict__ qkv, T* __restrict__ ctx,
                                                       float* __restrict__ lse, int S, int H, int dh, int Spad) {
  extern __shared__ float sm[];
  const int D = H * dh;
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * TQ;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float* Qs = sm;                      // [TQ][dh]
  float* KVs = Qs + TQ * dh;           // [TK][dh+1]
  float* P = KVs + TK * (dh + 1);      // [TQ][Spad]
  float* inv = P + TQ * Spad;          // [TQ]
  const float scale = rsqrtf((float)dh);
  const T* base = qkv + (int64_t)b * S * 3 * D + h * dh;

  for (int i = tid; i < TQ * dh; i += 256) {
    const int r = i / dh, d = i % dh;
    Qs[i] = (q0 + r < S) ? to_f32(base[(int64_t)(q0 + r) * 3 * D + d]) * scale : 0.f;
  }
  const int tq = tid >> 3, tk = tid & 7;
  for (int k0 = 0; k0 < S; k0 += TK) {
    __syncthreads();
    for (int i = tid; i < TK * dh; i += 256) {
      const int r = i / dh, d = i % dh;
      KVs[r * (dh + 1) + d] = (k0 + r < S) ? to_f32(base[(int64_t)(k0 + r) * 3 * D + D + d]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int key = tk + 8 * j;
      float s = 0.f;
      for (int d = 0; d < dh; ++d) s = fmaf(Qs[tq * dh + d], KVs[key * (dh + 1) + d], s);
      P[tq * Spad + k0 + key] = (k0 + key < S) ? s : -INFINITY;
    }
  }
  __syncthreads();
  // row softmax: each wave takes rows wave, wave+4, ...
  for (int r = wave; r < TQ; r += 4) {
    float mx = -INFINITY;
    for (int c = lane; c < Spad; c += 64) mx = fmaxf(mx, P[r * Spad + c]);
    mx = wave_max(mx);
    float sum = 0.f;
    for (int c = lane; c < Spad; c += 64) {
      const float e = __expf(P[r * Spad + c] - mx);
      P[r * Spad + c] = e;
      sum += e;
    }
    sum = wave_sum(sum);
    if (lane == 0) {
      inv[r] = 1.0f / sum;
      if (lse && q0 + r < S) lse[((int64_t)b * H + h) * S + q0 + r] = mx + __logf(sum);
    }
  }
  // context = P V
  const int nd = dh >> 3;  // outputs per thread (dh <= 128 -> at most 16)
  float acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.f;
  for (int k0 = 0; k0 < S; k0 += TK) {
    __syncthreads();
    for (int i = tid; i < TK * dh; i += 256) {
      const int r = i / dh, d = i % dh;
      KVs[r * dh + d] = (k0 + r < S) ? to_f32(base[(int64_t)(k0 + r) * 3 * D + 2 * D + d]) : 0.f;
    }
    __syncthreads();
    for (int key = 0; key < TK; ++key) {
      const float p = P[tq * Spad + k0 + key];
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (j < nd) acc[j] = fmaf(p, KVs[key * dh + tk + 8 * j], acc[j]);
    }
  }
  if (q0 + tq < S) {
    const float is = inv[tq];
    T* o = ctx + ((int64_t)b * S + q0 + tq) * D + h * dh;
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (j < nd) o[tk + 8 * j] = from_f32<T>(acc[j] * is);
  }
}

// ---------------------------------------------------------------------------
// backward, part 1: delta = rowsum(dO * O), dQ
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const T* __restrict__ qkv, const T* __restrict__ ctx,
                                                          const T* __restrict__ dctx, const float* __restrict__ lse,
                                                          T* __restrict__ dqkv, float* __restrict__ delta, int S, int H,
                                                          int dh) {
  extern __shared__ float sm[];
  const int D = H * dh;
  const int b = blockIdx.z, h = blockIdx.y, q0 = blockIdx.x * TQ;
  const int tid = threadIdx.x;
  float* Qs = sm;                       // [TQ][dh]
  float* dOs = Qs + TQ * dh;            // [TQ][dh]
  float* Ks = dOs + TQ * dh;            // [TK][dh+1]
  float* Vs = Ks + TK * (dh + 1);       // [TK][dh+1]
  float* dSs = Vs + TK * (dh + 1);      // [TQ][TK]
  float* dl = dSs + TQ * TK;            // [TQ] delta
  float* ls = dl + TQ;                  // [TQ] lse
  const float scale = rsqrtf((float)dh);
  const T* base = qkv + (int64_t)b * S * 3 * D + h * dh;

  for (int i = tid; i < TQ * dh; i += 256) {
    const int r = i / dh, d = i % dh;
    const bool ok = q0 + r < S;
    Qs[i] = ok ? to_f32(base[(int64_t)(q0 + r) * 3 * D + d]) : 0.f;
    dOs[i] = ok ? to_f32(dctx[((int64_t)b * S + q0 + r) * D + h * dh + d]) : 0.f;
  }
  __syncthreads();
  if (tid < TQ) {
    float s = 0.f;
    if (q0 + tid < S) {
      const T* o = ctx + ((int64_t)b * S + q0 + tid) * D + h * dh;
      for (int d = 0; d < dh; ++d) s = fmaf(dOs[tid * dh + d], to_f32(o[d]), s);
      delta[((int64_t)b * H + h) * S + q0 + tid] = s;
      ls[tid] = lse[((int64_t)b * H + h) * S + q0 + tid];
    } else {
      ls[tid] = 0.f;
    }
    dl[tid] = s;
  }
  const int tq = tid >> 3, tk = tid & 7;
  const int nd = dh >> 3;
  float acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.f;
  for (int k0 = 0; k0 < S; k0 += TK) {
    __syncthreads();
    for (int i = tid; i < TK * dh; i += 256) {
      const int r = i / dh, d = i % dh;
      const bool ok = k0 + r < S;
      Ks[r * (dh + 1) + d] = ok ? to_f32(base[(int64_t)(k0 + r) * 3 * D + D + d]) : 0.f;
      Vs[r * (dh + 1) + d] = ok ? to_f32(base[(int64_t)(k0 + r) * 3 * D + 2 * D + d]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int key = tk + 8 * j;
      float s = 0.f, dp = 0.f;
      for (int d = 0; d < dh; ++d) {
        s = fmaf(Qs[tq * dh + d], Ks[key * (dh + 1) + d], s);
        dp = fmaf(dOs[tq * dh + d], Vs[key * (dh + 1) + d], dp);
      }
      const float p = (k0 + key < S) ? __expf(s * scale - ls[tq]) : 0.f;
      dSs[tq * TK + key] = p * (dp - dl[tq]);
    }
    __syncthreads();
    for (int key = 0; key < TK; ++key) {
      const float ds = dSs[tq * TK + key];
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (j < nd) acc[j] = fmaf(ds, Ks[key * (dh + 1) + tk + 8 * j], acc[j]);
    }
  }
  if (q0 + tq < S) {
    T* o = dqkv + ((int64_t)b * S + q0 + tq) * 3 * D + h * dh;
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (j < nd) o[tk + 8 * j] = from_f32<T>(acc[j] * scale);
  }
}

// ---------------------------------------------------------------------------
// backward, part 2: dK, dV for a tile of TQ keys, streaming query tiles of TQ
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const T* __restrict__ qkv, const T* __restrict__ dctx,
                                                           const float* __restrict__ lse,
                                                           const float* __restrict__ delta, T* __restrict__ dqkv, int S,
                                                           int H, int dh) {
  extern __shared__ float sm[];
  const int D = H * dh;
  const int b = blockIdx.z, h = blockIdx.y, k0 = blockIdx.x * TQ;
  const int tid = threadIdx.x;
  const int ldk = dh + 1;
  float* Ks = sm;                  // [TQ][dh+1]
  float* Vs = Ks + TQ * ldk;       // [TQ][dh+1]
  float* Qs = Vs + TQ * ldk;       // [TQ][dh+1]
  float* dOs = Qs + TQ * ldk;      // [TQ][dh+1]
  float* Ps = dOs + TQ * ldk;      // [TQ(query)][TQ(key)]
  float* dSs = Ps + TQ * TQ;       // [TQ][TQ]
  float* ls = dSs + TQ * TQ;       // [TQ]
  float* dl = ls + TQ;             // [TQ]
  const float scale = rsqrtf((float)dh);
  const T* base = qkv + (int64_t)b * S * 3 * D + h * dh;

  for (int i = tid; i < TQ * dh; i += 256) {
    const int r = i / dh, d = i % dh;
    const bool ok = k0 + r < S;
    Ks[r * ldk + d] = ok ? to_f32(base[(int64_t)(k0 + r) * 3 * D + D + d]) : 0.f;
    Vs[r * ldk + d] = ok ? to_f32(base[(int64_t)(k0 + r) * 3 * D + 2 * D + d]) : 0.f;
  }
  const int tr = tid >> 3, tc = tid & 7;   // (row, 1/8 of the columns)
  const int nd = dh >> 3;
  float ak[16], av[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) { ak[j] = 0.f; av[j] = 0.f; }
  for (int q0 = 0; q0 < S; q0 += TQ) {
    __syncthreads();
    for (int i = tid; i < TQ * dh; i += 256) {
      const int r = i / dh, d = i % dh;
      const bool ok = q0 + r < S;
      Qs[r * ldk + d] = ok ? to_f32(base[(int64_t)(q0 + r) * 3 * D + d]) : 0.f;
      dOs[r * ldk + d] = ok ? to_f32(dctx[((int64_t)b * S + q0 + r) * D + h * dh + d]) : 0.f;
    }
    if (tid < TQ) {
      const bool ok = q0 + tid < S;
      ls[tid] = ok ? lse[((int64_t)b * H + h) * S + q0 + tid] : 0.f;
      dl[tid] = ok ? delta[((int64_t)b * H + h) * S + q0 + tid] : 0.f;
    }
    __syncthreads();
    // thread (query tr, keys tc + 8j), 4 pairs
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int key = tc + 8 * j;
      float s = 0.f, dp = 0.f;
      for (int d = 0; d < dh; ++d) {
        s = fmaf(Qs[tr * ldk + d], Ks[key * ldk + d], s);
        dp = fmaf(dOs[tr * ldk + d], Vs[key * ldk + d], dp);
      }
      const float p = (q0 + tr < S && k0 + key < S) ? __expf(s * scale - ls[tr]) : 0.f;
      Ps[tr * TQ + key] = p;
      dSs[tr * TQ + key] = p * (dp - dl[tr]);
    }
    __syncthreads();
    // thread (key tr, columns tc + 8j)
    for (int i = 0; i < TQ; ++i) {
      const float p = Ps[i * TQ + tr], ds = dSs[i * TQ + tr];
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (j < nd) {
          av[j] = fmaf(p, dOs[i * ldk + tc + 8 * j], av[j]);
          ak[j] = fmaf(ds, Qs[i * ldk + tc + 8 * j], ak[j]);
        }
    }
  }
  if (k0 + tr < S) {
    T* o = dqkv + ((int64_t)b * S + k0 + tr) * 3 * D + h * dh;
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (j < nd) {
        o[D + tc + 8 * j] = from_f32<T>(ak[j] * scale);
        o[2 * D + tc + 8 * j] = from_f32<T>(av[j]);
      }
  }
}

// ---------------------------------------------------------------------------
template <typename T>
static void attention_fwd_t(const void* qkv, void* ctx, float* lse, int nb, int S, int H, int dh, hipStream_t st) {
  const int Spad = cdiv(S, TK) * TK;
  const size_t shm = sizeof(float) * ((size_t)TQ * dh + (size_t)TK * (dh + 1) + (size_t)TQ * Spad + TQ);
  static size_t configured = 0;
  if (shm > 65536 && shm > configured) {
    // a refusal stays behind as the runtime's last error, which the calling entry point reports; nothing is launched
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<T>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)shm) != hipSuccess) return;
    configured = shm;
  }
  hipLaunchKernelGGL(attn_fwd_kernel<T>, dim3(cdiv(S, TQ), H, nb), dim3(256), shm, st, (const T*)qkv, (T*)ctx, lse, S, H,
                     dh, Spad);
}
// 8 consecutive elements as floats / from floats (16-byte accesses for bf16)
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16* p, float (&v)[8]) {
  union { uint4 u; bf16 h[8]; } t;
  t.u = *reinterpret_cast<const uint4*>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = to_f32(t.h[i]);
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
  union { uint4 u; bf16 h[8]; } t;
#pragma unroll
  for (int i = 0; i < 8; ++i) t.h[i] = from_f32<bf16>(v[i]);
  *reinterpret_cast<uint4*>(p) = t.u;
}
// ---------------------------------------------------------------------------
// forward for each sample's first query only (the top block under a first-token head: no other row of its
// output is read).  One workgroup per (sample, head): s_t = scale q.k_t, p = softmax(s), o = sum_t p_t v_t.
// ctx_rows is dense: [nb, D]; the log-sum-exp goes to entry (b, h, 0) of the [nb, H, S] array the backward
// kernels read.  dh / 8 lanes share a key (whole rows are read); partial sums over keys are combined in
// a fixed order.
// ---------------------------------------------------------------------------
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void attn_fwd_first_query_kernel(const T* __restrict__ qkv, T* __restrict__ ctx_rows,
                                                                   float* __restrict__ lse, int S, int H, int dh) {
  extern __shared__ float sm[];
  float* qs = sm;            // [dh]
  float* sc = qs + dh;       // [S] scores, then unnormalised probabilities
  float* part = sc + S;      // [256 / (dh / 8)][dh] partial outputs of the key groups (VEC)
  __shared__ float red[4];
  const int D = H * dh;
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
  const T* base = qkv + (int64_t)b * S * 3 * D + h * dh;
  const float scale = rsqrtf((float)dh);
  for (int d = tid; d < dh; d += 256) qs[d] = to_f32(base[d]);
  __syncthreads();
  const int lpr = VEC ? dh >> 3 : 1, j = tid % lpr, d0 = 8 * j, kpi = 256 / lpr;   // keys per iteration
  if (VEC) {
    for (int t0 = 0; t0 < S; t0 += kpi) {
      const int t = t0 + tid / lpr;
      const bool ok = t < S;
      float kv[8];
      load8(base + (int64_t)(ok ? t : 0) * 3 * D + D + d0, kv);
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) s = fmaf(qs[d0 + i], kv[i], s);
      for (int o = 1; o < lpr; o <<= 1) s += __shfl_xor(s, o, 64);
      if (ok && j == 0) sc[t] = s * scale;
    }
  } else {
    for (int t = tid; t < S; t += 256) {
      const T* kr = base + (int64_t)t * 3 * D + D;
      float s = 0.f;
      for (int d = 0; d < dh; ++d) s = fmaf(qs[d], to_f32(kr[d]), s);
      sc[t] = s * scale;
    }
  }
  __syncthreads();
  float lm = -INFINITY;
  for (int t = tid; t < S; t += 256) lm = fmaxf(lm, sc[t]);
  const float m = block_max<4>(lm, red);
  float ls = 0.f;
  for (int t = tid; t < S; t += 256) {
    const float p = __expf(sc[t] - m);
    sc[t] = p;
    ls += p;
  }
  const float l = block_sum<4>(ls, red);   // its barriers also publish sc
  const float inv = 1.0f / l;
  T* o = ctx_rows + (int64_t)b * D + h * dh;
  if (VEC) {
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int t0 = 0; t0 < S; t0 += kpi) {
      const int t = t0 + tid / lpr;
      if (t < S) {
        float vv[8];
        load8(base + (int64_t)t * 3 * D + 2 * D + d0, vv);
        const float p = sc[t];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(p, vv[i], acc[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) part[(tid / lpr) * dh + d0 + i] = acc[i];
    __syncthreads();
    for (int d = tid; d < dh; d += 256) {
      float a = 0.f;
      for (int g = 0; g < kpi; ++g) a += part[g * dh + d];
      o[d] = from_f32<T>(a * inv);
    }
  } else {
    for (int d = tid; d < dh; d += 256) {
      float a = 0.f;
      for (int t = 0; t < S; ++t) a = fmaf(sc[t], to_f32(base[(int64_t)t * 3 * D + 2 * D + d]), a);
      o[d] = from_f32<T>(a * inv);
    }
  }
  if (tid == 0 && lse) lse[((int64_t)b * H + h) * S] = m + __logf(l);
}
void attention_fwd_first_query(int dt, const void* qkv, void* ctx_rows, float* lse, int nb, int S, int H, int dh,
                               hipStream_t st) {
  if (nb <= 0) return;
  const bool vec = dh % 8 == 0 && 64 % (dh / 8) == 0 &&
                   (reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(ctx_rows)) % 16 == 0;
  const size_t shm = sizeof(float) * ((size_t)dh + S + (vec ? (size_t)(256 / (dh / 8)) * dh : 0));
#define PT_FQF(T, V)                                                                                                 \
  hipLaunchKernelGGL((attn_fwd_first_query_kernel<T, V>), dim3(H, nb), dim3(256), shm, st, (const T*)qkv, (T*)ctx_rows, \
                     lse, S, H, dh)
  if (dt == 0) { if (vec) PT_FQF(float, true); else PT_FQF(float, false); }
  else { if (vec) PT_FQF(bf16, true); else PT_FQF(bf16, false); }
#undef PT_FQF
}

// ---------------------------------------------------------------------------
// backward when only each sample's first query has a non-zero output gradient (the top block under a
// first-token head).  One workgroup per (sample, head): p_t = exp(q.k_t * scale - lse), dV_t = p_t dO,
// dS_t = p_t (dO.v_t - dO.o), dK_t = scale dS_t q, dQ_0 = scale sum_t dS_t k_t, dQ_t = 0 otherwise.
// ctx_rows and do_rows are dense: [nb, D], the first tokens' rows only.  One thread per key; the sum over
// keys for dQ_0 is taken by dh threads in key order (fixed, so reproducible).
// ---------------------------------------------------------------------------
// VEC: dh is a multiple of 8, so every head slice of a row starts on a 16-byte boundary and is moved in
// 8-element pieces
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void attn_bwd_first_query_kernel(const T* __restrict__ qkv, const T* __restrict__ ctx_rows,
                                                                   const T* __restrict__ do_rows,
                                                                   const float* __restrict__ lse, T* __restrict__ dqkv,
                                                                   int S, int H, int dh) {
  extern __shared__ float sm[];
  float* qs = sm;            // [dh]
  float* dos = qs + dh;      // [dh]
  float* dss = dos + dh;     // [S]
  __shared__ float delta_s;
  const int D = H * dh;
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
  const T* base = qkv + (int64_t)b * S * 3 * D + h * dh;
  T* obase = dqkv + (int64_t)b * S * 3 * D + h * dh;
  const float scale = rsqrtf((float)dh);
  for (int d = tid; d < dh; d += 256) {
    qs[d] = to_f32(base[d]);
    dos[d] = to_f32(do_rows[(int64_t)b * D + h * dh + d]);
  }
  __syncthreads();
  if (tid == 0) {
    const T* o = ctx_rows + (int64_t)b * D + h * dh;
    float s = 0.f;
    for (int d = 0; d < dh; ++d) s = fmaf(dos[d], to_f32(o[d]), s);
    delta_s = s;
  }
  __syncthreads();
  const float l0 = lse[((int64_t)b * H + h) * S], dl = delta_s;
  float dqa_out[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (VEC) {
    // dh / 8 lanes share a key: each moves one 16-byte piece of the key's rows, so a wave reads and writes
    // whole rows; the two dot products are finished with lane exchanges inside the group
    const int lpr = dh >> 3, j = tid % lpr, d0 = 8 * j, kpp = 256 / lpr;   // kpp keys per pass
    float dqa[8];   // this thread's share of dQ of the first token: sum over its keys of dS k
#pragma unroll
    for (int i = 0; i < 8; ++i) dqa[i] = 0.f;
    for (int t0 = 0; t0 < S; t0 += 4 * kpp) {   // four passes' rows in flight together
      float kv[4][8], vv[4][8];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = t0 + u * kpp + tid / lpr;
        const T* kr = base + (int64_t)(t < S ? t : 0) * 3 * D + D;
        load8(kr + d0, kv[u]);
        load8(kr + D + d0, vv[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = t0 + u * kpp + tid / lpr;
        float sc = 0.f, dp = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) { sc = fmaf(qs[d0 + i], kv[u][i], sc); dp = fmaf(dos[d0 + i], vv[u][i], dp); }
        for (int o = 1; o < lpr; o <<= 1) { sc += __shfl_xor(sc, o, 64); dp += __shfl_xor(dp, o, 64); }
        if (t < S) {
          const float pt = __expf(sc * scale - l0);
          const float ds = pt * (dp - dl);
          T* dq = obase + (int64_t)t * 3 * D;
          const float dsk = ds * scale;
          float z[8], a[8], c2[8];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            z[i] = 0.f; a[i] = dsk * qs[d0 + i]; c2[i] = pt * dos[d0 + i];
            dqa[i] = fmaf(ds, kv[u][i], dqa[i]);
          }
          if (t > 0) store8(dq + d0, z);
          store8(dq + D + d0, a);
          store8(dq + 2 * D + d0, c2);
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) dqa_out[i] = dqa[i];
  } else {
    for (int t = tid; t < S; t += 256) {
      const T* kr = base + (int64_t)t * 3 * D + D;
      const T* vr = kr + D;
      float sc = 0.f, dp = 0.f;
      for (int d = 0; d < dh; ++d) { sc = fmaf(qs[d], to_f32(kr[d]), sc); dp = fmaf(dos[d], to_f32(vr[d]), dp); }
      const float pt = __expf(sc * scale - l0);
      const float ds = pt * (dp - dl);
      dss[t] = ds;
      T* dq = obase + (int64_t)t * 3 * D;
      T* dk = dq + D;
      T* dv = dk + D;
      const float dsk = ds * scale;
      for (int d = 0; d < dh; ++d) {
        if (t > 0) dq[d] = from_f32<T>(0.f);
        dk[d] = from_f32<T>(dsk * qs[d]);
        dv[d] = from_f32<T>(pt * dos[d]);
      }
    }
  }
  if (VEC) {
    // dQ of the first token: the threads' partial sums, combined in a fixed order (thread = pass slot * lpr + j)
    __shared__ float dqp[256 * 8];
    const int lpr = dh >> 3, kpp = 256 / lpr;
#pragma unroll
    for (int i = 0; i < 8; ++i) dqp[tid * 8 + i] = dqa_out[i];
    __syncthreads();
    for (int d = tid; d < dh; d += 256) {
      float acc = 0.f;
      for (int g = 0; g < kpp; ++g) acc += dqp[(g * lpr + (d >> 3)) * 8 + (d & 7)];
      obase[d] = from_f32<T>(acc * scale);
    }
    return;
  }
  __syncthreads();
  for (int d = tid; d < dh; d += 256) {
    float acc = 0.f;
    for (int t = 0; t < S; ++t) acc = fmaf(dss[t], to_f32(base[(int64_t)t * 3 * D + D + d]), acc);
    obase[d] = from_f32<T>(acc * scale);
  }
}
void attention_bwd_first_query(int dt, const void* qkv, const void* ctx_rows, const void* do_rows, const float* lse,
                               void* dqkv, int nb, int S, int H, int dh, hipStream_t st) {
  if (nb <= 0) return;
  const size_t shm = sizeof(float) * ((size_t)2 * dh + S);
  // the vector form needs 8 | dh, dh / 8 lanes per key dividing the wave, and 16-byte aligned tensors
  const bool vec = dh % 8 == 0 && 64 % (dh / 8) == 0 && (reinterpret_cast<uintptr_t>(qkv) | reinterpret_cast<uintptr_t>(dqkv)) % 16 == 0;
#define PT_FQ(T, V)                                                                                                   \
  hipLaunchKernelGGL((attn_bwd_first_query_kernel<T, V>), dim3(H, nb), dim3(256), shm, st, (const T*)qkv, (const T*)ctx_rows, \
                     (const T*)do_rows, lse, (T*)dqkv, S, H, dh)
  if (dt == 0) { if (vec) PT_FQ(float, true); else PT_FQ(float, false); }
  else { if (vec) PT_FQ(bf16, true); else PT_FQ(bf16, false); }
#undef PT_FQ
}

// matrix-core kernels for bf16, head size 64 (attention_mfma.hip)
void attention_fwd_mfma(const void* qkv, void* ctx, float* lse, int nb, int S, int H, hipStream_t st);
void attention_bwd_mfma(const void* qkv, const void* ctx, const void* dctx, const float* lse, void* dqkv, float* delta,
                        int nb, int S, int H, hipStream_t st);

size_t attention_generic_lds_bytes(int S, int dh) {
  const size_t Spad = (size_t)cdiv(S, TK) * TK;
  const size_t fwd = sizeof(float) * ((size_t)TQ * dh + (size_t)TK * (dh + 1) + (size_t)TQ * Spad + TQ);
  const size_t dq = sizeof(float) * ((size_t)2 * TQ * dh + (size_t)2 * TK * (dh + 1) + (size_t)TQ * TK + 2 * TQ);
  const size_t dkv = sizeof(float) * ((size_t)4 * TQ * (dh + 1) + (size_t)2 * TQ * TQ + 2 * TQ);
  return std::max(std::max(fwd, dq), dkv);
}
size_t attention_first_query_lds_bytes(int S, int dh) {
  const size_t fwd = sizeof(float) * ((size_t)dh + S + (dh % 8 == 0 ? (size_t)(256 / (dh / 8)) * dh : 0));
  const size_t bwd = sizeof(float) * ((size_t)2 * dh + S);
  return std::max(fwd, bwd);
}
bool attention_uses_mfma(int dt, int dh) { return dt == 1 && dh == 64; }

void attention_fwd(int dt, const void* qkv, void* ctx, float* lse, int nb, int S, int H, int dh, hipStream_t st) {
  if (nb <= 0) return;
  if (dt == 1 && dh == 64) { attention_fwd_mfma(qkv, ctx, lse, nb, S, H, st); return; }
  if (dt == 0) attention_fwd_t<float>(qkv, ctx, lse, nb, S, H, dh, st);
  else attention_fwd_t<bf16>(qkv, ctx, lse, nb, S, H, dh, st);
}

template <typename T>
static void attention_bwd_t(const void* qkv, const void* ctx, const void* dctx, const float* lse, void* dqkv,
                            float* delta, int nb, int S, int H, int dh, hipStream_t st) {
  const size_t shm1 = sizeof(float) * ((size_t)2 * TQ * dh + (size_t)2 * TK * (dh + 1) + (size_t)TQ * TK + 2 * TQ);
  const size_t shm2 = sizeof(float) * ((size_t)4 * TQ * (dh + 1) + (size_t)2 * TQ * TQ + 2 * TQ);
  static size_t configured = 0;
  if (shm1 > 65536 && shm1 > configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dq_kernel<T>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm1) != hipSuccess) return;
    configured = shm1;
  }
  dim3 grid(cdiv(S, TQ), H, nb);
  hipLaunchKernelGGL(attn_bwd_dq_kernel<T>, grid, dim3(256), shm1, st, (const T*)qkv, (const T*)ctx, (const T*)dctx, lse,
                     (T*)dqkv, delta, S, H, dh);
  hipLaunchKernelGGL(attn_bwd_dkv_kernel<T>, grid, dim3(256), shm2, st, (const T*)qkv, (const T*)dctx, lse, delta,
                     (T*)dqkv, S, H, dh);
}
void attention_bwd(int dt, const void* qkv, const void* ctx, const void* dctx, const float* lse, void* dqkv,
                   float* delta_ws, int nb, int S, int H, int dh, hipStream_t st) {
  if (nb <= 0) return;
  if (dt == 1 && dh == 64) { attention_bwd_mfma(qkv, ctx, dctx, lse, dqkv, delta_ws, nb, S, H, st); return; }
  if (dt == 0) attention_bwd_t<float>(qkv, ctx, dctx, lse, dqkv, delta_ws, nb, S, H, dh, st);
  else attention_bwd_t<bf16>(qkv, ctx, dctx, lse, dqkv, delta_ws, nb, S, H, dh, st);
}

}  // namespace pt
