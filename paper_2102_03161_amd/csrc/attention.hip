// Multi-head softmax attention over a packed qkv tensor [nb, S, 3D]
// (columns [Q|K|V], head h = columns h*dh..(h+1)*dh-1 of each third), no mask.
//
// Generic fp32-FMA kernels for any element type, sequence length and head
// size (dh a multiple of 8, dh <= 128).  One workgroup owns a (sample, head,
// 32-row tile); keys/values stream through LDS in tiles.  The backward pass
// recomputes the probabilities from the saved row log-sum-exp and is split in
// a dq kernel (per query tile) and a dk/dv kernel (per key tile) so that no
// atomics are needed and results are reproducible.
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
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_kernel<T>), hipFuncAttributeMaxDynamicSharedMemorySize,
                        (int)shm);
    configured = shm;
  }
  hipLaunchKernelGGL(attn_fwd_kernel<T>, dim3(cdiv(S, TQ), H, nb), dim3(256), shm, st, (const T*)qkv, (T*)ctx, lse, S, H,
                     dh, Spad);
}
// matrix-core kernels for bf16, head size 64 (attention_mfma.hip)
void attention_fwd_mfma(const void* qkv, void* ctx, float* lse, int nb, int S, int H, hipStream_t st);
void attention_bwd_mfma(const void* qkv, const void* ctx, const void* dctx, const float* lse, void* dqkv, float* delta,
                        int nb, int S, int H, hipStream_t st);

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
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_dq_kernel<T>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm1);
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
