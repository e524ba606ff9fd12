// Per-layer gradient norms (Eq. 1's ||g_l||) and the fused optimizers.
//
// All parameter tensors live in one arena, each padded to a multiple of
// kChunk floats, ordered front end, block 0 .. L-1, head.  A layer is therefore
// a contiguous chunk range and the active set [block k .. head] a contiguous
// suffix, so both passes are single launches that stream the arena once with
// 16-byte accesses.  Padding is zero in every arena and stays zero under both
// update rules.
#include <mutex>

#include "common.h"
#include "kernels.h"

namespace pt {

// The arenas these kernels stream (gradients, master weights, moments) are far larger than the caches and are
// touched once per step: their loads and stores go past the caches (AdamW 5.7 -> 6.7 TB/s).
typedef float f32x4_nt __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld_nt4(const float* p) {
  const f32x4_nt t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_nt*>(p));
  return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void st_nt4(float* p, const float4& v) {
  f32x4_nt t; t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  __builtin_nontemporal_store(t, reinterpret_cast<f32x4_nt*>(p));
}

// sum of the squares of a chunk's 1024 gradient values, 4 per thread, in a fixed order (the norm pass and the
// updates that take the norms along share it, so both give the same bits)
__device__ __forceinline__ void chunk_sumsq(const float4& v, float* red, float* __restrict__ chunk_sq, int64_t c) {
  float s = (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
  s = block_sum<4>(s, red);
  if (threadIdx.x == 0) chunk_sq[c] = s;
}

__global__ __launch_bounds__(256) void sumsq_kernel(const float* __restrict__ g, float* __restrict__ chunk_sq,
                                                    int64_t first_chunk) {
  __shared__ float red[4];
  const int64_t c = first_chunk + blockIdx.x;
  // cached loads: what stays of the gradient in the last-level cache is read again by the update
  const float4 v = reinterpret_cast<const float4*>(g + c * kChunk)[threadIdx.x];
  chunk_sumsq(v, red, chunk_sq, c);
}
void sumsq_chunks(const float* g, float* chunk_sq, int64_t first_chunk, int64_t n_chunks, hipStream_t st) {
  if (n_chunks <= 0) return;
  hipLaunchKernelGGL(sumsq_kernel, dim3((unsigned)n_chunks), dim3(256), 0, st, g, chunk_sq, first_chunk);
}

// one workgroup per layer: fp64 sum of its chunk partials in a fixed order
constexpr int kFinThreads = 1024;   // one workgroup per group; the front end of BERT spans 23k chunks
__global__ __launch_bounds__(kFinThreads) void finalize_norms_kernel(const float* __restrict__ chunk_sq,
                                                             const int64_t* __restrict__ group_first, int G,
                                                             int first_active, int front_active,
                                                             float* __restrict__ norms) {
  __shared__ double red[kFinThreads];
  const int grp = blockIdx.x;
  const bool active = (grp == 0) ? (front_active != 0) : (grp >= first_active);
  if (!active) {
    if (threadIdx.x == 0) norms[grp] = 0.f;
    return;
  }
  const int64_t lo = group_first[grp], hi = group_first[grp + 1];
  double s = 0.0;
  for (int64_t c0 = lo + threadIdx.x; c0 < hi; c0 += 8 * kFinThreads) {   // eight loads in flight, added in chunk order
    float t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = c0 + u * kFinThreads < hi ? chunk_sq[c0 + u * kFinThreads] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) s += (double)t[u];
  }
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = kFinThreads / 2; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) norms[grp] = (float)sqrt(red[0]);
}
void finalize_norms(const float* chunk_sq, const int64_t* group_first_chunk, int G, int first_active, int front_active,
                    float* norms, hipStream_t st) {
  hipLaunchKernelGGL(finalize_norms_kernel, dim3(G), dim3(kFinThreads), 0, st, chunk_sq, group_first_chunk, G, first_active,
                     front_active, norms);
}

// ---- per-chunk sums for callers that may not allocate ----------------------------------------------------
// pt_layer_grad_norms_static keeps its per-chunk partial sums here instead of in the caller's work arena.
// Every GPU the library runs on holds its own copy of this array (2 MB) at its own address until the process
// ends; host code may only use the address hipGetSymbolAddress reports for the current device, never the
// array's name.  All calls on one GPU share the array, so calls that overlap on one GPU race.
constexpr int64_t kStaticChunks = 512 * 1024;   // 2^19 chunks of 1024 values: models up to 536 870 912 padded parameters
static __device__ __align__(256) float scratch[kStaticChunks];

constexpr int kMaxDevices = 64;
static float* g_scratch_ptr[kMaxDevices] = {};
static bool g_scratch_known[kMaxDevices] = {};

int64_t static_chunk_capacity() { return kStaticChunks; }

hipError_t static_chunk_sums(float** out) {
  static std::mutex mu;
  std::lock_guard<std::mutex> lock(mu);
  *out = nullptr;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  if (!g_scratch_known[dev]) {
    float* ptr = nullptr;
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
    g_scratch_known[dev] = true;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

__device__ __forceinline__ void store_shadow4(bf16* p, float a, float b, float c, float d) {
  union { bf16 h[4]; uint2 u; } t;
  t.h[0] = from_f32<bf16>(a); t.h[1] = from_f32<bf16>(b); t.h[2] = from_f32<bf16>(c); t.h[3] = from_f32<bf16>(d);
  *reinterpret_cast<uint2*>(p) = t.u;
}

// SQ: also leave the chunk's sum of squared gradients in chunk_sq (the norm pass folded into the update, which
// reads the gradient anyway)
template <bool SQ>
__global__ __launch_bounds__(256) void adamw_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                    float* __restrict__ m, float* __restrict__ v,
                                                    bf16* __restrict__ shadow, const uint8_t* __restrict__ chunk_decay,
                                                    int64_t first_chunk, OptArgs a, float* __restrict__ chunk_sq) {
  __shared__ float red[4];
  // last chunk first: the norm pass went through the gradient front to back, so its tail is what the
  // last-level cache still holds
  const int64_t c = first_chunk + (gridDim.x - 1 - blockIdx.x);
  const int64_t i = c * kChunk + 4 * threadIdx.x;
  const float shrink = chunk_decay[c] ? (1.0f - a.lr * a.weight_decay) : 1.0f;
  float4 wv = ld_nt4(w + i);
  const float4 gv = ld_nt4(g + i);
  float4 mv = ld_nt4(m + i);
  float4 vv = ld_nt4(v + i);
  if (SQ) chunk_sumsq(gv, red, chunk_sq, c);
  float* wp = &wv.x; const float* gp = &gv.x; float* mp = &mv.x; float* vp = &vv.x;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float gg = gp[e];
    const float mm = a.beta1 * mp[e] + (1.0f - a.beta1) * gg;
    const float v2 = a.beta2 * vp[e] + (1.0f - a.beta2) * gg * gg;
    mp[e] = mm;
    vp[e] = v2;
    wp[e] = wp[e] * shrink - a.lr * (mm / a.bias_c1) / (sqrtf(v2 / a.bias_c2) + a.eps);
  }
  st_nt4(w + i, wv);
  st_nt4(m + i, mv);
  st_nt4(v + i, vv);
  if (shadow) store_shadow4(shadow + i, wv.x, wv.y, wv.z, wv.w);
}
void adamw_chunks(float* w, const float* g, float* m, float* v, void* shadow, const uint8_t* chunk_decay,
                  int64_t first_chunk, int64_t n_chunks, OptArgs a, float* chunk_sq, hipStream_t st) {
  if (n_chunks <= 0) return;
  if (chunk_sq)
    hipLaunchKernelGGL(adamw_kernel<true>, dim3((unsigned)n_chunks), dim3(256), 0, st, w, g, m, v, (bf16*)shadow,
                       chunk_decay, first_chunk, a, chunk_sq);
  else
    hipLaunchKernelGGL(adamw_kernel<false>, dim3((unsigned)n_chunks), dim3(256), 0, st, w, g, m, v, (bf16*)shadow,
                       chunk_decay, first_chunk, a, chunk_sq);
}

template <bool SQ>
__global__ __launch_bounds__(256) void sgdm_kernel(float* __restrict__ w, const float* __restrict__ g,
                                                   float* __restrict__ m, bf16* __restrict__ shadow,
                                                   const uint8_t* __restrict__ chunk_decay, int64_t first_chunk,
                                                   OptArgs a, float* __restrict__ chunk_sq) {
  __shared__ float red[4];
  // last chunk first: the norm pass went through the gradient front to back, so its tail is what the
  // last-level cache still holds
  const int64_t c = first_chunk + (gridDim.x - 1 - blockIdx.x);
  const int64_t i = c * kChunk + 4 * threadIdx.x;
  const float wd = chunk_decay[c] ? a.weight_decay : 0.0f;
  float4 wv = ld_nt4(w + i);
  const float4 gv = ld_nt4(g + i);
  float4 mv = ld_nt4(m + i);
  if (SQ) chunk_sumsq(gv, red, chunk_sq, c);
  float* wp = &wv.x; const float* gp = &gv.x; float* mp = &mv.x;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float gg = gp[e] + wd * wp[e];
    const float mm = a.momentum * mp[e] + gg;
    mp[e] = mm;
    wp[e] = wp[e] - a.lr * mm;
  }
  st_nt4(w + i, wv);
  st_nt4(m + i, mv);
  if (shadow) store_shadow4(shadow + i, wv.x, wv.y, wv.z, wv.w);
}
void sgdm_chunks(float* w, const float* g, float* m, void* shadow, const uint8_t* chunk_decay, int64_t first_chunk,
                 int64_t n_chunks, OptArgs a, float* chunk_sq, hipStream_t st) {
  if (n_chunks <= 0) return;
  if (chunk_sq)
    hipLaunchKernelGGL(sgdm_kernel<true>, dim3((unsigned)n_chunks), dim3(256), 0, st, w, g, m, (bf16*)shadow, chunk_decay,
                       first_chunk, a, chunk_sq);
  else
    hipLaunchKernelGGL(sgdm_kernel<false>, dim3((unsigned)n_chunks), dim3(256), 0, st, w, g, m, (bf16*)shadow, chunk_decay,
                       first_chunk, a, chunk_sq);
}

// acc = (first ? 0 : acc) + weight * g over whole chunks; lane 0 of workgroup 0 folds the loss the same way
__global__ __launch_bounds__(256) void grad_accumulate_kernel(float* __restrict__ acc, const float* __restrict__ g,
                                                              int64_t first_chunk, float weight, int first,
                                                              const float* __restrict__ loss, float* __restrict__ loss_acc) {
  const int64_t i = (first_chunk + blockIdx.x) * kChunk + 4 * threadIdx.x;
  const float4 gv = ld_nt4(g + i);
  float4 av = make_float4(0.f, 0.f, 0.f, 0.f);
  if (!first) av = ld_nt4(acc + i);
  av.x += weight * gv.x; av.y += weight * gv.y; av.z += weight * gv.z; av.w += weight * gv.w;
  st_nt4(acc + i, av);
  if (blockIdx.x == 0 && threadIdx.x == 0) *loss_acc = (first ? 0.f : *loss_acc) + weight * *loss;
}
void grad_accumulate_chunks(float* acc, const float* g, int64_t first_chunk, int64_t n_chunks, float weight, bool first,
                            const float* loss, float* loss_acc, hipStream_t st) {
  if (n_chunks <= 0) return;
  hipLaunchKernelGGL(grad_accumulate_kernel, dim3((unsigned)n_chunks), dim3(256), 0, st, acc, g, first_chunk, weight,
                     first ? 1 : 0, loss, loss_acc);
}

// g = acc * inv over whole chunks; loss = loss_acc * inv
__global__ __launch_bounds__(256) void grad_average_kernel(float* __restrict__ g, const float* __restrict__ acc,
                                                           int64_t first_chunk, float inv, float* __restrict__ loss,
                                                           const float* __restrict__ loss_acc) {
  const int64_t i = (first_chunk + blockIdx.x) * kChunk + 4 * threadIdx.x;
  float4 av = ld_nt4(acc + i);
  av.x *= inv; av.y *= inv; av.z *= inv; av.w *= inv;
  *reinterpret_cast<float4*>(g + i) = av;
  if (blockIdx.x == 0 && threadIdx.x == 0) *loss = *loss_acc * inv;
}
void grad_average_chunks(float* g, const float* acc, int64_t first_chunk, int64_t n_chunks, float inv, float* loss,
                         const float* loss_acc, hipStream_t st) {
  if (n_chunks <= 0) return;
  hipLaunchKernelGGL(grad_average_kernel, dim3((unsigned)n_chunks), dim3(256), 0, st, g, acc, first_chunk, inv, loss,
                     loss_acc);
}

}  // namespace pt
