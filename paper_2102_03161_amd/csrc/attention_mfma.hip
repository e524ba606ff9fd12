// bf16 softmax attention on the gfx950 matrix cores, head size 64, no mask.
//
// Layout trick shared by the three kernels: the score tile is always computed
// with the dimension a wave OWNS (32 queries in forward / dQ, 32 keys in dK/dV)
// as the MFMA output column, i.e. one lane = one owned row.  Then
//   * every per-row quantity (running max, sum, log-sum-exp, delta, the O
//     rescale factor) is a per-lane scalar: the only cross-lane traffic is one
//     xor-32 shuffle between the two half-waves;
//   * the fp32 score/probability accumulator, converted to bf16, already IS the
//     B operand of the next MFMA (contraction over the streamed dimension), so
//     probabilities never leave registers;
//   * the other operand of that MFMA must be read "transposed" (8 streamed rows
//     for one feature), which the cooperative tile loader provides by writing a
//     transposed copy of each streamed 32x64 tile into LDS (2x2 16-bit
//     transposes in registers, 4-byte LDS writes).
// The streamed dimension goes through LDS in 32-row tiles shared by the four
// waves of a workgroup.  No atomics: dQ and dK/dV are separate kernels, each
// recomputing the probabilities from the saved row log-sum-exp, so results are
// reproducible.
#include "common.h"
#include "kernels.h"

namespace pt {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace {

constexpr int DH = 64;
constexpr int LDR = DH + 8;   // row-major tile: 144-byte rows, conflict-free 16-byte operand reads
constexpr int LDT = 32 + 4;   // transposed tile [64][32]: 72-byte rows, conflict-free 8-byte operand reads

// Cooperative load (256 threads) of rows r0..r0+31 of a [*, 64] bf16 matrix with row stride ld, in two
// halves so that the global loads of the next tile can be in flight while the current one is consumed:
// tile_gload fetches this thread's two 8-byte pieces (rows 2rp, 2rp+1; features 4dc..4dc+3; rows >= nrows
// read as 0), tile_sstore writes them to a row-major tile Xs[32][LDR] and / or a transposed tile Xt[64][LDT].
struct TileRegs { uint2 a, b; };
__device__ __forceinline__ TileRegs tile_gload(const bf16* __restrict__ src, int64_t ld, int r0, int nrows, int tid) {
  const int rp = tid >> 4, dc = tid & 15;
  const int r = r0 + 2 * rp;
  TileRegs t;
  t.a = make_uint2(0, 0);
  t.b = make_uint2(0, 0);
  if (r < nrows) t.a = *reinterpret_cast<const uint2*>(src + (int64_t)r * ld + 4 * dc);
  if (r + 1 < nrows) t.b = *reinterpret_cast<const uint2*>(src + (int64_t)(r + 1) * ld + 4 * dc);
  return t;
}
__device__ __forceinline__ void tile_sstore(const TileRegs& r, bf16* Xs, bf16* Xt, int tid) {
  const int rp = tid >> 4, dc = tid & 15;
  const uint2 a = r.a, b = r.b;
  if (Xs) {
    *reinterpret_cast<uint2*>(Xs + (2 * rp) * LDR + 4 * dc) = a;
    *reinterpret_cast<uint2*>(Xs + (2 * rp + 1) * LDR + 4 * dc) = b;
  }
  if (Xt) {
    uint32_t* t = reinterpret_cast<uint32_t*>(Xt);
    const int o = (4 * dc) * (LDT / 2) + rp;  // dword index of Xt[4dc][2rp]
    t[o] = (a.x & 0xffffu) | (b.x << 16);
    t[o + (LDT / 2)] = (a.x >> 16) | (b.x & 0xffff0000u);
    t[o + 2 * (LDT / 2)] = (a.y & 0xffffu) | (b.y << 16);
    t[o + 3 * (LDT / 2)] = (a.y >> 16) | (b.y & 0xffff0000u);
  }
}

// A operand from a row-major tile: row lane%32, features 16*ks + 8*half .. +7
__device__ __forceinline__ bf16x8 frag_rows(const bf16* Xs, int lane, int ks) {
  return *reinterpret_cast<const bf16x8*>(Xs + (lane & 31) * LDR + ks * 16 + (lane >> 5) * 8);
}
// A operand from a transposed tile: feature 32*dt + lane%32, streamed rows in accumulator order:
// slot i of k-step ks2 is row 16*ks2 + 8*(i/4) + 4*half + i%4
__device__ __forceinline__ bf16x8 frag_cols(const bf16* Xt, int lane, int dt, int ks2) {
  const bf16* p = Xt + (dt * 32 + (lane & 31)) * LDT + 16 * ks2 + 4 * (lane >> 5);
  union { uint2 u[2]; bf16x8 v; } t;
  t.u[0] = *reinterpret_cast<const uint2*>(p);
  t.u[1] = *reinterpret_cast<const uint2*>(p + 8);
  return t.v;
}
// B operand straight from global memory: the lane's own row, features 16*ks + 8*half .. +7
__device__ __forceinline__ bf16x8 own_row_frag(const bf16* row, bool ok, int lane, int ks) {
  union { uint4 u; bf16x8 v; } t;
  t.u = make_uint4(0, 0, 0, 0);
  if (ok) t.u = *reinterpret_cast<const uint4*>(row + ks * 16 + (lane >> 5) * 8);
  return t.v;
}
// 2^x by the hardware instruction (results below the normal range flush to zero, which softmax tolerates)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ bf16x8 pack8(const f32x16& a, int first) {
  bf16x8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = from_f32<bf16>(a[first + i]);
  return r;
}
// accumulator register v of a 32x32 tile holds tile row 8*(v/4) + 4*half + v%4 (column = lane%32)
__device__ __forceinline__ int acc_row(int v, int half) { return 8 * (v >> 2) + 4 * half + (v & 3); }

// store one accumulator pair [feature rows][owned column] as 8-byte pieces of the owner's row
__device__ __forceinline__ void store_owned_row(bf16* row, const f32x16 (&acc)[2], float mul, int half) {
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      union { bf16 h[4]; uint2 u; } t;
#pragma unroll
      for (int e = 0; e < 4; ++e) t.h[e] = from_f32<bf16>(acc[dt][4 * g4 + e] * mul);
      *reinterpret_cast<uint2*>(row + dt * 32 + 8 * g4 + 4 * half) = t.u;
    }
}

// ---------------------------------------------------------------------------
// forward: a wave owns 32 queries, K/V stream through LDS
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ ctx,
                                                            float* __restrict__ lse, int S, int H) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[32 * LDR];
  __shared__ __attribute__((aligned(16))) bf16 Vt[64 * LDT];
  const int D = H * DH;
  const int b = blockIdx.z, h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int q = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const bool qok = q < S;
  const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
  const float c = 0.125f * 1.44269504088896f;  // 1/sqrt(64) * log2(e): scores are handled in the log2 domain
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qf[ks] = own_row_frag(base + (int64_t)q * 3 * D, qok, lane, ks);
  f32x16 o[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.f;
  float m = -INFINITY, lsum = 0.f;
  const int ntile = (S + 31) / 32;
  TileRegs rk = tile_gload(base + D, 3 * D, 0, S, tid), rv = tile_gload(base + 2 * D, 3 * D, 0, S, tid);
  for (int kt = 0; kt < ntile; ++kt) {
    __syncthreads();
    tile_sstore(rk, Ks, nullptr, tid);
    tile_sstore(rv, nullptr, Vt, tid);
    __syncthreads();
    if (kt + 1 < ntile) {
      rk = tile_gload(base + D, 3 * D, (kt + 1) * 32, S, tid);
      rv = tile_gload(base + 2 * D, 3 * D, (kt + 1) * 32, S, tid);
    }
    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Ks, lane, ks), qf[ks], s, 0, 0, 0);
    if (kt == ntile - 1 && (S & 31)) {  // keys past the end exist only in the last tile
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = (kt * 32 + acc_row(v, half) < S) ? s[v] : -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c;
    // softmax is invariant under the shift m, so the reference maximum only has to keep exp2 in range: it is
    // moved (and the running sums rescaled) only when a row's maximum has grown by more than 2^8
    if (__any(mx > m + 8.f)) {
      const float m_new = mx > m + 8.f ? mx : m;
      const float alpha = fast_exp2(m - m_new);
      lsum *= alpha;
      m = m_new;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
    }
    float rs = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s[v] = fast_exp2(fmaf(s[v], c, -m));
      rs += s[v];
    }
    lsum += rs + __shfl_xor(rs, 32, 64);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const bf16x8 pb = pack8(s, 8 * ks2);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(Vt, lane, dt, ks2), pb, o[dt], 0, 0, 0);
    }
  }
  if (qok) {
    store_owned_row(ctx + ((int64_t)b * S + q) * D + h * DH, o, 1.0f / lsum, half);
    if (lse && half == 0) lse[((int64_t)b * H + h) * S + q] = (m + __log2f(lsum)) * 0.693147180559945f;
  }
}

// ---------------------------------------------------------------------------
// backward part 1: delta = rowsum(dO * O) and dQ; a wave owns 32 queries
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ ctx,
                                                               const bf16* __restrict__ dctx,
                                                               const float* __restrict__ lse, bf16* __restrict__ dqkv,
                                                               float* __restrict__ delta, int S, int H) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[32 * LDR];
  __shared__ __attribute__((aligned(16))) bf16 Vs[32 * LDR];
  __shared__ __attribute__((aligned(16))) bf16 Kt[64 * LDT];
  const int D = H * DH;
  const int b = blockIdx.z, h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int q = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const bool qok = q < S;
  const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
  const float scale = 0.125f, c = scale * 1.44269504088896f;
  bf16x8 qf[4], dof[4];
  float part = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qf[ks] = own_row_frag(base + (int64_t)q * 3 * D, qok, lane, ks);
    dof[ks] = own_row_frag(dctx + ((int64_t)b * S + q) * D + h * DH, qok, lane, ks);
    const bf16x8 of = own_row_frag(ctx + ((int64_t)b * S + q) * D + h * DH, qok, lane, ks);
#pragma unroll
    for (int i = 0; i < 8; ++i) part += to_f32(dof[ks][i]) * to_f32(of[i]);
  }
  const float dl = part + __shfl_xor(part, 32, 64);
  // rows past the end keep finite values (their dQ is never stored)
  const float lq2 = (qok ? lse[((int64_t)b * H + h) * S + q] : 0.f) * 1.44269504088896f;
  if (qok && half == 0) delta[((int64_t)b * H + h) * S + q] = dl;
  f32x16 dq[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) dq[dt][v] = 0.f;
  const int ntile = (S + 31) / 32;
  TileRegs rk = tile_gload(base + D, 3 * D, 0, S, tid), rv = tile_gload(base + 2 * D, 3 * D, 0, S, tid);
  for (int kt = 0; kt < ntile; ++kt) {
    __syncthreads();
    tile_sstore(rk, Ks, Kt, tid);
    tile_sstore(rv, Vs, nullptr, tid);
    __syncthreads();
    if (kt + 1 < ntile) {
      rk = tile_gload(base + D, 3 * D, (kt + 1) * 32, S, tid);
      rv = tile_gload(base + 2 * D, 3 * D, (kt + 1) * 32, S, tid);
    }
    f32x16 s, dp;
#pragma unroll
    for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Ks, lane, ks), qf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Vs, lane, ks), dof[ks], dp, 0, 0, 0);
    }
    if (kt == ntile - 1 && (S & 31)) {  // keys past the end: probability 0
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = (kt * 32 + acc_row(v, half) < S) ? s[v] : -INFINITY;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float p = fast_exp2(fmaf(s[v], c, -lq2));
      s[v] = p * (dp[v] - dl);  // dS^T
    }
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const bf16x8 dsb = pack8(s, 8 * ks2);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
        dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(Kt, lane, dt, ks2), dsb, dq[dt], 0, 0, 0);
    }
  }
  if (qok) store_owned_row(dqkv + ((int64_t)b * S + q) * 3 * D + h * DH, dq, scale, half);
}

// ---------------------------------------------------------------------------
// backward part 2: dK, dV; a wave owns 32 keys, Q / dO stream through LDS
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(const bf16* __restrict__ qkv,
                                                                const bf16* __restrict__ dctx,
                                                                const float* __restrict__ lse,
                                                                const float* __restrict__ delta,
                                                                bf16* __restrict__ dqkv, int S, int H) {
  __shared__ __attribute__((aligned(16))) bf16 Qs[32 * LDR];
  __shared__ __attribute__((aligned(16))) bf16 dOs[32 * LDR];
  __shared__ __attribute__((aligned(16))) bf16 Qt[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 dOt[64 * LDT];
  __shared__ __attribute__((aligned(16))) float ls[32], dls[32];  // row log-sum-exp (log2 domain) and delta of the tile
  const int D = H * DH;
  const int b = blockIdx.z, h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int key = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const bool kok = key < S;
  const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
  const bf16* dobase = dctx + (int64_t)b * S * D + h * DH;
  const float scale = 0.125f, c = scale * 1.44269504088896f;
  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    kf[ks] = own_row_frag(base + (int64_t)key * 3 * D + D, kok, lane, ks);
    vf[ks] = own_row_frag(base + (int64_t)key * 3 * D + 2 * D, kok, lane, ks);
  }
  f32x16 dk[2], dv[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[dt][v] = 0.f; dv[dt][v] = 0.f; }
  const int ntile = (S + 31) / 32;
  TileRegs rq = tile_gload(base, 3 * D, 0, S, tid), rdo = tile_gload(dobase, D, 0, S, tid);
  // a query row past the end gets log-sum-exp +inf, hence probability exp2(-inf) = 0, and delta 0
  float nls = INFINITY, ndl = 0.f;
  if (tid < 32 && tid < S) {
    nls = lse[((int64_t)b * H + h) * S + tid] * 1.44269504088896f;
    ndl = delta[((int64_t)b * H + h) * S + tid];
  }
  for (int qt = 0; qt < ntile; ++qt) {
    __syncthreads();
    tile_sstore(rq, Qs, Qt, tid);
    tile_sstore(rdo, dOs, dOt, tid);
    if (tid < 32) { ls[tid] = nls; dls[tid] = ndl; }
    __syncthreads();
    if (qt + 1 < ntile) {
      rq = tile_gload(base, 3 * D, (qt + 1) * 32, S, tid);
      rdo = tile_gload(dobase, D, (qt + 1) * 32, S, tid);
      if (tid < 32) {
        const int qq = (qt + 1) * 32 + tid;
        nls = qq < S ? lse[((int64_t)b * H + h) * S + qq] * 1.44269504088896f : INFINITY;
        ndl = qq < S ? delta[((int64_t)b * H + h) * S + qq] : 0.f;
      }
    }
    f32x16 s, dp;
#pragma unroll
    for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Qs, lane, ks), kf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(dOs, lane, ks), vf[ks], dp, 0, 0, 0);
    }
    f32x16 pr;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {  // accumulator registers 4g..4g+3 are tile rows 8g + 4*half + 0..3
      const float4 l4 = *reinterpret_cast<const float4*>(ls + 8 * g4 + 4 * half);
      const float4 d4 = *reinterpret_cast<const float4*>(dls + 8 * g4 + 4 * half);
      const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int v = 4 * g4 + e;
        const float p = fast_exp2(fmaf(s[v], c, -lv[e]));
        pr[v] = p;
        s[v] = p * (dp[v] - dv4[e]);  // dS
      }
    }
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const bf16x8 pb = pack8(pr, 8 * ks2), dsb = pack8(s, 8 * ks2);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(dOt, lane, dt, ks2), pb, dv[dt], 0, 0, 0);
        dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols(Qt, lane, dt, ks2), dsb, dk[dt], 0, 0, 0);
      }
    }
  }
  if (kok) {
    bf16* row = dqkv + ((int64_t)b * S + key) * 3 * D + h * DH;
    store_owned_row(row + D, dk, scale, half);
    store_owned_row(row + 2 * D, dv, 1.0f, half);
  }
}


// ===========================================================================
// Resident variants: when the whole streamed side of one (sample, head) fits in LDS, it is loaded once with
// every global load in flight at the same time, and the tile loop then runs without barriers or further
// global loads (the streaming kernels above pay one global-load latency per 32-row tile).  Tiles stay
// row-major; the operand that must be read "transposed" comes from the LDS transpose read
// ds_read_b64_tr_b16, which hands a lane four consecutive rows of one feature.  A workgroup has one wave per
// 32 owned rows (at most 8 waves; longer sequences split the owned rows over blockIdx.x).
// ===========================================================================
__device__ __forceinline__ unsigned lds_addr(const void* p) {
  return (unsigned)(size_t)((__attribute__((address_space(3))) const void*)(p));
}
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4v;

// rows [0, rows_pad) of two [*, 64] matrices into row-major LDS images (rows >= nrows read as 0).  Eight
// 16-byte global loads per thread are issued before the first LDS store, so a workgroup pays the global
// latency once per round instead of once per piece.
__device__ __forceinline__ void load_resident2(bf16* dst_a, const bf16* __restrict__ src_a, int64_t ld_a, bf16* dst_b,
                                               const bf16* __restrict__ src_b, int64_t ld_b, int nrows, int rows_pad,
                                               int tid, int nthreads) {
  const int total = rows_pad * 8;
  for (int c0 = tid; c0 < total; c0 += 4 * nthreads) {
    uint4 va[4], vb[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * nthreads, row = c >> 3, ch = c & 7;
      va[u] = make_uint4(0, 0, 0, 0);
      vb[u] = make_uint4(0, 0, 0, 0);
      if (c < total && row < nrows) {
        va[u] = *reinterpret_cast<const uint4*>(src_a + (int64_t)row * ld_a + ch * 8);
        vb[u] = *reinterpret_cast<const uint4*>(src_b + (int64_t)row * ld_b + ch * 8);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * nthreads, row = c >> 3, ch = c & 7;
      if (c < total) {
        *reinterpret_cast<uint4*>(dst_a + row * LDR + ch * 8) = va[u];
        *reinterpret_cast<uint4*>(dst_b + row * LDR + ch * 8) = vb[u];
      }
    }
  }
}
// A operand "feature dt*32 + lane%32 over 8 streamed rows in accumulator order" from a row-major tile:
// two transpose reads of rows 16*ks2 + 4*half + {0..3} and the same + 8.  The 16 lanes of a group address a
// 4 x 16 block (lane l: row l/4, features 4*(l%4)..+3) and lane i receives the four rows of feature i.
// The caller waits for the reads (lds_wait) before the fragment is used.
__device__ __forceinline__ void frag_cols_tr(const bf16* X, int lane, int dt, int ks2, bf16x8& f) {
  const int l16 = lane & 15, grp = lane >> 4;
  const int row = 16 * ks2 + 4 * (grp >> 1) + (l16 >> 2);
  const int col = dt * 32 + 16 * (grp & 1) + 4 * (l16 & 3);
  const unsigned addr = lds_addr(X + row * LDR + col);
  union { u32x2 h[2]; bf16x8 v; } t;
  asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(t.h[0]) : "v"(addr));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(t.h[1]) : "v"(addr), "n"(8 * LDR * 2));
  f = t.v;
}
// A operand "row lane%32, features 16*ks + 8*half .. +7" of a row-major tile, issued without a wait so that
// the reads of a whole tile are in flight together (the compiler would otherwise wait for each fragment right
// before the MFMA that uses it).  base = address of the lane's row start + 16*half bytes.
__device__ __forceinline__ void frag_rows_issue(unsigned base, bf16x8 (&f)[4]) {
  asm volatile("ds_read_b128 %0, %1" : "=v"(f[0]) : "v"(base));
  asm volatile("ds_read_b128 %0, %1 offset:32" : "=v"(f[1]) : "v"(base));
  asm volatile("ds_read_b128 %0, %1 offset:64" : "=v"(f[2]) : "v"(base));
  asm volatile("ds_read_b128 %0, %1 offset:96" : "=v"(f[3]) : "v"(base));
}
// waits until at most PENDING LDS operations are outstanding (they return in order) and makes the given
// fragments depend on the wait, so that no MFMA reading them is scheduled before it
template <int PENDING, int N>
__device__ __forceinline__ void lds_wait(bf16x8 (&f)[N]) {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(PENDING) : "memory");
#pragma unroll
  for (int i = 0; i < N; ++i) asm volatile("" : "+v"(f[i]));
}

__global__ __launch_bounds__(512) void attn_fwd_res_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ ctx,
                                                           float* __restrict__ lse, int S, int H, int ntile) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Ks = reinterpret_cast<bf16*>(smem);
  bf16* Vs = Ks + ntile * 32 * LDR;
  const int D = H * DH;
  const int b = blockIdx.z, h = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int nw = blockDim.x >> 6;
  const int q = (blockIdx.x * nw + wave) * 32 + (lane & 31);
  const bool qok = q < S;
  const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
  const float c = 0.125f * 1.44269504088896f;
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qf[ks] = own_row_frag(base + (int64_t)q * 3 * D, qok, lane, ks);
  load_resident2(Ks, base + D, 3 * D, Vs, base + 2 * D, 3 * D, S, ntile * 32, tid, blockDim.x);
  __syncthreads();
  if ((blockIdx.x * nw + wave) * 32 >= S) return;   // a wave without queries (no barrier follows)
  f32x16 o[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[dt][v] = 0.f;
  float m = -INFINITY, lsum = 0.f;
  const unsigned rows_base = lds_addr(Ks + (lane & 31) * LDR + half * 8);
  for (int kt = 0; kt < ntile; ++kt) {
    const bf16* Vt = Vs + kt * 32 * LDR;
    bf16x8 kr[4], vf[4];   // K rows [ks]; V columns [ks2][dt]
    frag_rows_issue(rows_base + kt * (32 * LDR * 2), kr);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) frag_cols_tr(Vt, lane, dt, ks2, vf[2 * ks2 + dt]);
    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
    lds_wait<8>(kr);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[ks], qf[ks], s, 0, 0, 0);
    if (kt == ntile - 1 && (S & 31)) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = (kt * 32 + acc_row(v, half) < S) ? s[v] : -INFINITY;
    }
    float mx = s[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c;
    if (__any(mx > m + 8.f)) {
      const float m_new = mx > m + 8.f ? mx : m;
      const float alpha = fast_exp2(m - m_new);
      lsum *= alpha;
      m = m_new;
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[dt][v] *= alpha;
    }
    float rs = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s[v] = fast_exp2(fmaf(s[v], c, -m));
      rs += s[v];
    }
    lsum += rs + __shfl_xor(rs, 32, 64);
    lds_wait<0>(vf);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const bf16x8 pb = pack8(s, 8 * ks2);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[2 * ks2 + dt], pb, o[dt], 0, 0, 0);
    }
  }
  if (qok) {
    store_owned_row(ctx + ((int64_t)b * S + q) * D + h * DH, o, 1.0f / lsum, half);
    if (lse && half == 0) lse[((int64_t)b * H + h) * S + q] = (m + __log2f(lsum)) * 0.693147180559945f;
  }
}

// A workgroup takes `upw` consecutive units (unit = nblk * (b * H + h) + block of queries): when only one
// workgroup fits a CU and there are more units than CUs, a workgroup walks over several, and the K and V images
// stay in LDS from one unit to the next of the same head (a head's two query blocks at S = 384 or 512).
__global__ __launch_bounds__(512, 4) void attn_bwd_dq_res_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ ctx,
                                                              const bf16* __restrict__ dctx,
                                                              const float* __restrict__ lse, bf16* __restrict__ dqkv,
                                                              float* __restrict__ delta, int S, int H, int ntile, int nblk,
                                                              int upw, int nunits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Ks = reinterpret_cast<bf16*>(smem);
  bf16* Vs = Ks + ntile * 32 * LDR;
  const int D = H * DH;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int nw = blockDim.x >> 6;
  const float scale = 0.125f, c = scale * 1.44269504088896f;
  int loaded = -1;   // the head whose K and V are in LDS
  const int u_end = ((int)blockIdx.x + 1) * upw < nunits ? ((int)blockIdx.x + 1) * upw : nunits;
  for (int u = (int)blockIdx.x * upw; u < u_end; ++u) {
  const int bh = u / nblk, blk = u - bh * nblk;
  const int b = bh / H, h = bh - b * H;
  const int q = (blk * nw + wave) * 32 + (lane & 31);
  const bool qok = q < S;
  const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
  bf16x8 qf[4], dof[4];
  float part = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qf[ks] = own_row_frag(base + (int64_t)q * 3 * D, qok, lane, ks);
    dof[ks] = own_row_frag(dctx + ((int64_t)b * S + q) * D + h * DH, qok, lane, ks);
    const bf16x8 of = own_row_frag(ctx + ((int64_t)b * S + q) * D + h * DH, qok, lane, ks);
#pragma unroll
    for (int i = 0; i < 8; ++i) part += to_f32(dof[ks][i]) * to_f32(of[i]);
  }
  if (loaded != bh) {
    if (loaded >= 0) __syncthreads();   // everybody is done with the previous head's images
    load_resident2(Ks, base + D, 3 * D, Vs, base + 2 * D, 3 * D, S, ntile * 32, tid, blockDim.x);
    loaded = bh;
    __syncthreads();
  }
  if ((blk * nw + wave) * 32 >= S) continue;   // a wave without queries (it still meets the barriers above)
  const float dl = part + __shfl_xor(part, 32, 64);
  const float lq2 = (qok ? lse[((int64_t)b * H + h) * S + q] : 0.f) * 1.44269504088896f;
  if (qok && half == 0) delta[((int64_t)b * H + h) * S + q] = dl;
  f32x16 dq[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) dq[dt][v] = 0.f;
  const unsigned k_base = lds_addr(Ks + (lane & 31) * LDR + half * 8);
  const unsigned v_base = lds_addr(Vs + (lane & 31) * LDR + half * 8);
  for (int kt = 0; kt < ntile; ++kt) {
    const bf16* Kt = Ks + kt * 32 * LDR;
    // Fragments are fetched in the order they are used and each set's registers are free again before the
    // next set arrives: 16 registers of fragments in flight instead of 48, which is what lets two
    // workgroups share a CU (one loads its head while the other computes).
    bf16x8 kr[4], vr[4], kc[4];
    frag_rows_issue(k_base + kt * (32 * LDR * 2), kr);
    frag_rows_issue(v_base + kt * (32 * LDR * 2), vr);
    f32x16 s, dp;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
    lds_wait<4>(kr);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[ks], qf[ks], s, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int v = 0; v < 16; ++v) dp[v] = 0.f;
    lds_wait<0>(vr);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[ks], dof[ks], dp, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) frag_cols_tr(Kt, lane, dt, ks2, kc[2 * ks2 + dt]);
    if (kt == ntile - 1 && (S & 31)) {
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = (kt * 32 + acc_row(v, half) < S) ? s[v] : -INFINITY;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float p = fast_exp2(fmaf(s[v], c, -lq2));
      s[v] = p * (dp[v] - dl);  // dS^T
    }
    lds_wait<0>(kc);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const bf16x8 dsb = pack8(s, 8 * ks2);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kc[2 * ks2 + dt], dsb, dq[dt], 0, 0, 0);
    }
  }
  if (qok) store_owned_row(dqkv + ((int64_t)b * S + q) * 3 * D + h * DH, dq, scale, half);
  }
}

// units as in attn_bwd_dq_res_kernel (here a unit's block is a block of keys, and Q, dO and the two float rows stay)
__global__ __launch_bounds__(512) void attn_bwd_dkv_res_kernel(const bf16* __restrict__ qkv,
                                                               const bf16* __restrict__ dctx,
                                                               const float* __restrict__ lse,
                                                               const float* __restrict__ delta,
                                                               bf16* __restrict__ dqkv, int S, int H, int ntile, int nblk,
                                                               int upw, int nunits) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Qs = reinterpret_cast<bf16*>(smem);
  bf16* dOs = Qs + ntile * 32 * LDR;
  float* ls = reinterpret_cast<float*>(dOs + ntile * 32 * LDR);   // row log-sum-exp in the log2 domain
  float* dls = ls + ntile * 32;
  const int D = H * DH;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int nw = blockDim.x >> 6;
  const float scale = 0.125f, c = scale * 1.44269504088896f;
  int loaded = -1;
  const int u_end = ((int)blockIdx.x + 1) * upw < nunits ? ((int)blockIdx.x + 1) * upw : nunits;
  for (int u = (int)blockIdx.x * upw; u < u_end; ++u) {
  const int bh = u / nblk, blk = u - bh * nblk;
  const int b = bh / H, h = bh - b * H;
  const int key = (blk * nw + wave) * 32 + (lane & 31);
  const bool kok = key < S;
  const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
  const bf16* dobase = dctx + (int64_t)b * S * D + h * DH;
  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    kf[ks] = own_row_frag(base + (int64_t)key * 3 * D + D, kok, lane, ks);
    vf[ks] = own_row_frag(base + (int64_t)key * 3 * D + 2 * D, kok, lane, ks);
  }
  if (loaded != bh) {
    if (loaded >= 0) __syncthreads();
    load_resident2(Qs, base, 3 * D, dOs, dobase, D, S, ntile * 32, tid, blockDim.x);
    // a query row past the end gets log-sum-exp +inf, hence probability exp2(-inf) = 0, and delta 0
    for (int r = tid; r < ntile * 32; r += blockDim.x) {
      ls[r] = r < S ? lse[((int64_t)b * H + h) * S + r] * 1.44269504088896f : INFINITY;
      dls[r] = r < S ? delta[((int64_t)b * H + h) * S + r] : 0.f;
    }
    loaded = bh;
    __syncthreads();
  }
  if ((blk * nw + wave) * 32 >= S) continue;
  f32x16 dk[2], dv[2];
#pragma unroll
  for (int dt = 0; dt < 2; ++dt)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[dt][v] = 0.f; dv[dt][v] = 0.f; }
  const unsigned q_base = lds_addr(Qs + (lane & 31) * LDR + half * 8);
  const unsigned do_base = lds_addr(dOs + (lane & 31) * LDR + half * 8);
  for (int qt = 0; qt < ntile; ++qt) {
    const bf16* Qt = Qs + qt * 32 * LDR;
    const bf16* dOt = dOs + qt * 32 * LDR;
    bf16x8 qr[4], dor[4], tc[8];   // rows of Q and dO; columns [ks2][dt] of dO, then of Q
    frag_rows_issue(q_base + qt * (32 * LDR * 2), qr);
    frag_rows_issue(do_base + qt * (32 * LDR * 2), dor);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) frag_cols_tr(dOt, lane, dt, ks2, tc[2 * ks2 + dt]);
    f32x16 s, dp;
#pragma unroll
    for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
    lds_wait<8>(qr);
    lds_wait<8>(dor);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) frag_cols_tr(Qt, lane, dt, ks2, tc[4 + 2 * ks2 + dt]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qr[ks], kf[ks], s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dor[ks], vf[ks], dp, 0, 0, 0);
    }
    f32x16 pr;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      const float4 l4 = *reinterpret_cast<const float4*>(ls + qt * 32 + 8 * g4 + 4 * half);
      const float4 d4 = *reinterpret_cast<const float4*>(dls + qt * 32 + 8 * g4 + 4 * half);
      const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int v = 4 * g4 + e;
        const float p = fast_exp2(fmaf(s[v], c, -lv[e]));
        pr[v] = p;
        s[v] = p * (dp[v] - dv4[e]);  // dS
      }
    }
    lds_wait<0>(tc);
#pragma unroll
    for (int ks2 = 0; ks2 < 2; ++ks2) {
      const bf16x8 pb = pack8(pr, 8 * ks2), dsb = pack8(s, 8 * ks2);
#pragma unroll
      for (int dt = 0; dt < 2; ++dt) {
        dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tc[2 * ks2 + dt], pb, dv[dt], 0, 0, 0);
        dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tc[4 + 2 * ks2 + dt], dsb, dk[dt], 0, 0, 0);
      }
    }
  }
  if (kok) {
    bf16* row = dqkv + ((int64_t)b * S + key) * 3 * D + h * DH;
    store_owned_row(row + D, dk, scale, half);
    store_owned_row(row + 2 * D, dv, 1.0f, half);
  }
  }
}

// ---------------------------------------------------------------------------
// Fused backward for short sequences (S <= 256): one workgroup per (sample, head) holds Q, K, V and dO of the
// head in LDS, so the packed qkv and dO are read from memory once instead of once per kernel and the
// row statistics (log-sum-exp, delta = dO.O) never leave the chip.  Wave w owns rows 32w..32w+31: first as
// queries (the dQ loop of attn_bwd_dq_res_kernel over the key tiles), then as keys (the dK/dV loop of
// attn_bwd_dkv_res_kernel over the query tiles).  No atomics; the scores are recomputed in the second pass.
// ---------------------------------------------------------------------------
// v, or zeros (a select of the four words in registers; a conditional on the struct goes through memory)
__device__ __forceinline__ uint4 keep(uint4 v, bool on) {
  const unsigned m = on ? 0xffffffffu : 0u;
  return make_uint4(v.x & m, v.y & m, v.z & m, v.w & m);
}
__global__ __launch_bounds__(512) void attn_bwd_fused_res_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ ctx,
                                                                 const bf16* __restrict__ dctx,
                                                                 const float* __restrict__ lse, bf16* __restrict__ dqkv,
                                                                 int S, int H, int ntile) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tile_elems = ntile * 32 * LDR;
  bf16* Qs = reinterpret_cast<bf16*>(smem);
  bf16* Ks = Qs + tile_elems;
  bf16* Vs = Ks + tile_elems;
  bf16* dOs = Vs + tile_elems;
  float* ls = reinterpret_cast<float*>(dOs + tile_elems);   // row log-sum-exp in the log2 domain
  float* dls = ls + ntile * 32;                             // row delta
  const int D = H * DH;
  const int b = blockIdx.y, h = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
  const int own = wave * 32 + (lane & 31);   // the row this lane owns, as a query and as a key
  const bool ok = own < S;
  const bool active = wave * 32 < S;
  const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
  const bf16* dobase = dctx + (int64_t)b * S * D + h * DH;
  bf16* obase = dqkv + (int64_t)b * S * 3 * D + h * DH;
  const float scale = 0.125f, c = scale * 1.44269504088896f;

  // The loads the first pass waits for go out together: the lane's own query row with its dO and O (the
  // lines are the ones the image loads bring in), its log-sum-exp, and the K and V images (a workgroup has
  // one wave per 32 rows, so four 16-byte chunks per thread cover an image).  Rows past the end read row
  // S - 1 and are zeroed afterwards: unconditional loads let the compiler count exactly which ones a wait
  // needs, where loads under a branch make it wait for all of them.  The Q and dO images, which only the
  // second pass reads, are requested once K and V are in LDS and stay in registers over the first pass.  The barriers are bare s_barrier instructions behind an LDS wait:
  // __syncthreads() would also wait for the loads still in flight.
  const int ownc = ok ? own : S - 1;
  union Frag { uint4 u; bf16x8 v; };
  Frag qf_[4], dof_[4], of_[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int off = ks * 16 + half * 8;
    qf_[ks].u = *reinterpret_cast<const uint4*>(base + (int64_t)ownc * 3 * D + off);
    dof_[ks].u = *reinterpret_cast<const uint4*>(dobase + (int64_t)ownc * D + off);
    of_[ks].u = *reinterpret_cast<const uint4*>(ctx + ((int64_t)b * S + ownc) * D + h * DH + off);
  }
  const float lse_own = lse[((int64_t)b * H + h) * S + ownc];
  uint4 vk[4], vv[4], vq[4], vd[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int ch = tid + u * (int)blockDim.x, row = ch >> 3, col = (ch & 7) * 8, rc = row < S ? row : S - 1;
    vk[u] = *reinterpret_cast<const uint4*>(base + (int64_t)rc * 3 * D + D + col);
    vv[u] = *reinterpret_cast<const uint4*>(base + (int64_t)rc * 3 * D + 2 * D + col);
  }
  bf16x8 qf[4], dof[4];
  float part = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qf_[ks].u = keep(qf_[ks].u, ok);
    dof_[ks].u = keep(dof_[ks].u, ok);
    of_[ks].u = keep(of_[ks].u, ok);
    qf[ks] = qf_[ks].v;
    dof[ks] = dof_[ks].v;
#pragma unroll
    for (int i = 0; i < 8; ++i) part += to_f32(dof[ks][i]) * to_f32(of_[ks].v[i]);
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int ch = tid + u * (int)blockDim.x, row = ch >> 3, col = (ch & 7) * 8;
    *reinterpret_cast<uint4*>(Ks + row * LDR + col) = keep(vk[u], row < S);
    *reinterpret_cast<uint4*>(Vs + row * LDR + col) = keep(vv[u], row < S);
  }
  __builtin_amdgcn_sched_barrier(0);   // the second pass's images are requested once K and V have left their registers
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int ch = tid + u * (int)blockDim.x, row = ch >> 3, col = (ch & 7) * 8, rc = row < S ? row : S - 1;
    vq[u] = *reinterpret_cast<const uint4*>(base + (int64_t)rc * 3 * D + col);
    vd[u] = *reinterpret_cast<const uint4*>(dobase + (int64_t)rc * D + col);
  }
  const float dl = part + __shfl_xor(part, 32, 64);
  const float lq2 = (ok ? lse_own : 0.f) * 1.44269504088896f;
  // a row past the end gets log-sum-exp +inf, hence probability exp2(-inf) = 0, and delta 0
  if (half == 0) {
    ls[own] = ok ? lq2 : INFINITY;
    dls[own] = ok ? dl : 0.f;
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");

  // ---- pass 1: the wave's rows as queries ----
  if (active) {
    f32x16 dq[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) dq[dt][v] = 0.f;
    const unsigned k_base = lds_addr(Ks + (lane & 31) * LDR + half * 8);
    const unsigned v_base = lds_addr(Vs + (lane & 31) * LDR + half * 8);
    for (int kt = 0; kt < ntile; ++kt) {
      const bf16* Kt = Ks + kt * 32 * LDR;
      bf16x8 kr[4], vr[4], kc[4];
      frag_rows_issue(k_base + kt * (32 * LDR * 2), kr);
      frag_rows_issue(v_base + kt * (32 * LDR * 2), vr);
      f32x16 s, dp;
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = 0.f;
      lds_wait<4>(kr);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[ks], qf[ks], s, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int v = 0; v < 16; ++v) dp[v] = 0.f;
      lds_wait<0>(vr);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[ks], dof[ks], dp, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) frag_cols_tr(Kt, lane, dt, ks2, kc[2 * ks2 + dt]);
      if (kt == ntile - 1 && (S & 31)) {
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = (kt * 32 + acc_row(v, half) < S) ? s[v] : -INFINITY;
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float p = fast_exp2(fmaf(s[v], c, -lq2));
        s[v] = p * (dp[v] - dl);  // dS^T
      }
      lds_wait<0>(kc);
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        const bf16x8 dsb = pack8(s, 8 * ks2);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kc[2 * ks2 + dt], dsb, dq[dt], 0, 0, 0);
      }
    }
    if (ok) store_owned_row(obase + (int64_t)own * 3 * D, dq, scale, half);
  }

  // ---- pass 2: the wave's rows as keys ----
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const int ch = tid + u * (int)blockDim.x, row = ch >> 3, col = (ch & 7) * 8;
    *reinterpret_cast<uint4*>(Qs + row * LDR + col) = keep(vq[u], row < S);
    *reinterpret_cast<uint4*>(dOs + row * LDR + col) = keep(vd[u], row < S);
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  if (active) {
    bf16x8 kf[4], vf[4];
    frag_rows_issue(lds_addr(Ks + own * LDR + half * 8), kf);
    frag_rows_issue(lds_addr(Vs + own * LDR + half * 8), vf);
    lds_wait<0>(kf);
    lds_wait<0>(vf);
    f32x16 dk[2], dv[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) { dk[dt][v] = 0.f; dv[dt][v] = 0.f; }
    const unsigned q_base = lds_addr(Qs + (lane & 31) * LDR + half * 8);
    const unsigned do_base = lds_addr(dOs + (lane & 31) * LDR + half * 8);
    for (int qt = 0; qt < ntile; ++qt) {
      const bf16* Qt = Qs + qt * 32 * LDR;
      const bf16* dOt = dOs + qt * 32 * LDR;
      bf16x8 qr[4], dor[4], tc[8];   // rows of Q and dO; columns [ks2][dt] of dO, then of Q
      frag_rows_issue(q_base + qt * (32 * LDR * 2), qr);
      frag_rows_issue(do_base + qt * (32 * LDR * 2), dor);
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) frag_cols_tr(dOt, lane, dt, ks2, tc[2 * ks2 + dt]);
      f32x16 s, dp;
#pragma unroll
      for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
      lds_wait<8>(qr);
      lds_wait<8>(dor);
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) frag_cols_tr(Qt, lane, dt, ks2, tc[4 + 2 * ks2 + dt]);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qr[ks], kf[ks], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dor[ks], vf[ks], dp, 0, 0, 0);
      }
      f32x16 pr;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const float4 l4 = *reinterpret_cast<const float4*>(ls + qt * 32 + 8 * g4 + 4 * half);
        const float4 d4 = *reinterpret_cast<const float4*>(dls + qt * 32 + 8 * g4 + 4 * half);
        const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dv4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = 4 * g4 + e;
          const float p = fast_exp2(fmaf(s[v], c, -lv[e]));
          pr[v] = p;
          s[v] = p * (dp[v] - dv4[e]);  // dS
        }
      }
      lds_wait<0>(tc);
#pragma unroll
      for (int ks2 = 0; ks2 < 2; ++ks2) {
        const bf16x8 pb = pack8(pr, 8 * ks2), dsb = pack8(s, 8 * ks2);
#pragma unroll
        for (int dt = 0; dt < 2; ++dt) {
          dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tc[2 * ks2 + dt], pb, dv[dt], 0, 0, 0);
          dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tc[4 + 2 * ks2 + dt], dsb, dk[dt], 0, 0, 0);
        }
      }
    }
    if (ok) {
      bf16* row = obase + (int64_t)own * 3 * D;
      store_owned_row(row + D, dk, scale, half);
      store_owned_row(row + 2 * D, dv, 1.0f, half);
    }
  }
}

// ---------------------------------------------------------------------------
// Pipelined fused backward (S <= 208): the fused kernel above spends half of a head's time waiting for the
// head's four [S,64] matrices, with every CU of the chip loading at the same moment and computing at the same
// moment.  Here a workgroup stays on its CU and walks over its heads, and the matrices of the next head arrive
// while the current one is computed: they travel straight from global memory into LDS (global_load_lds, no
// staging registers) into image slots that the current head no longer reads.
//
// LDS holds six images of rows_pad = ceil16(S) rows of 128 bytes, in three pairs that rotate per head:
//   pair (n mod 3)      Q and dO of head n   (read by pass 2, and for the lanes' own rows at the head's start)
//   pair (n + 1 mod 3)  K and V of head n    (read by pass 1, and for the lanes' own rows when pass 2 starts)
//   pair (n + 2 mod 3)  free: K and V of head n + 1 are requested into it when head n starts;
//                       Q and dO of head n + 1 go into head n's K/V pair once pass 1 is over.
// An image has no padding (a wave-wide load writes 64 consecutive 16-byte slots = eight rows); slot (row, p)
// holds the row's 16-byte chunk p ^ img_swz(row), the permutation being applied to the global address a lane
// fetches.  img_swz makes both kinds of fragment reads conflict-free: the 16 rows a quarter-wave reads with
// ds_read_b128 fall into 16 different 16-byte bank groups, and so do the 4 rows x 32 bytes that a half-wave's
// two 16-lane groups address in a transpose read.  XOR-ing a chunk index is XOR-ing bits 4-6 of the byte
// address, so a lane keeps two offsets and derives the others with one XOR.
// Tiles are 32 rows and the last one may reach up to 16 rows past an image: those reads land in the next
// image or in a zeroed pad behind the last one.  Everything there is finite (the whole LDS is zeroed first,
// and rows past S of an image are copies of row S - 1), and it only meets probabilities that are exactly 0.
// ---------------------------------------------------------------------------
#define PT_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PT_GLB(p) ((const __attribute__((address_space(1))) void*)(p))
constexpr int kImgRowBytes = 2 * DH;   // 128
constexpr int kImgPadBytes = 16 * kImgRowBytes;
__device__ __forceinline__ constexpr int img_swz(int row) {
  const int t = (row >> 1) & 7;
  return ((t & 1) << 2) | (t >> 1);
}
// requests rows [0, rows_pad) of a [nrows, 64] matrix (row stride ld elements) into the image at `img`; the
// wave-wide loads are dealt to the nw waves round-robin
__device__ __forceinline__ void img_request(unsigned char* img, const bf16* __restrict__ src, int64_t ld, int nrows, int rows_pad,
                                            int wave, int nw, int lane) {
  for (int i = wave; i < (rows_pad >> 3); i += nw) {
    const int row = 8 * i + (lane >> 3);
    const int c = (lane & 7) ^ img_swz(row);
    const int rc = row < nrows ? row : nrows - 1;
    __builtin_amdgcn_global_load_lds(PT_GLB(src + (int64_t)rc * ld + 8 * c), PT_LDS(img + i * 1024), 16, 0, 0);
  }
}
// the four 16-byte fragments (features 16 ks + 8 half .. + 7, ks = 0..3) of the lane's row: rb is the lane's
// offset of chunk `half` in a 32-row tile, base the tile's LDS address
__device__ __forceinline__ void img_rows_issue(unsigned base, unsigned rb, bf16x8 (&f)[4]) {
  asm volatile("ds_read_b128 %0, %1" : "=v"(f[0]) : "v"(base + rb));
  asm volatile("ds_read_b128 %0, %1" : "=v"(f[1]) : "v"(base + (rb ^ 32u)));
  asm volatile("ds_read_b128 %0, %1" : "=v"(f[2]) : "v"(base + (rb ^ 64u)));
  asm volatile("ds_read_b128 %0, %1" : "=v"(f[3]) : "v"(base + (rb ^ 96u)));
}
// the same reads from address registers that the caller advances by one tile per iteration: a[ks] is the
// address of the lane's chunk (2 ks + half) in the current tile, t[] the four transposed-read addresses
// {dt = 0, dt = 1} x {rows 0..7, rows 8..15}; delta moves to the neighbouring image of a pair
__device__ __forceinline__ void img_rows_issue_at(const unsigned (&a)[4], unsigned delta, bf16x8 (&f)[4]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) asm volatile("ds_read_b128 %0, %1" : "=v"(f[ks]) : "v"(a[ks] + delta));
}
template <int KS2>
__device__ __forceinline__ void img_cols_tr_at(unsigned a0, unsigned a1, bf16x8& f) {
  union { u32x2 h[2]; bf16x8 v; } t;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(t.h[0]) : "v"(a0), "n"(KS2 * 16 * kImgRowBytes));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(t.h[1]) : "v"(a1), "n"(KS2 * 16 * kImgRowBytes + 8 * kImgRowBytes));
  f = t.v;
}
__device__ __forceinline__ f32x4v lds_read_f4(unsigned addr) {
  f32x4v r;
  asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"(addr));
  return r;
}

// A wave's [32 rows x 64] result (accumulator pair: feature rows, owned column) goes out through the wave's
// own 32 rows of an image that nobody reads any more: written as 8-byte pieces in the image layout, read back
// eight rows per instruction and stored as whole 128-byte lines (the direct form, 8 bytes per lane and
// instruction, touches every line sixteen times).  Only the wave itself touches these LDS rows, and LDS
// operations of a wave complete in order, so no barrier is involved.  tile_a = LDS address of the wave's row 0.
__device__ __forceinline__ void store_rows_staged(unsigned tile_a, const f32x16 (&acc)[2], float mul, bf16* __restrict__ gbase,
                                                  int64_t ld, int row0, int S, int lane) {
  asm volatile("" : "+v"(lane));   // recompute the addresses here: hoisted, they would occupy registers over the passes
  const int r = lane & 31, half = lane >> 5;
  if (row0 + r < S) {   // rows past the end may lie outside the image
    const unsigned wa = tile_a + r * kImgRowBytes + 8 * half;
    const unsigned f = img_swz(r);
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        union { bf16 h[4]; u32x2 u; } t;
#pragma unroll
        for (int e = 0; e < 4; ++e) t.h[e] = from_f32<bf16>(acc[dt][4 * g4 + e] * mul);
        asm volatile("ds_write_b64 %0, %1" ::"v"(wa + (((4 * dt + g4) ^ f) << 4)), "v"(t.u) : "memory");
      }
  }
  typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
  u32x4v d[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(d[j]) : "v"(tile_a + lane * 16), "n"(j * 1024) : "memory");
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    asm volatile("" : "+v"(d[j]));
    const int row = row0 + 8 * j + (lane >> 3);
    const int ch = (lane & 7) ^ img_swz(row);
    if (row < S) *reinterpret_cast<u32x4v*>(gbase + (int64_t)row * ld + 8 * ch) = d[j];
  }
}

__global__ __launch_bounds__(512) void attn_bwd_pipe_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ ctx,
                                                            const bf16* __restrict__ dctx, const float* __restrict__ lse,
                                                            bf16* __restrict__ dqkv, int S, int H, int ntile, int rows_pad,
                                                            int nheads) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int img_bytes = rows_pad * kImgRowBytes;
  float* ls = reinterpret_cast<float*>(smem + 6 * img_bytes + kImgPadBytes);   // row log-sum-exp in the log2 domain
  float* dls = ls + ntile * 32;                                                // row delta
  const int D = H * DH;
  const int tid = threadIdx.x, lane = tid & 63, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // one wave per 32 rows
  const int own = wave * 32 + (lane & 31);                     // the row this lane owns, as a query and as a key
  const bool ok = own < S;
  const int ownc = ok ? own : S - 1;
  const float scale = 0.125f, c = scale * 1.44269504088896f;
  // per-lane offsets inside a 32-row tile of an image
  const unsigned rb = (unsigned)((lane & 31) * kImgRowBytes + ((half ^ img_swz(lane & 31)) << 4));
  unsigned tr;
  {
    const int l16 = lane & 15, grp = lane >> 4;
    const int row = 4 * (grp >> 1) + (l16 >> 2), ch = 2 * (grp & 1) + ((l16 & 3) >> 1);
    tr = (unsigned)(row * kImgRowBytes + ((ch ^ img_swz(row)) << 4) + (l16 & 1) * 8);
  }
  const unsigned smem_a = lds_addr(smem);
  const unsigned ls_a = lds_addr(ls), dls_a = lds_addr(dls);
  const unsigned own_tile = wave * (32 * kImgRowBytes);   // the wave's own rows inside an image
  // A wave requests its own 32 rows of an image (four wave-wide loads of eight rows): rows [0, rows_pad) of
  // a [S, 64] matrix at src with row stride ld; rows past the end are copies of row S - 1.
  auto request_own = [&](int slot, const bf16* __restrict__ src, int ld) {
    int lane = tid & 63;
    asm volatile("" : "+v"(lane));   // recompute the addresses here: hoisted, they would occupy registers over the passes
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row0 = 32 * wave + 8 * j;
      if (row0 < rows_pad) {
        const int row = row0 + (lane >> 3);
        const int ch = (lane & 7) ^ img_swz(row);
        const int rc = row < S ? row : S - 1;
        __builtin_amdgcn_global_load_lds(PT_GLB(src + (int64_t)rc * ld + 8 * ch),
                                         PT_LDS(smem + slot * img_bytes + (4 * wave + j) * 1024), 16, 0, 0);
      }
    }
  };

  // zero the images and the pad once (see above); no load is in flight yet
  for (int i = tid; i < (6 * img_bytes + kImgPadBytes) / 16; i += blockDim.x)
    reinterpret_cast<uint4*>(smem)[i] = make_uint4(0, 0, 0, 0);
  __syncthreads();

  int head = blockIdx.x;
  if (head >= nheads) return;
  int pq = 0;   // pair of the current head's Q and dO images; K and V are in pair pq + 1, pair pq + 2 is free
  union Frag { uint4 u; bf16x8 v; };
  Frag of_[4];
  float lse_own;
  {
    const int b = head / H, h = head - b * H;
    const bf16* base = qkv + (int64_t)b * S * 3 * D + h * DH;
    request_own(0, base, 3 * D);
    request_own(1, dctx + (int64_t)b * S * D + h * DH, D);
    request_own(2, base + D, 3 * D);
    request_own(3, base + 2 * D, 3 * D);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      of_[ks].u = *reinterpret_cast<const uint4*>(ctx + ((int64_t)b * S + ownc) * D + h * DH + ks * 16 + half * 8);
    lse_own = lse[((int64_t)b * H + h) * S + ownc];
  }
  f32x16 dk[2], dv[2];       // the previous head's dK and dV wait here until its Q and dO images are free
  bf16* obase_prev = nullptr;

  for (;;) {
    const int b = head / H, h = head - b * H;
    bf16* obase = dqkv + (int64_t)b * S * 3 * D + h * DH;
    const int pk = pq == 2 ? 0 : pq + 1, pf = pk == 2 ? 0 : pk + 1;
    const unsigned q_a = smem_a + 2 * pq * img_bytes, do_a = q_a + img_bytes;
    const unsigned k_a = smem_a + 2 * pk * img_bytes, v_a = k_a + img_bytes;
    const unsigned f_a = smem_a + 2 * pf * img_bytes;
    const int next = head + gridDim.x;
    const bool has_next = next < nheads;
    const int nb_ = next / H, nh_ = next - nb_ * H;
    const bf16* nbase = qkv + (int64_t)nb_ * S * 3 * D + nh_ * DH;

    // ---- head start: the four images (and the lane's O row) have arrived ----
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();   // and nobody reads the previous head's Q and dO images (the free pair) any more
    asm volatile("" ::: "memory");
    if (obase_prev) {
      store_rows_staged(f_a + own_tile, dk, scale, obase_prev + D, 3 * D, 32 * wave, S, lane);
      store_rows_staged(f_a + img_bytes + own_tile, dv, 1.0f, obase_prev + 2 * D, 3 * D, 32 * wave, S, lane);
    }
    if (has_next) {
      request_own(2 * pf, nbase + D, 3 * D);
      request_own(2 * pf + 1, nbase + 2 * D, 3 * D);
    }
    bf16x8 qf[4], dof[4];
    img_rows_issue(q_a + own_tile, rb, qf);
    img_rows_issue(do_a + own_tile, rb, dof);
    lds_wait<0>(qf);
    lds_wait<0>(dof);
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int i = 0; i < 8; ++i) part += to_f32(dof[ks][i]) * to_f32(of_[ks].v[i]);
    const float dl = part + __shfl_xor(part, 32, 64);
    // a row past the end gets log-sum-exp +inf, hence probability exp2(-inf) = 0, and delta 0
    const float lq2 = ok ? lse_own * 1.44269504088896f : INFINITY;
    if (half == 0) {
      ls[own] = lq2;
      dls[own] = ok ? dl : 0.f;
    }

    // ---- pass 1: the wave's rows as queries ----
    f32x16 dq[2];
    {
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) dq[dt][v] = 0.f;
      // addresses of the current tile's fragments in the K image, advanced once per tile (V = K + one image)
      unsigned ka[4] = {k_a + rb, k_a + (rb ^ 32u), k_a + (rb ^ 64u), k_a + (rb ^ 96u)};
      unsigned kta[4] = {k_a + tr, k_a + (tr ^ 64u), k_a + (tr ^ 32u), k_a + (tr ^ 96u)};
      for (int kt = 0; kt < ntile; ++kt) {
        // The two waves of a SIMD take turns at the higher priority, tile by tile: with equal priorities the
        // older wave is served first throughout, finishes its pass early and leaves the younger one to run
        // the rest alone, one dependent instruction after the other.
        if ((kt ^ (wave >> 2)) & 1) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
        bf16x8 kr[4], vr[4], kc[4];
        img_rows_issue_at(ka, 0u, kr);
        img_rows_issue_at(ka, (unsigned)img_bytes, vr);
        f32x16 s, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
        lds_wait<4>(kr);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kr[ks], qf[ks], s, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int v = 0; v < 16; ++v) dp[v] = 0.f;
        lds_wait<0>(vr);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vr[ks], dof[ks], dp, 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        img_cols_tr_at<0>(kta[0], kta[2], kc[0]);
        img_cols_tr_at<0>(kta[1], kta[3], kc[1]);
        img_cols_tr_at<1>(kta[0], kta[2], kc[2]);
        img_cols_tr_at<1>(kta[1], kta[3], kc[3]);
#pragma unroll
        for (int i = 0; i < 4; ++i) { ka[i] += 32 * kImgRowBytes; kta[i] += 32 * kImgRowBytes; }
        if (kt == ntile - 1 && (S & 31)) {
#pragma unroll
          for (int v = 0; v < 16; ++v) s[v] = (kt * 32 + acc_row(v, half) < S) ? s[v] : -INFINITY;
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const float p = fast_exp2(fmaf(s[v], c, -lq2));
          s[v] = p * (dp[v] - dl);  // dS^T
        }
        lds_wait<0>(kc);
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          const bf16x8 dsb = pack8(s, 8 * ks2);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) dq[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kc[2 * ks2 + dt], dsb, dq[dt], 0, 0, 0);
        }
      }
    }

    // ---- pass 2: the wave's rows as keys ----
    bf16x8 kf[4], vf[4];
    img_rows_issue(k_a + own_tile, rb, kf);
    img_rows_issue(v_a + own_tile, rb, vf);
    lds_wait<0>(kf);
    lds_wait<0>(vf);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // ls / dls are written
    __builtin_amdgcn_s_barrier();                          // nobody reads this head's K and V images any more
    asm volatile("" ::: "memory");
    store_rows_staged(k_a + own_tile, dq, scale, obase, 3 * D, 32 * wave, S, lane);
    if (has_next) {
      request_own(2 * pk, nbase, 3 * D);
      request_own(2 * pk + 1, dctx + (int64_t)nb_ * S * D + nh_ * DH, D);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        of_[ks].u = *reinterpret_cast<const uint4*>(ctx + ((int64_t)nb_ * S + ownc) * D + nh_ * DH + ks * 16 + half * 8);
      lse_own = lse[((int64_t)nb_ * H + nh_) * S + ownc];
    }
    {
#pragma unroll
      for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) { dk[dt][v] = 0.f; dv[dt][v] = 0.f; }
      unsigned qa[4] = {q_a + rb, q_a + (rb ^ 32u), q_a + (rb ^ 64u), q_a + (rb ^ 96u)};   // dO = Q + one image
      unsigned qta[4] = {q_a + tr, q_a + (tr ^ 64u), q_a + (tr ^ 32u), q_a + (tr ^ 96u)};
      for (int qt = 0; qt < ntile; ++qt) {
        if ((qt ^ (wave >> 2)) & 1) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
        // The dO columns and the Q columns share four registers' worth of fragments each in turn, and the
        // rows' log-sum-exp and delta come in two at a time: the pass keeps 64 accumulator registers and the
        // wave's own K and V rows, and there must be room left for the next head's O row.
        bf16x8 qr[4], dor[4], tc[4];
        img_rows_issue_at(qa, 0u, qr);
        img_rows_issue_at(qa, (unsigned)img_bytes, dor);
        img_cols_tr_at<0>(qta[0] + img_bytes, qta[2] + img_bytes, tc[0]);
        img_cols_tr_at<0>(qta[1] + img_bytes, qta[3] + img_bytes, tc[1]);
        img_cols_tr_at<1>(qta[0] + img_bytes, qta[2] + img_bytes, tc[2]);
        img_cols_tr_at<1>(qta[1] + img_bytes, qta[3] + img_bytes, tc[3]);
        f32x16 s, dp;
#pragma unroll
        for (int v = 0; v < 16; ++v) { s[v] = 0.f; dp[v] = 0.f; }
        lds_wait<8>(qr);
        lds_wait<8>(dor);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qr[ks], kf[ks], s, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dor[ks], vf[ks], dp, 0, 0, 0);
        }
        f32x16 pr;
        const unsigned l_a = ls_a + (qt * 32 + 4 * half) * 4, d_a = dls_a + (qt * 32 + 4 * half) * 4;
        f32x4v lc = lds_read_f4(l_a), dc = lds_read_f4(d_a);
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          f32x4v ln = lc, dn = dc;
          if (g4 + 1 < 4) {
            ln = lds_read_f4(l_a + 32 * (g4 + 1));
            dn = lds_read_f4(d_a + 32 * (g4 + 1));
            asm volatile("s_waitcnt lgkmcnt(2)" ::: "memory");
          } else {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          }
          asm volatile("" : "+v"(lc), "+v"(dc));
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int v = 4 * g4 + e;
            const float p = fast_exp2(fmaf(s[v], c, -lc[e]));
            pr[v] = p;
            s[v] = p * (dp[v] - dc[e]);  // dS
          }
          lc = ln;
          dc = dn;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(tc[i]));   // everything issued so far has arrived
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          const bf16x8 pb = pack8(pr, 8 * ks2);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) dv[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tc[2 * ks2 + dt], pb, dv[dt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        img_cols_tr_at<0>(qta[0], qta[2], tc[0]);
        img_cols_tr_at<0>(qta[1], qta[3], tc[1]);
        img_cols_tr_at<1>(qta[0], qta[2], tc[2]);
        img_cols_tr_at<1>(qta[1], qta[3], tc[3]);
#pragma unroll
        for (int i = 0; i < 4; ++i) { qa[i] += 32 * kImgRowBytes; qta[i] += 32 * kImgRowBytes; }
        lds_wait<0>(tc);
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          const bf16x8 dsb = pack8(s, 8 * ks2);
#pragma unroll
          for (int dt = 0; dt < 2; ++dt) dk[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tc[2 * ks2 + dt], dsb, dk[dt], 0, 0, 0);
        }
      }
    }
    obase_prev = obase;
    if (!has_next) break;
    head = next;
    pq = pk;
  }
  // the last head's dK and dV: through its Q and dO images once every wave is done with them
  {
    const unsigned q_a = smem_a + 2 * pq * img_bytes;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    store_rows_staged(q_a + own_tile, dk, scale, obase_prev + D, 3 * D, 32 * wave, S, lane);
    store_rows_staged(q_a + img_bytes + own_tile, dv, 1.0f, obase_prev + 2 * D, 3 * D, 32 * wave, S, lane);
  }
}

// Sequence lengths the resident kernels take (the LDS image of two [S,64] matrices and two float rows must
// fit in 160 KB, i.e. S <= 512).  Measured: forward wins at S = 197 (25 vs 33 us per layer at ViT-B, batch
// 64) but loses at S = 384, where only one workgroup fits a CU (44 vs 39 us); backward wins at both.
constexpr int g_attn_resident_max_s = 224;
constexpr int g_attn_resident_max_s_bwd = 512;
constexpr int g_attn_fused_max_s_bwd = 256;   // four [S,64] images and two float rows in 160 KB, eight waves
#ifdef PT_TUNING_HOOKS   // stand-alone experiments only; the library is built without it
int g_attn_bwd_pipe = 1;
#else
constexpr int g_attn_bwd_pipe = 1;            // the pipelined fused backward where its six images fit (S <= 208)
#endif
struct ResPlan { int ntile, nw, nblk; size_t lds; };
ResPlan resident_plan(int S, bool with_rows) {
  ResPlan r;
  r.ntile = cdiv(S, 32);
  r.nblk = cdiv(r.ntile, 8);
  r.nw = cdiv(r.ntile, r.nblk);
  r.lds = (size_t)2 * r.ntile * 32 * LDR * sizeof(bf16) + (with_rows ? (size_t)2 * r.ntile * 32 * sizeof(float) : 0);
  return r;
}
// compute units of the current device (0 if the query fails); asked once per device
int device_cu_count() {
  static int count[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  if (count[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = 0;
    count[dev] = n > 0 ? n : -1;
  }
  return count[dev] > 0 ? count[dev] : 0;
}
template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

#ifdef PT_TUNING_HOOKS
void attention_set_bwd_pipe(int v) { g_attn_bwd_pipe = v; }
#endif
void attention_fwd_mfma(const void* qkv, void* ctx, float* lse, int nb, int S, int H, hipStream_t st) {
  if (S <= g_attn_resident_max_s) {
    const ResPlan r = resident_plan(S, false);
    if (allow_lds(attn_fwd_res_kernel, r.lds) == hipSuccess) {
      hipLaunchKernelGGL(attn_fwd_res_kernel, dim3(r.nblk, H, nb), dim3(64 * r.nw), r.lds, st, (const bf16*)qkv, (bf16*)ctx,
                         lse, S, H, r.ntile);
      return;
    }
    (void)hipGetLastError();
  }
  hipLaunchKernelGGL(attn_fwd_mfma_kernel, dim3(cdiv(S, 128), H, nb), dim3(256), 0, st, (const bf16*)qkv, (bf16*)ctx, lse,
                     S, H);
}
void attention_bwd_mfma(const void* qkv, const void* ctx, const void* dctx, const float* lse, void* dqkv, float* delta,
                        int nb, int S, int H, hipStream_t st) {
  {
    // The pipelined kernel where it pays: its six unpadded images, the pad and the two float rows must fit in
    // 160 KB (S <= 208); the fused kernel below must be down to one workgroup per CU (from 129 rows on: with
    // shorter sequences several of its workgroups share a CU and overlap each other's loads anyway; measured
    // 10.5 against 11.1 us at S = 128); and there must be more heads than CUs, or no workgroup has a next head.
    const int ntile = cdiv(S, 32), rows_pad = 16 * cdiv(S, 16);
    const size_t lds = (size_t)6 * rows_pad * kImgRowBytes + kImgPadBytes + (size_t)2 * ntile * 32 * sizeof(float);
    const int cus = device_cu_count();
    const int nheads = nb * H;
    if (g_attn_bwd_pipe && ntile >= 5 && ntile <= 8 && lds <= 160 * 1024 && cus > 0 && nheads > cus &&
        allow_lds(attn_bwd_pipe_kernel, lds) == hipSuccess) {
      hipLaunchKernelGGL(attn_bwd_pipe_kernel, dim3(nheads < cus ? nheads : cus), dim3(64 * ntile), lds, st,
                         (const bf16*)qkv, (const bf16*)ctx, (const bf16*)dctx, lse, (bf16*)dqkv, S, H, ntile, rows_pad,
                         nheads);
      return;
    }
    (void)hipGetLastError();
  }
  if (S <= g_attn_fused_max_s_bwd) {
    const int ntile = cdiv(S, 32);
    const size_t lds = (size_t)4 * ntile * 32 * LDR * sizeof(bf16) + (size_t)2 * ntile * 32 * sizeof(float);
    if (allow_lds(attn_bwd_fused_res_kernel, lds) == hipSuccess) {
      hipLaunchKernelGGL(attn_bwd_fused_res_kernel, dim3(H, nb), dim3(64 * ntile), lds, st, (const bf16*)qkv,
                         (const bf16*)ctx, (const bf16*)dctx, lse, (bf16*)dqkv, S, H, ntile);
      return;
    }
    (void)hipGetLastError();
  }
  if (S <= g_attn_resident_max_s_bwd) {
    const ResPlan r = resident_plan(S, false), r2 = resident_plan(S, true);
    if (allow_lds(attn_bwd_dq_res_kernel, r.lds) == hipSuccess && allow_lds(attn_bwd_dkv_res_kernel, r2.lds) == hipSuccess) {
      // one workgroup per CU (more than 80 KB of LDS) and more units than CUs: workgroups walk over units
      const int nunits = r.nblk * H * nb, cus = device_cu_count();
      const int upw = (r.lds > 80 * 1024 && cus > 0 && nunits > cus) ? cdiv(nunits, cus) : 1;
      hipLaunchKernelGGL(attn_bwd_dq_res_kernel, dim3(cdiv(nunits, upw)), dim3(64 * r.nw), r.lds, st, (const bf16*)qkv,
                         (const bf16*)ctx, (const bf16*)dctx, lse, (bf16*)dqkv, delta, S, H, r.ntile, r.nblk, upw, nunits);
      hipLaunchKernelGGL(attn_bwd_dkv_res_kernel, dim3(cdiv(nunits, upw)), dim3(64 * r2.nw), r2.lds, st, (const bf16*)qkv,
                         (const bf16*)dctx, lse, delta, (bf16*)dqkv, S, H, r2.ntile, r2.nblk, upw, nunits);
      return;
    }
    (void)hipGetLastError();
  }
  dim3 grid(cdiv(S, 128), H, nb);
  hipLaunchKernelGGL(attn_bwd_dq_mfma_kernel, grid, dim3(256), 0, st, (const bf16*)qkv, (const bf16*)ctx,
                     (const bf16*)dctx, lse, (bf16*)dqkv, delta, S, H);
  hipLaunchKernelGGL(attn_bwd_dkv_mfma_kernel, grid, dim3(256), 0, st, (const bf16*)qkv, (const bf16*)dctx, lse, delta,
                     (bf16*)dqkv, S, H);
}

}  // namespace pt
