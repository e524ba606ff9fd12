// Dense contractions of the encoder block: C = epilogue(A x B).
//
//  * gemm_mfma_kernel: bf16 inputs, fp32 accumulation on the gfx950 matrix
//    cores (v_mfma_f32_32x32x16_bf16), LDS-staged double-buffered tiles.  Both
//    operands may be stored with the contraction index contiguous ("k-major")
//    or strided; a strided operand is transposed in registers on its way from
//    HBM to LDS so the MFMA operand reads are always 16-byte LDS reads.
//  * gemm_generic_kernel: any element type, any strides and sizes, plain FMA.
//    Serves fp32 mode and the few small / unaligned products (task heads).
//
// The K loop runs in a fixed order and there is no split-K, so every output
// element is a deterministic function of its own row and column only.
#include "common.h"
#include "kernels.h"

namespace pt {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

template <typename T>
struct GemmDev {
  const T* A;
  const T* B;
  void* C;
  int M, N, K;
  int64_t lda, ldb, ldc;
  const T* bias;
  const T* aux;
  T* aux_out;
  int64_t ld_aux;
};

template <typename T, typename TC, int EPI>
__device__ __forceinline__ void epilogue_store(const GemmDev<T>& g, int row, int col, float acc) {
  float v = acc;
  if (EPI == EPI_BIAS || EPI == EPI_BIAS_RES || EPI == EPI_BIAS_GELU) v += to_f32(g.bias[col]);
  if (EPI == EPI_BIAS_RES) v += to_f32(g.aux[(int64_t)row * g.ld_aux + col]);
  if (EPI == EPI_RES) {  // an fp32 output adds the fp32 gradient stream
    if (sizeof(TC) == 4) v += reinterpret_cast<const float*>(g.aux)[(int64_t)row * g.ld_aux + col];
    else v += to_f32(g.aux[(int64_t)row * g.ld_aux + col]);
  }
  if (EPI == EPI_BIAS_GELU) {
    if (g.aux_out) g.aux_out[(int64_t)row * g.ld_aux + col] = from_f32<T>(v);  // pre-activation for the backward pass
    v = gelu_f(v);
  }
  if (EPI == EPI_MUL_DGELU) v *= dgelu_f(to_f32(g.aux[(int64_t)row * g.ld_aux + col]));
  reinterpret_cast<TC*>(g.C)[(int64_t)row * g.ldc + col] = from_f32<TC>(v);
}

// ---------------------------------------------------------------------------
// generic FMA kernel: 64x64 tile, 16-deep, 256 threads, 4x4 outputs per thread
// ---------------------------------------------------------------------------
template <typename T, typename TC, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmDev<T> g, int64_t a_sm, int64_t a_sk, int64_t b_sk,
                                                           int64_t b_sn) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < g.K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      int mm, kk;
      if (a_sk == 1) { kk = idx & 15; mm = idx >> 4; } else { mm = idx & 63; kk = idx >> 6; }
      const int gm = m0 + mm, gk = k0 + kk;
      As[kk][mm] = (gm < g.M && gk < g.K) ? to_f32(g.A[gm * a_sm + gk * a_sk]) : 0.f;
      int nn, kb;
      if (b_sk == 1) { kb = idx & 15; nn = idx >> 4; } else { nn = idx & 63; kb = idx >> 6; }
      const int gn = n0 + nn, gkb = k0 + kb;
      Bs[kb][nn] = (gn < g.N && gkb < g.K) ? to_f32(g.B[gkb * b_sk + gn * b_sn]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty * 4 + i;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx * 4 + j;
      if (col < g.N) epilogue_store<T, TC, EPI>(g, row, col, acc[i][j]);
    }
  }
}

// ---------------------------------------------------------------------------
// bf16 MFMA kernel: 128x128x32 tile, 4 waves (2x2), 64x64 per wave
// ---------------------------------------------------------------------------
constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDSK = BK + 8;  // 80-byte rows: 16-byte operand reads of 8 consecutive rows hit distinct banks

// Stage one 128 x 32 operand tile into 8 dwords per thread.
// k-major operand (element (r,k) at p[r*ld + k]): two 16-byte loads per thread.
__device__ __forceinline__ void load_kmajor(const bf16* p, int64_t ld, int R, int K, int r0, int k0, int tid,
                                            uint32_t (&reg)[8]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = tid + i * 256;
    const int row = c >> 2, kc = (c & 3) * 8;
    const int gr = r0 + row, gk = k0 + kc;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (gr < R && gk < K) v = *reinterpret_cast<const uint4*>(p + (int64_t)gr * ld + gk);
    reg[4 * i + 0] = v.x; reg[4 * i + 1] = v.y; reg[4 * i + 2] = v.z; reg[4 * i + 3] = v.w;
  }
}
__device__ __forceinline__ void store_kmajor(bf16* s, int tid, const uint32_t (&reg)[8]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = tid + i * 256;
    const int row = c >> 2, kc = (c & 3) * 8;
    *reinterpret_cast<uint4*>(s + row * LDSK + kc) = make_uint4(reg[4 * i], reg[4 * i + 1], reg[4 * i + 2], reg[4 * i + 3]);
  }
}
// strided operand (element (r,k) at p[k*ld + r]): each thread owns rows 2q,2q+1
// and eight consecutive k; eight 4-byte loads, 64 lanes cover 256 contiguous bytes.
__device__ __forceinline__ void load_strided(const bf16* p, int64_t ld, int R, int K, int r0, int k0, int tid,
                                             uint32_t (&reg)[8]) {
  const int q = tid & 63, kg = tid >> 6;
  const int gr = r0 + 2 * q;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int gk = k0 + kg * 8 + j;
    reg[j] = (gr < R && gk < K) ? *reinterpret_cast<const uint32_t*>(p + (int64_t)gk * ld + gr) : 0u;
  }
}
__device__ __forceinline__ void store_strided(bf16* s, int tid, const uint32_t (&reg)[8]) {
  const int q = tid & 63, kg = tid >> 6;
  uint4 even, odd;  // 2x2 transposes of 16-bit halves
  even.x = (reg[0] & 0xffffu) | (reg[1] << 16); odd.x = (reg[0] >> 16) | (reg[1] & 0xffff0000u);
  even.y = (reg[2] & 0xffffu) | (reg[3] << 16); odd.y = (reg[2] >> 16) | (reg[3] & 0xffff0000u);
  even.z = (reg[4] & 0xffffu) | (reg[5] << 16); odd.z = (reg[4] >> 16) | (reg[5] & 0xffff0000u);
  even.w = (reg[6] & 0xffffu) | (reg[7] << 16); odd.w = (reg[6] >> 16) | (reg[7] & 0xffff0000u);
  *reinterpret_cast<uint4*>(s + (2 * q) * LDSK + kg * 8) = even;
  *reinterpret_cast<uint4*>(s + (2 * q + 1) * LDSK + kg * 8) = odd;
}

template <bool TA, bool TB, int EPI, typename TC>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmDev<bf16> g) {
  __shared__ __attribute__((aligned(16))) bf16 As[2][BM * LDSK];
  __shared__ __attribute__((aligned(16))) bf16 Bs[2][BN * LDSK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint32_t ra[8], rb[8];
  auto gload = [&](int k0) {
    if (TA) load_strided(g.A, g.lda, g.M, g.K, m0, k0, tid, ra); else load_kmajor(g.A, g.lda, g.M, g.K, m0, k0, tid, ra);
    // B is "k-major" when stored [N,K] (tb), strided when stored [K,N]
    if (TB) load_kmajor(g.B, g.ldb, g.N, g.K, n0, k0, tid, rb); else load_strided(g.B, g.ldb, g.N, g.K, n0, k0, tid, rb);
  };
  auto sstore = [&](int buf) {
    if (TA) store_strided(As[buf], tid, ra); else store_kmajor(As[buf], tid, ra);
    if (TB) store_kmajor(Bs[buf], tid, rb); else store_strided(Bs[buf], tid, rb);
  };

  const int nk = (g.K + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  int cur = 0;
  for (int kt = 0; kt < nk; ++kt) {
    if (kt + 1 < nk) gload((kt + 1) * BK);
    const bf16* as = As[cur] + (wm * 64 + (lane & 31)) * LDSK + (lane >> 5) * 8;
    const bf16* bs = Bs[cur] + (wn * 64 + (lane & 31)) * LDSK + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDSK + ks * 16);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * LDSK + ks * 16);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(cur ^ 1);
    __syncthreads();
    cur ^= 1;
  }
  // accumulator layout of the 32x32 MFMA: lane holds column lane%32, rows 8*(v/4) + 4*(lane/32) + v%4
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int col = n0 + wn * 64 + j * 32 + (lane & 31);
      if (col >= g.N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (row < g.M) epilogue_store<bf16, TC, EPI>(g, row, col, acc[i][j][v]);
      }
    }
}

// ---------------------------------------------------------------------------
// dispatch
// ---------------------------------------------------------------------------
template <typename T, typename TC, int EPI>
static void launch_generic(const Gemm& a, hipStream_t st) {
  GemmDev<T> g{(const T*)a.A, (const T*)a.B, a.C, a.M, a.N, a.K, a.lda, a.ldb, a.ldc,
               (const T*)a.bias, (const T*)a.aux, (T*)a.aux_out, a.ld_aux};
  const int64_t a_sm = a.ta ? 1 : a.lda, a_sk = a.ta ? a.lda : 1;
  const int64_t b_sk = a.tb ? 1 : a.ldb, b_sn = a.tb ? a.ldb : 1;
  dim3 grid(cdiv(a.N, 64), cdiv(a.M, 64));
  hipLaunchKernelGGL((gemm_generic_kernel<T, TC, EPI>), grid, dim3(256), 0, st, g, a_sm, a_sk, b_sk, b_sn);
}

template <typename T, typename TC>
static void launch_generic_epi(const Gemm& a, hipStream_t st) {
  switch (a.epi) {
    case EPI_STORE: launch_generic<T, TC, EPI_STORE>(a, st); break;
    case EPI_BIAS: launch_generic<T, TC, EPI_BIAS>(a, st); break;
    case EPI_BIAS_RES: launch_generic<T, TC, EPI_BIAS_RES>(a, st); break;
    case EPI_BIAS_GELU: launch_generic<T, TC, EPI_BIAS_GELU>(a, st); break;
    case EPI_MUL_DGELU: launch_generic<T, TC, EPI_MUL_DGELU>(a, st); break;
    case EPI_RES: launch_generic<T, TC, EPI_RES>(a, st); break;
  }
}

template <bool TA, bool TB, typename TC>
static void launch_mfma_epi(const Gemm& a, hipStream_t st) {
  GemmDev<bf16> g{(const bf16*)a.A, (const bf16*)a.B, a.C, a.M, a.N, a.K, a.lda, a.ldb, a.ldc,
                  (const bf16*)a.bias, (const bf16*)a.aux, (bf16*)a.aux_out, a.ld_aux};
  dim3 grid(cdiv(a.N, BN), cdiv(a.M, BM));
  dim3 blk(256);
  if constexpr (sizeof(TC) == 4) {  // fp32 outputs: weight gradients, logits (+bias), gradient stream (+residual)
    if (a.epi == EPI_STORE) hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_STORE, TC>), grid, blk, 0, st, g);
    else if (a.epi == EPI_BIAS) hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_BIAS, TC>), grid, blk, 0, st, g);
    else if (a.epi == EPI_BIAS_RES) hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_BIAS_RES, TC>), grid, blk, 0, st, g);
    else hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_RES, TC>), grid, blk, 0, st, g);
    return;
  }
  switch (a.epi) {
    case EPI_STORE: hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_STORE, TC>), grid, blk, 0, st, g); break;
    case EPI_BIAS: hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_BIAS, TC>), grid, blk, 0, st, g); break;
    case EPI_BIAS_RES: hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_BIAS_RES, TC>), grid, blk, 0, st, g); break;
    case EPI_BIAS_GELU: hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_BIAS_GELU, TC>), grid, blk, 0, st, g); break;
    case EPI_MUL_DGELU: hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_MUL_DGELU, TC>), grid, blk, 0, st, g); break;
    case EPI_RES: hipLaunchKernelGGL((gemm_mfma_kernel<TA, TB, EPI_RES, TC>), grid, blk, 0, st, g); break;
  }
}

static bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// The MFMA path needs 16-byte vectors along k for k-major operands and 4-byte
// pairs along the row index for strided ones.
static bool mfma_ok(const Gemm& a) {
  const bool a_ok = a.ta ? (a.M % 2 == 0 && a.lda % 2 == 0 && aligned(a.A, 4))
                         : (a.K % 8 == 0 && a.lda % 8 == 0 && aligned(a.A, 16));
  const bool b_ok = a.tb ? (a.K % 8 == 0 && a.ldb % 8 == 0 && aligned(a.B, 16))
                         : (a.N % 2 == 0 && a.ldb % 2 == 0 && aligned(a.B, 4));
  return a_ok && b_ok && a.M >= 32 && a.N >= 32;
}

bool gemm_uses_mfma(int dt, const Gemm& a) { return dt != 0 && mfma_ok(a); }

void gemm(int dt, const Gemm& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return;
  if (a.c_f32 && (a.epi == EPI_BIAS_GELU || a.epi == EPI_MUL_DGELU)) return;  // not used by the step
  if (dt == 0) {
    launch_generic_epi<float, float>(a, st);
    return;
  }
  if (mfma_ok(a)) {
    if (a.c_f32) {
      if (!a.ta && !a.tb) launch_mfma_epi<false, false, float>(a, st);
      else if (!a.ta && a.tb) launch_mfma_epi<false, true, float>(a, st);
      else if (a.ta && !a.tb) launch_mfma_epi<true, false, float>(a, st);
      else launch_mfma_epi<true, true, float>(a, st);
    } else {
      if (!a.ta && !a.tb) launch_mfma_epi<false, false, bf16>(a, st);
      else if (!a.ta && a.tb) launch_mfma_epi<false, true, bf16>(a, st);
      else if (a.ta && !a.tb) launch_mfma_epi<true, false, bf16>(a, st);
      else launch_mfma_epi<true, true, bf16>(a, st);
    }
    return;
  }
  if (a.c_f32) launch_generic_epi<bf16, float>(a, st); else launch_generic_epi<bf16, bf16>(a, st);
}

}  // namespace pt
