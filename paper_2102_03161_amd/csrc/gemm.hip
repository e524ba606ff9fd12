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
#include <algorithm>
#include "common.h"
#include "kernels.h"
#include "gemm_epilogue.h"

namespace pt {

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
// bf16 MFMA kernel, tile shape given by Cfg
// ---------------------------------------------------------------------------
template <int BM_, int BN_, int BK_, int WGM_, int WGN_>
struct Cfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
  static constexpr int NT = 64 * WGM * WGN;          // threads
  static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // per-wave tile
  static constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 MFMA tiles per wave
  static constexpr int LDSK = BK + 8;  // padded rows: 16-byte operand reads of 8 consecutive rows hit distinct banks
  static constexpr int KC = BK / 8;    // 16-byte chunks per row
};

// Staging of one ROWS x BK operand tile in registers: NR dwords per thread.
// k-major operand (element (r,k) at p[r*ld + k]): 16-byte loads.
template <int ROWS, int BK, int NT>
struct KMajor {
  static constexpr int KC = BK / 8, CH = ROWS * KC / NT, NR = 4 * CH, LDSK = BK + 8;
  static_assert(ROWS * KC % NT == 0, "tile does not divide over the threads");
  static __device__ __forceinline__ void load(const bf16* p, int64_t ld, int R, int K, int r0, int k0, int tid,
                                              uint32_t (&reg)[NR]) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * NT;
      const int row = c / KC, kc = (c % KC) * 8;
      const int gr = r0 + row, gk = k0 + kc;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (gr < R && gk < K) v = *reinterpret_cast<const uint4*>(p + (int64_t)gr * ld + gk);
      reg[4 * i + 0] = v.x; reg[4 * i + 1] = v.y; reg[4 * i + 2] = v.z; reg[4 * i + 3] = v.w;
    }
  }
  static __device__ __forceinline__ void store(bf16* s, int tid, const uint32_t (&reg)[NR]) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int c = tid + i * NT;
      const int row = c / KC, kc = (c % KC) * 8;
      *reinterpret_cast<uint4*>(s + row * LDSK + kc) = make_uint4(reg[4 * i], reg[4 * i + 1], reg[4 * i + 2], reg[4 * i + 3]);
    }
  }
};
// strided operand (element (r,k) at p[k*ld + r]): a task owns rows 2q,2q+1 and eight consecutive k;
// eight 4-byte loads (64 lanes cover 256 contiguous bytes), 2x2 16-bit transposes, two 16-byte LDS writes.
template <int ROWS, int BK, int NT>
struct Strided {
  static constexpr int QN = ROWS / 2, TASKS = QN * (BK / 8), TP = TASKS / NT, NR = 8 * TP, LDSK = BK + 8;
  static_assert(TASKS % NT == 0, "tile does not divide over the threads");
  static __device__ __forceinline__ void load(const bf16* p, int64_t ld, int R, int K, int r0, int k0, int tid,
                                              uint32_t (&reg)[NR]) {
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      const int t = tid + i * NT;
      const int q = t % QN, kg = t / QN;
      const int gr = r0 + 2 * q;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int gk = k0 + kg * 8 + j;
        reg[8 * i + j] = (gr < R && gk < K) ? *reinterpret_cast<const uint32_t*>(p + (int64_t)gk * ld + gr) : 0u;
      }
    }
  }
  static __device__ __forceinline__ void store(bf16* s, int tid, const uint32_t (&reg)[NR]) {
#pragma unroll
    for (int i = 0; i < TP; ++i) {
      const int t = tid + i * NT;
      const int q = t % QN, kg = t / QN;
      const uint32_t* r = reg + 8 * i;
      uint4 even, odd;
      even.x = (r[0] & 0xffffu) | (r[1] << 16); odd.x = (r[0] >> 16) | (r[1] & 0xffff0000u);
      even.y = (r[2] & 0xffffu) | (r[3] << 16); odd.y = (r[2] >> 16) | (r[3] & 0xffff0000u);
      even.z = (r[4] & 0xffffu) | (r[5] << 16); odd.z = (r[4] >> 16) | (r[5] & 0xffff0000u);
      even.w = (r[6] & 0xffffu) | (r[7] << 16); odd.w = (r[6] >> 16) | (r[7] & 0xffff0000u);
      *reinterpret_cast<uint4*>(s + (2 * q) * LDSK + kg * 8) = even;
      *reinterpret_cast<uint4*>(s + (2 * q + 1) * LDSK + kg * 8) = odd;
    }
  }
  // column sums over k of the staged values: lo[i] += rows 2q, hi[i] += rows 2q+1
  static __device__ __forceinline__ void colsum(const uint32_t (&reg)[NR], float (&lo)[TP], float (&hi)[TP]) {
#pragma unroll
    for (int i = 0; i < TP; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        lo[i] += __uint_as_float(reg[8 * i + j] << 16);
        hi[i] += __uint_as_float(reg[8 * i + j] & 0xffff0000u);
      }
  }
};

template <bool T, int ROWS, int BK, int NT> struct LoaderSel { typedef KMajor<ROWS, BK, NT> type; };
template <int ROWS, int BK, int NT> struct LoaderSel<true, ROWS, BK, NT> { typedef Strided<ROWS, BK, NT> type; };

template <typename C, bool TA, bool TB, int EPI, typename TC>
__global__ __launch_bounds__(C::NT, 4) void gemm_mfma_kernel(GemmDev<bf16> g, SplitArgs sp, int tiles_n, int total_tiles,
                                                          int vec_ok) {
  typedef typename LoaderSel<TA, C::BM, C::BK, C::NT>::type LA;     // A strided when stored [K,M]
  typedef typename LoaderSel<!TB, C::BN, C::BK, C::NT>::type LB;    // B strided when stored [K,N]
  constexpr int LDSK = C::LDSK;
  constexpr int STAGE_LD = C::WTN + 4;
  constexpr int OPER_BYTES = 2 * (C::BM + C::BN) * LDSK * 2;
  constexpr int STAGE_BYTES = C::WGM * C::WGN * 32 * STAGE_LD * 4;
  constexpr int LDS_BYTES = OPER_BYTES > STAGE_BYTES ? OPER_BYTES : STAGE_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char lds[LDS_BYTES];
  bf16* As = reinterpret_cast<bf16*>(lds);                       // [2][BM*LDSK]
  bf16* Bs = As + 2 * C::BM * LDSK;                              // [2][BN*LDSK]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / C::WGN, wn = wave % C::WGN;
  // Workgroups go round-robin to the 8 XCDs, each with its own L2: give every XCD a contiguous
  // run of tiles (n fastest) so that tiles sharing an A row panel meet in one L2.
  const int per = (total_tiles + 7) >> 3;
  const int lin = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if (lin >= total_tiles) return;
  const int m0 = (lin / tiles_n) * C::BM, n0 = (lin % tiles_n) * C::BN;
  const int split = blockIdx.z;

  f32x16 acc[C::TM][C::TN];
#pragma unroll
  for (int i = 0; i < C::TM; ++i)
#pragma unroll
    for (int j = 0; j < C::TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  uint32_t ra[LA::NR], rb[LB::NR];
  constexpr int CSN = TB ? 1 : LB::NR / 8;
  float cs_lo[CSN], cs_hi[CSN];
#pragma unroll
  for (int i = 0; i < CSN; ++i) { cs_lo[i] = 0.f; cs_hi[i] = 0.f; }
  const bool do_colsum = !TB && sp.colsum != nullptr && m0 == 0;

  const int nk_all = (g.K + C::BK - 1) / C::BK;
  const int kt0 = split * sp.tiles_per_split;
  const int kt1 = (kt0 + sp.tiles_per_split < nk_all) ? kt0 + sp.tiles_per_split : nk_all;

  auto gload = [&](int kt) {
    LA::load(g.A, g.lda, g.M, g.K, m0, kt * C::BK, tid, ra);
    LB::load(g.B, g.ldb, g.N, g.K, n0, kt * C::BK, tid, rb);
    if constexpr (!TB) {
      if (do_colsum) LB::colsum(rb, cs_lo, cs_hi);
    }
  };
  auto sstore = [&](int buf) {
    LA::store(As + buf * C::BM * LDSK, tid, ra);
    LB::store(Bs + buf * C::BN * LDSK, tid, rb);
  };

  if (kt0 < kt1) {
    gload(kt0);
    sstore(0);
  }
  __syncthreads();
  int cur = 0;
  for (int kt = kt0; kt < kt1; ++kt) {
    if (kt + 1 < kt1) gload(kt + 1);
    const bf16* as = As + cur * C::BM * LDSK + (wm * C::WTM + (lane & 31)) * LDSK + (lane >> 5) * 8;
    const bf16* bs = Bs + cur * C::BN * LDSK + (wn * C::WTN + (lane & 31)) * LDSK + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < C::BK / 16; ++ks) {
      bf16x8 a[C::TM], b[C::TN];
#pragma unroll
      for (int i = 0; i < C::TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDSK + ks * 16);
#pragma unroll
      for (int j = 0; j < C::TN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * LDSK + ks * 16);
#pragma unroll
      for (int i = 0; i < C::TM; ++i)
#pragma unroll
        for (int j = 0; j < C::TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < kt1) sstore(cur ^ 1);
    __syncthreads();
    cur ^= 1;
  }

  // ---- column sums of B (bias gradient riding on the weight-gradient product) ----
  if constexpr (!TB) {
    if (do_colsum) {  // uniform over the workgroup; the main loop ended with a barrier
      float* red = reinterpret_cast<float*>(lds);  // [BK/8][BN]
#pragma unroll
      for (int i = 0; i < CSN; ++i) {
        const int t = tid + i * C::NT;
        const int q = t % (C::BN / 2), kg = t / (C::BN / 2);
        red[kg * C::BN + 2 * q] = cs_lo[i];
        red[kg * C::BN + 2 * q + 1] = cs_hi[i];
      }
      __syncthreads();
      for (int n = tid; n < C::BN; n += C::NT) {
        float s = 0.f;
#pragma unroll
        for (int kg = 0; kg < C::BK / 8; ++kg) s += red[kg * C::BN + n];
        if (n0 + n < g.N) sp.colsum[(int64_t)split * g.N + n0 + n] = s;
      }
      __syncthreads();
    }
  }

  void* Cbase = sizeof(TC) == 4 ? (void*)(reinterpret_cast<float*>(g.C) + split * sp.slab)
                                : (void*)(reinterpret_cast<bf16*>(g.C) + split * sp.slab);
  // one operand buffer: this kernel lives on having four small workgroups per CU
  staged_epilogue<C::TM, C::TN, C::WTM, C::WTN, EPI, TC, 1>(g, Cbase, acc, reinterpret_cast<float*>(lds) + wave * 32 * STAGE_LD,
                                                            m0 + wm * C::WTM, n0 + wn * C::WTN, lane, vec_ok);
}

// A second, short vector (the column-sum partials of the same product) may ride along in the last workgroups.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int splits, int64_t n,
                                                            float* __restrict__ out, int vec, int blocks_main,
                                                            const float* __restrict__ part2, int64_t n2,
                                                            float* __restrict__ out2, int vec2) {
  if ((int)blockIdx.x < blocks_main) {
    splitk_sum4(part, splits, n, out, vec, ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4);
  } else {
    const int64_t i = ((int64_t)(blockIdx.x - blocks_main) * 256 + threadIdx.x) * 4;
    if (i < n2) splitk_sum4(part2, splits, n2, out2, vec2, i);
  }
}

int splitk_vec_ok4(const float* part, int64_t n, const float* out) {
  return (n % 4 == 0 && (reinterpret_cast<uintptr_t>(part) % 16) == 0 && (reinterpret_cast<uintptr_t>(out) % 16) == 0) ? 1 : 0;
}
static int vec_ok4(const float* part, int64_t n, const float* out) { return splitk_vec_ok4(part, n, out); }
void gemm_splitk_reduce(const float* part, int splits, int64_t n, float* out, const float* part2, int64_t n2, float* out2,
                        hipStream_t st) {
  const int blocks_main = (int)cdiv64(n, 1024);
  const int blocks2 = part2 ? (int)cdiv64(n2, 1024) : 0;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)(blocks_main + blocks2)), dim3(256), 0, st, part, splits, n, out,
                     vec_ok4(part, n, out), blocks_main, part2, part2 ? n2 : 0, out2, part2 ? vec_ok4(part2, n2, out2) : 0);
}

// the reductions of up to four products in one launch (same split count)
struct ReduceGroup {
  const float* part[4]; float* out[4]; int64_t n[4]; int vec[4];
  const float* part2[4]; float* out2[4]; int64_t n2[4]; int vec2[4];
  int block0[5];      // first workgroup of each product
  int blocks_main[4];
  int nprob, splits;
};
__global__ __launch_bounds__(256) void splitk_reduce_group_kernel(ReduceGroup rg) {
  int p = 0;
  while (p + 1 < rg.nprob && (int)blockIdx.x >= rg.block0[p + 1]) ++p;
  const int b = (int)blockIdx.x - rg.block0[p];
  if (b < rg.blocks_main[p]) {
    splitk_sum4(rg.part[p], rg.splits, rg.n[p], rg.out[p], rg.vec[p], ((int64_t)b * 256 + threadIdx.x) * 4);
  } else {
    const int64_t i = ((int64_t)(b - rg.blocks_main[p]) * 256 + threadIdx.x) * 4;
    if (i < rg.n2[p]) splitk_sum4(rg.part2[p], rg.splits, rg.n2[p], rg.out2[p], rg.vec2[p], i);
  }
}
void gemm_splitk_reduce_group(int nprob, int splits, const float* const* part, const int64_t* n, float* const* out,
                              const float* const* part2, const int64_t* n2, float* const* out2, hipStream_t st) {
  ReduceGroup rg{};
  rg.nprob = nprob;
  rg.splits = splits;
  int b0 = 0;
  for (int i = 0; i < nprob; ++i) {
    rg.part[i] = part[i]; rg.out[i] = out[i]; rg.n[i] = n[i]; rg.vec[i] = vec_ok4(part[i], n[i], out[i]);
    rg.part2[i] = part2[i]; rg.out2[i] = out2[i]; rg.n2[i] = part2[i] ? n2[i] : 0;
    rg.vec2[i] = part2[i] ? vec_ok4(part2[i], n2[i], out2[i]) : 0;
    rg.block0[i] = b0;
    rg.blocks_main[i] = (int)cdiv64(n[i], 1024);
    b0 += rg.blocks_main[i] + (part2[i] ? (int)cdiv64(n2[i], 1024) : 0);
  }
  rg.block0[nprob] = b0;
  hipLaunchKernelGGL(splitk_reduce_group_kernel, dim3((unsigned)b0), dim3(256), 0, st, rg);
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
// whether (layout, epilogue, output type) is one of the combinations the training step uses
static bool combo_used(const Gemm& a) {
  if (a.ta && a.tb) return false;
  if (a.ta) return a.c_f32 && a.epi == EPI_STORE;                                             // weight gradient
  if (a.tb) return a.c_f32 ? (a.epi == EPI_RES) : (a.epi == EPI_STORE || a.epi == EPI_MUL_DGELU);  // input gradient
  return a.c_f32 ? (a.epi == EPI_BIAS || a.epi == EPI_BIAS_RES)                                 // forward
                 : (a.epi == EPI_BIAS || a.epi == EPI_BIAS_RES || a.epi == EPI_BIAS_GELU);
}
// 16-byte epilogue accesses need 8-element alignment of everything the epilogue touches
bool gemm_epilogue_vec_ok(const Gemm& a) {
  bool ok = a.N % 8 == 0 && a.ldc % 8 == 0 && aligned(a.C, 16);
  if (a.bias) ok = ok && aligned(a.bias, 16);
  if (a.aux) ok = ok && a.ld_aux % 8 == 0 && aligned(a.aux, 16);
  if (a.aux_out) ok = ok && a.ld_aux % 8 == 0 && aligned(a.aux_out, 16);
  return ok;
}

bool gemm_uses_mfma(int dt, const Gemm& a) { return dt != 0 && mfma_ok(a) && combo_used(a); }

typedef Cfg<128, 128, 32, 2, 2> Cfg0;

// kernel selection; -1 = choose by problem shape.  0: register-staged kernel; 10 + v: variant v of
// the asynchronous global->LDS kernel (tuning hook for experiments)
#ifdef PT_TUNING_HOOKS   // stand-alone experiments only; the library is built without it
static int g_cfg_override = -1;
void gemm_set_config(int c) { g_cfg_override = c; }
#else
constexpr int g_cfg_override = -1;
#endif

template <typename C, bool TA, bool TB, int EPI, typename TC>
static void launch_mfma(const Gemm& a, int splits, float* cbase, int64_t slab, float* colsum_part, hipStream_t st) {
  GemmDev<bf16> g{(const bf16*)a.A, (const bf16*)a.B, cbase ? (void*)cbase : a.C, a.M, a.N, a.K, a.lda, a.ldb, a.ldc,
                  (const bf16*)a.bias, (const bf16*)a.aux, (bf16*)a.aux_out, a.ld_aux};
  const int tiles_m = cdiv(a.M, C::BM), tiles_n = cdiv(a.N, C::BN), total = tiles_m * tiles_n;
  const int nk = cdiv(a.K, C::BK);
  SplitArgs sp{splits, cdiv(nk, splits), slab, colsum_part};
  dim3 grid(8 * cdiv(total, 8), 1, splits);
  hipLaunchKernelGGL((gemm_mfma_kernel<C, TA, TB, EPI, TC>), grid, dim3(C::NT), 0, st, g, sp, tiles_n, total,
                     gemm_epilogue_vec_ok(a) ? 1 : 0);
}

template <typename C>
static void dispatch_mfma(const Gemm& a, hipStream_t st) {
  if (a.ta) {
    // weight gradient: few output tiles and a long contraction -> split K over grid.z into fp32
    // slabs, then add the slabs in a fixed order; the bias gradient rides along as column sums of B.
    const int tiles = cdiv(a.M, C::BM) * cdiv(a.N, C::BN), nk = cdiv(a.K, C::BK);
    int splits = 1;
    const int64_t mn = (int64_t)a.M * a.N;
    if (a.ws) {
      splits = 768 / tiles;
      if (splits < 1) splits = 1;
      if (splits > nk / 8) splits = nk / 8;
      if (splits > 16) splits = 16;
      while (splits > 1 && (size_t)(splits * (mn + a.N)) > a.ws_floats) --splits;
      if (splits < 1) splits = 1;
    }
    float* cs_part = nullptr;
    if (a.colsum_out) cs_part = splits > 1 ? a.ws + splits * mn : a.colsum_out;
    if (splits > 1) {
      launch_mfma<C, true, false, EPI_STORE, float>(a, splits, a.ws, mn, cs_part, st);
      // ldc == N is required for the slab layout
      gemm_splitk_reduce(a.ws, splits, mn, (float*)a.C, a.colsum_out ? cs_part : nullptr, a.N, a.colsum_out, st);
    } else {
      launch_mfma<C, true, false, EPI_STORE, float>(a, 1, nullptr, 0, cs_part, st);
    }
    return;
  }
  if (a.tb) {
    if (a.c_f32) launch_mfma<C, false, true, EPI_RES, float>(a, 1, nullptr, 0, nullptr, st);
    else if (a.epi == EPI_STORE) launch_mfma<C, false, true, EPI_STORE, bf16>(a, 1, nullptr, 0, nullptr, st);
    else launch_mfma<C, false, true, EPI_MUL_DGELU, bf16>(a, 1, nullptr, 0, nullptr, st);
    return;
  }
  if (a.c_f32) {
    if (a.epi == EPI_BIAS) launch_mfma<C, false, false, EPI_BIAS, float>(a, 1, nullptr, 0, nullptr, st);
    else launch_mfma<C, false, false, EPI_BIAS_RES, float>(a, 1, nullptr, 0, nullptr, st);
  } else {
    if (a.epi == EPI_BIAS) launch_mfma<C, false, false, EPI_BIAS, bf16>(a, 1, nullptr, 0, nullptr, st);
    else if (a.epi == EPI_BIAS_RES) launch_mfma<C, false, false, EPI_BIAS_RES, bf16>(a, 1, nullptr, 0, nullptr, st);
    else launch_mfma<C, false, false, EPI_BIAS_GELU, bf16>(a, 1, nullptr, 0, nullptr, st);
  }
}

void gemm(int dt, const Gemm& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return;
  if (a.c_f32 && (a.epi == EPI_BIAS_GELU || a.epi == EPI_MUL_DGELU)) return;  // not used by the step
  if (gemm_uses_mfma(dt, a) && (!a.ta || a.ldc == a.N)) {
    if (g_cfg_override != 0 && gemm_dma_ok(a)) {
      // Weight gradients: 256x128 tiles (128x128 for small outputs), split over K.
      // Forward and input-gradient products with at least 4096 rows and K a multiple of 64: the two-group
      // kernel with 256x256 or 192x256 tiles, one workgroup per CU, whichever fills whole rounds of 256
      // CUs better (M = 12608, N = 768: 198 tiles of 192x256 against 150 of 256x256); wide outputs with
      // a short K do better with 256x128 tiles, two workgroups per CU, whose prologues and epilogues
      // overlap.  Everything else, and products whose large tiles would leave many CUs idle: 128x128 tiles,
      // three per CU.
      if (g_cfg_override < 0 && gemm_dma_skinny(a, st)) return;
      int v = g_cfg_override >= 10 ? g_cfg_override - 10 : 1;
      if (g_cfg_override < 0) {
        v = (a.ta || a.N >= 3072) ? 2 : 1;
        if (a.ta && (int64_t)a.M * a.N <= 1024 * 1024) v = 1;
        if (!a.ta && a.M >= 4096 && a.K % 64 == 0) {
          const int tn = cdiv(a.N, 256);
          const int t192 = cdiv(a.M, 192) * tn, t256 = cdiv(a.M, 256) * tn;
          if (a.N >= 3072 && (a.K < 1024 || a.tb)) {
            // wide and short: 192-row tiles only when their last round of 256 is (nearly) full, as for the
            // 12288 tokens of BERT-base (768 tiles at N = 3072; 9-10 % faster than 256x128 there)
            const int last = t192 % 256;
            if (last == 0 || last >= 224) v = 6;
          } else {
            v = cdiv(t192, 256) * 192 < cdiv(t256, 256) * 256 ? 6 : 5;
            // fewer tiles than 60 % of the CUs of their rounds (8192 tokens at N = 768: 129 tiles): 128x128 tiles,
            // three workgroups per CU, fill the chip better (6-13 % faster on those five products)
            const int tiles = v == 6 ? t192 : t256;
            if (tiles * 10 < cdiv(tiles, 256) * 256 * 6) v = 1;
          }
        }
      }
      gemm_dma(a, v, st);
      return;
    }
    dispatch_mfma<Cfg0>(a, st);
    return;
  }
  if (dt == 0) launch_generic_epi<float, float>(a, st);
  else if (a.c_f32) launch_generic_epi<bf16, float>(a, st);
  else launch_generic_epi<bf16, bf16>(a, st);
  // column sums of B requested alongside a weight gradient: separate pass on this path
  if (a.colsum_out && a.ta && !a.tb && a.ws) colsum(dt, a.B, a.ldb, a.K, a.N, a.colsum_out, a.ws, st);
}

void gemm_wgrad_flush(WgradCarry* carry, hipStream_t st) {
  if (!carry || carry->nprob <= 0) return;
  gemm_splitk_reduce_group(carry->nprob, carry->splits, carry->part, carry->n, carry->out, carry->part2, carry->n2,
                           carry->out2, st);
  carry->nprob = 0;
}

void gemm_wgrad_batch(int dt, const Gemm* g, int n, hipStream_t st, hipEvent_t mid, WgradCarry* carry, LnBwdRide* ln) {
  if (ln) ln->taken_np = 0;
  if (n <= 0) return;
  bool mfma = dt != 0 && g_cfg_override != 0;
  for (int i = 0; i < n && mfma; ++i) mfma = gemm_uses_mfma(dt, g[i]);
  // one product alone goes to the grouped kernel too when its contraction is long (the tokens of a batch)
  if (mfma && (n > 1 || g[0].K >= 2048) && gemm_wgrad_group(g, n, st, mid, carry, ln)) return;
  gemm_wgrad_flush(carry, st);
  for (int i = 0; i < n; ++i) gemm(dt, g[i], st);
  if (mid) (void)hipEventRecord(mid, st);
}

size_t gemm_wgrad_batch_ws_floats(int D, int F) {
  const int64_t shapes[4][2] = {{D, 3 * D}, {D, D}, {D, F}, {F, D}};
  int64_t tiles = 0, per_split = 0;
  for (auto& sh : shapes) {
    tiles += ((sh[0] + 255) / 256) * ((sh[1] + 255) / 256);
    per_split += sh[0] * sh[1] + sh[1];
  }
  const int64_t splits = std::min<int64_t>(16, std::max<int64_t>(1, 256 / std::max<int64_t>(tiles, 1)));
  return (size_t)(splits * per_split);
}

}  // namespace pt
