// Pieces shared by the matrix-core GEMM kernels: the device-side problem
// descriptor, the fused epilogues, and the LDS-staged store path.
#pragma once
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
    // what the backward pass needs of the pre-activation is GELU'(h): it is stored instead of h, so that the
    // input-gradient epilogue is one multiplication and the exponential is evaluated once per element
    float dg;
    v = gelu_both(v, &dg);
    if (g.aux_out) g.aux_out[(int64_t)row * g.ld_aux + col] = from_f32<T>(dg);
  }
  if (EPI == EPI_MUL_DGELU) v *= to_f32(g.aux[(int64_t)row * g.ld_aux + col]);   // aux = GELU'(h) saved by the forward
  reinterpret_cast<TC*>(g.C)[(int64_t)row * g.ldc + col] = from_f32<TC>(v);
}

struct SplitArgs {
  int splits;         // grid.z; each split owns a contiguous range of k tiles and its own output slab
  int tiles_per_split;
  int64_t slab;       // elements between the output slabs of consecutive splits
  float* colsum;      // [splits][N] column sums of B over the split's k range (TB == false only), or null
};

typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));   // operand type of the nontemporal builtins

// What an 8-column chunk of one output row reads besides the accumulators: the residual / saved GELU'(h) in
// bf16 (one 16-byte load) or the fp32 gradient stream (two).  Loading is separate from applying so that the
// loads of a whole 32-row block can be in flight before the first of them is needed.
template <int EPI, typename TC>
struct Aux8 {
  static constexpr bool BF = EPI == EPI_BIAS_RES || (EPI == EPI_RES && sizeof(TC) == 2) || EPI == EPI_MUL_DGELU;
  static constexpr bool F32 = EPI == EPI_RES && sizeof(TC) == 4;
  union { uint4 u; u32x4_nt v; bf16 h[8]; float f[4]; } r[F32 ? 2 : 1];
  __device__ __forceinline__ void load(const GemmDev<bf16>& g, int row, int col) {
    if (BF) {
      const bf16* ap = g.aux + (int64_t)row * g.ld_aux + col;
      // the saved GELU'(h) is read exactly once, here: past the caches; a residual input was just written
      if (EPI == EPI_MUL_DGELU) r[0].v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt*>(ap));
      else r[0].u = *reinterpret_cast<const uint4*>(ap);
    }
    if (F32) {
      const float* ap = reinterpret_cast<const float*>(g.aux) + (int64_t)row * g.ld_aux + col;
      r[0].u = *reinterpret_cast<const uint4*>(ap);
      r[F32 ? 1 : 0].u = *reinterpret_cast<const uint4*>(ap + 4);
    }
  }
  __device__ __forceinline__ void apply(float (&v)[8]) const {
    if (BF) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (EPI == EPI_MUL_DGELU) v[e] *= to_f32(r[0].h[e]); else v[e] += to_f32(r[0].h[e]);
      }
    }
    if (F32) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += r[F32 ? e >> 2 : 0].f[e & 3];
    }
  }
};

// the bias of 8 consecutive columns
template <int EPI>
struct Bias8 {
  static constexpr bool ON = EPI == EPI_BIAS || EPI == EPI_BIAS_RES || EPI == EPI_BIAS_GELU;
  union { uint4 u; bf16 h[8]; } b;
  __device__ __forceinline__ void load(const GemmDev<bf16>& g, int col) {
    if (ON) b.u = *reinterpret_cast<const uint4*>(g.bias + col);
  }
  __device__ __forceinline__ void apply(float (&v)[8]) const {
    if (ON) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += to_f32(b.h[e]);
    }
  }
};

// 8 consecutive output columns of one row, bias and auxiliary operand already in registers: epilogue math
// and 16-byte stores
template <int EPI, typename TC>
__device__ __forceinline__ void epilogue_finish8(const GemmDev<bf16>& g, void* Cbase, int row, int col, float (&v)[8],
                                                 const Bias8<EPI>& bias, const Aux8<EPI, TC>& aux) {
  bias.apply(v);
  aux.apply(v);
  if (EPI == EPI_BIAS_GELU) {
    float dg[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = gelu_both(v[e], &dg[e]);
    if (g.aux_out) {
      union { uint4 u; bf16 h[8]; } o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o.h[e] = from_f32<bf16>(dg[e]);
      // GELU'(h) is read again only in the backward pass: written past the caches
      union { uint4 u; u32x4_nt v; } nt;
      nt.u = o.u;
      __builtin_nontemporal_store(nt.v, reinterpret_cast<u32x4_nt*>(g.aux_out + (int64_t)row * g.ld_aux + col));
    }
  }
  if (sizeof(TC) == 4) {
    float* c = reinterpret_cast<float*>(Cbase) + (int64_t)row * g.ldc + col;
    *reinterpret_cast<float4*>(c) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(c + 4) = make_float4(v[4], v[5], v[6], v[7]);
  } else {
    union { uint4 u; bf16 h[8]; } o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o.h[e] = from_f32<bf16>(v[e]);
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16*>(Cbase) + (int64_t)row * g.ldc + col) = o.u;
  }
}

template <int EPI, typename TC>
__device__ __forceinline__ void epilogue_store8(const GemmDev<bf16>& g, void* Cbase, int row, int col, float (&v)[8]) {
  Bias8<EPI> bias;
  Aux8<EPI, TC> aux;
  bias.load(g, col);
  aux.load(g, row, col);
  epilogue_finish8<EPI, TC>(g, Cbase, row, col, v, bias, aux);
}

// Accumulators of one wave (TM x TN tiles of 32x32) -> per-wave LDS staging -> 16-byte row-contiguous
// stores with the epilogue applied.  `stage` is this wave's private 32 x (WTN+4) float area; (row0, col0)
// is the wave tile's origin in C.  A wave reads back only what it wrote itself, so no workgroup barrier
// is needed (LDS operations of one wave complete in order); the wave barriers only stop the compiler
// from moving accesses across them.
// A wave tile that lies wholly inside C (all but the last tile row or column) takes a path without
// branches: the auxiliary loads of the next 32-row block are issued while the current block is staged, and
// stores are never waited for.  With the bounds checks in the loop every 8-row pass became a chain of
// store-acknowledge wait, LDS read, auxiliary load, wait, store (8.5 us of a 34 us workgroup for the
// 256x128 GELU tiles, 11.4 us for the tiles that multiply by the saved GELU').
// accumulator layout of the 32x32 MFMA: lane holds column lane%32, rows 8*(v/4) + 4*(lane/32) + v%4
// NBUF = 2 keeps two blocks' operands in registers (the next one loading while this one is used); NBUF = 1
// loads each block's operand while that block is staged, for kernels with no registers to spare.
template <int TM, int TN, int WTM, int WTN, int EPI, typename TC, int NBUF = 2>
__device__ __forceinline__ void staged_epilogue(const GemmDev<bf16>& g, void* Cbase, const f32x16 (&acc)[TM][TN],
                                                float* stage, int row0, int col0, int lane, int vec_ok) {
  constexpr int STAGE_LD = WTN + 4;
  constexpr int CPR = WTN / 8;   // 8-column chunks per row of the wave tile
  constexpr int RPP = 64 / CPR;  // rows per pass
  constexpr int NP = 32 / RPP;   // passes per 32-row block
  const int cc = (lane % CPR) * 8, rl = lane / CPR;
  const bool interior =
      __builtin_amdgcn_readfirstlane(vec_ok && row0 + TM * 32 <= g.M && col0 + WTN <= g.N ? 1 : 0) != 0;
  Bias8<EPI> bias;
  Aux8<EPI, TC> aux[NBUF][NP];
  if (interior) {
    bias.load(g, col0 + cc);
    if (NBUF == 2) {
#pragma unroll
      for (int pss = 0; pss < NP; ++pss) aux[0][pss].load(g, row0 + pss * RPP + rl, col0 + cc);
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        stage[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * STAGE_LD + j * 32 + (lane & 31)] = acc[i][j][v];
    // the next block's operand takes the registers that this block's accumulators have just left
    if (interior && NBUF == 2 && i + 1 < TM) {
#pragma unroll
      for (int pss = 0; pss < NP; ++pss) aux[(i + 1) & 1][pss].load(g, row0 + (i + 1) * 32 + pss * RPP + rl, col0 + cc);
    }
    if (interior && NBUF == 1) {
#pragma unroll
      for (int pss = 0; pss < NP; ++pss) aux[0][pss].load(g, row0 + i * 32 + pss * RPP + rl, col0 + cc);
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int pss = 0; pss < NP; ++pss) {
      const int r = pss * RPP + rl;
      const int row = row0 + i * 32 + r, col = col0 + cc;
      float v8[8];
      const float4 x0 = *reinterpret_cast<const float4*>(stage + r * STAGE_LD + cc);
      const float4 x1 = *reinterpret_cast<const float4*>(stage + r * STAGE_LD + cc + 4);
      v8[0] = x0.x; v8[1] = x0.y; v8[2] = x0.z; v8[3] = x0.w; v8[4] = x1.x; v8[5] = x1.y; v8[6] = x1.z; v8[7] = x1.w;
      if (interior) {
        epilogue_finish8<EPI, TC>(g, Cbase, row, col, v8, bias, aux[NBUF == 2 ? i & 1 : 0][pss]);
      } else if (row < g.M && col < g.N) {
        if (vec_ok && col + 8 <= g.N) {
          epilogue_store8<EPI, TC>(g, Cbase, row, col, v8);
        } else {
          GemmDev<bf16> gs = g;
          gs.C = Cbase;
          for (int e = 0; e < 8 && col + e < g.N; ++e) epilogue_store<bf16, TC, EPI>(gs, row, col + e, v8[e]);
        }
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

typedef float f32x4_st __attribute__((ext_vector_type(4)));   // operand type of the nontemporal store builtin
// out[i] = sum over splits of part[z][i], z in increasing order (4 floats per thread).
__device__ __forceinline__ void splitk_sum4(const float* __restrict__ part, int splits, int64_t n, float* __restrict__ out,
                                            int vec, int64_t i) {
  if (vec && i + 3 < n) {
    float4 s = *reinterpret_cast<const float4*>(part + i);
    for (int z = 1; z < splits; ++z) {
      const float4 t = *reinterpret_cast<const float4*>(part + (int64_t)z * n + i);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    // a weight gradient is next read by the norm and update passes, after the rest of the backward pass
    // has gone through the caches: stored past them
    f32x4_st o; o.x = s.x; o.y = s.y; o.z = s.z; o.w = s.w;
    __builtin_nontemporal_store(o, reinterpret_cast<f32x4_st*>(out + i));
  } else {
    for (int64_t j = i; j < n && j < i + 4; ++j) {
      float s = part[j];
      for (int z = 1; z < splits; ++z) s += part[(int64_t)z * n + j];
      out[j] = s;
    }
  }
}

// host side
bool gemm_epilogue_vec_ok(const Gemm& a);
void gemm_splitk_reduce(const float* part, int splits, int64_t n, float* out, const float* part2, int64_t n2, float* out2,
                        hipStream_t st);
bool gemm_dma_ok(const Gemm& a);
void gemm_dma(const Gemm& a, int variant, hipStream_t st);
// few rows, long K, workspace given: split-K with a summing epilogue pass; false if the shape is not taken
bool gemm_dma_skinny(const Gemm& a, hipStream_t st);
bool gemm_wgrad_group(const Gemm* a, int n, hipStream_t st, hipEvent_t mid, WgradCarry* carry, LnBwdRide* ln);
int splitk_vec_ok4(const float* part, int64_t n, const float* out);
// the split-K reductions of up to four products (part2 entries may be null) in one launch
void gemm_splitk_reduce_group(int nprob, int splits, const float* const* part, const int64_t* n, float* const* out,
                              const float* const* part2, const int64_t* n2, float* const* out2, hipStream_t st);

}  // namespace pt
