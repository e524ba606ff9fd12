// bf16 matrix-core GEMM with an asynchronous HBM -> LDS pipeline (gfx950).
//
// Operand tiles travel from global memory straight into LDS with
// global_load_lds_dwordx4 (no staging registers), NS tiles deep, so that the
// HBM/L2 latency of a tile is hidden behind the MFMA work of the NS-1 tiles
// before it.  The only synchronisation per k-tile is one s_waitcnt vmcnt(n)
// (this wave's own tile has landed) and one s_barrier (everybody's has).
//
// LDS layouts follow the operand's memory layout, because a wave-wide DMA load
// writes 64 consecutive 16-byte slots:
//   k-major operand  (element (r,k) at p[r*ld + k]) : tile [ROWS][BK], read as
//       16-byte MFMA fragments;
//   strided operand  (element (r,k) at p[k*ld + r]) : tile [BK][ROWS], read with
//       ds_read_b64_tr_b16, the LDS transpose read that hands each lane four
//       consecutive k of one row.
// Both use an XOR swizzle of the 16-byte slot index (applied to the global
// address each lane fetches), which makes the fragment reads bank-conflict free.
//
// Requirements checked by the host: K a multiple of BK (no zero fill exists on
// this path), 16-byte aligned rows.  Rows / columns past the edge are clamped to
// the last valid one: they only feed outputs that are never stored.
#include "common.h"
#include "kernels.h"
#include "gemm_epilogue.h"
#include "ln_bwd_rows.h"

namespace pt {

namespace {

#define PT_LDS(p) ((__attribute__((address_space(3))) void*)(p))
#define PT_GLB(p) ((const __attribute__((address_space(1))) void*)(p))
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;

constexpr int kBK = 32;

__device__ __forceinline__ void compiler_fence() { asm volatile("" ::: "memory"); }

typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

__device__ __forceinline__ unsigned lds_addr(const void* p) {
  return (unsigned)(size_t)((__attribute__((address_space(3))) const void*)(p));
}

// ---- k-major tile [ROWS][BK]: rows of 2*BK bytes ----
// BK = 64 makes a row segment a whole 128-byte cache line.  With BK = 32 every line is requested twice, half
// a line at a time, one k-tile apart, and the L2 -> L1 path, which moves whole lines, carries twice the bytes:
// a kernel that only issues these loads (the 12608 x 768 x 3072 product's 128x128 tiling, three workgroups
// per CU) takes 76.6 us with 64-byte segments and 49.9 us with 128-byte ones, and the product itself ran in
// 85 us, i.e. at the speed of its loads.
// Slot (row, c') holds chunk c' ^ swzk(row); swzk spreads the 16 rows that the lanes of a quarter-wave read
// together over all 64 banks.
template <int ROWS, int NW, int NFRAG, int BK>
struct TileK {
  static constexpr int ROWB = BK * 2, CPR = ROWB / 16, RPL = 1024 / ROWB;   // row bytes, chunks per row, rows per load
  static constexpr int BYTES = ROWS * ROWB, LOADS = ROWS / RPL / NW;        // wave-wide loads per wave
  static constexpr int KS = BK / 16;                                        // k-steps per tile
  static_assert(ROWS % (RPL * NW) == 0, "rows must divide over the waves");
  static_assert(BK == 32 || BK == 64, "64- or 128-byte rows");
  const bf16* gp[LOADS];   // this lane's source of each load, advanced by one tile per issue
  unsigned foff[KS];       // fragment byte offsets within the tile per k-step (row block 0)

  static __device__ __forceinline__ constexpr int swzk(int row) { return BK == 32 ? ((row >> 2) & 3) : ((row >> 1) & 7); }
  __device__ __forceinline__ void setup(const bf16* p, int64_t ld, int R, int r0, int k0, int rbase, int wave,
                                        int lane) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int row = RPL * (wave * LOADS + i) + lane / CPR;
      const int c = (lane % CPR) ^ swzk(row);
      int gr = r0 + row;
      gr = gr < R ? gr : R - 1;
      gp[i] = p + (int64_t)gr * ld + k0 + 8 * c;
    }
    const int row = rbase + (lane & 31);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) foff[ks] = row * ROWB + (((2 * ks + (lane >> 5)) ^ swzk(row)) << 4);
  }
  __device__ __forceinline__ void issue_one(unsigned char* tile, int wave, int i) {
    __builtin_amdgcn_global_load_lds(PT_GLB(gp[i]), PT_LDS(tile + (wave * LOADS + i) * 1024), 16, 0, 0);
    gp[i] += BK;
  }
  __device__ __forceinline__ void issue(unsigned char* tile, int wave) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) issue_one(tile, wave, i);
  }
  // fragments of all row blocks for one k-step, issued as inline assembly (see TileS::read)
  static constexpr int READS = NFRAG;   // LDS instructions per k-step
  __device__ __forceinline__ void read(const unsigned char* tile, int ks, bf16x8 (&f)[NFRAG]) const {
    const unsigned addr = lds_addr(tile) + foff[ks];
#pragma unroll
    for (int i = 0; i < NFRAG; ++i)
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(f[i]) : "v"(addr), "n"(i * 32 * ROWB));
  }
};

// ---- strided tile [BK][ROWS]: rows of ROWS*2 bytes, slot (k, c') holds chunk c' ^ swz(k) ----
// A transpose read has its 16-lane groups address 4 k rows x 32 bytes; the groups of one half-wave differ by
// 32 bytes in the row (or by 8 k rows).  Rows are a multiple of 256 bytes, so only the chunk index decides
// the bank: swz moves the four k rows of a group to four different 64-byte quarters of the bank space and
// the k+8 group to the other 32 bytes of each, which makes any two groups served together conflict-free
// (checked against a bank model; the earlier (k & 3) << 1 left two-way conflicts, 21 % of the cycles of the
// weight-gradient kernel by SQ_LDS_BANK_CONFLICT).
__device__ __forceinline__ constexpr int swz(int k) { return ((k & 3) << 2) ^ (((k >> 3) & 1) << 1); }
// Fragments come from ds_read_b64_tr_b16 (each lane gets four consecutive k of one row).  All fragment
// reads are issued as inline assembly: the compiler would otherwise wait for every outstanding
// global->LDS load before a transpose read, which serialises the pipeline, and explicit lgkmcnt waits
// let the reads of the second k-step overlap the MFMAs of the first.  LDS operations return in order,
// so "at most n outstanding" means everything issued before the last n has arrived.
template <int ROWS, int NW, int NFRAG, int BK>
struct TileS {
  static constexpr int ROWB = ROWS * 2, KPL = 1024 / ROWB;       // k rows per wave-wide load
  static constexpr int BYTES = BK * ROWB, LOADS = BK / KPL / NW;
  static constexpr int CPR = ROWS / 8;                           // 16-byte chunks per k row
  static constexpr int KS = BK / 16;
  static_assert(BK % (KPL * NW) == 0 && KPL >= 1, "tile must divide over the waves");
  static_assert(CPR >= 16, "swz permutes chunks within groups of 16");
  const bf16* gp[LOADS];
  int64_t gstep;
  unsigned foff[NFRAG];    // fragment byte offsets (k-step 0, first half) per 32-row block

  __device__ __forceinline__ void setup(const bf16* p, int64_t ld, int R, int r0, int k0, int rbase, int wave,
                                        int lane) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int k = KPL * (wave * LOADS + i) + lane / CPR;
      const int c = (lane % CPR) ^ swz(k);
      int gr = r0 + 8 * c;
      gr = gr + 8 <= R ? gr : (R - 8);   // R >= 8 and R % 8 == 0 are checked by the host
      gp[i] = p + (int64_t)(k0 + k) * ld + gr;
    }
    gstep = (int64_t)BK * ld;
    const int l16 = lane & 15, grp = lane >> 4;
    const int k = 8 * (grp >> 1) + (l16 >> 2);
#pragma unroll
    for (int j = 0; j < NFRAG; ++j) {
      const int col = rbase + j * 32 + (grp & 1) * 16 + 4 * (l16 & 3);
      foff[j] = k * ROWB + (((col >> 3) ^ swz(k)) << 4) + (col & 7) * 2;
    }
  }
  __device__ __forceinline__ void issue_one(unsigned char* tile, int wave, int i) {
    __builtin_amdgcn_global_load_lds(PT_GLB(gp[i]), PT_LDS(tile + (wave * LOADS + i) * 1024), 16, 0, 0);
    gp[i] += gstep;
  }
  __device__ __forceinline__ void issue(unsigned char* tile, int wave) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) issue_one(tile, wave, i);
  }
  static constexpr int READS = 2 * NFRAG;
  // ks is a compile-time constant at every call site (unrolled), so the offsets fold to immediates
  __device__ __forceinline__ void read(const unsigned char* tile, int ks, bf16x8 (&f)[NFRAG]) const {
    const unsigned base = lds_addr(tile);
#pragma unroll
    for (int j = 0; j < NFRAG; ++j) {
      union { u32x2 h[2]; bf16x8 v; } t;
      const unsigned addr = base + foff[j] + 16 * ks * ROWB;
      // k rows 16*ks + 8*half + {0..3} and {4..7}: +4 and +16*ks rows are constant offsets (swz uses bits 0, 1, 3 of k)
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(t.h[0]) : "v"(addr));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(t.h[1]) : "v"(addr), "n"(4 * ROWB));
      f[j] = t.v;
    }
  }
  // sum over the tile's k rows of column n (for the fused bias gradient)
  static __device__ __forceinline__ float colsum(const unsigned char* lds, int n) {
    float s = 0.f;
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      const int c = (n >> 3) ^ swz(k);
      s += to_f32(*reinterpret_cast<const bf16*>(lds + k * ROWB + c * 16 + (n & 7) * 2));
    }
    return s;
  }
};

template <bool STRIDED, int ROWS, int NW, int NFRAG, int BK> struct TileSel { typedef TileK<ROWS, NW, NFRAG, BK> type; };
template <int ROWS, int NW, int NFRAG, int BK> struct TileSel<true, ROWS, NW, NFRAG, BK> { typedef TileS<ROWS, NW, NFRAG, BK> type; };

// s_waitcnt lgkmcnt(PENDING) that the given fragments depend on, so that no MFMA using them can be
// scheduled before it
template <int PENDING, int NA, int NB>
__device__ __forceinline__ void wait_lds(bf16x8 (&a)[NA], bf16x8 (&b)[NB]) {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(PENDING) : "memory");
#pragma unroll
  for (int i = 0; i < NA; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
  for (int i = 0; i < NB; ++i) asm volatile("" : "+v"(b[i]));
}

// s_waitcnt vmcnt(n), n < 64 (the count is split over two bit fields); expcnt and lgkmcnt are left open
template <int N>
__device__ __forceinline__ void wait_vm() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// The LDS footprint allows two workgroups per CU with 256x128 tiles (eight waves each) and three with
// 128x128 tiles (four waves each).  The second launch bound is the number of waves per SIMD that this
// amounts to: the register allocation is held to it, whatever the epilogue would like to use.
constexpr int dma_waves_per_simd(int lds_bytes, int waves) {
  return (lds_bytes <= 48 * 1024 ? 3 : (lds_bytes <= 80 * 1024 ? 2 : 1)) * waves / 4;
}
template <int BM, int BN, int WGM, int WGN, int kNS, int BK, bool TA, bool TB, int EPI, typename TC>
__global__ __launch_bounds__(64 * WGM * WGN, dma_waves_per_simd((BM + BN) * BK * 2 * kNS, WGM * WGN))
void gemm_dma_kernel(GemmDev<bf16> g, SplitArgs sp, int tiles_m, int tiles_n,
                                                                  int group_n, int vec_ok) {
  constexpr int NW = WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
  typedef typename TileSel<TA, BM, NW, TM, BK>::type LA;    // A strided when stored [K,M]
  typedef typename TileSel<!TB, BN, NW, TN, BK>::type LB;   // B strided when stored [K,N]
  constexpr int KS = BK / 16;                                // k-steps (MFMA depth 16) per tile
  constexpr int STAGE = LA::BYTES + LB::BYTES;
  constexpr int STAGE_LD = WTN + 4;
  constexpr int EPI_BYTES = NW * 32 * STAGE_LD * 4;
  constexpr int LDS_BYTES = kNS * STAGE > EPI_BYTES ? kNS * STAGE : EPI_BYTES;
  constexpr int LPT = LA::LOADS + LB::LOADS;  // DMA loads per thread per tile
  constexpr int RPS = LA::READS + LB::READS;  // LDS read instructions per k-step
  static_assert(LPT * (kNS >= 4 ? 2 : 1) < 64, "vmcnt is a 6-bit counter");
  static_assert(RPS <= 15, "lgkmcnt is a 4-bit counter");
  static_assert(kNS >= 2 && LDS_BYTES <= 160 * 1024, "stages must fit the LDS");
  __shared__ __attribute__((aligned(1024))) unsigned char lds[LDS_BYTES];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // Workgroups are dealt to the 8 XCDs round-robin by their index, and each XCD has an L2 of its own.  The
  // index is remapped so that one XCD works through a contiguous range of the sequence
  //   for split: for column group (group_n tile columns): for tile row: for tile column in the group
  // which keeps a K slice (split-K) or a band of B panels small enough to stay in that L2 while the A panels
  // stream past it once.
  const int total_tiles = tiles_m * tiles_n, total_work = total_tiles * sp.splits;
  const int per = (total_work + 7) >> 3;
  const int work = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if (work >= total_work) return;
  const int split = work / total_tiles;
  const int t = work - split * total_tiles;
  const int grp = t / (group_n * tiles_m);
  const int rem = t - grp * group_n * tiles_m;
  const int gw = tiles_n - grp * group_n < group_n ? tiles_n - grp * group_n : group_n;
  const int m0 = (rem / gw) * BM, n0 = (grp * group_n + rem % gw) * BN;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nk_all = g.K / BK;
  const int kt0 = split * sp.tiles_per_split;
  const int kt1 = (kt0 + sp.tiles_per_split < nk_all) ? kt0 + sp.tiles_per_split : nk_all;
  const int n = kt1 > kt0 ? kt1 - kt0 : 0;
  const bool do_colsum = !TB && sp.colsum != nullptr && m0 == 0;
  float cs = 0.f;

  LA ta;
  LB tb;
  ta.setup(g.A, g.lda, g.M, m0, kt0 * BK, wm * WTM, wave, lane);
  tb.setup(g.B, g.ldb, g.N, n0, kt0 * BK, wn * WTN, wave, lane);

  int fill = 0;  // stage the next issued tile goes to
#pragma unroll
  for (int s = 0; s < kNS - 1; ++s)
    if (s < n) {
      ta.issue(lds + s * STAGE, wave);
      tb.issue(lds + s * STAGE + LA::BYTES, wave);
    }
  fill = kNS - 1;
  int cur = 0;   // stage of the tile being consumed

  for (int it = 0; it < n; ++it) {
    // this wave's loads of tile `it` have landed when at most the loads of the later tiles are pending
    if (kNS >= 4 && it + 2 < n) wait_vm<2 * LPT>();
    else if (kNS >= 3 && it + 1 < n) wait_vm<LPT>();
    else wait_vm<0>();
    compiler_fence();
    __builtin_amdgcn_s_barrier();   // everybody's loads of tile `it` have landed, and tile it-1 is fully consumed
    compiler_fence();
    if (it + kNS - 1 < n) {
      ta.issue(lds + fill * STAGE, wave);
      tb.issue(lds + fill * STAGE + LA::BYTES, wave);
    }
    fill = fill + 1 == kNS ? 0 : fill + 1;
    const unsigned char* sa = lds + cur * STAGE;
    const unsigned char* sb = sa + LA::BYTES;
    cur = cur + 1 == kNS ? 0 : cur + 1;
    // Two fragment sets in registers.  The reads of k-steps 0 and 1 are issued up front; the MFMAs of a
    // k-step start as soon as its fragments are in, and the reads of k-step s+2 are issued behind the
    // MFMAs of k-step s into the set those MFMAs have just consumed, so LDS reads overlap matrix work.
    // LDS operations return in order: "at most RPS outstanding" means the older set has arrived.
    bf16x8 fa[2][TM], fb[2][TN];
    ta.read(sa, 0, fa[0]);
    tb.read(sb, 0, fb[0]);
    ta.read(sa, 1, fa[1]);
    tb.read(sb, 1, fb[1]);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (ks + 1 < KS) wait_lds<RPS>(fa[ks & 1], fb[ks & 1]);
      else wait_lds<0>(fa[ks & 1], fb[ks & 1]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
      // nothing may be scheduled across this point: without it the compiler sinks the MFMAs above below the
      // next wait, and every fragment read of the tile is then waited for before the first MFMA issues
      __builtin_amdgcn_sched_barrier(0);
      if (ks + 2 < KS) {
        ta.read(sa, ks + 2, fa[ks & 1]);
        tb.read(sb, ks + 2, fb[ks & 1]);
      }
    }
    if constexpr (!TB) {
      if (do_colsum && tid < BN) cs += LB::colsum(sb, tid);
    }
  }
  compiler_fence();
  __builtin_amdgcn_s_barrier();   // all fragment reads done: the LDS can be reused for the epilogue
  compiler_fence();
  if constexpr (!TB) {
    if (do_colsum && tid < BN && n0 + tid < g.N) sp.colsum[(int64_t)split * g.N + n0 + tid] = cs;
  }
  void* Cbase = sizeof(TC) == 4 ? (void*)(reinterpret_cast<float*>(g.C) + split * sp.slab)
                                : (void*)(reinterpret_cast<bf16*>(g.C) + split * sp.slab);
  // four waves per SIMD leave 128 registers each: only the long-latency read of the saved GELU' is double-buffered
  constexpr int NBUF = (EPI == EPI_MUL_DGELU || dma_waves_per_simd((BM + BN) * BK * 2 * kNS, NW) < 4) ? 2 : 1;
  staged_epilogue<TM, TN, WTM, WTN, EPI, TC, NBUF>(g, Cbase, acc, reinterpret_cast<float*>(lds) + wave * 32 * STAGE_LD,
                                                   m0 + wm * WTM, n0 + wn * WTN, lane, vec_ok);
}


// ---- 256x256x64 (or 192x256x64) tiles, two wave groups in alternating roles ----
// The eight waves form two groups of four, one wave of each group per SIMD.  Time is cut into phases that
// end in a workgroup barrier.  In a phase one group only issues matrix instructions, on fragments it
// already holds in registers, while the other group reads its next fragments from LDS; at the barrier they
// swap.  The matrix cores therefore always have a wave whose operands are complete, and LDS reads are
// spread evenly over time instead of arriving from all eight waves right after a tile barrier.  Measured on
// the single-role pipeline above (12608 x 768 x 3072, cycles per k tile and CU; 2048 are MFMA issue): MFMAs
// alone 2380, with LDS reads 2710, with the global->LDS loads 2720-3250, all three 3500-3700.
//
// A group holds the fragments of half a k tile at a time (WHOLE = false: 16 MFMAs per phase, four phases and
// barriers per tile) or, where the registers allow it (192-row tiles), of a whole k tile (WHOLE = true: two
// phases per tile, 4-5 % faster).  Group 1 runs one phase behind group 0.  A tiles live in a ring of three
// stages and B tiles in a ring of two, 160 KB (136 KB) in all: A (the activations, streamed from HBM) is
// requested two tiles ahead, B (weights, mostly L2 hits) one tile ahead.  Loads are issued a few per phase:
// B(t+1) in the first phase of tile t and A(t+2) in equal parts over the other phases, between MFMAs where
// the issuing wave computes and in one go where it fetches, so that "at most LA::LOADS loads outstanding" at
// the end of a tile's last phase means A(t+1) and B(t+1) have landed.
//
// pp_run computes one output tile (rows m0.., columns n0..) over the k tiles kt0 .. kt0 + n - 1 and stores it
// to slab `split`; all 512 threads of the workgroup take part.
// the LDS of the two-group kernels: one array per size, so that a kernel's other roles can use the same bytes
template <int BYTES>
__device__ __forceinline__ unsigned char* pp_lds() {
  __shared__ __attribute__((aligned(1024))) unsigned char lds[BYTES];
  return lds;
}
constexpr int kPpLdsBytes256 = 160 * 1024;   // 256-row tiles: three A stages and two B stages of 32 KB
template <int BM, bool WHOLE, bool TA, bool TB, int EPI, typename TC>
__device__ __forceinline__ void pp_run(const GemmDev<bf16>& g, const SplitArgs& sp, int split, int kt0, int n, int m0, int n0,
                                       int vec_ok) {
  constexpr int BN = 256, WGN = 4, BK = 64, NW = 8, NSA = 3, NSB = 2;
  constexpr int WTM = BM / 2, WTN = 64, TM = WTM / 32, TN = 2;
  static_assert(BM == 256 || BM == 192, "two rows of waves, 32-row fragments");
  typedef typename TileSel<TA, BM, NW, TM, BK>::type LA;
  typedef typename TileSel<!TB, BN, NW, TN, BK>::type LB;
  constexpr int STAGE_LD = WTN + 4;
  constexpr int LDS_BYTES = NSA * LA::BYTES + NSB * LB::BYTES;
  static_assert(NW * 32 * STAGE_LD * 4 <= LDS_BYTES && LDS_BYTES <= 160 * 1024, "LDS budget");
  constexpr int NH = WHOLE ? 1 : 2;        // halves of a k tile whose fragments a group holds at a time
  constexpr int KSF = 4 / NH;              // k-steps (MFMA depth 16) per half
  constexpr int NPART = 2 * NH - 1;        // A(t+2) goes out in this many parts, one per phase after the first
  static_assert(LA::LOADS >= NPART, "A loads are spread over the phases");
  static_assert(BM != 256 || LDS_BYTES == kPpLdsBytes256, "kPpLdsBytes256 names the 256-row kernels' array");
  unsigned char* const lds = pp_lds<LDS_BYTES>();
  unsigned char* const ldsB = lds + NSA * LA::BYTES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int grp = __builtin_amdgcn_readfirstlane(wave >> 2);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const bool do_colsum = !TB && sp.colsum != nullptr && m0 == 0;
  float cs = 0.f;

  LA ta;
  LB tb;
  ta.setup(g.A, g.lda, g.M, m0, kt0 * BK, wm * WTM, wave, lane);
  tb.setup(g.B, g.ldb, g.N, n0, kt0 * BK, wn * WTN, wave, lane);

  bf16x8 fa[KSF][TM], fb[KSF][TN];
  // fragment reads of one half (k-steps KSF*half ..), complete once fetched() returns
  auto fetch = [&](const unsigned char* sa, const unsigned char* sb, int half) {
#pragma unroll
    for (int ks = 0; ks < KSF; ++ks) {
      ta.read(sa, KSF * half + ks, fa[ks]);
      tb.read(sb, KSF * half + ks, fb[ks]);
    }
  };
  auto fetched = [&]() {
#pragma unroll
    for (int ks = 0; ks < KSF; ++ks) wait_lds<0>(fa[ks], fb[ks]);
  };
  // the MFMAs on the fragments held; `load(q)` for q in [0, nq) goes out between them
  auto compute = [&](bool on, int nq, auto load) {
#pragma unroll
    for (int ks = 0; ks < KSF; ++ks)
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
        const int slot = ks * TM + i;
        if (slot < nq) {
          if (on) load(slot);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
  };
  // part q of A(t+2)'s loads: [part_lo(q), part_lo(q + 1))
  auto part_lo = [](int q) constexpr { return q * LA::LOADS / NPART; };
  // End of a phase.  Nothing may be scheduled across it: MFMAs have no side effects, and left to itself the
  // compiler sinks most of a compute phase's MFMAs below the barrier into the wave's next fetch phase (to hide
  // its LDS latency), which leaves compute phases with one or two MFMAs and puts both groups' MFMAs into
  // the same phase: the alternation of the two groups exists only if the phases stay as written.
  auto phase_end = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  auto tile_done = [&](bool moreA) {   // A(t+1) and B(t+1) have landed; everybody is past tile t
    __builtin_amdgcn_sched_barrier(0);
    if (moreA) wait_vm<LA::LOADS>();
    else wait_vm<0>();
    compiler_fence();
    __builtin_amdgcn_s_barrier();
    compiler_fence();
    __builtin_amdgcn_sched_barrier(0);
  };

  if (n > 0) {
    ta.issue(lds, wave);
    tb.issue(ldsB, wave);
  }
  if (n > 1) {
    ta.issue(lds + LA::BYTES, wave);
    wait_vm<LA::LOADS>();
  } else {
    wait_vm<0>();
  }
  compiler_fence();
  __builtin_amdgcn_s_barrier();
  compiler_fence();

  // The two groups run separate loops (straight-line code each, which the register allocator handles far
  // better than one loop with a branch per phase); both execute 2 * NH barriers per tile.
  if (grp == 0) {
    int ia = 0, ib = 0;   // stages of tile t
    for (int t = 0; t < n; ++t) {
      const bool moreB = t + 1 < n, moreA = t + 2 < n;
      const unsigned char* sa = lds + ia * LA::BYTES;
      const unsigned char* sb = ldsB + ib * LB::BYTES;
      unsigned char* const dstB = ldsB + (ib ^ 1) * LB::BYTES;
      unsigned char* const dstA = lds + (ia == 0 ? NSA - 1 : ia - 1) * LA::BYTES;   // stage (t + 2) % 3
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        // fetch phase: B(t+1) with the first half, a part of A(t+2) with the others
        fetch(sa, sb, h);
        if (h == 0) {
          if (moreB) tb.issue(dstB, wave);
        } else if (moreA) {
#pragma unroll
          for (int q = part_lo(2 * h - 1); q < part_lo(2 * h); ++q) ta.issue_one(dstA, wave, q);
        }
        fetched();
        phase_end();
        // compute phase
        compute(moreA, part_lo(2 * h + 1) - part_lo(2 * h), [&](int q) { ta.issue_one(dstA, wave, part_lo(2 * h) + q); });
        if constexpr (!TB) {
          if (h == 0 && do_colsum) cs += LB::colsum(sb, tid);   // threads 0..255 are this group
        }
        if (h == NH - 1) tile_done(moreA);
        else phase_end();
      }
      ia = ia + 1 == NSA ? 0 : ia + 1;
      ib ^= 1;
    }
  } else {
    int ia = 0, ib = 0;
    // first phase of tile 0: nothing to compute yet
    if (n > 1) tb.issue(ldsB + LB::BYTES, wave);
    if (n > 0) phase_end();
    for (int t = 0; t < n; ++t) {
      const bool moreA = t + 2 < n;
      const unsigned char* sa = lds + ia * LA::BYTES;
      const unsigned char* sb = ldsB + ib * LB::BYTES;
      unsigned char* const dstA = lds + (ia == 0 ? NSA - 1 : ia - 1) * LA::BYTES;
#pragma unroll
      for (int h = 0; h < NH; ++h) {
        // fetch phase, with a part of A(t+2)
        fetch(sa, sb, h);
        if (moreA) {
#pragma unroll
          for (int q = part_lo(2 * h); q < part_lo(2 * h + 1); ++q) ta.issue_one(dstA, wave, q);
        }
        fetched();
        if (h == NH - 1) tile_done(moreA);
        else phase_end();
        // compute phase: the next part of A(t+2), or, in the first phase of tile t + 1, B(t+2) into the stage
        // tile t's B has just left
        if (h < NH - 1) {
          compute(moreA, part_lo(2 * h + 2) - part_lo(2 * h + 1), [&](int q) { ta.issue_one(dstA, wave, part_lo(2 * h + 1) + q); });
          phase_end();
        } else if (t + 1 < n) {
          unsigned char* const dstB = ldsB + ib * LB::BYTES;
          compute(moreA, LB::LOADS, [&](int q) { tb.issue_one(dstB, wave, q); });
          phase_end();
        }
      }
      ia = ia + 1 == NSA ? 0 : ia + 1;
      ib ^= 1;
    }
    if (n > 0) compute(false, 0, [](int) {});
  }
  compiler_fence();
  __builtin_amdgcn_s_barrier();   // all fragment reads done: the LDS can be reused for the epilogue
  compiler_fence();
  if constexpr (!TB) {
    if (do_colsum && tid < BN && n0 + tid < g.N) sp.colsum[(int64_t)split * g.N + n0 + tid] = cs;
  }
  void* Cbase = sizeof(TC) == 4 ? (void*)(reinterpret_cast<float*>(g.C) + split * sp.slab)
                                : (void*)(reinterpret_cast<bf16*>(g.C) + split * sp.slab);
  staged_epilogue<TM, TN, WTM, WTN, EPI, TC>(g, Cbase, acc, reinterpret_cast<float*>(lds) + wave * 32 * STAGE_LD, m0 + wm * WTM,
                                             n0 + wn * WTN, lane, vec_ok);
}

// Several weight gradients dW_p = X_p^T dY_p over the same tokens in one launch.  One encoder block has
// only 108 output tiles of 256x256 in its four weight matrices; launched one matrix at a time each needs a
// 7- to 16-way split over K to occupy the chip and then writes and re-reads that many fp32 slabs.  Together
// they fill the CUs with a two-way split.
constexpr int kMaxGroup = 4;
struct GroupArgs {
  GemmDev<bf16> g[kMaxGroup];   // C = this problem's slab area (or the destination when splits == 1)
  float* colsum[kMaxGroup];
  int64_t slab[kMaxGroup];
  int tile0[kMaxGroup + 1];     // first tile of each problem in the launch's tile order
  int tiles_n[kMaxGroup];
  int vec_ok[kMaxGroup];
  int nprob, splits, tiles_per_split;
  // the slab reduction of an earlier launch, done by the workgroups behind this launch's own
  const float* c_part[kMaxGroup]; float* c_out[kMaxGroup]; int64_t c_n[kMaxGroup];
  const float* c_part2[kMaxGroup]; float* c_out2[kMaxGroup]; int64_t c_n2[kMaxGroup];
  int c_vec[kMaxGroup], c_vec2[kMaxGroup];
  int c_nprob, c_splits;
  // a LayerNorm backward pass that is independent of the products, run by the same workgroups first
  LnBwdArgs<bf16, bf16, bf16> ln;   // dy and x are fp32 when ln_on == 2 (the pointers are cast back)
  int ln_on;
};
__global__ __launch_bounds__(512) void gemm_wgrad_group_kernel(GroupArgs ga) {
  const int total_tiles = ga.tile0[ga.nprob], total_work = total_tiles * ga.splits;
  const int per = (total_work + 7) >> 3;
  if ((int)blockIdx.x >= 8 * per) {
    // One encoder block's tiles leave 40 of the 256 CUs without a workgroup.  The workgroups placed there sum
    // the split-K slabs that the previous launch left behind (85 MB of streaming beside a launch that is bound
    // by its matrix work), which therefore needs no launch of its own.
    // The same workgroups first run a LayerNorm backward pass that does not depend on these products (the
    // block's last one, whose result only the next block reads): 135 MB more, still well inside what 40 CUs
    // stream while the others work through their 98 k tiles.
    float* red = reinterpret_cast<float*>(pp_lds<kPpLdsBytes256>());
    const int rid = (int)blockIdx.x - 8 * per, nred = (int)gridDim.x - 8 * per;
    if (ga.ln_on == 1) {
      if (ga.ln.D <= 768) ln_bwd_rows<bf16, bf16, bf16, 3, 8>(ga.ln, red, rid, nred);
      else ln_bwd_rows<bf16, bf16, bf16, 4, 8>(ga.ln, red, rid, nred);
    } else if (ga.ln_on == 2) {
      const LnBwdArgs<bf16, float, float> a{reinterpret_cast<const float*>(ga.ln.dy), ga.ln.lddy,
                                            reinterpret_cast<const float*>(ga.ln.x), ga.ln.ldx, ga.ln.mean, ga.ln.rstd,
                                            ga.ln.gamma, ga.ln.dres, ga.ln.lddres, ga.ln.dx_s, ga.ln.dx_o, ga.ln.lddx,
                                            ga.ln.partial, ga.ln.rows, ga.ln.D};
      if (ga.ln.D <= 768) ln_bwd_rows<bf16, float, float, 3, 8>(a, red, rid, nred);
      else ln_bwd_rows<bf16, float, float, 4, 8>(a, red, rid, nred);
    }
    const int64_t first = ((int64_t)((int)blockIdx.x - 8 * per) * 512 + threadIdx.x) * 4;
    const int64_t step = (int64_t)((int)gridDim.x - 8 * per) * 512 * 4;
    for (int p = 0; p < ga.c_nprob; ++p) {
      for (int64_t i = first; i < ga.c_n[p]; i += step) splitk_sum4(ga.c_part[p], ga.c_splits, ga.c_n[p], ga.c_out[p], ga.c_vec[p], i);
      if (ga.c_part2[p])
        for (int64_t i = first; i < ga.c_n2[p]; i += step)
          splitk_sum4(ga.c_part2[p], ga.c_splits, ga.c_n2[p], ga.c_out2[p], ga.c_vec2[p], i);
    }
    return;
  }
  const int work = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if (work >= total_work) return;
  const int split = work / total_tiles;
  const int tt = work - split * total_tiles;
  int p = 0;
  while (p + 1 < ga.nprob && tt >= ga.tile0[p + 1]) ++p;
  const int local = tt - ga.tile0[p];
  const SplitArgs sp{ga.splits, ga.tiles_per_split, ga.slab[p], ga.colsum[p]};
  const int nk_all = ga.g[p].K / 64;
  const int kt0 = split * ga.tiles_per_split;
  const int kt1 = (kt0 + ga.tiles_per_split < nk_all) ? kt0 + ga.tiles_per_split : nk_all;
  pp_run<256, false, true, false, EPI_STORE, float>(ga.g[p], sp, split, kt0, kt1 > kt0 ? kt1 - kt0 : 0, (local / ga.tiles_n[p]) * 256,
                                             (local % ga.tiles_n[p]) * 256, ga.vec_ok[p]);
}

// Workgroups are dealt to the 8 XCDs round-robin by their index; the index is remapped so that one XCD works
// through a contiguous range of {split, column group, tile row, tile column} (see gemm_dma_kernel).
template <int BM, bool WHOLE, bool TA, bool TB, int EPI, typename TC>
__global__ __launch_bounds__(512) void gemm_pp_kernel(GemmDev<bf16> g, SplitArgs sp, int tiles_m, int tiles_n, int group_n,
                                                      int vec_ok) {
  const int total_tiles = tiles_m * tiles_n, total_work = total_tiles * sp.splits;
  const int per = (total_work + 7) >> 3;
  const int work = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
  if (work >= total_work) return;
  const int split = work / total_tiles;
  const int tt = work - split * total_tiles;
  const int cg = tt / (group_n * tiles_m);
  const int rem = tt - cg * group_n * tiles_m;
  const int gw = tiles_n - cg * group_n < group_n ? tiles_n - cg * group_n : group_n;
  const int m0 = (rem / gw) * BM, n0 = (cg * group_n + rem % gw) * 256;
  const int nk_all = g.K / 64;
  const int kt0 = split * sp.tiles_per_split;
  const int kt1 = (kt0 + sp.tiles_per_split < nk_all) ? kt0 + sp.tiles_per_split : nk_all;
  const int n = kt1 > kt0 ? kt1 - kt0 : 0;
  pp_run<BM, WHOLE, TA, TB, EPI, TC>(g, sp, split, kt0, n, m0, n0, vec_ok);
}

#ifdef PT_TUNING_HOOKS   // stand-alone experiments only; the library is built without it
int g_group_n = 0;                  // forced column-group width; 0 = derive from g_group_bytes
int64_t g_group_bytes = 1536 << 10;
#else
constexpr int g_group_n = 0;
constexpr int64_t g_group_bytes = 1536 << 10;  // L2 bytes a column group's B panels may take
#endif

template <int BM, int BN, int WGM, int WGN, int NS, int BK, bool TA, bool TB, int EPI, typename TC>
void launch_dma(const Gemm& a, int splits, float* cbase, int64_t slab, float* colsum_part, hipStream_t st) {
  GemmDev<bf16> g{(const bf16*)a.A, (const bf16*)a.B, cbase ? (void*)cbase : a.C, a.M, a.N, a.K, a.lda, a.ldb, a.ldc,
                  (const bf16*)a.bias, (const bf16*)a.aux, (bf16*)a.aux_out, a.ld_aux};
  const int tiles_m = cdiv(a.M, BM), tiles_n = cdiv(a.N, BN), total = tiles_m * tiles_n;
  const int nk = a.K / BK;
  SplitArgs sp{splits, cdiv(nk, splits), slab, colsum_part};
  dim3 grid(8 * cdiv(total * splits, 8), 1, 1);
  // column-group width: the B panels of a group (whole K) should fit beside the streaming A panels in a 4 MB L2
  int group_n = g_group_n;
  if (group_n <= 0) {
    const int64_t panel = (int64_t)BN * (a.K / splits) * 2;
    group_n = (int)(g_group_bytes / (panel > 0 ? panel : 1));
    if (group_n < 1) group_n = 1;
  }
  if (group_n > tiles_n) group_n = tiles_n;
  hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WGM, WGN, NS, BK, TA, TB, EPI, TC>), grid, dim3(64 * WGM * WGN), 0, st, g, sp,
                     tiles_m, tiles_n, group_n, gemm_epilogue_vec_ok(a) ? 1 : 0);
}

template <int BM, bool TA, bool TB, int EPI, typename TC>
void launch_pp(const Gemm& a, int splits, float* cbase, int64_t slab, float* colsum_part, hipStream_t st) {
  constexpr int BN = 256, BK = 64;
  GemmDev<bf16> g{(const bf16*)a.A, (const bf16*)a.B, cbase ? (void*)cbase : a.C, a.M, a.N, a.K, a.lda, a.ldb, a.ldc,
                  (const bf16*)a.bias, (const bf16*)a.aux, (bf16*)a.aux_out, a.ld_aux};
  const int tiles_m = cdiv(a.M, BM), tiles_n = cdiv(a.N, BN), total = tiles_m * tiles_n;
  const int nk = a.K / BK;
  SplitArgs sp{splits, cdiv(nk, splits), slab, colsum_part};
  dim3 grid(8 * cdiv(total * splits, 8), 1, 1);
  int group_n = g_group_n;
  if (group_n <= 0) {
    const int64_t panel = (int64_t)BN * (a.K / splits) * 2;
    group_n = (int)(g_group_bytes / (panel > 0 ? panel : 1));
    if (group_n < 1) group_n = 1;
  }
  if (group_n > tiles_n) group_n = tiles_n;
  // 192-row tiles leave room for a whole k tile of fragments in registers (whole-tile phases, 4-5 % faster);
  // 256-row tiles do not
  hipLaunchKernelGGL((gemm_pp_kernel<BM, BM == 192, TA, TB, EPI, TC>), grid, dim3(512), 0, st, g, sp, tiles_m, tiles_n,
                     group_n, gemm_epilogue_vec_ok(a) ? 1 : 0);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// sums the fp32 slabs of a split product in slab order and applies the product's epilogue
template <int EPI, typename TC>
__global__ __launch_bounds__(256) void split_epilogue_kernel(GemmDev<bf16> g, const float* __restrict__ part, int splits,
                                                             int64_t slab) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= slab) return;
  // eight slabs' loads in flight at a time; the additions keep the slab order
  float v = 0.f;
  for (int s0 = 0; s0 < splits; s0 += 8) {
    float t[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) t[u] = s0 + u < splits ? part[(s0 + u) * slab + i] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) v += t[u];
  }
  epilogue_store<bf16, TC, EPI>(g, (int)(i / g.N), (int)(i % g.N), v);
}
template <int EPI, typename TC>
void launch_split_epilogue(const Gemm& a, const float* part, int splits, hipStream_t st) {
  GemmDev<bf16> g{(const bf16*)a.A, (const bf16*)a.B, a.C, a.M, a.N, a.K, a.lda, a.ldb, a.ldc,
                  (const bf16*)a.bias, (const bf16*)a.aux, (bf16*)a.aux_out, a.ld_aux};
  const int64_t mn = (int64_t)a.M * a.N;
  hipLaunchKernelGGL((split_epilogue_kernel<EPI, TC>), dim3((unsigned)cdiv64(mn, 256)), dim3(256), 0, st, g, part, splits, mn);
}

}  // namespace

bool gemm_dma_ok(const Gemm& a) {
  if (a.K % kBK != 0 || a.K < kBK) return false;
  if (!aligned16(a.A) || !aligned16(a.B) || a.lda % 8 || a.ldb % 8) return false;
  if (a.ta && (a.M % 8 || a.M < 8)) return false;
  if (!a.tb && (a.N % 8 || a.N < 8)) return false;
  return a.M >= 32 && a.N >= 32;
}

// workgroups a split-K weight gradient aims for: two 256x128 workgroups per CU
#ifdef PT_TUNING_HOOKS
int g_split_target = 512;
void gemm_set_split_target(int t) { g_split_target = t; }
void gemm_set_group(int tiles, long bytes) {
  g_group_n = tiles;
  if (bytes > 0) g_group_bytes = bytes;
}
#else
constexpr int g_split_target = 512;
#endif

// weight gradients (both operands strided in memory: whole cache lines whatever BK): BK = 32, three stages
template <int BM, int BN, int WGM, int WGN>
static void dispatch_wgrad(const Gemm& a, hipStream_t st) {
  constexpr int NS = 3, BK = 32;
  const int tiles = cdiv(a.M, BM) * cdiv(a.N, BN), nk = a.K / BK;
  int splits = 1;
  const int64_t mn = (int64_t)a.M * a.N;
  if (a.ws) {
    splits = g_split_target / tiles;
    if (splits > nk / 8) splits = nk / 8;
    if (splits > 16) splits = 16;
    if (splits < 1) splits = 1;
    while (splits > 1 && (size_t)(splits * (mn + a.N)) > a.ws_floats) --splits;
  }
  float* cs_part = nullptr;
  if (a.colsum_out) cs_part = splits > 1 ? a.ws + splits * mn : a.colsum_out;
  if (splits > 1) {
    launch_dma<BM, BN, WGM, WGN, NS, BK, true, false, EPI_STORE, float>(a, splits, a.ws, mn, cs_part, st);
    gemm_splitk_reduce(a.ws, splits, mn, (float*)a.C, a.colsum_out ? cs_part : nullptr, a.N, a.colsum_out, st);
  } else {
    launch_dma<BM, BN, WGM, WGN, NS, BK, true, false, EPI_STORE, float>(a, 1, nullptr, 0, cs_part, st);
  }
}

bool gemm_wgrad_group(const Gemm* a, int n, hipStream_t st, hipEvent_t mid, WgradCarry* carry, LnBwdRide* ln) {
  if (n < 1 || n > kMaxGroup) return false;
  int64_t total = 0, per_split = 0;
  for (int i = 0; i < n; ++i) {
    const Gemm& m = a[i];
    if (!m.ta || m.tb || !m.c_f32 || m.ldc != m.N || m.epi != EPI_STORE || !gemm_dma_ok(m) || m.K % 64 != 0) return false;
    if (m.K != a[0].K || m.ws != a[0].ws || m.ws_floats != a[0].ws_floats || !m.ws) return false;
    total += (int64_t)cdiv(m.M, 256) * cdiv(m.N, 256);
    per_split += (int64_t)m.M * m.N + m.N;
  }
  const int nk = a[0].K / 64;
  int splits = (int)(256 / total);
  if (splits > nk / 4) splits = nk / 4;
  if (splits > 16) splits = 16;
  if (splits < 1) splits = 1;
  while (splits > 1 && (size_t)(splits * per_split) > a[0].ws_floats) --splits;
  GroupArgs ga{};
  ga.nprob = n;
  ga.splits = splits;
  ga.tiles_per_split = cdiv(nk, splits);
  float* ws = a[0].ws;
  const float* part[kMaxGroup];
  const float* cpart[kMaxGroup];
  int t0 = 0;
  for (int i = 0; i < n; ++i) {
    const Gemm& m = a[i];
    const int64_t mn = (int64_t)m.M * m.N;
    float* cbase = splits > 1 ? ws : (float*)m.C;
    float* cs = !m.colsum_out ? nullptr : (splits > 1 ? ws + splits * mn : m.colsum_out);
    part[i] = cbase;
    cpart[i] = cs;
    ga.g[i] = GemmDev<bf16>{(const bf16*)m.A, (const bf16*)m.B, (void*)cbase, m.M, m.N, m.K, m.lda, m.ldb, m.ldc,
                            nullptr, nullptr, nullptr, 0};
    ga.colsum[i] = cs;
    ga.slab[i] = splits > 1 ? mn : 0;
    ga.tile0[i] = t0;
    ga.tiles_n[i] = cdiv(m.N, 256);
    ga.vec_ok[i] = gemm_epilogue_vec_ok(m) && aligned16(cbase) ? 1 : 0;
    t0 += cdiv(m.M, 256) * cdiv(m.N, 256);
    if (splits > 1) ws += splits * (mn + m.N);
  }
  ga.tile0[n] = t0;
  const int own = 8 * cdiv(t0 * splits, 8);
  // a carried reduction rides on the workgroups that fit beside this launch's own (one per CU, 256 CUs), in
  // multiples of eight (one per XCD); with fewer than eight to spare it runs on its own first
  int extra = ((256 - own) / 8) * 8;
  if (extra < 8) extra = 0;
  const bool host_ln = ln && extra > 0 && ln->D <= 1024 && ln->D % 4 == 0 && ln->rows > 0 && ln->partial;
  if (host_ln) {
    ga.ln = LnBwdArgs<bf16, bf16, bf16>{(const bf16*)ln->dy, ln->lddy, (const bf16*)ln->x, ln->ldx, ln->mean, ln->rstd,
                                        (const bf16*)ln->gamma, ln->dres, ln->lddres, ln->dx_s, (bf16*)ln->dx_o, ln->lddx,
                                        ln->partial, ln->rows, ln->D};
    ga.ln_on = ln->f32_in ? 2 : 1;
    ln->taken_np = extra;
  }
  if (!(carry && carry->nprob > 0)) {
    if (!host_ln) extra = 0;
  } else {
    if (extra == 0) {
      gemm_wgrad_flush(carry, st);
    } else {
      ga.c_nprob = carry->nprob;
      ga.c_splits = carry->splits;
      for (int i = 0; i < carry->nprob; ++i) {
        ga.c_part[i] = carry->part[i]; ga.c_out[i] = carry->out[i]; ga.c_n[i] = carry->n[i];
        ga.c_vec[i] = splitk_vec_ok4(carry->part[i], carry->n[i], carry->out[i]);
        ga.c_part2[i] = carry->part2[i]; ga.c_out2[i] = carry->out2[i]; ga.c_n2[i] = carry->part2[i] ? carry->n2[i] : 0;
        ga.c_vec2[i] = carry->part2[i] ? splitk_vec_ok4(carry->part2[i], carry->n2[i], carry->out2[i]) : 0;
      }
      carry->nprob = 0;
    }
  }
  hipLaunchKernelGGL(gemm_wgrad_group_kernel, dim3(own + extra), dim3(512), 0, st, ga);
  if (mid) (void)hipEventRecord(mid, st);
  if (splits > 1) {
    WgradCarry now;
    now.nprob = n;
    now.splits = splits;
    for (int i = 0; i < n; ++i) {
      now.part[i] = part[i]; now.out[i] = (float*)a[i].C; now.n[i] = (int64_t)a[i].M * a[i].N;
      now.part2[i] = a[i].colsum_out ? cpart[i] : nullptr; now.out2[i] = a[i].colsum_out; now.n2[i] = a[i].N;
    }
    if (carry) *carry = now;               // summed by the next launch or by gemm_wgrad_flush
    else gemm_wgrad_flush(&now, st);
  }
  return true;
}

template <int BM>
static void dispatch_pp_fwd(const Gemm& a, hipStream_t st) {
#define PT_L(TB_, EPI_, TC_) launch_pp<BM, false, TB_, EPI_, TC_>(a, 1, nullptr, 0, nullptr, st)
  if (a.tb) {
    if (a.c_f32) PT_L(true, EPI_RES, float);
    else if (a.epi == EPI_STORE) PT_L(true, EPI_STORE, bf16);
    else PT_L(true, EPI_MUL_DGELU, bf16);
    return;
  }
  if (a.c_f32) {
    if (a.epi == EPI_BIAS) PT_L(false, EPI_BIAS, float);
    else PT_L(false, EPI_BIAS_RES, float);
  } else {
    if (a.epi == EPI_BIAS) PT_L(false, EPI_BIAS, bf16);
    else if (a.epi == EPI_BIAS_RES) PT_L(false, EPI_BIAS_RES, bf16);
    else PT_L(false, EPI_BIAS_GELU, bf16);
  }
#undef PT_L
}

// forward and input-gradient products (at least one k-major operand)
template <int BM, int BN, int WGM, int WGN, int NS, int BK>
static void dispatch_fwd(const Gemm& a, hipStream_t st) {
#define PT_L(TB_, EPI_, TC_) launch_dma<BM, BN, WGM, WGN, NS, BK, false, TB_, EPI_, TC_>(a, 1, nullptr, 0, nullptr, st)
  if (a.tb) {
    if (a.c_f32) PT_L(true, EPI_RES, float);
    else if (a.epi == EPI_STORE) PT_L(true, EPI_STORE, bf16);
    else PT_L(true, EPI_MUL_DGELU, bf16);
    return;
  }
  if (a.c_f32) {
    if (a.epi == EPI_BIAS) PT_L(false, EPI_BIAS, float);
    else PT_L(false, EPI_BIAS_RES, float);
  } else {
    if (a.epi == EPI_BIAS) PT_L(false, EPI_BIAS, bf16);
    else if (a.epi == EPI_BIAS_RES) PT_L(false, EPI_BIAS_RES, bf16);
    else PT_L(false, EPI_BIAS_GELU, bf16);
  }
#undef PT_L
}

// Few rows and a long contraction (the products of a top block that works on first-token rows, e.g.
// 64 x 768 x 3072): the six workgroups of the output would each walk all of K one tile latency at a time
// (45 us).  K is split over more workgroups into fp32 slabs in the caller's workspace, and a small kernel
// sums the slabs in order and applies the epilogue.
bool gemm_dma_skinny(const Gemm& a, hipStream_t st) {
  if (a.ta || a.M > 128 || !a.ws || !gemm_dma_ok(a)) return false;
  const int nk = a.K / 32;
  int splits = nk / 12;   // at least 12 k tiles per split
  if (splits > 16) splits = 16;
  const int64_t mn = (int64_t)a.M * a.N;
  while (splits > 1 && (size_t)(splits * mn) > a.ws_floats) --splits;
  if (splits < 2) return false;
  Gemm p = a;
  p.C = a.ws; p.ldc = a.N; p.c_f32 = true; p.epi = EPI_STORE; p.bias = nullptr; p.aux = nullptr; p.aux_out = nullptr;
  if (a.tb) launch_dma<128, 128, 2, 2, 3, 32, false, true, EPI_STORE, float>(p, splits, a.ws, mn, nullptr, st);
  else launch_dma<128, 128, 2, 2, 3, 32, false, false, EPI_STORE, float>(p, splits, a.ws, mn, nullptr, st);
#define PT_SE(EPI_, TC_) launch_split_epilogue<EPI_, TC_>(a, a.ws, splits, st)
  if (a.tb) {
    if (a.c_f32) PT_SE(EPI_RES, float);
    else if (a.epi == EPI_STORE) PT_SE(EPI_STORE, bf16);
    else PT_SE(EPI_MUL_DGELU, bf16);
  } else if (a.c_f32) {
    if (a.epi == EPI_BIAS) PT_SE(EPI_BIAS, float);
    else PT_SE(EPI_BIAS_RES, float);
  } else {
    if (a.epi == EPI_BIAS) PT_SE(EPI_BIAS, bf16);
    else if (a.epi == EPI_BIAS_RES) PT_SE(EPI_BIAS_RES, bf16);
    else PT_SE(EPI_BIAS_GELU, bf16);
  }
#undef PT_SE
  return true;
}

void gemm_dma(const Gemm& a, int variant, hipStream_t st) {
  // variants: 1 = 128x128 tiles, 2 = 256x128, 5 / 6 = the two-group kernel with 256 / 192-row tiles
  if (a.ta) {   // a single weight gradient (a block's four go through gemm_wgrad_group)
    if (variant == 1) dispatch_wgrad<128, 128, 2, 2>(a, st);
    else dispatch_wgrad<256, 128, 4, 2>(a, st);
    return;
  }
  if ((variant == 5 || variant == 6) && a.K % 64 == 0) {
    if (variant == 5) dispatch_pp_fwd<256>(a, st);
    else dispatch_pp_fwd<192>(a, st);
    return;
  }
  // The single-role tilings keep 32-wide k tiles and three stages: with 64-wide tiles they fit one workgroup
  // less per CU and lose more than the whole-line loads gain.
  if (variant == 2 && a.K % 64 == 0) dispatch_fwd<256, 128, 4, 2, 3, 32>(a, st);
  else dispatch_fwd<128, 128, 2, 2, 3, 32>(a, st);
}

}  // namespace pt
