// Host-side launchers of the gfx950 kernels.  `dt` selects the activation /
// compute-parameter element type: 0 = fp32, 1 = bf16 (fp32 accumulation).
// Every launcher validates nothing: the orchestrator checks shapes first.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pt {

enum Epi {
  EPI_STORE = 0,      // C = acc
  EPI_BIAS = 1,       // C = acc + bias[n]
  EPI_BIAS_RES = 2,   // C = acc + bias[n] + aux[m,n]
  EPI_BIAS_GELU = 3,  // h = acc + bias[n]; aux_out[m,n] = GELU'(h) (if non-null); C = GELU(h)
  EPI_MUL_DGELU = 4,  // C = acc * aux[m,n], aux = the GELU'(h) that EPI_BIAS_GELU saved
  EPI_RES = 5         // C = acc + aux[m,n]
};

struct Gemm {
  const void* A = nullptr;  // ta ? [K,M] : [M,K], leading dimension lda
  const void* B = nullptr;  // tb ? [N,K] : [K,N], leading dimension ldb
  void* C = nullptr;        // [M,N], leading dimension ldc; T, or float when c_f32
  int M = 0, N = 0, K = 0;
  int64_t lda = 0, ldb = 0, ldc = 0;
  bool ta = false, tb = false;
  Epi epi = EPI_STORE;
  const void* bias = nullptr;  // T [N]
  const void* aux = nullptr;   // T [M,N] ld_aux (fp32 when c_f32: the gradient stream)
  void* aux_out = nullptr;     // T [M,N] ld_aux
  int64_t ld_aux = 0;
  bool c_f32 = false;
  // weight-gradient products (ta && !tb, fp32 C with ldc == N) may split K over several workgroups
  // through `ws` (ws_floats fp32 of scratch) and can also return the column sums of B over K
  // (the bias gradient) in colsum_out[N]
  float* ws = nullptr;
  size_t ws_floats = 0;
  float* colsum_out = nullptr;
};
void gemm(int dt, const Gemm& g, hipStream_t st);
// n weight-gradient products (ta, fp32 C with ldc == N) over the same K and sharing one workspace.  With
// bf16 operands up to four of them run as one launch (one encoder block has too few output tiles per matrix
// to fill the chip without a deep split over K); otherwise they run one after the other.
// `mid` (may be null): an event recorded behind the product kernels and in front of the reduction of the
// split-K slabs, so that a caller can time the two parts separately.
// `carry` (may be null): with it the reduction of this launch's split-K slabs is not launched but described
// in *carry, and a reduction that *carry describes on entry is done by this launch, on workgroups added for
// the CUs that its own tiles leave idle (or on its own first, if this launch cannot host it).  The weight
// gradients of a launch are therefore final only after the next call with the same carry or after
// gemm_wgrad_flush; successive calls must use different workspaces (the carried slabs stay where they are).
struct WgradCarry {
  int nprob = 0, splits = 0;
  const float* part[4] = {}; float* out[4] = {}; int64_t n[4] = {};      // slabs -> weight gradient
  const float* part2[4] = {}; float* out2[4] = {}; int64_t n2[4] = {};   // column-sum partials -> bias gradient (or null)
};
// `ln` (may be null): a LayerNorm backward pass in bf16 mode with D <= 1024 (the arguments of
// layernorm_bwd) that is independent of these products.  A grouped launch that has workgroups to spare runs
// it beside the matrix work, leaves one partial row per such workgroup in ln->partial and sets ln->taken_np
// to their number; the caller then owes the sum over those rows (layernorm_bwd_reduce).  taken_np == 0: the
// pass was not taken and is still to be run.
struct LnBwdRide {
  const void* dy; int64_t lddy; const void* x; int64_t ldx; const float* mean; const float* rstd; const void* gamma;
  const float* dres; int64_t lddres; float* dx_s; void* dx_o; int64_t lddx; float* partial; int rows, D;
  bool f32_in = false;   // dy and x are fp32 (the post-LN passes), else both bf16
  int taken_np = 0;
};
void gemm_wgrad_batch(int dt, const Gemm* g, int n, hipStream_t st, hipEvent_t mid = nullptr, WgradCarry* carry = nullptr,
                      LnBwdRide* ln = nullptr);
void gemm_wgrad_flush(WgradCarry* carry, hipStream_t st);
// workspace floats gemm_wgrad_batch may use for a block's four matrices (D x 3D, D x D, D x F, F x D)
size_t gemm_wgrad_batch_ws_floats(int D, int F);
// true when gemm() will run the matrix-core kernel for this problem
bool gemm_uses_mfma(int dt, const Gemm& g);

// ---- attention (softmax(q k^T / sqrt(dh)) v, no mask) over packed qkv [nb,S,3D]
void attention_fwd(int dt, const void* qkv, void* ctx, float* lse /*[nb,H,S] or null*/, int nb, int S, int H,
                   int dh, hipStream_t st);
void attention_bwd(int dt, const void* qkv, const void* ctx, const void* dctx, const float* lse, void* dqkv,
                   float* delta_ws /*[nb,H,S]*/, int nb, int S, int H, int dh, hipStream_t st);
// Dynamic LDS bytes the kernels without matrix cores (fp32 mode, or a head size other than 64) and the
// first-query kernels ask for at sequence length S; the orchestrator rejects configurations above the 160 KB
// of a CU before anything is launched.
size_t attention_generic_lds_bytes(int S, int dh);
size_t attention_first_query_lds_bytes(int S, int dh);
bool attention_uses_mfma(int dt, int dh);
// the same for each sample's first query only (nothing else of the output is read, or has a gradient):
// ctx_rows and do_rows [nb, D] hold the first tokens' rows; lse entry (b, h, 0) of [nb,H,S] is written / read
void attention_fwd_first_query(int dt, const void* qkv, void* ctx_rows, float* lse, int nb, int S, int H, int dh,
                               hipStream_t st);
void attention_bwd_first_query(int dt, const void* qkv, const void* ctx_rows, const void* do_rows, const float* lse,
                               void* dqkv, int nb, int S, int H, int dh, hipStream_t st);

// ---- LayerNorm over rows of length D
// y[r] = LN(x[r]); rows addressed r*ldx / r*ldy (elements).  x is fp32 when x_f32, else T.
// mean/rstd may be null.
void layernorm_fwd(int dt, bool x_f32, const void* x, int64_t ldx, const void* gamma, const void* beta, void* y,
                   int64_t ldy, float* mean, float* rstd, int rows, int D, float eps, hipStream_t st);
// dx[r] = LNbwd(dy[r]) (+ dres[r] if non-null).  dy is the fp32 gradient stream when dy_f32, else T.
// The result is written to dx_s (fp32) and / or dx_o (T), either may be null; both null computes the
// parameter gradients only.  dgamma/dbeta fp32 [D] via `partial` scratch of ln_partial_floats(D) floats.
// dxsum (may be null): fp32 [D] column sums of the result over the rows, i.e. the bias gradient of the
// linear map that produced this LayerNorm's input side.
size_t ln_partial_floats(int D);
// x_s[i * row_stride + d] += r[i * D + d] for i < n (fp32), x_o (T, may be null) gets the rounded sums of those
// rows, colsum[d] (may be null) += sum_i r[i * D + d]: adds a gradient that only every row_stride / D-th row has
void add_rows(int dt, const float* r, float* x_s, void* x_o, int64_t row_stride, float* colsum, int n, int D,
              hipStream_t st);
// With `deferred` non-null the pass leaves dgamma, dbeta and dxsum unwritten and describes in *deferred the
// sum over its partial rows that produces them (np = 0: nothing to sum); layernorm_bwd_reduce then does that
// for any number of passes in one launch per kLnReduceBatch of them.  Each such pass needs a `partial` of its own.
constexpr int kLnReduceBatch = 64;
struct LnReduceJob { const float* partial; int np; float* dgamma; float* dbeta; float* dxsum; };
void layernorm_bwd(int dt, bool dy_f32, bool x_f32, const void* dy, int64_t lddy, const void* x, int64_t ldx,
                   const float* mean, const float* rstd, const void* gamma, const float* dres, int64_t lddres,
                   float* dx_s, void* dx_o, int64_t lddx, float* dgamma, float* dbeta, float* dxsum, float* partial,
                   int rows, int D, hipStream_t st, LnReduceJob* deferred = nullptr);
void layernorm_bwd_reduce(const LnReduceJob* jobs, int n, int D, hipStream_t st);

// out[n] = sum_m X[m,n] (fp32), X is T [M,N] with leading dimension ld.
size_t colsum_partial_floats(int N);
void colsum(int dt, const void* X, int64_t ld, int M, int N, float* out, float* partial, hipStream_t st);

// ---- ViT front end
// sample b of the output reads image map[b] (map null = identity)
void vit_patchify(int dt, const float* images, const int64_t* map, void* patches, int nb, int chans, int img, int patch,
                  hipStream_t st);
void vit_assemble(int dt, const void* E, const void* cls, const void* pos, void* X, int nb, int S, int D,
                  hipStream_t st);
// dE[b*N+i] = dX[b,1+i]; dpos[s] = sum_b dX[b,s]; dcls = sum_b dX[b,0]
void vit_front_bwd(int dt, const float* dX, void* dE, float* dpos, float* dcls, int nb, int S, int D, hipStream_t st);

// ---- BERT front end
// ids outside [0, vocab) are clamped into the table
void bert_embed(int dt, const int32_t* ids, const int64_t* map, const void* Ew, const void* Ep, float* emb, int nb, int S,
                int D, int vocab, hipStream_t st);
// dEp[s] = sum_b demb[b,s] for s < S (rows >= S untouched); dEw rows: deterministic
// segmented sum over equal ids.  `dEw` must be zero on entry.
// `ws`: 2*nb*S + 4 int32 of scratch.
size_t bert_embed_ws_ints(int ntok, int vocab);
void bert_embed_bwd(const int32_t* ids, const float* demb, float* dEw, float* dEp, int32_t* ws, int nb, int S, int D,
                    int vocab, hipStream_t st);

// ---- losses
// ViT: z fp32 [nb,C]; writes per-sample loss, dz (T) = (softmax - onehot)/nb.
void ce_rows(int dt, const float* z, const int32_t* labels, float* loss_rows, void* dz, int nb, int C, hipStream_t st);
// BERT QA: x [nb,S,D] (T), W [D,2], b[2] (T).  z fp32 [nb,S,2] -> CE over S per column.
void qa_logits(int dt, const void* x, const void* W, const void* b, float* z, int rows, int D, hipStream_t st);
void qa_ce(int dt, const float* z, const int32_t* labels, float* loss_rows /*[nb]*/, float* dz /*fp32 [nb,S,2]*/, int nb,
           int S, hipStream_t st);
// dx[t] = dz[t,0] W[:,0] + dz[t,1] W[:,1]; dW[d,c] = sum_t x[t,d] dz[t,c]; db[c] = sum_t dz[t,c]
size_t qa_partial_floats(int D);
void qa_head_bwd(int dt, const void* x, const void* W, const float* dz, float* dx, float* dW, float* db, float* partial,
                 int rows, int D, hipStream_t st);
// loss = (sum_i rows[i]) / n, fixed order
void mean_reduce(const float* rows, int n, float* out, hipStream_t st);

// ---- plumbing
void fill_zero(void* p, size_t bytes, hipStream_t st);
// dst[dst_idx[i]] = src[src_idx[i]] for rows of row_bytes (multiple of 16); idx null = identity
void copy_rows(void* dst, const int64_t* dst_idx, const void* src, const int64_t* src_idx, int nrows,
               size_t row_bytes, hipStream_t st);
// nrows rows of row_bytes each from src + i * src_stride to dst + i * dst_stride (bytes), several such copies
// per launch: gathers every S-th row of a tensor into a dense block and scatters it back
struct RowCopy {
  const void* src;
  void* dst;
  int64_t src_stride, dst_stride;
  int row_bytes;
};
constexpr int kMaxRowCopies = 12;
void strided_rows_copy(const RowCopy* d, int n, int nrows, hipStream_t st);
void f32_to_bf16(const float* src, void* dst, size_t n, hipStream_t st);
void bf16_to_f32(const void* src, float* dst, size_t n, hipStream_t st);

// ---- gradient norms and optimizers over the padded, contiguous tensor arenas.
// Arenas are cut into chunks of kChunk floats; chunk c belongs to group chunk_group[c].
constexpr int kChunk = 1024;
void grad_accumulate_chunks(float* acc, const float* g, int64_t first_chunk, int64_t n_chunks, float weight, bool first,
                            const float* loss, float* loss_acc, hipStream_t st);
void grad_average_chunks(float* g, const float* acc, int64_t first_chunk, int64_t n_chunks, float inv, float* loss,
                         const float* loss_acc, hipStream_t st);
void sumsq_chunks(const float* g, float* chunk_sq, int64_t first_chunk, int64_t n_chunks, hipStream_t st);
// norms[grp] = sqrt(sum of chunk_sq over the chunk range of grp) for active groups, 0 otherwise
void finalize_norms(const float* chunk_sq, const int64_t* group_first_chunk /*[G+1] device*/, int G, int first_active,
                    int front_active, float* norms, hipStream_t st);
// Device address, on the current GPU, of the library's own array of static_chunk_capacity() per-chunk sums
// (resolved once per device; no allocation).  Calls that use it on one GPU must not overlap.
int64_t static_chunk_capacity();
hipError_t static_chunk_sums(float** out);
struct OptArgs {
  float lr, momentum, beta1, beta2, eps, weight_decay;
  float bias_c1, bias_c2;  // 1-beta1^t, 1-beta2^t
};
// chunk_sq non-null: the update also leaves each chunk's sum of squared gradients there, as sumsq_chunks would
void adamw_chunks(float* w, const float* g, float* m, float* v, void* shadow /*bf16 or null*/,
                  const uint8_t* chunk_decay, int64_t first_chunk, int64_t n_chunks, OptArgs a, float* chunk_sq,
                  hipStream_t st);
void sgdm_chunks(float* w, const float* g, float* m, void* shadow, const uint8_t* chunk_decay, int64_t first_chunk,
                 int64_t n_chunks, OptArgs a, float* chunk_sq, hipStream_t st);

}  // namespace pt
