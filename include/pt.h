/*
 * pt.h - C ABI of the freeze-boundary training step for MI355X (gfx950).
 *
 * One training iteration of a Transformer encoder (ViT pre-LN / BERT post-LN,
 * paper App. A.1) whose L layers f_0 .. f_{L-1} (Sec. 2.1) are split at a
 * freeze boundary k = L_frozen (Sec. 3.1, Eq. 1):
 *
 *   pt_set_freeze_boundary(k)   F = F_frozen o F_pipe            (Sec. 3.2.1)
 *   pt_frozen_forward           forward-only through the front end and blocks
 *                               0..k-1, served from / written to the per-sample
 *                               activation cache           (Sec. 3.4, App. D.1)
 *   pt_active_fwd_bwd           forward + backward through blocks k..L-1 + head
 *   pt_layer_grad_norms         ||g_l|| for every layer               (Eq. 1)
 *   pt_optimizer_step           update of F_pipe's parameters only
 *                                                        (Sec. 3.3, App. D.2)
 *
 * General rules
 *  - Every pointer argument is marked HOST or DEVICE below.  The library never
 *    allocates device memory: the caller owns the four arenas handed to
 *    pt_create (sizes from pt_query_arena_bytes), the input / label buffers and
 *    the HIP stream.  pt_ctx owns host bookkeeping only.
 *  - All device work is enqueued on the stream given to pt_create.  Calls that
 *    return host scalars (loss, norms, reads) synchronise that stream.
 *  - Errors: every call returns a pt_status; nothing throws or aborts across
 *    the ABI.  Arguments and resources (arena sizes, LDS needs of the attention
 *    kernels, window slots of the host tier) are validated before anything is
 *    enqueued, so on PT_EINVAL / PT_ESTATE / PT_ENOMEM / PT_ECACHE_MISS the
 *    context is unchanged.  PT_EDEVICE reports a failed HIP call or kernel:
 *    work may have been enqueued by then, the step's results are undefined and
 *    the context should be destroyed.  pt_last_error gives a message.
 *  - Call order per step: pt_frozen_forward -> pt_active_fwd_bwd ->
 *    [pt_layer_grad_norms] -> pt_optimizer_step.  Out of order: PT_ESTATE.
 *    (pt_layer_grad_norms_begin takes the place of pt_layer_grad_norms in this
 *    order; its _end half may come any time later.)
 *  - Layouts: activations [B,S,D] row-major; linear maps y = x W + b with W
 *    stored [in,out] row-major; packed QKV weight columns [Q|K|V], head h owns
 *    columns h*dh..(h+1)*dh-1 of each third.  In PT_BF16 mode activations are
 *    bf16, accumulation / LayerNorm / softmax statistics / gradients of
 *    parameters / optimizer state are fp32, and forward/backward kernels read a
 *    bf16 shadow (round-to-nearest-even) of the fp32 master parameters.
 */
#ifndef PT_H_
#define PT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The shared library is built with hidden visibility: these entry points are all it exports. */
#define PT_API __attribute__((visibility("default")))

typedef struct pt_ctx pt_ctx;

typedef enum {
  PT_OK = 0,
  PT_EINVAL = 1,      /* bad argument (NULL, out of range, decreasing boundary) */
  PT_ESTATE = 2,      /* call out of order                                      */
  PT_ENOMEM = 3,      /* host allocation failed or an arena is too small        */
  PT_EDEVICE = 4,     /* a HIP call or kernel reported an error                 */
  PT_ECACHE_MISS = 5  /* pt_cache_row: the slot holds nothing                   */
} pt_status;

enum { PT_VIT_PRELN = 0, PT_BERT_POSTLN = 1 };   /* App. A.1: where LayerNorm sits */
enum { PT_F32 = 0, PT_BF16 = 1 };
enum { PT_SGDM = 0, PT_ADAMW = 1 };
/* Task head.  DEFAULT: ViT = final LayerNorm + CLS token + linear classifier (image classification,
 * Sec. 4.1); BERT = per-token start / end logits (span QA, Sec. 4.1).  CLS (BERT only): the first
 * token's final activation -> linear classifier over n_out classes (sequence classification). */
enum { PT_HEAD_DEFAULT = 0, PT_HEAD_CLS = 1 };

typedef struct {
  int32_t arch;        /* PT_VIT_PRELN | PT_BERT_POSTLN                              */
  int32_t dtype;       /* PT_F32 | PT_BF16                                           */
  int32_t L, D, H, F;  /* blocks, hidden, heads, MLP width; D % H == 0, D/H % 8 == 0 and <= 128, D <= 2048, F % 4 == 0 */
  int32_t S;           /* sequence length (ViT: (img/patch)^2 + 1).  Without matrix-core attention (PT_F32, or
                          D/H != 64) a strip of 32 score rows lives in LDS: S <= about 1100 at D/H = 64      */
  int32_t B;           /* largest batch any call will pass                           */
  int32_t n_out;       /* classes (ViT, BERT with PT_HEAD_CLS) or 2 (BERT span QA)   */
  int32_t img, patch, chans;  /* ViT front end                                       */
  int32_t vocab, max_pos;     /* BERT front end, max_pos >= S                        */
  float ln_eps;
  int32_t optimizer;   /* PT_SGDM | PT_ADAMW                                         */
  int32_t head;        /* PT_HEAD_DEFAULT | PT_HEAD_CLS                              */
  int32_t grad_accum;  /* 1: the state arena also holds a gradient accumulator, see pt_accumulate_grads */
  int32_t k_min;       /* the boundary this context starts at and can never be below (0 = everything may train).
                          Blocks 0..k_min-1 (and the front end when k_min >= 1) are frozen for good, so nothing a
                          frozen layer does not need (Sec. 3.2.1 item 2) is planned for them: the state arena holds
                          gradients and moments of the tensors from block k_min on only, and the work arena no
                          saved activations of theirs                                                */
  int64_t cache_slots; /* 0 = no cache; slot i belongs to sample id i                */
  int64_t host_slots;  /* rows of the host tier: sample ids cache_slots .. cache_slots+host_slots-1 (0 = none) */
  int64_t window_slots;/* device rows the host tier is staged through, >= 2 B when host_slots > 0; they are
                          the last rows of the cache arena                            */
} pt_config;

typedef struct {
  float lr, momentum, beta1, beta2, eps, weight_decay;
} pt_opt_hparams;

/* Bytes of the four caller-owned DEVICE arenas for this configuration:
 * params (fp32 masters + bf16 shadows), state (fp32 gradients + optimizer
 * moments, + one gradient accumulator when grad_accum is set), work (activations, saved tensors, scratch), cache (cache_slots rows
 * of S*D activations).  state and work shrink with cfg->k_min: a context that
 * resumes training at a boundary k_min >= 1 is sized for F_pipe = blocks
 * k_min..L-1 plus a forward-only F_frozen.  Each must be 256-byte aligned.
 * PT_EINVAL on a bad configuration. */
PT_API pt_status pt_query_arena_bytes(const pt_config* cfg /*HOST*/, size_t* params, size_t* state,
                               size_t* work, size_t* cache /*HOST out*/);

/* Creates a context over the arenas (DEVICE pointers, sizes as queried).  The
 * params and state arenas are cleared (enqueued); parameters are then set with
 * pt_write_tensor.  hip_stream is a hipStream_t (NULL = default stream).  The
 * boundary starts at k = k_min (0 unless the configuration says otherwise) and
 * the step counter at 0 (Eq. 1: L_frozen^(0)=0). */
PT_API pt_status pt_create(const pt_config* cfg /*HOST*/, void* d_params, void* d_state, void* d_work,
                    void* d_cache /*DEVICE, may be NULL iff cache_slots==0*/, void* hip_stream,
                    pt_ctx** out /*HOST out*/);
PT_API pt_status pt_destroy(pt_ctx* ctx);

/* Moves the freeze boundary: blocks 0..k-1 (and, for k >= 1, the front end)
 * become F_frozen.  0 <= k <= L and k >= current boundary, otherwise PT_EINVAL
 * and nothing changes (the argmin of Eq. 1 ranges over layers at or above the
 * previous boundary, so the boundary never moves down).  Gradients and
 * optimizer moments of newly frozen tensors are cleared and never used again
 * (Sec. 3.2.1); cache rows written at a smaller k become stale and are advanced
 * on their next use (Sec. 3.4). */
PT_API pt_status pt_set_freeze_boundary(pt_ctx* ctx, int32_t k);
PT_API pt_status pt_get_freeze_boundary(const pt_ctx* ctx, int32_t* k /*HOST out*/);

/* F_frozen for one batch of nb <= B samples.
 *  d_input    DEVICE. ViT: fp32 images [nb,chans,img,img]; BERT: int32 ids [nb,S].
 *             Read by kernels enqueued in this call only (the ids that the
 *             token-table gradient needs at k == 0 are copied into the work
 *             arena), so the buffer may be released or reused, in stream
 *             order, once the call returns.  Token ids are not read on the
 *             host: an id outside [0,vocab) is clamped to the nearest valid
 *             row of the table instead of being reported.
 *  sample_ids HOST, nb unique ids in [0,cache_slots+host_slots), or NULL to bypass the
 *             cache.  Ignored when k == 0 (nothing is frozen, the front end is
 *             being trained).  Per sample: a row written at the current k is a
 *             hit (copied, no block runs); a row written at k' < k is advanced
 *             through blocks k'..k-1 only; otherwise the front end and blocks
 *             0..k-1 run.  Updated rows are written back (App. D.1 item 2).
 *  d_hk_out   HOST out: DEVICE pointer to the boundary activation [nb,S,D]
 *             inside the work arena, valid until the next pt_frozen_forward.
 * Results per sample do not depend on the sample's position in the batch. */
PT_API pt_status pt_frozen_forward(pt_ctx* ctx, const void* d_input, int32_t nb, const int64_t* sample_ids,
                            void** d_hk_out);

/* The timing profiler of the cache (Sec. 3.4: caching is switched on only once it is faster than
 * recomputing the frozen prefix; Sec. 4.3.5 reports from which boundary that held on the paper's
 * cluster).  Runs pt_frozen_forward for this batch once to write or advance its rows, then `reps`
 * times bypassing the cache and `reps` times from the cache (all hits), timed with events on the
 * context's stream, and returns the mean milliseconds per call of each (HOST out).  The caller passes
 * sample_ids = NULL to later calls while ms_cached >= ms_recompute.  Needs k >= 1 and a cache;
 * synchronises; leaves the context as after a pt_frozen_forward of this batch. */
PT_API pt_status pt_time_frozen_forward(pt_ctx* ctx, const void* d_input /*DEVICE*/, int32_t nb,
                                 const int64_t* sample_ids /*HOST*/, int32_t reps, float* ms_recompute,
                                 float* ms_cached);

/* F_pipe: forward through blocks k..L-1 and the task head, loss, backward down
 * to block k (and the front end iff k == 0), for the batch of the preceding
 * pt_frozen_forward.
 *  d_hk      DEVICE [nb,S,D] boundary activation (normally *d_hk_out); read only.
 *  d_labels  DEVICE int32: ViT and BERT with PT_HEAD_CLS [nb] class ids; BERT span QA [nb,2]
 *             (start,end) positions.
 *  loss_out  HOST out, mean loss over the batch; the call synchronises.  May be
 *            NULL: then nothing synchronises and pt_last_loss fetches it later.
 * Gradients of all active tensors are overwritten (not accumulated). */
PT_API pt_status pt_active_fwd_bwd(pt_ctx* ctx, const void* d_hk, const int32_t* d_labels, float* loss_out);
PT_API pt_status pt_last_loss(pt_ctx* ctx, float* loss_out /*HOST out*/);

/* L2 norm of the gradient of every layer taken as one vector (Eq. 1's ||g_l||,
 * on the raw gradient of the mean loss of the last pt_active_fwd_bwd).
 * norms_out HOST, L+2 floats: [front end, block 0 .. block L-1, head]; frozen
 * layers (and the front end when k >= 1) read exactly 0.  Synchronises. */
PT_API pt_status pt_layer_grad_norms(pt_ctx* ctx, float* norms_out);

/* The same in two halves, for callers that do not want the stream to run dry
 * while the host waits, nor the gradient to be read twice:
 * pt_layer_grad_norms_begin (same preconditions as pt_layer_grad_norms) asks
 * for the norms of the gradients as they are now and returns at once;
 * pt_layer_grad_norms_end waits for them and copies the L+2 norms to norms_out
 * (HOST).  If pt_optimizer_step comes between the two, its pass over the
 * gradient (which it reads and does not change) leaves the sums of squares as a
 * by-product and the host's wait comes after the update is queued; any other
 * call that would change the gradients or the boundary first has the norm
 * kernels enqueued ahead of it.  Either way the values are, bit for bit, what
 * pt_layer_grad_norms would have returned at the point of _begin.  One set of
 * norms can be pending at a time: a second _begin (or pt_layer_grad_norms)
 * before _end, or _end without _begin, is PT_ESTATE. */
PT_API pt_status pt_layer_grad_norms_begin(pt_ctx* ctx);
PT_API pt_status pt_layer_grad_norms_end(pt_ctx* ctx, float* norms_out);

/* pt_layer_grad_norms for callers that cannot allocate device memory and have
 * no scratch to lend (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same kernels, with the per-chunk partial
 * sums in a 2 MB array that the library holds in static device memory on every
 * GPU it runs on, instead of in the work arena.  Same preconditions, arguments
 * and results (bit for bit) as pt_layer_grad_norms; calls no allocating
 * routine.  Limit: models of at most 2^19 * 1024 = 536 870 912 parameters after
 * padding each tensor to a multiple of 1024 (larger: PT_EINVAL, nothing
 * enqueued).  All contexts on one GPU share the array and it keeps the last
 * call's contents (nothing needs clearing: every value read was written by the
 * same call): calls that overlap on one GPU race and must be serialised by the
 * caller.  Synchronises. */
PT_API pt_status pt_layer_grad_norms_static(pt_ctx* ctx, float* norms_out /*HOST, L+2*/);

/* Micro-batch gradient accumulation (Sec. 2.1 pipeline parallelism and Sec. 3.2.3:
 * a mini-batch is processed as M micro-batches whose gradients are combined
 * before the single optimizer step).  For configurations with grad_accum = 1:
 * after each micro-batch's pt_active_fwd_bwd, pt_accumulate_grads adds
 * nb * gradient (nb = that micro-batch's size; first != 0 starts a new sum) and
 * nb * loss into the accumulator and readies the context for the next
 * micro-batch; pt_finish_accumulation then leaves the sample-weighted mean
 * gradient (= the gradient of the mean loss over all accumulated samples) where
 * pt_layer_grad_norms and pt_optimizer_step read it, and returns the mean loss
 * (mean_loss_out HOST, may be NULL; a non-NULL pointer synchronises).  Only the
 * active tensors are touched.  PT_ESTATE if called out of order, if grad_accum
 * is 0, or if the boundary is moved while a sum is in progress. */
PT_API pt_status pt_accumulate_grads(pt_ctx* ctx, int32_t first);
PT_API pt_status pt_finish_accumulation(pt_ctx* ctx, float* mean_loss_out);

/* One optimizer step over the active tensors only; frozen bytes are untouched.
 * SGD-momentum: v <- mu v + g (+ wd w on decayed tensors), w <- w - lr v.
 * AdamW: decoupled decay, bias-corrected moments, one shared step counter.
 * Decayed tensors: weight matrices and the token table.  Also refreshes the
 * bf16 shadow in PT_BF16 mode. */
PT_API pt_status pt_optimizer_step(pt_ctx* ctx, const pt_opt_hparams* hp /*HOST*/);

/* Eq. 1 with the readings: argmin over blocks k_prev..L-1, bound
 * floor(k_prev + alpha (L - k_prev)) evaluated in double precision (alpha is a
 * double so that e.g. 0.7 * 10 is not read as 6.9999998), ties to the lowest
 * index.  norms HOST, L+2 floats as returned by pt_layer_grad_norms.  Pure host
 * arithmetic; does not move the boundary.  PT_EINVAL unless 0 < alpha < 1. */
PT_API pt_status pt_next_boundary(const float* norms, int32_t L, int32_t k_prev, double alpha, int32_t* k_next);

/* ---- tensor table and state access (synchronising host copies) ---------- */
enum { PT_KIND_PARAM = 0, PT_KIND_GRAD = 1, PT_KIND_MOMENT1 = 2, PT_KIND_MOMENT2 = 3,
       PT_KIND_SHADOW = 4 /* bf16 shadow widened to fp32; PT_BF16 mode only */ };

PT_API pt_status pt_num_tensors(const pt_ctx* ctx, int32_t* n /*HOST out*/);
/* name: HOST buffer of name_cap bytes (NUL-terminated on return); group is the
 * grad-norm slot (0 front, 1+l block l, L+1 head). */
PT_API pt_status pt_tensor_info(const pt_ctx* ctx, int32_t id, char* name, size_t name_cap, int64_t* numel,
                         int32_t* rows, int32_t* cols, int32_t* group, int32_t* decayed);
/* fp32 HOST buffers of numel elements.  pt_write_tensor(PT_KIND_PARAM) also
 * refreshes the bf16 shadow.  PT_KIND_SHADOW is read-only.  A tensor below
 * k_min has no gradient or moments: reading them gives zeros, writing them is
 * PT_EINVAL. */
PT_API pt_status pt_write_tensor(pt_ctx* ctx, int32_t id, int32_t kind, const float* src);
PT_API pt_status pt_read_tensor(pt_ctx* ctx, int32_t id, int32_t kind, float* dst);
PT_API pt_status pt_get_step_count(const pt_ctx* ctx, int64_t* t);
PT_API pt_status pt_set_step_count(pt_ctx* ctx, int64_t t);

/* Activations of the last step widened to fp32 (parity checks).  PT_ACT_HL: when the head reads only each
 * sample's first token (ViT; BERT with the classification head), S >= 4 and the top block is active, that
 * block computes only those rows of its output: rows [b, 0, :] are defined, the others unspecified. */
enum { PT_ACT_HK = 0 /*[nb,S,D]*/, PT_ACT_HL = 1 /*[nb,S,D]*/, PT_ACT_LOGITS = 2 /*ViT [nb,n_out]; BERT [nb,S,2]*/,
       PT_ACT_DHK = 3 /*[nb,S,D] gradient wrt the boundary activation; valid when k == 0 or arch-internal*/ };
PT_API pt_status pt_read_activation(pt_ctx* ctx, int32_t which, float* dst /*HOST*/, size_t numel);

/* Cache inspection.  pt_cache_row copies the raw row bytes (S*D elements of the
 * activation type) to HOST and reports the boundary it was written at;
 * PT_ECACHE_MISS if the slot is empty.  pt_cache_stats: counters since creation
 * of per-sample decisions and of (sample, block) forward evaluations spent in
 * pt_frozen_forward. */
PT_API pt_status pt_cache_row(pt_ctx* ctx, int64_t sample_id, void* dst, size_t dst_bytes, int32_t* written_at_k);

/* Host tier of the cache (Sec. 3.4, App. E: when the cached activations do not
 * fit the fast tier they live one level down and pass through a sliding window
 * that is filled ahead of use and emptied as rows are consumed).  Here the fast
 * tier is HBM (sample ids below cache_slots) and the lower tier is pinned HOST
 * memory of host_slots rows (S*D elements of the activation type each), owned by
 * the caller and attached once after pt_create.  Host rows travel on a copy
 * stream of the library's own: pt_cache_prefetch stages the valid host rows of
 * the given ids (typically the NEXT batch's) into free window slots while the
 * current step computes (best effort: it stops when the window is full;
 * staged_out HOST, may be NULL); pt_frozen_forward uses staged rows, stages the
 * others on demand, writes new or advanced rows back to the host asynchronously
 * and releases window slots as rows are consumed.  Decisions (hit / advance /
 * miss) and the bytes of h_k do not depend on the tier.  pt_host_tier_stats:
 * rows moved each way, rows staged by pt_cache_prefetch, and how many of those
 * were then used. */
PT_API pt_status pt_attach_host_tier(pt_ctx* ctx, void* h_rows /*pinned HOST*/, size_t bytes);
PT_API pt_status pt_cache_prefetch(pt_ctx* ctx, const int64_t* sample_ids /*HOST*/, int32_t n, int32_t* staged_out);
PT_API pt_status pt_host_tier_stats(const pt_ctx* ctx, int64_t* rows_to_device, int64_t* rows_to_host,
                             int64_t* prefetched, int64_t* prefetched_used);
PT_API pt_status pt_cache_stats(const pt_ctx* ctx, int64_t* hits, int64_t* advances, int64_t* misses,
                         int64_t* block_runs);

/* Optional kernel timing.  While enabled, every launcher call of the listed
 * categories is bracketed by two HIP events on the context's stream; totals are
 * folded in when the optimizer step ends or when they are read (synchronises).
 * `work` sums the algorithmic FLOPs (GEMM and attention categories) or bytes
 * (optimizer, norms) of the timed launches, 0 for the others.  Timing costs a few
 * microseconds per launch, so throughput is measured with it off. */
enum { PT_PROF_GEMM_GENERIC = 0, PT_PROF_GEMM_NN = 1 /* y = x W */, PT_PROF_GEMM_NT = 2 /* dx = dy W^T */,
       PT_PROF_GEMM_TN = 3 /* dW = x^T dy */, PT_PROF_ATTN_FWD = 4, PT_PROF_ATTN_BWD = 5, PT_PROF_LN_FWD = 6,
       PT_PROF_LN_BWD = 7, PT_PROF_COLSUM = 8, PT_PROF_OPT = 9, PT_PROF_NORMS = 10, PT_PROF_CACHE = 11,
       PT_PROF_WGRAD_BLOCK = 12 /* the four weight gradients of one block as one grouped kernel launch; the
                                   reduction of its split-K slabs is booked under the next category */,
       PT_PROF_SPLITK_REDUCE = 13, PT_PROF_COUNT = 14 };
PT_API pt_status pt_profile_enable(pt_ctx* ctx, int32_t on);
PT_API pt_status pt_profile_reset(pt_ctx* ctx);
PT_API pt_status pt_profile_read(pt_ctx* ctx, int32_t category, double* total_ms, int64_t* launches, double* work /*HOST out*/);

PT_API const char* pt_last_error(const pt_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PT_H_ */
