// C ABI and step orchestration: tensor table, arena plan, freeze-boundary
// state machine, activation-cache index, and the sequence of kernel launches
// for F_frozen (forward only, nothing kept) and F_pipe (forward with saved
// tensors, loss, backward).  Host code only; kernels live in the other files.
#include "../../include/pt.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <unordered_map>
#include <unordered_set>
#include <vector>

#include "kernels.h"

using namespace pt;

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t x, size_t a = kAlign) { return (x + a - 1) / a * a; }

struct TensorDesc {
  std::string name;
  int64_t numel;
  int rows, cols;
  int group;
  bool decayed;
  int64_t offset;  // floats from the start of each per-parameter arena, multiple of kChunk
  int64_t padded;
};

const char* const kBlockNames[12] = {"ln1_g", "ln1_b", "Wqkv", "bqkv", "Wo", "bo",
                                     "ln2_g", "ln2_b", "W1",   "b1",   "W2", "b2"};
enum BlockTensor { LN1_G, LN1_B, WQKV, BQKV, WO, BO, LN2_G, LN2_B, W1, B1, W2, B2 };

// byte offsets into the work arena of the tensors one block keeps
struct Slot {
  size_t U, QKV, CTX, Y, WN, HP, G, LSE, MU1, RS1, MU2, RS2;   // HP: GELU'(pre-activation), G: GELU(pre-activation)
};

struct Plan {
  std::vector<TensorDesc> tensors;
  int64_t arena_floats = 0;
  int64_t state_lo = 0;     // floats of the parameter arena in front of the first tensor that can ever be trained
                            // (k_min > 0): the gradient / moment arenas hold the tensors from there on only
  std::vector<int64_t> group_first_chunk;  // G+1
  size_t params_bytes = 0, state_bytes = 0, work_bytes = 0, cache_bytes = 0;
  // work arena
  std::vector<size_t> X;   // L+1 block inputs / outputs
  std::vector<Slot> slot;  // L+1 (slot L: scratch of the forward-only prefix)
  size_t HKOUT, sA, sB, sC, sD, oA, oB, oC, oD, oE, oE2, dF, dQKV, DELTA;
  // dense copies of the first token's rows (top block's backward under a first-token head)
  size_t rG, rHP, rDF, rXa, rXb, rCTX, rDO, rOC, rOD, rDCTX, rS0, rS1, rS2, rST;  // s*: fp32 gradient stream, o*: T operand copies
  size_t PATCH, EMB, DEMB, MUE, RSE, CHAINWS, IDS;  // front ends (EMB: ViT patch embeddings / BERT embedding sum; IDS: the batch's token ids)
  size_t CFEAT, MUF, RSF, LOGITS, DZ, DC, LOSSROWS;  // heads
  int ln_slots = 1;
  size_t LOSS, LOSSACC, NORMS, LNPART, GEMMWS, QAPART, CHUNKDECAY, GROUPFIRST, CHUNKSQ, IDX, STAGE;
  size_t idx_capacity = 0, stage_floats = 0, gemmws_floats = 0;
};

bool validate(const pt_config& c, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (c.arch != PT_VIT_PRELN && c.arch != PT_BERT_POSTLN) return bad("arch");
  if (c.dtype != PT_F32 && c.dtype != PT_BF16) return bad("dtype");
  if (c.optimizer != PT_SGDM && c.optimizer != PT_ADAMW) return bad("optimizer");
  if (c.head != PT_HEAD_DEFAULT && c.head != PT_HEAD_CLS) return bad("head");
  if (c.L < 1 || c.L > 512 || c.D < 8 || c.H < 1 || c.F < 4 || c.S < 1 || c.B < 1 || c.n_out < 1) return bad("sizes");
  if (c.D % c.H) return bad("D % H");
  const int dh = c.D / c.H;
  if (dh % 8 || dh > 128) return bad("head size must be a multiple of 8 and at most 128");
  if (c.D > 2048 || c.F % 4) return bad("D <= 2048, F % 4 == 0");
  if (c.arch == PT_VIT_PRELN) {
    if (c.img < 1 || c.patch < 1 || c.chans < 1 || c.img % c.patch) return bad("image / patch");
    const int g = c.img / c.patch;
    if (g * g + 1 != c.S) return bad("S must be (img/patch)^2 + 1");
  } else {
    if (c.vocab < 1 || c.max_pos < c.S) return bad("vocab / max_pos");
    if (c.head == PT_HEAD_DEFAULT && c.n_out != 2) return bad("BERT span-QA head has n_out = 2");
  }
  if (c.cache_slots < 0 || c.host_slots < 0 || c.window_slots < 0) return bad("cache_slots / host_slots / window_slots");
  if (c.host_slots > 0 && c.window_slots < 2 * (int64_t)c.B) return bad("a host tier needs window_slots >= 2 B");
  if (c.host_slots == 0 && c.window_slots != 0) return bad("window_slots without host_slots");
  if (!(c.ln_eps >= 0.f)) return bad("ln_eps");
  if (c.k_min < 0 || c.k_min > c.L) return bad("k_min outside 0..L");
  if ((int64_t)c.B * c.S > (1 << 24)) return bad("B*S too large");
  // attention kernels that keep a score row (or strip) of the whole sequence in LDS
  constexpr size_t kLdsPerCu = 160 * 1024;
  if (!attention_uses_mfma(c.dtype == PT_BF16 ? 1 : 0, dh) && attention_generic_lds_bytes(c.S, dh) > kLdsPerCu)
    return bad("sequence too long for the attention kernels of this mode (fp32, or head size other than 64)");
  if (c.S >= 4 && (c.arch == PT_VIT_PRELN || c.head == PT_HEAD_CLS) && attention_first_query_lds_bytes(c.S, dh) > kLdsPerCu)
    return bad("sequence too long for the first-token attention kernels");
  return true;
}

void make_plan(const pt_config& c, Plan* p) {
  const int L = c.L, D = c.D, F = c.F, S = c.S, B = c.B;
  const size_t e = c.dtype == PT_BF16 ? 2 : 4;
  auto add = [&](const std::string& name, int rows, int cols, int group, bool dec) {
    TensorDesc t;
    t.name = name; t.rows = rows; t.cols = cols; t.numel = (int64_t)rows * cols; t.group = group; t.decayed = dec;
    t.offset = p->arena_floats;
    t.padded = (t.numel + kChunk - 1) / kChunk * kChunk;
    p->arena_floats += t.padded;
    p->tensors.push_back(t);
  };
  p->group_first_chunk.push_back(0);
  if (c.arch == PT_VIT_PRELN) {
    add("front.W_pe", c.chans * c.patch * c.patch, D, 0, true);
    add("front.b_pe", 1, D, 0, false);
    add("front.cls", 1, D, 0, false);
    add("front.pos", S, D, 0, false);
  } else {
    add("front.E_w", c.vocab, D, 0, true);
    add("front.E_p", c.max_pos, D, 0, false);
    add("front.ln_g", 1, D, 0, false);
    add("front.ln_b", 1, D, 0, false);
  }
  p->group_first_chunk.push_back(p->arena_floats / kChunk);
  for (int l = 0; l < L; ++l) {
    const std::string pre = "blk" + std::to_string(l) + ".";
    const int rows[12] = {1, 1, D, 1, D, 1, 1, 1, D, 1, F, 1};
    const int cols[12] = {D, D, 3 * D, 3 * D, D, D, D, D, F, F, D, D};
    for (int j = 0; j < 12; ++j) add(pre + kBlockNames[j], rows[j], cols[j], 1 + l, j == WQKV || j == WO || j == W1 || j == W2);
    p->group_first_chunk.push_back(p->arena_floats / kChunk);
  }
  if (c.arch == PT_VIT_PRELN) {
    add("head.ln_g", 1, D, L + 1, false);
    add("head.ln_b", 1, D, L + 1, false);
  }
  add("head.W", D, c.n_out, L + 1, true);
  add("head.b", 1, c.n_out, L + 1, false);
  p->group_first_chunk.push_back(p->arena_floats / kChunk);

  const size_t P = (size_t)p->arena_floats;
  p->params_bytes = align_up(P * 4) + (c.dtype == PT_BF16 ? align_up(P * 2) : 0);
  // A layer that is frozen for good keeps no gradient and no optimizer state (Sec. 3.2.1 item 2): with k_min > 0
  // the state arenas start at block k_min's first tensor.
  p->state_lo = c.k_min == 0 ? 0 : p->group_first_chunk[c.k_min + 1] * kChunk;
  const size_t Ps = P - (size_t)p->state_lo;
  p->state_bytes = align_up(Ps * 4) * ((c.optimizer == PT_ADAMW ? 3 : 2) + (c.grad_accum ? 1 : 0));
  p->cache_bytes = (size_t)(c.cache_slots + c.window_slots) * S * D * e;

  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
  const size_t T = (size_t)B * S;
  const size_t TD = T * D * e, TF = T * F * e, BHS = (size_t)B * c.H * S * 4;
  // Blocks below k_min only ever run forward-only: their inputs ping-pong between two buffers and they keep
  // no saved tensors (Sec. 3.2.1 item 2); every block from k_min on has an input buffer and a slot of its own.
  p->X.resize(L + 1);
  {
    size_t ping[2] = {0, 0};
    if (c.k_min > 0) ping[0] = take(TD);
    if (c.k_min > 1) ping[1] = take(TD);
    for (int l = 0; l <= L; ++l) p->X[l] = l < c.k_min ? ping[l & 1] : take(TD);
  }
  p->slot.resize(L + 1);
  for (int l = c.k_min < L ? c.k_min : L; l <= L; ++l) {
    Slot& s = p->slot[l];
    // post-LN keeps the two pre-LayerNorm sums (U, WN) in fp32
    const size_t TDsum = c.arch == PT_BERT_POSTLN ? T * D * 4 : TD;
    s.U = take(TDsum); s.QKV = take(3 * TD); s.CTX = take(TD); s.Y = take(TD); s.WN = take(TDsum);
    s.HP = take(TF); s.G = take(TF); s.LSE = take(BHS);
    s.MU1 = take(T * 4); s.RS1 = take(T * 4); s.MU2 = take(T * 4); s.RS2 = take(T * 4);
  }
  for (int l = 0; l < c.k_min && l < L; ++l) p->slot[l] = p->slot[L];   // never used: these blocks take the prefix's scratch slot
  p->HKOUT = take(TD);
  const size_t TD4 = T * D * 4;
  p->sA = take(TD4); p->sB = take(TD4); p->sC = take(TD4); p->sD = take(TD4);
  p->oA = take(TD); p->oB = take(TD); p->oC = take(TD); p->oD = take(TD); p->oE = take(TD); p->dF = take(TF);
  p->oE2 = c.arch == PT_BERT_POSTLN ? take(TD) : p->oE;   // post-LN: successive blocks alternate (see block_backward)
  p->dQKV = take(3 * TD); p->DELTA = take(BHS);
  {
    const size_t BD = (size_t)B * D, BF = (size_t)B * F;
    p->rG = take(BF * e); p->rHP = take(BF * e); p->rDF = take(BF * e);
    p->rXa = take(BD * 4); p->rXb = take(BD * 4); p->rCTX = take(BD * e); p->rDO = take(BD * e);
    p->rOC = take(BD * e); p->rOD = take(BD * e); p->rDCTX = take(BD * e);
    p->rS0 = take(BD * 4); p->rS1 = take(BD * 4); p->rS2 = take(BD * 4);
    p->rST = take((size_t)B * 4 * 4);
  }
  if (c.arch == PT_VIT_PRELN) {
    const size_t np = (size_t)B * (S - 1);
    p->PATCH = take(np * c.chans * c.patch * c.patch * e);
    p->EMB = take(np * D * e);
    p->DEMB = take(np * D * e);
    p->MUE = p->RSE = p->CHAINWS = p->IDS = 0;
    p->CFEAT = take((size_t)B * D * e); p->MUF = take((size_t)B * 4); p->RSF = take((size_t)B * 4);
    p->LOGITS = take((size_t)B * c.n_out * 4); p->DZ = take((size_t)B * c.n_out * e); p->DC = take((size_t)B * D * e);
  } else {
    p->PATCH = 0;
    p->EMB = take(TD4); p->DEMB = take(TD4); p->MUE = take(T * 4); p->RSE = take(T * 4); p->CHAINWS = take(bert_embed_ws_ints((int)T, c.vocab) * 4);
    p->IDS = take(T * 4);
    p->CFEAT = p->MUF = p->RSF = p->DC = 0;
    if (c.head == PT_HEAD_CLS) { p->LOGITS = take((size_t)B * c.n_out * 4); p->DZ = take((size_t)B * c.n_out * e); }
    else { p->LOGITS = take(T * 2 * 4); p->DZ = take(T * 2 * 4); }
  }
  p->LOSSROWS = take((size_t)B * 4);
  p->LOSS = take(4);
  p->LOSSACC = take(4);
  p->NORMS = take((size_t)(L + 2) * 4);
  // one slot of partial sums per LayerNorm backward pass of a sweep: two per block that can be active, the
  // final LayerNorm (ViT) or the embedding LayerNorm (BERT), and one to spare
  p->ln_slots = 2 * (L - std::min(c.k_min, L)) + 2;
  p->LNPART = take(ln_partial_floats(D) * 4 * p->ln_slots);
  // scratch of the weight-gradient products: split-K slabs (up to 16 splits, about 768 workgroups in
  // flight) plus their column-sum partials; also serves the separate column-sum pass of the FMA path
  {
    const int maxn = std::max(std::max(3 * D, F), c.n_out);
    size_t need = colsum_partial_floats(maxn);
    const int64_t shapes[6][2] = {{D, 3 * D}, {D, D}, {D, F}, {F, D}, {c.chans * c.patch * c.patch, D}, {D, c.n_out}};
    for (auto& sh : shapes) {
      const int64_t tiles = ((sh[0] + 127) / 128) * ((sh[1] + 127) / 128);
      if (tiles <= 0) continue;
      const int64_t splits = std::min<int64_t>(16, std::max<int64_t>(1, 1024 / tiles));
      need = std::max(need, (size_t)(splits * (sh[0] * sh[1] + sh[1])));
    }
    need = std::max(need, 2 * (gemm_wgrad_batch_ws_floats(D, F) + 64));   // two blocks' slabs (see run_wgrads)
    p->gemmws_floats = need;
    p->GEMMWS = take(need * 4);
  }
  p->QAPART = take(qa_partial_floats(D) * 4);
  const size_t nchunks = P / kChunk;
  p->CHUNKDECAY = take(nchunks);
  p->GROUPFIRST = take((size_t)(L + 3) * 8);
  p->CHUNKSQ = take(nchunks * 4);
  p->idx_capacity = (size_t)16 * B;  // two turns of up to 8 index arrays of B entries
  p->IDX = take(p->idx_capacity * 8);
  int64_t maxt = 0;
  for (auto& t : p->tensors) maxt = std::max(maxt, t.numel);
  p->stage_floats = std::max<size_t>({(size_t)maxt, T * D, T * 2, (size_t)B * c.n_out});
  p->STAGE = take(p->stage_floats * 4);
  p->work_bytes = off;
}

}  // namespace

struct pt_ctx {
  pt_config cfg;
  Plan plan;
  int dt = 0;
  size_t esz = 4;
  hipStream_t st = nullptr;
  float* master = nullptr;
  char* shadow = nullptr;  // bf16 [P] or null
  float* grads = nullptr;
  float* mom1 = nullptr;
  float* mom2 = nullptr;
  float* gacc = nullptr;      // gradient accumulator over micro-batches (grad_accum configurations)
  std::vector<LnReduceJob> ln_jobs;   // LayerNorm backward passes whose partial sums are not summed yet
  Gemm pending_wg[4];                 // post-LN: a block's weight gradients, held back until the next block starts
  int pending_nwg = 0;
  WgradCarry wgrad_carry;             // split-K slabs of the last block's weight gradients, not summed yet
  int wgrad_parity = 0;               // which half of the GEMM workspace the next block's slabs go to
  int64_t acc_samples = 0;    // samples accumulated so far; 0 = no accumulation in progress
  char* work = nullptr;
  char* cache = nullptr;
  int k = 0;
  int64_t step = 0;
  int phase = 0;  // 0 idle, 1 frozen forward done, 2 backward done
  int nb = 0;
  void* last_hk = nullptr;
  void* last_dhk = nullptr;
  std::vector<int32_t> slot_k;  // boundary a cache row was written at, -1 = empty (HBM rows, then host rows)
  // host tier: rows of sample ids >= cache_slots live in pinned host memory and pass through a window of
  // device rows (the last window_slots rows of the cache arena) on a copy stream of their own
  struct WinSlot { int64_t id = -1; int state = 0; hipEvent_t ev = nullptr; int64_t stamp = 0; };  // 0 free, 1 staged, 2 write-back
  char* host_rows = nullptr;
  hipStream_t copy_st = nullptr;
  hipEvent_t ev_copy = nullptr, ev_main = nullptr;
  std::vector<WinSlot> win;
  std::unordered_map<int64_t, int> win_of;  // staged rows: sample id -> window slot
  int64_t call_stamp = 0;
  int64_t n_h2d = 0, n_d2h = 0, n_prefetched = 0, n_prefetch_used = 0;
  int64_t n_hit = 0, n_adv = 0, n_miss = 0, n_runs = 0;
  // pinned host staging for index arrays, double-buffered by call parity
  int64_t* h_idx[2] = {nullptr, nullptr};
  float* h_norms = nullptr;   // pinned host memory: L + 2 norms, written by the norm kernel itself, and the loss
  float* static_sq = nullptr;      // this GPU's copy of the library's static per-chunk sums (pt_layer_grad_norms_static)
  hipEvent_t norms_ev = nullptr;   // recorded behind the norm kernels by pt_layer_grad_norms_begin
  bool norms_pending = false;      // begun and not yet fetched
  bool norms_deferred = false;     // pending, and the norm kernels are not enqueued yet: the next update takes them along
  hipEvent_t idx_ev[2] = {nullptr, nullptr};
  bool idx_ev_used[2] = {false, false};
  int idx_turn = 0;
  mutable std::string err;
  // optional per-category kernel timing with HIP events on the context's stream
  struct ProfRec { hipEvent_t a, b, m; int cat, cat2; double work; };   // m, cat2: optional split of the bracket in two
  bool prof_on = false;
  std::vector<ProfRec> prof_pool;
  size_t prof_used = 0;
  double prof_ms[PT_PROF_COUNT] = {};
  double prof_work[PT_PROF_COUNT] = {};
  int64_t prof_n[PT_PROF_COUNT] = {};

  const void* cp(int id) const {  // parameter as the kernels read it
    const TensorDesc& t = plan.tensors[id];
    return dt ? (const void*)(shadow + t.offset * 2) : (const void*)(master + t.offset);
  }
  float* gp(int id) const { return grads + plan.tensors[id].offset; }
  void* w(size_t off) const { return work + off; }
  float* wf(size_t off) const { return reinterpret_cast<float*>(work + off); }
  int blk(int l, int j) const { return 4 + 12 * l + j; }
  int head(int j) const { return 4 + 12 * cfg.L + j; }  // ViT: ln_g, ln_b, W, b; BERT: W, b
};

namespace {

// Brackets one launcher call with two events when profiling is on.
struct ProfScope {
  pt_ctx* c;
  pt_ctx::ProfRec* r = nullptr;
  ProfScope(pt_ctx* ctx, int cat, double work) : c(ctx) {
    if (!c->prof_on) return;
    if (c->prof_used == c->prof_pool.size()) {
      pt_ctx::ProfRec n{};
      if (hipEventCreate(&n.a) != hipSuccess || hipEventCreate(&n.b) != hipSuccess || hipEventCreate(&n.m) != hipSuccess) return;
      c->prof_pool.push_back(n);
    }
    r = &c->prof_pool[c->prof_used++];
    r->cat = cat;
    r->cat2 = -1;
    r->work = work;
    (void)hipEventRecord(r->a, c->st);
  }
  // the bracket is cut in two at an event the launcher records: [a, m) stays in the scope's category, [m, b) goes to cat2
  hipEvent_t split(int cat2) {
    if (!r) return nullptr;
    r->cat2 = cat2;
    return r->m;
  }
  ~ProfScope() {
    if (r) (void)hipEventRecord(r->b, c->st);
  }
};

// the slab reduction that the last block's weight-gradient launch left for a successor
void flush_wgrad_carry(pt_ctx* c) {
  if (c->wgrad_carry.nprob <= 0) return;
  ProfScope ps_(c, PT_PROF_SPLITK_REDUCE, 0.0);
  gemm_wgrad_flush(&c->wgrad_carry, c->st);
}

// sums the partial rows of every LayerNorm backward pass enqueued since the last call (one launch)
void flush_ln_reductions(pt_ctx* c) {
  if (c->ln_jobs.empty()) return;
  ProfScope ps_(c, PT_PROF_LN_BWD, 0.0);
  layernorm_bwd_reduce(c->ln_jobs.data(), (int)c->ln_jobs.size(), c->cfg.D, c->st);
  c->ln_jobs.clear();
}

// where the next LayerNorm backward pass of the sweep puts its workgroups' partial sums
float* ln_partial_slot(pt_ctx* c) {
  if (c->ln_jobs.size() == (size_t)c->plan.ln_slots) flush_ln_reductions(c);
  return c->wf(c->plan.LNPART) + c->ln_jobs.size() * ln_partial_floats(c->cfg.D);
}

// memory-bound launches timed with their algorithmic bytes (what must be read and written once)
void prof_ln_fwd(pt_ctx* c, int dt, bool x_f32, const void* x, int64_t ldx, const void* gamma, const void* beta, void* y,
                 int64_t ldy, float* mean, float* rstd, int rows, int D, float eps, hipStream_t st) {
  ProfScope ps_(c, PT_PROF_LN_FWD, (double)rows * D * ((x_f32 ? 4 : c->esz) + c->esz));
  layernorm_fwd(dt, x_f32, x, ldx, gamma, beta, y, ldy, mean, rstd, rows, D, eps, st);
}
void prof_ln_bwd(pt_ctx* c, int dt, bool dy_f32, bool x_f32, const void* dy, int64_t lddy, const void* x, int64_t ldx,
                 const float* mean, const float* rstd, const void* gamma, const float* dres, int64_t lddres, float* dx_s,
                 void* dx_o, int64_t lddx, float* dgamma, float* dbeta, float* dxsum, int rows, int D, hipStream_t st,
                 bool reduce_now = false) {
  const double per = (dy_f32 ? 4 : c->esz) + (x_f32 ? 4 : c->esz) + (dres ? 4 : 0) + (dx_s ? 4 : 0) + (dx_o ? c->esz : 0);
  // Each pass of a backward sweep writes its workgroups' partial sums of d(gamma), d(beta) and the column sums
  // to a slot of its own; nothing reads those three results before the sweep ends, so they are summed for
  // all passes in one launch there (flush_ln_reductions) unless the caller needs them at once.
  float* partial = ln_partial_slot(c);
  LnReduceJob job;
  {
    ProfScope ps_(c, PT_PROF_LN_BWD, (double)rows * D * per);
    layernorm_bwd(dt, dy_f32, x_f32, dy, lddy, x, ldx, mean, rstd, gamma, dres, lddres, dx_s, dx_o, lddx, dgamma, dbeta, dxsum,
                  partial, rows, D, st, reduce_now ? nullptr : &job);
  }
  if (!reduce_now && job.np > 0) c->ln_jobs.push_back(job);
}
void prof_copy_rows(pt_ctx* c, void* dst, const int64_t* dst_idx, const void* src, const int64_t* src_idx, int nrows,
                    size_t row_bytes, hipStream_t st) {
  ProfScope ps_(c, PT_PROF_CACHE, 2.0 * nrows * row_bytes);
  copy_rows(dst, dst_idx, src, src_idx, nrows, row_bytes, st);
}

// folds finished event pairs into the per-category totals (synchronises)
void prof_collect(pt_ctx* c) {
  if (c->prof_used == 0) return;
  (void)hipStreamSynchronize(c->st);
  for (size_t i = 0; i < c->prof_used; ++i) {
    const auto& r = c->prof_pool[i];
    float ms = 0.f, ms2 = 0.f;
    if (r.cat2 >= 0) {
      if (hipEventElapsedTime(&ms, r.a, r.m) == hipSuccess && hipEventElapsedTime(&ms2, r.m, r.b) == hipSuccess) {
        c->prof_ms[r.cat] += ms;
        c->prof_work[r.cat] += r.work;
        c->prof_n[r.cat] += 1;
        c->prof_ms[r.cat2] += ms2;
        c->prof_n[r.cat2] += 1;
      }
    } else if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
      c->prof_ms[r.cat] += ms;
      c->prof_work[r.cat] += r.work;
      c->prof_n[r.cat] += 1;
    }
  }
  c->prof_used = 0;
}

int gemm_cat(int dt, const Gemm& m) {
  if (!gemm_uses_mfma(dt, m)) return PT_PROF_GEMM_GENERIC;
  if (m.ta) return PT_PROF_GEMM_TN;
  return m.tb ? PT_PROF_GEMM_NT : PT_PROF_GEMM_NN;
}

pt_status fail(const pt_ctx* c, pt_status s, const std::string& m) {
  if (c) c->err = m;
  return s;
}
pt_status flush_deferred_norms(pt_ctx* c);   // norms begun but not enqueued yet: enqueue them now
#define HIP_TRY(ctx, expr)                                                                  \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(ctx, PT_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

// ---------------------------------------------------------------------------
// one encoder block, forward.  save == false: forward-only (nothing kept).
// ---------------------------------------------------------------------------
void block_forward(pt_ctx* c, int l, const void* xin, void* xout, const Slot& s, int ns, bool save) {
  const pt_config& g = c->cfg;
  const int D = g.D, F = g.F, Tn = ns * g.S, dt = c->dt;
  hipStream_t st = c->st;
  float* lse = save ? c->wf(s.LSE) : nullptr;
  float* mu1 = save ? c->wf(s.MU1) : nullptr; float* rs1 = save ? c->wf(s.RS1) : nullptr;
  float* mu2 = save ? c->wf(s.MU2) : nullptr; float* rs2 = save ? c->wf(s.RS2) : nullptr;
  auto lin = [&](const void* A, int K, int wid, int bid, void* C, int N, Epi epi, const void* aux, void* aux_out,
                 bool out_f32 = false) {
    Gemm m;
    m.A = A; m.lda = K; m.B = c->cp(wid); m.ldb = N; m.C = C; m.ldc = N; m.M = Tn; m.N = N; m.K = K;
    m.epi = epi; m.bias = c->cp(bid); m.aux = aux; m.aux_out = aux_out; m.ld_aux = N; m.c_f32 = out_f32;
    { ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K); gemm(dt, m, st); }
  };
  if (g.arch == PT_VIT_PRELN) {
    { prof_ln_fwd(c, dt, false, xin, D, c->cp(c->blk(l, LN1_G)), c->cp(c->blk(l, LN1_B)), c->w(s.U), D, mu1, rs1, Tn, D, g.ln_eps, st); }
    lin(c->w(s.U), D, c->blk(l, WQKV), c->blk(l, BQKV), c->w(s.QKV), 3 * D, EPI_BIAS, nullptr, nullptr);
    { ProfScope ps_(c, PT_PROF_ATTN_FWD, 4.0 * ns * g.H * (double)g.S * g.S * (D / g.H)); attention_fwd(dt, c->w(s.QKV), c->w(s.CTX), lse, ns, g.S, g.H, D / g.H, st); }
    lin(c->w(s.CTX), D, c->blk(l, WO), c->blk(l, BO), c->w(s.Y), D, EPI_BIAS_RES, xin, nullptr);
    { prof_ln_fwd(c, dt, false, c->w(s.Y), D, c->cp(c->blk(l, LN2_G)), c->cp(c->blk(l, LN2_B)), c->w(s.WN), D, mu2, rs2, Tn, D, g.ln_eps, st); }
    lin(c->w(s.WN), D, c->blk(l, W1), c->blk(l, B1), c->w(s.G), F, EPI_BIAS_GELU, nullptr, save ? c->w(s.HP) : nullptr);
    lin(c->w(s.G), F, c->blk(l, W2), c->blk(l, B2), xout, D, EPI_BIAS_RES, c->w(s.Y), nullptr);
  } else {
    // post-LN: U holds x + Attn(x) in fp32, Y = LN1(U), WN holds Y + MLP(Y) in fp32, out = LN2(WN)
    lin(xin, D, c->blk(l, WQKV), c->blk(l, BQKV), c->w(s.QKV), 3 * D, EPI_BIAS, nullptr, nullptr);
    { ProfScope ps_(c, PT_PROF_ATTN_FWD, 4.0 * ns * g.H * (double)g.S * g.S * (D / g.H)); attention_fwd(dt, c->w(s.QKV), c->w(s.CTX), lse, ns, g.S, g.H, D / g.H, st); }
    lin(c->w(s.CTX), D, c->blk(l, WO), c->blk(l, BO), c->w(s.U), D, EPI_BIAS_RES, xin, nullptr, true);
    { prof_ln_fwd(c, dt, true, c->w(s.U), D, c->cp(c->blk(l, LN1_G)), c->cp(c->blk(l, LN1_B)), c->w(s.Y), D, mu1, rs1, Tn, D, g.ln_eps, st); }
    lin(c->w(s.Y), D, c->blk(l, W1), c->blk(l, B1), c->w(s.G), F, EPI_BIAS_GELU, nullptr, save ? c->w(s.HP) : nullptr);
    lin(c->w(s.G), F, c->blk(l, W2), c->blk(l, B2), c->w(s.WN), D, EPI_BIAS_RES, c->w(s.Y), nullptr, true);
    { prof_ln_fwd(c, dt, true, c->w(s.WN), D, c->cp(c->blk(l, LN2_G)), c->cp(c->blk(l, LN2_B)), xout, D, mu2, rs2, Tn, D, g.ln_eps, st); }
  }
}

// ---------------------------------------------------------------------------
// one encoder block, backward.  The gradient of the residual stream is carried
// in fp32 between blocks (its per-token sums cancel heavily, so bf16 rounding
// along that path would dominate the bias / LayerNorm-shift gradients); tensors
// that feed the matrix cores get a T copy written by the kernel that makes them.
// In: dout_s (fp32) and, for pre-LN, its T copy dout_o.  Out: dx_s / dx_o.
// lower_b2 (pre-LN, may be null): where the column sums of dx go, i.e. the gradient of the second MLP
// bias of the block below, whose output gradient dx is.
// ---------------------------------------------------------------------------
// The weight gradients of one block (all its products, one grouped launch in the matrix-core path).  `ln`: a
// LayerNorm backward pass that does not depend on them and may ride on the launch (see gemm_wgrad_batch).
void launch_wgrads(pt_ctx* c, Gemm* wg, int nwg, LnBwdRide* ln) {
  if (nwg <= 0) return;
  const Plan& p = c->plan;
  const int dt = c->dt;
  double fl = 0;
  for (int i = 0; i < nwg; ++i) fl += 2.0 * wg[i].M * wg[i].N * wg[i].K;
  // the four products of a whole block in the matrix-core path: the grouped kernel is timed on its own, the
  // reduction of its split-K slabs separately
  const bool grouped = nwg == 4 && gemm_cat(dt, wg[0]) == PT_PROF_GEMM_TN;
  // Successive blocks alternate between the two halves of the workspace: the slabs of a split launch are
  // summed by the next block's launch, on the CUs its tiles leave idle, or at the end of the sweep
  // (flush_wgrad_carry), so they must survive that launch.
  const size_t half = (p.gemmws_floats / 2) & ~(size_t)63;
  float* ws = c->wf(p.GEMMWS) + (c->wgrad_parity ? half : 0);
  c->wgrad_parity ^= 1;
  for (int i = 0; i < nwg; ++i) { wg[i].ws = ws; wg[i].ws_floats = half; }
  ProfScope ps_(c, grouped ? PT_PROF_WGRAD_BLOCK : gemm_cat(dt, wg[0]), fl);
  gemm_wgrad_batch(dt, wg, nwg, c->st, grouped ? ps_.split(PT_PROF_SPLITK_REDUCE) : nullptr, &c->wgrad_carry, ln);
}
// post-LN: the weight gradients of the block above, held back for the next block's first LayerNorm pass
void launch_pending_wgrads(pt_ctx* c, LnBwdRide* ln) {
  if (c->pending_nwg > 0) launch_wgrads(c, c->pending_wg, c->pending_nwg, ln);
  c->pending_nwg = 0;
}

struct GradBufs {
  float* s;  // fp32 stream
  void* o;   // T copy (pre-LN only)
};

void block_backward(pt_ctx* c, int l, const void* xin, const Slot& s, GradBufs dout, GradBufs dx, int ns, bool need_dx,
                    float* lower_b2) {
  const pt_config& g = c->cfg;
  const int D = g.D, F = g.F, Tn = ns * g.S, dt = c->dt;
  hipStream_t st = c->st;
  const Plan& p = c->plan;
  float* sC = c->wf(p.sC); float* sD = c->wf(p.sD);
  void* oC = c->w(p.oC); void* oD = c->w(p.oD); void* dF = c->w(p.dF); void* dQKV = c->w(p.dQKV);
  // post-LN: the block above may still be reading its oE (its weight gradients are launched with this block's
  // first LayerNorm pass on board, which writes this block's oE), so successive blocks alternate
  void* oE = c->w((l & 1) ? p.oE2 : p.oE);
  // dW[K_in, N_out] = X^T dY ; db = colsum over tokens of dY (bias_dt 0: fp32 source, else T)
  // bid >= 0: also db = column sums of dY over the tokens, riding on the same product
  // The four weight gradients of the block are collected and run together at its end: every dY they read
  // stays in a buffer of its own until then, and one launch over all four fills the chip where each alone
  // would need a deep split over the tokens.
  Gemm wg[4];
  int nwg = 0;
  auto wgrad = [&](const void* X, int Kin, const void* dY, int Nout, int wid, int bid) {
    Gemm& m = wg[nwg++];
    m.A = X; m.lda = Kin; m.ta = true; m.B = dY; m.ldb = Nout; m.C = c->gp(wid); m.ldc = Nout;
    m.M = Kin; m.N = Nout; m.K = Tn; m.c_f32 = true;
    m.ws = c->wf(p.GEMMWS); m.ws_floats = p.gemmws_floats; m.colsum_out = bid >= 0 ? c->gp(bid) : nullptr;
  };
  auto run_wgrads = [&](LnBwdRide* ln = nullptr) { launch_wgrads(c, wg, nwg, ln); };
  // dX[Tn, K_in] = dY W^T (+ epilogue)
  auto dgrad = [&](const void* dY, int Nout, int wid, void* dX, int Kin, Epi epi, const void* aux, bool out_f32) {
    Gemm m;
    m.A = dY; m.lda = Nout; m.B = c->cp(wid); m.ldb = Nout; m.tb = true; m.C = dX; m.ldc = Kin;
    m.M = Tn; m.N = Kin; m.K = Nout; m.epi = epi; m.aux = aux; m.ld_aux = Kin; m.c_f32 = out_f32;
    { ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K); gemm(dt, m, st); }
  };
  if (g.arch == PT_VIT_PRELN) {
    // the gradient of b2 (column sums of dout) came with the kernel that produced dout
    wgrad(c->w(s.G), F, dout.o, D, c->blk(l, W2), -1);
    dgrad(dout.o, D, c->blk(l, W2), dF, F, EPI_MUL_DGELU, c->w(s.HP), false);
    wgrad(c->w(s.WN), D, dF, F, c->blk(l, W1), c->blk(l, B1));
    dgrad(dF, F, c->blk(l, W1), oC, D, EPI_STORE, nullptr, false);                      // oC = dL/dLN2out
    { prof_ln_bwd(c, dt, false, false, oC, D, c->w(s.Y), D, c->wf(s.MU2), c->wf(s.RS2), c->cp(c->blk(l, LN2_G)), dout.s, D, sC, oD,
                  D, c->gp(c->blk(l, LN2_G)), c->gp(c->blk(l, LN2_B)), c->gp(c->blk(l, BO)), Tn, D, st); }  // sC / oD = dL/dY
    wgrad(c->w(s.CTX), D, oD, D, c->blk(l, WO), -1);
    dgrad(oD, D, c->blk(l, WO), oC, D, EPI_STORE, nullptr, false);                      // oC = dL/dCTX
    { ProfScope ps_(c, PT_PROF_ATTN_BWD, 8.0 * ns * g.H * (double)g.S * g.S * (D / g.H)); attention_bwd(dt, c->w(s.QKV), c->w(s.CTX), oC, c->wf(s.LSE), dQKV, c->wf(p.DELTA), ns, g.S, g.H, D / g.H, st); }
    wgrad(c->w(s.U), D, dQKV, 3 * D, c->blk(l, WQKV), c->blk(l, BQKV));
    dgrad(dQKV, 3 * D, c->blk(l, WQKV), oC, D, EPI_STORE, nullptr, false);              // oC = dL/dU
    // The block's last LayerNorm backward pass (-> dx) and its weight gradients do not depend on each other:
    // the pass is offered to the weight-gradient launch, which runs it on its spare workgroups where it has
    // them (gemm_wgrad_batch); otherwise it runs here as a launch of its own.
    bool ln1_done = false;
    if (dt != 0) {
      LnBwdRide ride{oC, D, xin, D, c->wf(s.MU1), c->wf(s.RS1), c->cp(c->blk(l, LN1_G)), sC, D,
                     need_dx ? dx.s : nullptr, need_dx ? dx.o : nullptr, D, ln_partial_slot(c), Tn, D};
      run_wgrads(&ride);
      if (ride.taken_np > 0) {
        c->ln_jobs.push_back(LnReduceJob{ride.partial, ride.taken_np, c->gp(c->blk(l, LN1_G)), c->gp(c->blk(l, LN1_B)), lower_b2});
        ln1_done = true;
      }
    }
    if (!ln1_done)
    { prof_ln_bwd(c, dt, false, false, oC, D, xin, D, c->wf(s.MU1), c->wf(s.RS1), c->cp(c->blk(l, LN1_G)), sC, D,
                  need_dx ? dx.s : nullptr, need_dx ? dx.o : nullptr, D, c->gp(c->blk(l, LN1_G)),
                  c->gp(c->blk(l, LN1_B)), lower_b2, Tn, D, st); }
    if (dt != 0) return;   // the products went out with the offer above
  } else {
    // The block's first LayerNorm backward pass does not depend on the weight gradients of the block above,
    // which were held back for it: it is offered to their launch, which runs it on its spare workgroups
    // where it has them; otherwise it runs as a launch of its own behind them.
    bool ln2_done = false;
    if (dt != 0 && c->pending_nwg > 0) {
      LnBwdRide ride{dout.s, D, c->w(s.WN), D, c->wf(s.MU2), c->wf(s.RS2), c->cp(c->blk(l, LN2_G)), nullptr, 0, sC, oE, D,
                     ln_partial_slot(c), Tn, D};
      ride.f32_in = true;
      launch_pending_wgrads(c, &ride);
      if (ride.taken_np > 0) {
        c->ln_jobs.push_back(LnReduceJob{ride.partial, ride.taken_np, c->gp(c->blk(l, LN2_G)), c->gp(c->blk(l, LN2_B)), c->gp(c->blk(l, B2))});
        ln2_done = true;
      }
    }
    if (!ln2_done)
    { prof_ln_bwd(c, dt, true, true, dout.s, D, c->w(s.WN), D, c->wf(s.MU2), c->wf(s.RS2), c->cp(c->blk(l, LN2_G)), nullptr, 0, sC,
                  oE, D, c->gp(c->blk(l, LN2_G)), c->gp(c->blk(l, LN2_B)), c->gp(c->blk(l, B2)), Tn, D, st); }  // sC / oE = dL/d(Y+MLP)
    wgrad(c->w(s.G), F, oE, D, c->blk(l, W2), -1);
    dgrad(oE, D, c->blk(l, W2), dF, F, EPI_MUL_DGELU, c->w(s.HP), false);
    wgrad(c->w(s.Y), D, dF, F, c->blk(l, W1), c->blk(l, B1));
    dgrad(dF, F, c->blk(l, W1), sD, D, EPI_RES, sC, true);                              // sD = dL/dY
    { prof_ln_bwd(c, dt, true, true, sD, D, c->w(s.U), D, c->wf(s.MU1), c->wf(s.RS1), c->cp(c->blk(l, LN1_G)), nullptr, 0, sC, oC,
                  D, c->gp(c->blk(l, LN1_G)), c->gp(c->blk(l, LN1_B)), c->gp(c->blk(l, BO)), Tn, D, st); }  // sC / oC = dL/d(x+Attn)
    wgrad(c->w(s.CTX), D, oC, D, c->blk(l, WO), -1);
    dgrad(oC, D, c->blk(l, WO), oD, D, EPI_STORE, nullptr, false);                      // oD = dL/dCTX
    { ProfScope ps_(c, PT_PROF_ATTN_BWD, 8.0 * ns * g.H * (double)g.S * g.S * (D / g.H)); attention_bwd(dt, c->w(s.QKV), c->w(s.CTX), oD, c->wf(s.LSE), dQKV, c->wf(p.DELTA), ns, g.S, g.H, D / g.H, st); }
    wgrad(xin, D, dQKV, 3 * D, c->blk(l, WQKV), c->blk(l, BQKV));
    if (need_dx) dgrad(dQKV, 3 * D, c->blk(l, WQKV), dx.s, D, EPI_RES, sC, true);
    if (dt != 0) {   // held back for the next block's first LayerNorm pass (or the end of the sweep)
      for (int i = 0; i < nwg; ++i) c->pending_wg[i] = wg[i];
      c->pending_nwg = nwg;
      return;
    }
  }
  run_wgrads();
}


// ---------------------------------------------------------------------------
// Forward of the top block when the head reads only each sample's first token (ViT class token, BERT
// sequence classification): of this block's output nothing but those ns rows is ever read, so everything
// behind the attention (output projection, LayerNorms, both MLP products) runs on ns rows, and the attention
// itself on one query per sample; keys and values still need every token, hence the full LayerNorm and QKV
// product in front.  The first-token rows of the intermediate tensors are kept dense, in the row buffers
// block_backward_first_rows works on, instead of in the block's slot; xout gets its first-token rows only.
// ---------------------------------------------------------------------------
void block_forward_first_rows(pt_ctx* c, int l, const void* xin, void* xout, const Slot& s, int ns) {
  const pt_config& g = c->cfg;
  const int D = g.D, F = g.F, S = g.S, Tn = ns * g.S, dt = c->dt;
  const int64_t SD = (int64_t)S * D;
  hipStream_t st = c->st;
  const Plan& p = c->plan;
  void* rG = c->w(p.rG); void* rHP = c->w(p.rHP); void* rXa = c->w(p.rXa); void* rXb = c->w(p.rXb);
  void* rCTX = c->w(p.rCTX); void* rDO = c->w(p.rDO);
  float* rmu1 = c->wf(p.rST); float* rrs1 = rmu1 + ns; float* rmu2 = rrs1 + ns; float* rrs2 = rmu2 + ns;
  auto lin = [&](const void* A, int64_t lda, int K, int wid, int bid, void* C, int64_t ldc, int N, int M, Epi epi,
                 const void* aux, void* aux_out, int64_t ld_aux, bool out_f32) {
    Gemm m;
    m.A = A; m.lda = lda; m.B = c->cp(wid); m.ldb = N; m.C = C; m.ldc = ldc; m.M = M; m.N = N; m.K = K;
    m.epi = epi; m.bias = c->cp(bid); m.aux = aux; m.aux_out = aux_out; m.ld_aux = ld_aux; m.c_f32 = out_f32;
    if (M == ns) { m.ws = c->wf(p.GEMMWS); m.ws_floats = p.gemmws_floats; }   // lets a few-row product split its K
    { ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K); gemm(dt, m, st); }
  };
  auto attn = [&]() {
    ProfScope ps_(c, PT_PROF_ATTN_FWD, 4.0 * ns * g.H * (double)g.S * (D / g.H));
    attention_fwd_first_query(dt, c->w(s.QKV), rCTX, c->wf(s.LSE), ns, g.S, g.H, D / g.H, st);
  };
  if (g.arch == PT_VIT_PRELN) {
    { prof_ln_fwd(c, dt, false, xin, D, c->cp(c->blk(l, LN1_G)), c->cp(c->blk(l, LN1_B)), c->w(s.U), D, c->wf(s.MU1), c->wf(s.RS1), Tn, D, g.ln_eps, st); }
    lin(c->w(s.U), D, D, c->blk(l, WQKV), c->blk(l, BQKV), c->w(s.QKV), 3 * D, 3 * D, Tn, EPI_BIAS, nullptr, nullptr, 3 * D, false);
    attn();
    lin(rCTX, D, D, c->blk(l, WO), c->blk(l, BO), rXb, D, D, ns, EPI_BIAS_RES, xin, nullptr, SD, false);          // rows of Y
    { prof_ln_fwd(c, dt, false, rXb, D, c->cp(c->blk(l, LN2_G)), c->cp(c->blk(l, LN2_B)), rXa, D, rmu2, rrs2, ns, D, g.ln_eps, st); }
    lin(rXa, D, D, c->blk(l, W1), c->blk(l, B1), rG, F, F, ns, EPI_BIAS_GELU, nullptr, rHP, F, false);
    lin(rG, F, F, c->blk(l, W2), c->blk(l, B2), xout, SD, D, ns, EPI_BIAS_RES, rXb, nullptr, D, false);
  } else {
    lin(xin, D, D, c->blk(l, WQKV), c->blk(l, BQKV), c->w(s.QKV), 3 * D, 3 * D, Tn, EPI_BIAS, nullptr, nullptr, 3 * D, false);
    attn();
    lin(rCTX, D, D, c->blk(l, WO), c->blk(l, BO), rXb, D, D, ns, EPI_BIAS_RES, xin, nullptr, SD, true);           // rows of U, fp32
    { prof_ln_fwd(c, dt, true, rXb, D, c->cp(c->blk(l, LN1_G)), c->cp(c->blk(l, LN1_B)), rDO, D, rmu1, rrs1, ns, D, g.ln_eps, st); }  // rows of Y
    lin(rDO, D, D, c->blk(l, W1), c->blk(l, B1), rG, F, F, ns, EPI_BIAS_GELU, nullptr, rHP, F, false);
    lin(rG, F, F, c->blk(l, W2), c->blk(l, B2), rXa, D, D, ns, EPI_BIAS_RES, rDO, nullptr, D, true);               // rows of WN, fp32
    { prof_ln_fwd(c, dt, true, rXa, D, c->cp(c->blk(l, LN2_G)), c->cp(c->blk(l, LN2_B)), xout, SD, rmu2, rrs2, ns, D, g.ln_eps, st); }
  }
}

// ---------------------------------------------------------------------------
// Backward of the top block when the head reads only each sample's first token (ViT class token, BERT
// sequence classification): dL/dx_L is zero in every other row, so everything between the block's output and
// its attention (both MLP products and their weight gradients, the LayerNorms, the output projection) involves
// ns rows instead of ns * S.  Those rows are kept dense (block_forward_first_rows left the saved
// activations' rows in the row buffers) and pushed through the same kernels; the attention backward, which
// needs every token, takes the one row of dL/dCTX per sample that is not zero.  Pre-LN: the head's backward
// has put the first tokens' rows of dL/dx_L into rS0 / rDO, and the last LayerNorm backward adds dL/dY in
// those rows only (dout is not read).  Post-LN: the rows are gathered from dout.s, whose other rows must be
// zero on entry (the head backward zero-fills them) and serve as the zero background of the residual
// gradient that the last product adds.  The results equal those of block_backward (rows of zeros contribute
// nothing).
// ---------------------------------------------------------------------------
void block_backward_first_rows(pt_ctx* c, int l, const void* xin, const Slot& s, GradBufs dout, GradBufs dx, int ns,
                               bool need_dx, float* lower_b2) {
  const pt_config& g = c->cfg;
  const int D = g.D, F = g.F, S = g.S, Tn = ns * g.S, dt = c->dt;
  const int64_t SD = (int64_t)S * D;
  hipStream_t st = c->st;
  const Plan& p = c->plan;
  void* oC = c->w(p.oC); void* dQKV = c->w(p.dQKV);
  void* rG = c->w(p.rG); void* rHP = c->w(p.rHP); void* rDF = c->w(p.rDF); void* rXa = c->w(p.rXa); void* rXb = c->w(p.rXb);
  void* rCTX = c->w(p.rCTX); void* rDO = c->w(p.rDO); void* rOC = c->w(p.rOC); void* rOD = c->w(p.rOD);
  void* rDCTX = c->w(p.rDCTX);
  float* rS0 = c->wf(p.rS0); float* rS1 = c->wf(p.rS1); float* rS2 = c->wf(p.rS2);
  float* rmu1 = c->wf(p.rST); float* rrs1 = rmu1 + ns; float* rmu2 = rrs1 + ns; float* rrs2 = rmu2 + ns;
  auto wgrad = [&](const void* X, int Kin, const void* dY, int Nout, int wid, int bid, int rows) {
    Gemm m;
    m.A = X; m.lda = Kin; m.ta = true; m.B = dY; m.ldb = Nout; m.C = c->gp(wid); m.ldc = Nout;
    m.M = Kin; m.N = Nout; m.K = rows; m.c_f32 = true;
    m.ws = c->wf(p.GEMMWS); m.ws_floats = p.gemmws_floats; m.colsum_out = bid >= 0 ? c->gp(bid) : nullptr;
    ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K);
    gemm_wgrad_batch(dt, &m, 1, st);
  };
  // The three weight gradients over the first tokens' rows are tiny (ns tokens deep): they are noted here and
  // go out as one grouped launch once the last of their operands exists (each has row buffers of its own).
  Gemm rows_wg[3];
  int n_rows_wg = 0;
  double rows_wg_flops = 0.0;
  auto wgrad_rows = [&](const void* X, int Kin, const void* dY, int Nout, int wid, int bid) {
    Gemm& m = rows_wg[n_rows_wg++];
    m.A = X; m.lda = Kin; m.ta = true; m.B = dY; m.ldb = Nout; m.C = c->gp(wid); m.ldc = Nout;
    m.M = Kin; m.N = Nout; m.K = ns; m.c_f32 = true;
    m.ws = c->wf(p.GEMMWS); m.ws_floats = p.gemmws_floats; m.colsum_out = bid >= 0 ? c->gp(bid) : nullptr;
    rows_wg_flops += 2.0 * m.M * m.N * m.K;
  };
  auto wgrad_rows_launch = [&]() {
    ProfScope ps_(c, gemm_cat(dt, rows_wg[0]), rows_wg_flops);
    gemm_wgrad_batch(dt, rows_wg, n_rows_wg, st);
  };
  auto dgrad = [&](const void* dY, int Nout, int wid, void* dX, int Kin, Epi epi, const void* aux, bool out_f32, int rows) {
    Gemm m;
    m.A = dY; m.lda = Nout; m.B = c->cp(wid); m.ldb = Nout; m.tb = true; m.C = dX; m.ldc = Kin;
    m.M = rows; m.N = Kin; m.K = Nout; m.epi = epi; m.aux = aux; m.ld_aux = Kin; m.c_f32 = out_f32;
    if (rows == ns) { m.ws = c->wf(p.GEMMWS); m.ws_floats = p.gemmws_floats; }   // lets a few-row product split its K
    ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K);
    gemm(dt, m, st);
  };
  auto row = [&](const void* src, int64_t src_elems, int esz_, void* dst, int cols) {   // gather descriptor
    return RowCopy{src, dst, src_elems * esz_, (int64_t)cols * esz_, cols * esz_};
  };
  auto back = [&](const void* src, int cols, int esz_, void* dst, int64_t dst_elems) {   // scatter descriptor
    return RowCopy{src, dst, (int64_t)cols * esz_, dst_elems * esz_, cols * esz_};
  };
  if (g.arch == PT_VIT_PRELN) {
    // rG, rHP (GELU out and GELU'), rXa (LN2 out), rXb (Y), rCTX and the LN2 statistics come from the forward,
    // rDO / rS0 (the first tokens' rows of dL/dx_L) from the head's backward: nothing to gather
    wgrad_rows(rG, F, rDO, D, c->blk(l, W2), -1);
    dgrad(rDO, D, c->blk(l, W2), rDF, F, EPI_MUL_DGELU, rHP, false, ns);
    wgrad_rows(rXa, D, rDF, F, c->blk(l, W1), c->blk(l, B1));
    dgrad(rDF, F, c->blk(l, W1), rOC, D, EPI_STORE, nullptr, false, ns);                 // dL/dLN2out
    { prof_ln_bwd(c, dt, false, false, rOC, D, rXb, D, rmu2, rrs2, c->cp(c->blk(l, LN2_G)), rS0, D, rS1, rOD, D,
                  c->gp(c->blk(l, LN2_G)), c->gp(c->blk(l, LN2_B)), c->gp(c->blk(l, BO)), ns, D, st); }  // rS1 / rOD = dL/dY
    wgrad_rows(rCTX, D, rOD, D, c->blk(l, WO), -1);
    wgrad_rows_launch();
    dgrad(rOD, D, c->blk(l, WO), rDCTX, D, EPI_STORE, nullptr, false, ns);                // dL/dCTX
    { ProfScope ps_(c, PT_PROF_ATTN_BWD, 8.0 * ns * g.H * (double)g.S * (D / g.H)); attention_bwd_first_query(dt, c->w(s.QKV), rCTX, rDCTX, c->wf(s.LSE), dQKV, ns, g.S, g.H, D / g.H, st); }
    wgrad(c->w(s.U), D, dQKV, 3 * D, c->blk(l, WQKV), c->blk(l, BQKV), Tn);
    dgrad(dQKV, 3 * D, c->blk(l, WQKV), oC, D, EPI_STORE, nullptr, false, Tn);            // dL/dU
    // dL/dY (rS1), the residual branch of dL/dx, is non-zero in the first tokens' rows only: it is added to
    // those rows (and to the column sums) after the LayerNorm backward instead of being read as a full tensor
    { prof_ln_bwd(c, dt, false, false, oC, D, xin, D, c->wf(s.MU1), c->wf(s.RS1), c->cp(c->blk(l, LN1_G)), nullptr, 0,
                  need_dx ? dx.s : nullptr, need_dx ? dx.o : nullptr, D, c->gp(c->blk(l, LN1_G)),
                  c->gp(c->blk(l, LN1_B)), lower_b2, Tn, D, st, /*reduce_now=*/true); }   // add_rows adds to lower_b2
    if (need_dx) add_rows(dt, rS1, dx.s, dx.o, SD, lower_b2, ns, D, st);
  } else {
    // post-LN: U = x + Attn(x) and WN = Y + MLP(Y) are the fp32 sums in front of the two LayerNorms
    // rXa (WN), rXb (U), rG, rHP, rDO (rows of Y), rCTX and both LayerNorms' statistics come from the forward
    const RowCopy in[] = {row(dout.s, SD, 4, rS0, D)};
    strided_rows_copy(in, 1, ns, st);
    { prof_ln_bwd(c, dt, true, true, rS0, D, rXa, D, rmu2, rrs2, c->cp(c->blk(l, LN2_G)), nullptr, 0, rS1, rOD, D,
                  c->gp(c->blk(l, LN2_G)), c->gp(c->blk(l, LN2_B)), c->gp(c->blk(l, B2)), ns, D, st); }  // rS1 / rOD = dL/d(Y+MLP)
    wgrad_rows(rG, F, rOD, D, c->blk(l, W2), -1);
    dgrad(rOD, D, c->blk(l, W2), rDF, F, EPI_MUL_DGELU, rHP, false, ns);
    wgrad_rows(rDO, D, rDF, F, c->blk(l, W1), c->blk(l, B1));                              // rDO holds the rows of Y here
    dgrad(rDF, F, c->blk(l, W1), rS2, D, EPI_RES, rS1, true, ns);                          // rS2 = dL/dY
    { prof_ln_bwd(c, dt, true, true, rS2, D, rXb, D, rmu1, rrs1, c->cp(c->blk(l, LN1_G)), nullptr, 0, rS1, rOC, D,
                  c->gp(c->blk(l, LN1_G)), c->gp(c->blk(l, LN1_B)), c->gp(c->blk(l, BO)), ns, D, st); }  // rS1 / rOC = dL/d(x+Attn)
    wgrad_rows(rCTX, D, rOC, D, c->blk(l, WO), -1);
    wgrad_rows_launch();
    dgrad(rOC, D, c->blk(l, WO), rDCTX, D, EPI_STORE, nullptr, false, ns);                // dL/dCTX
    const RowCopy out[] = {back(rS1, D, 4, dout.s, SD)};
    strided_rows_copy(out, 1, ns, st);
    { ProfScope ps_(c, PT_PROF_ATTN_BWD, 8.0 * ns * g.H * (double)g.S * (D / g.H)); attention_bwd_first_query(dt, c->w(s.QKV), rCTX, rDCTX, c->wf(s.LSE), dQKV, ns, g.S, g.H, D / g.H, st); }
    wgrad(xin, D, dQKV, 3 * D, c->blk(l, WQKV), c->blk(l, BQKV), Tn);
    if (need_dx) dgrad(dQKV, 3 * D, c->blk(l, WQKV), dx.s, D, EPI_RES, dout.s, true, Tn);
  }
}

// front end over `ns` samples; sample i reads input map[i] (device, or null = identity)
void front_forward(pt_ctx* c, const void* d_input, const int64_t* d_map, void* xout, int ns, bool save) {
  const pt_config& g = c->cfg;
  const Plan& p = c->plan;
  const int D = g.D, dt = c->dt;
  hipStream_t st = c->st;
  if (g.arch == PT_VIT_PRELN) {
    const int pd = g.chans * g.patch * g.patch, np = ns * (g.S - 1);
    vit_patchify(dt, (const float*)d_input, d_map, c->w(p.PATCH), ns, g.chans, g.img, g.patch, st);
    Gemm m;
    m.A = c->w(p.PATCH); m.lda = pd; m.B = c->cp(0); m.ldb = D; m.C = c->w(p.EMB); m.ldc = D;
    m.M = np; m.N = D; m.K = pd; m.epi = EPI_BIAS; m.bias = c->cp(1);
    { ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K); gemm(dt, m, st); }
    vit_assemble(dt, c->w(p.EMB), c->cp(2), c->cp(3), xout, ns, g.S, D, st);
  } else {
    bert_embed(dt, (const int32_t*)d_input, d_map, c->cp(0), c->cp(1), c->wf(p.EMB), ns, g.S, D, g.vocab, st);
    // the token-table gradient needs the ids again: keep a copy, so the caller's buffer may go once this call returns
    if (save) (void)hipMemcpyAsync(c->w(p.IDS), d_input, (size_t)ns * g.S * 4, hipMemcpyDeviceToDevice, st);
    { prof_ln_fwd(c, dt, true, c->w(p.EMB), D, c->cp(2), c->cp(3), xout, D, save ? c->wf(p.MUE) : nullptr,
                  save ? c->wf(p.RSE) : nullptr, ns * g.S, D, g.ln_eps, st); }
  }
}

void front_backward(pt_ctx* c, const float* dx, int ns) {
  const pt_config& g = c->cfg;
  const Plan& p = c->plan;
  const int D = g.D, dt = c->dt;
  hipStream_t st = c->st;
  if (g.arch == PT_VIT_PRELN) {
    const int pd = g.chans * g.patch * g.patch, np = ns * (g.S - 1);
    vit_front_bwd(dt, dx, c->w(p.DEMB), c->gp(3), c->gp(2), ns, g.S, D, st);
    Gemm m;
    m.A = c->w(p.PATCH); m.lda = pd; m.ta = true; m.B = c->w(p.DEMB); m.ldb = D; m.C = c->gp(0); m.ldc = D;
    m.M = pd; m.N = D; m.K = np; m.c_f32 = true;
    m.ws = c->wf(p.GEMMWS); m.ws_floats = p.gemmws_floats; m.colsum_out = c->gp(1);
    { ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K); gemm(dt, m, st); }
  } else {
    { prof_ln_bwd(c, dt, true, true, dx, D, c->w(p.EMB), D, c->wf(p.MUE), c->wf(p.RSE), c->cp(2), nullptr, 0, c->wf(p.DEMB),
                  nullptr, D, c->gp(2), c->gp(3), nullptr, ns * g.S, D, st); }
    fill_zero(c->gp(0), (size_t)c->plan.tensors[0].padded * 4, st);
    fill_zero(c->gp(1), (size_t)c->plan.tensors[1].padded * 4, st);
    bert_embed_bwd(reinterpret_cast<const int32_t*>(c->w(p.IDS)), c->wf(p.DEMB), c->gp(0), c->gp(1),
                   reinterpret_cast<int32_t*>(c->w(p.CHAINWS)), ns, g.S, D, g.vocab, st);
  }
}

// stage `n` int64 values for the device; returns the device pointer
struct IdxStager {
  pt_ctx* c;
  int turn;
  size_t used = 0;
  explicit IdxStager(pt_ctx* ctx) : c(ctx), turn(ctx->idx_turn) {}
  hipError_t begin() {
    if (c->idx_ev_used[turn]) return hipEventSynchronize(c->idx_ev[turn]);
    return hipSuccess;
  }
  const int64_t* put(const std::vector<int64_t>& v, hipError_t* e) {
    if (v.empty()) return nullptr;
    int64_t* h = c->h_idx[turn] + used;
    std::memcpy(h, v.data(), v.size() * 8);
    int64_t* d = reinterpret_cast<int64_t*>(c->w(c->plan.IDX)) + (size_t)turn * (c->plan.idx_capacity / 2) + used;
    hipError_t r = hipMemcpyAsync(d, h, v.size() * 8, hipMemcpyHostToDevice, c->st);
    if (r != hipSuccess) *e = r;
    used += v.size();
    return d;
  }
  hipError_t end() {
    hipError_t r = hipEventRecord(c->idx_ev[turn], c->st);
    c->idx_ev_used[turn] = true;
    c->idx_turn ^= 1;
    return r;
  }
};

}  // namespace

// ===========================================================================
// C ABI (pt.h declares every entry point with C linkage and default visibility; nothing else is exported)
// ===========================================================================

pt_status pt_query_arena_bytes(const pt_config* cfg, size_t* params, size_t* state, size_t* work, size_t* cache) {
  if (!cfg || !params || !state || !work || !cache) return PT_EINVAL;
  if (!validate(*cfg, nullptr)) return PT_EINVAL;
  Plan p;
  make_plan(*cfg, &p);
  *params = p.params_bytes; *state = p.state_bytes; *work = p.work_bytes; *cache = p.cache_bytes;
  return PT_OK;
}

pt_status pt_create(const pt_config* cfg, void* d_params, void* d_state, void* d_work, void* d_cache, void* hip_stream,
                    pt_ctx** out) {
  if (!cfg || !out || !d_params || !d_state || !d_work) return PT_EINVAL;
  if (!validate(*cfg, nullptr)) return PT_EINVAL;
  if (cfg->cache_slots + cfg->window_slots > 0 && !d_cache) return PT_EINVAL;
  for (const void* q : {d_params, d_state, d_work, (void*)d_cache})
    if (reinterpret_cast<uintptr_t>(q) % kAlign) return PT_EINVAL;
  pt_ctx* c = new (std::nothrow) pt_ctx();
  if (!c) return PT_ENOMEM;
  c->cfg = *cfg;
  make_plan(*cfg, &c->plan);
  c->dt = cfg->dtype == PT_BF16 ? 1 : 0;
  c->esz = c->dt ? 2 : 4;
  c->st = reinterpret_cast<hipStream_t>(hip_stream);
  const size_t P = (size_t)c->plan.arena_floats;
  c->master = reinterpret_cast<float*>(d_params);
  c->shadow = c->dt ? reinterpret_cast<char*>(d_params) + align_up(P * 4) : nullptr;
  // The state arenas hold the tensors from offset state_lo on; the pointers are those of a (virtual) full-size
  // arena, so that a tensor's offset addresses all arenas alike.  Nothing below state_lo is ever touched.
  const size_t Ps = P - (size_t)c->plan.state_lo, Sb = align_up(Ps * 4);
  auto state_arena = [&](int i) { return reinterpret_cast<float*>(reinterpret_cast<char*>(d_state) + (size_t)i * Sb) - c->plan.state_lo; };
  c->grads = state_arena(0);
  c->mom1 = state_arena(1);
  c->mom2 = cfg->optimizer == PT_ADAMW ? state_arena(2) : nullptr;
  c->gacc = cfg->grad_accum ? state_arena(cfg->optimizer == PT_ADAMW ? 3 : 2) : nullptr;
  c->k = cfg->k_min;
  c->work = reinterpret_cast<char*>(d_work);
  c->cache = reinterpret_cast<char*>(d_cache);
  c->slot_k.assign((size_t)(cfg->cache_slots + cfg->host_slots), -1);
  auto cleanup = [&]() {
    for (int i = 0; i < 2; ++i) {
      if (c->h_idx[i]) (void)hipHostFree(c->h_idx[i]);
      if (c->idx_ev[i]) (void)hipEventDestroy(c->idx_ev[i]);
    }
    if (c->h_norms) (void)hipHostFree(c->h_norms);
    if (c->norms_ev) (void)hipEventDestroy(c->norms_ev);
    delete c;
  };
#define CREATE_TRY(expr)                         \
  do {                                           \
    if ((expr) != hipSuccess) { cleanup(); return PT_EDEVICE; } \
  } while (0)
  for (int i = 0; i < 2; ++i) {
    CREATE_TRY(hipHostMalloc(reinterpret_cast<void**>(&c->h_idx[i]), (c->plan.idx_capacity / 2) * 8, hipHostMallocDefault));
    CREATE_TRY(hipEventCreateWithFlags(&c->idx_ev[i], hipEventDisableTiming));
  }
  CREATE_TRY(hipHostMalloc(reinterpret_cast<void**>(&c->h_norms), (size_t)(cfg->L + 3) * 4, hipHostMallocDefault));   // norms, loss
  CREATE_TRY(hipEventCreateWithFlags(&c->norms_ev, hipEventDisableTiming));
  CREATE_TRY(static_chunk_sums(&c->static_sq));   // set-up of pt_layer_grad_norms_static: resolved here, with this GPU current
  fill_zero(d_params, c->plan.params_bytes, c->st);
  fill_zero(d_state, c->plan.state_bytes, c->st);
  // chunk tables
  const size_t nchunks = P / kChunk;
  std::vector<uint8_t> decay(nchunks, 0);
  for (auto& t : c->plan.tensors)
    if (t.decayed)
      for (int64_t ch = t.offset / kChunk; ch < (t.offset + t.padded) / kChunk; ++ch) decay[(size_t)ch] = 1;
  CREATE_TRY(hipMemcpyAsync(c->w(c->plan.CHUNKDECAY), decay.data(), nchunks, hipMemcpyHostToDevice, c->st));
  CREATE_TRY(hipMemcpyAsync(c->w(c->plan.GROUPFIRST), c->plan.group_first_chunk.data(),
                            c->plan.group_first_chunk.size() * 8, hipMemcpyHostToDevice, c->st));
  CREATE_TRY(hipStreamSynchronize(c->st));
#undef CREATE_TRY
  *out = c;
  return PT_OK;
}

pt_status pt_destroy(pt_ctx* c) {
  if (!c) return PT_EINVAL;
  (void)hipStreamSynchronize(c->st);
  for (int i = 0; i < 2; ++i) {
    if (c->h_idx[i]) (void)hipHostFree(c->h_idx[i]);
    if (c->idx_ev[i]) (void)hipEventDestroy(c->idx_ev[i]);
  }
  if (c->h_norms) (void)hipHostFree(c->h_norms);
  if (c->norms_ev) (void)hipEventDestroy(c->norms_ev);
  for (auto& r : c->prof_pool) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); (void)hipEventDestroy(r.m); }
  if (c->copy_st) {
    (void)hipStreamSynchronize(c->copy_st);
    for (auto& w : c->win) if (w.ev) (void)hipEventDestroy(w.ev);
    if (c->ev_copy) (void)hipEventDestroy(c->ev_copy);
    if (c->ev_main) (void)hipEventDestroy(c->ev_main);
    (void)hipStreamDestroy(c->copy_st);
  }
  delete c;
  return PT_OK;
}

const char* pt_last_error(const pt_ctx* c) { return c ? c->err.c_str() : "null context"; }

pt_status pt_get_freeze_boundary(const pt_ctx* c, int32_t* k) {
  if (!c || !k) return PT_EINVAL;
  *k = c->k;
  return PT_OK;
}

pt_status pt_set_freeze_boundary(pt_ctx* c, int32_t k) {
  if (!c) return PT_EINVAL;
  if (k < 0 || k > c->cfg.L) return fail(c, PT_EINVAL, "boundary outside 0..L");
  if (k < c->k) return fail(c, PT_EINVAL, "the boundary never moves down");
  if (k == c->k) return PT_OK;
  if (c->acc_samples) return fail(c, PT_ESTATE, "the boundary cannot move while gradients are being accumulated");
  { const pt_status fs = flush_deferred_norms(c); if (fs != PT_OK) return fs; }   // pending norms are of the gradients and boundary as they are now
  // newly frozen: front end (if the old boundary was 0) and blocks k_old..k-1
  const auto& gf = c->plan.group_first_chunk;
  const int64_t lo = (c->k == 0 ? gf[0] : gf[c->k + 1]) * kChunk, hi = gf[k + 1] * kChunk;
  fill_zero(c->grads + lo, (size_t)(hi - lo) * 4, c->st);
  fill_zero(c->mom1 + lo, (size_t)(hi - lo) * 4, c->st);
  if (c->mom2) fill_zero(c->mom2 + lo, (size_t)(hi - lo) * 4, c->st);
  c->k = k;
  c->phase = 0;
  return PT_OK;
}

// ---- host tier of the activation cache (Sec. 3.4 / App. E: hierarchical cache with a sliding window) ----
namespace {

size_t cache_row_bytes(const pt_ctx* c) { return (size_t)c->cfg.S * c->cfg.D * c->esz; }
char* window_row(const pt_ctx* c, int slot) { return c->cache + (size_t)(c->cfg.cache_slots + slot) * cache_row_bytes(c); }
char* host_row(const pt_ctx* c, int64_t id) { return c->host_rows + (size_t)(id - c->cfg.cache_slots) * cache_row_bytes(c); }

// A free window slot, or -1.  Write-back slots are reclaimed once their copy has completed; `evict` also gives
// up staged rows that this call does not use; `block` waits for the copy stream as the last resort.
int window_alloc(pt_ctx* c, bool evict, bool block) {
  for (int pass = 0; pass < 2; ++pass) {
    for (size_t i = 0; i < c->win.size(); ++i)
      if (c->win[i].state == 0) return (int)i;
    for (size_t i = 0; i < c->win.size(); ++i)
      if (c->win[i].state == 2) {
        if (hipEventQuery(c->win[i].ev) == hipSuccess) { c->win[i].state = 0; c->win[i].id = -1; return (int)i; }
        (void)hipGetLastError();   // "not ready" is an answer, not an error to be reported later
      }
    if (evict) {
      int best = -1;
      for (size_t i = 0; i < c->win.size(); ++i)
        if (c->win[i].state == 1 && c->win[i].stamp != c->call_stamp && (best < 0 || c->win[i].stamp < c->win[best].stamp)) best = (int)i;
      if (best >= 0) { c->win_of.erase(c->win[best].id); c->win[best].state = 0; c->win[best].id = -1; return best; }
    }
    if (!block || pass == 1) break;
    if (hipStreamSynchronize(c->copy_st) != hipSuccess) return -1;
    for (auto& w : c->win) if (w.state == 2) { w.state = 0; w.id = -1; }
  }
  return -1;
}

// Stages the host row of `id` into a window slot (asynchronously, on the copy stream); returns the slot or -1.
int window_stage(pt_ctx* c, int64_t id, bool evict, bool block, hipError_t* err) {
  auto it = c->win_of.find(id);
  if (it != c->win_of.end()) return it->second;
  const int slot = window_alloc(c, evict, block);
  if (slot < 0) return -1;
  const hipError_t e = hipMemcpyAsync(window_row(c, slot), host_row(c, id), cache_row_bytes(c), hipMemcpyHostToDevice, c->copy_st);
  if (e != hipSuccess) { if (err) *err = e; return -1; }
  c->win[slot].id = id; c->win[slot].state = 1; c->win[slot].stamp = c->call_stamp;
  c->win_of[id] = slot;
  c->n_h2d++;
  return slot;
}

}  // namespace

pt_status pt_attach_host_tier(pt_ctx* c, void* h_rows, size_t bytes) {
  if (!c || !h_rows) return PT_EINVAL;
  if (c->cfg.host_slots <= 0) return fail(c, PT_ESTATE, "the configuration has host_slots = 0");
  if (c->host_rows) return fail(c, PT_ESTATE, "a host tier is already attached");
  if (bytes < (size_t)c->cfg.host_slots * cache_row_bytes(c)) return fail(c, PT_ENOMEM, "host tier memory too small");
  HIP_TRY(c, hipStreamCreateWithFlags(&c->copy_st, hipStreamNonBlocking));
  HIP_TRY(c, hipEventCreateWithFlags(&c->ev_copy, hipEventDisableTiming));
  HIP_TRY(c, hipEventCreateWithFlags(&c->ev_main, hipEventDisableTiming));
  c->win.resize((size_t)c->cfg.window_slots);
  for (auto& w : c->win) HIP_TRY(c, hipEventCreateWithFlags(&w.ev, hipEventDisableTiming));
  c->host_rows = static_cast<char*>(h_rows);
  return PT_OK;
}

pt_status pt_cache_prefetch(pt_ctx* c, const int64_t* sample_ids, int32_t n, int32_t* staged_out) {
  if (!c || (!sample_ids && n > 0) || n < 0) return PT_EINVAL;
  if (staged_out) *staged_out = 0;
  if (!c->host_rows) return PT_OK;   // nothing lives on the host: every row is already in HBM
  const int64_t lo = c->cfg.cache_slots, hi = lo + c->cfg.host_slots;
  c->call_stamp++;
  hipError_t err = hipSuccess;
  int staged = 0;
  for (int i = 0; i < n; ++i) {
    const int64_t id = sample_ids[i];
    if (id < 0 || id >= hi) return fail(c, PT_EINVAL, "sample id outside the cache");
    if (id < lo || c->slot_k[(size_t)id] < 0 || c->win_of.count(id)) continue;
    if (window_stage(c, id, false, false, &err) < 0) break;   // best effort: the window is full
    ++staged;
  }
  if (err != hipSuccess) return fail(c, PT_EDEVICE, hipGetErrorString(err));
  c->n_prefetched += staged;
  if (staged_out) *staged_out = staged;
  return PT_OK;
}

pt_status pt_host_tier_stats(const pt_ctx* c, int64_t* rows_to_device, int64_t* rows_to_host, int64_t* prefetched,
                             int64_t* prefetched_used) {
  if (!c) return PT_EINVAL;
  if (rows_to_device) *rows_to_device = c->n_h2d;
  if (rows_to_host) *rows_to_host = c->n_d2h;
  if (prefetched) *prefetched = c->n_prefetched;
  if (prefetched_used) *prefetched_used = c->n_prefetch_used;
  return PT_OK;
}

pt_status pt_frozen_forward(pt_ctx* c, const void* d_input, int32_t nb, const int64_t* sample_ids, void** d_hk_out) {
  if (!c || !d_input || !d_hk_out) return PT_EINVAL;
  const pt_config& g = c->cfg;
  const Plan& p = c->plan;
  if (nb < 1 || nb > g.B) return fail(c, PT_EINVAL, "batch outside 1..B");
  const int k = c->k;
  const size_t row_bytes = (size_t)g.S * g.D * c->esz;
  if (k == 0) {
    front_forward(c, d_input, nullptr, c->w(p.X[0]), nb, true);
    c->last_hk = c->w(p.X[0]);
  } else {
    const bool use_cache = sample_ids && g.cache_slots + g.host_slots > 0;
    std::vector<int> kw(nb, -1);
    // device row of each sample in the cache arena: its own slot, or a window slot for the host tier
    std::vector<int64_t> row_r(nb, -1), row_w(nb, -1);
    bool host_used = false;
    if (use_cache) {
      if (g.host_slots > 0 && !c->host_rows) return fail(c, PT_ESTATE, "host_slots > 0 but no host tier is attached");
      std::unordered_set<int64_t> seen;
      for (int i = 0; i < nb; ++i) {
        if (sample_ids[i] < 0 || sample_ids[i] >= g.cache_slots + g.host_slots) return fail(c, PT_EINVAL, "sample id outside the cache");
        if (!seen.insert(sample_ids[i]).second) return fail(c, PT_EINVAL, "duplicate sample id in a batch");
        kw[i] = c->slot_k[(size_t)sample_ids[i]];
        if (sample_ids[i] < g.cache_slots) row_r[i] = row_w[i] = sample_ids[i];
      }
      // host tier: rows already staged by pt_cache_prefetch are used as they are, the others are staged now;
      // a row that will be (re)written gets a window slot to be copied back from.  All window slots are
      // chosen before the main stream is made to wait for the copy stream, so none of them is in flight
      // when a kernel below touches it.
      // Every window slot this call can need is known to exist before any is taken: a host-tier sample
      // needs one slot (its staged row, or a fresh one to be written back from), and any slot that does not
      // hold a row of this batch can be had (free, reclaimed after its write-back, or evicted).
      {
        int64_t needed = 0, own = 0;
        for (int i = 0; i < nb; ++i) {
          if (sample_ids[i] < g.cache_slots) continue;
          if (c->win_of.count(sample_ids[i])) ++own;
          else if (kw[i] >= 0 || kw[i] < k) ++needed;
        }
        if (needed + own > (int64_t)c->win.size()) return fail(c, PT_ENOMEM, "the window cannot hold this batch's host-tier rows");
      }
      c->call_stamp++;
      hipError_t herr = hipSuccess;
      for (int i = 0; i < nb; ++i) {
        if (sample_ids[i] < g.cache_slots || kw[i] < 0) continue;
        auto it = c->win_of.find(sample_ids[i]);
        if (it != c->win_of.end()) { c->win[it->second].stamp = c->call_stamp; c->n_prefetch_used++; }
      }
      for (int i = 0; i < nb; ++i) {
        if (sample_ids[i] < g.cache_slots) continue;
        host_used = true;
        int slot = -1;
        if (kw[i] >= 0) {
          slot = window_stage(c, sample_ids[i], true, true, &herr);
          if (slot < 0) return fail(c, herr != hipSuccess ? PT_EDEVICE : PT_ENOMEM, "no window slot for a host-tier row");
          c->win[slot].stamp = c->call_stamp;
          row_r[i] = g.cache_slots + slot;
        }
        if (kw[i] < k) {
          if (slot < 0) {
            slot = window_alloc(c, true, true);
            if (slot < 0) return fail(c, PT_ENOMEM, "no window slot for a host-tier row");
            c->win[slot].id = sample_ids[i]; c->win[slot].state = 1; c->win[slot].stamp = c->call_stamp;
          }
          row_w[i] = g.cache_slots + slot;
        }
      }
      if (host_used) {
        HIP_TRY(c, hipEventRecord(c->ev_copy, c->copy_st));
        HIP_TRY(c, hipStreamWaitEvent(c->st, c->ev_copy, 0));
      }
    }
    // sorted order: misses first, then by the boundary the row was written at (stable)
    std::vector<int> order(nb);
    for (int i = 0; i < nb; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return kw[a] < kw[b]; });
    bool identity = true;
    for (int i = 0; i < nb; ++i) identity = identity && order[i] == i;
    int n_miss = 0, n_hit = 0;
    for (int i = 0; i < nb; ++i) { n_miss += kw[i] < 0; n_hit += kw[i] == k; }
    IdxStager stg(c);
    HIP_TRY(c, stg.begin());
    hipError_t cerr = hipSuccess;
    if (n_hit == nb) {
      // every sample is a hit: one gather from the cache, no block runs
      std::vector<int64_t> src(nb);
      for (int i = 0; i < nb; ++i) src[i] = row_r[i];
      const int64_t* dsrc = stg.put(src, &cerr);
      { prof_copy_rows(c, c->w(p.HKOUT), nullptr, c->cache, dsrc, nb, row_bytes, c->st); }
      c->last_hk = c->w(p.HKOUT);
    } else {
      if (n_miss > 0) {
        const int64_t* dmap = nullptr;
        if (!(identity && n_miss == nb)) {
          std::vector<int64_t> map(n_miss);
          for (int i = 0; i < n_miss; ++i) map[i] = order[i];
          dmap = stg.put(map, &cerr);
        }
        front_forward(c, d_input, dmap, c->w(p.X[0]), n_miss, false);
      }
      // level j: rows written at j join at their sorted positions, then block j runs on the prefix
      for (int j = 0; j <= k; ++j) {
        std::vector<int64_t> dst, src;
        int n_le = 0;
        for (int i = 0; i < nb; ++i) {
          if (kw[order[i]] == j) { dst.push_back(i); src.push_back(row_r[order[i]]); }
          n_le += kw[order[i]] <= j;
        }
        if (!dst.empty()) {
          const int64_t* ddst = stg.put(dst, &cerr);
          const int64_t* dsrc = stg.put(src, &cerr);
          { prof_copy_rows(c, c->w(p.X[j]), ddst, c->cache, dsrc, (int)dst.size(), row_bytes, c->st); }
        }
        // the sorted prefix of n_le samples (misses and rows written at or below j) runs block j
        if (j < k && n_le > 0) {
          block_forward(c, j, c->w(p.X[j]), c->w(p.X[j + 1]), p.slot[g.L], n_le, false);
          c->n_runs += n_le;
        }
      }
      if (use_cache) {
        std::vector<int64_t> dst, src;
        for (int i = 0; i < nb; ++i)
          if (kw[order[i]] < k) { dst.push_back(row_w[order[i]]); src.push_back(i); }
        const int64_t* ddst = stg.put(dst, &cerr);
        const int64_t* dsrc = stg.put(src, &cerr);
        { prof_copy_rows(c, c->cache, ddst, c->w(p.X[k]), dsrc, (int)dst.size(), row_bytes, c->st); }
      }
      if (identity) {
        c->last_hk = c->w(p.X[k]);
      } else {
        std::vector<int64_t> dst(nb);
        for (int i = 0; i < nb; ++i) dst[i] = order[i];
        const int64_t* ddst = stg.put(dst, &cerr);
        { prof_copy_rows(c, c->w(p.HKOUT), ddst, c->w(p.X[k]), nullptr, nb, row_bytes, c->st); }
        c->last_hk = c->w(p.HKOUT);
      }
    }
    HIP_TRY(c, stg.end());
    if (cerr != hipSuccess) return fail(c, PT_EDEVICE, hipGetErrorString(cerr));
    if (host_used) {
      // the copy stream continues only after this call's kernels: rewritten rows go back to the host, rows that
      // were only read give their window slot back
      HIP_TRY(c, hipEventRecord(c->ev_main, c->st));
      HIP_TRY(c, hipStreamWaitEvent(c->copy_st, c->ev_main, 0));
      for (int i = 0; i < nb; ++i) {
        if (sample_ids[i] < g.cache_slots) continue;
        const int slot = (int)((row_w[i] >= 0 ? row_w[i] : row_r[i]) - g.cache_slots);
        c->win_of.erase(sample_ids[i]);
        if (row_w[i] >= 0) {
          HIP_TRY(c, hipMemcpyAsync(host_row(c, sample_ids[i]), window_row(c, slot), row_bytes, hipMemcpyDeviceToHost, c->copy_st));
          HIP_TRY(c, hipEventRecord(c->win[slot].ev, c->copy_st));
          c->win[slot].state = 2;
          c->n_d2h++;
        } else {
          c->win[slot].state = 0; c->win[slot].id = -1;
        }
      }
    }
    if (use_cache)
      for (int i = 0; i < nb; ++i) {
        if (kw[i] < 0) c->n_miss++; else if (kw[i] == k) c->n_hit++; else c->n_adv++;
        c->slot_k[(size_t)sample_ids[i]] = k;
      }
  }
  HIP_TRY(c, hipGetLastError());
  c->nb = nb;
  c->phase = 1;
  *d_hk_out = c->last_hk;
  return PT_OK;
}

pt_status pt_time_frozen_forward(pt_ctx* c, const void* d_input, int32_t nb, const int64_t* sample_ids, int32_t reps,
                                 float* ms_recompute, float* ms_cached) {
  if (!c || !d_input || !sample_ids || !ms_recompute || !ms_cached || reps < 1) return PT_EINVAL;
  if (c->k < 1) return fail(c, PT_ESTATE, "nothing is frozen: there is no prefix to time");
  if (c->cfg.cache_slots + c->cfg.host_slots <= 0) return fail(c, PT_ESTATE, "the configuration has no cache");
  void* hk = nullptr;
  pt_status st = pt_frozen_forward(c, d_input, nb, sample_ids, &hk);   // rows are written / advanced here, untimed
  if (st != PT_OK) return st;
  hipEvent_t e[3] = {nullptr, nullptr, nullptr};
  for (auto& ev : e) HIP_TRY(c, hipEventCreate(&ev));
  hipError_t herr = hipEventRecord(e[0], c->st);
  for (int i = 0; i < reps && st == PT_OK; ++i) st = pt_frozen_forward(c, d_input, nb, nullptr, &hk);
  if (herr == hipSuccess) herr = hipEventRecord(e[1], c->st);
  for (int i = 0; i < reps && st == PT_OK; ++i) st = pt_frozen_forward(c, d_input, nb, sample_ids, &hk);
  if (herr == hipSuccess) herr = hipEventRecord(e[2], c->st);
  if (herr == hipSuccess) herr = hipEventSynchronize(e[2]);
  float a = 0.f, b = 0.f;
  if (herr == hipSuccess) herr = hipEventElapsedTime(&a, e[0], e[1]);
  if (herr == hipSuccess) herr = hipEventElapsedTime(&b, e[1], e[2]);
  for (auto& ev : e) (void)hipEventDestroy(ev);
  if (st != PT_OK) return st;
  if (herr != hipSuccess) return fail(c, PT_EDEVICE, hipGetErrorString(herr));
  *ms_recompute = a / (float)reps;
  *ms_cached = b / (float)reps;
  return PT_OK;
}

pt_status pt_active_fwd_bwd(pt_ctx* c, const void* d_hk, const int32_t* d_labels, float* loss_out) {
  if (!c || !d_hk || !d_labels) return PT_EINVAL;
  if (c->phase < 1) return fail(c, PT_ESTATE, "pt_frozen_forward has not run for this step");
  if (reinterpret_cast<uintptr_t>(d_hk) % 16) return fail(c, PT_EINVAL, "d_hk must be 16-byte aligned");
  { const pt_status fs = flush_deferred_norms(c); if (fs != PT_OK) return fs; }   // pending norms are of the gradients and boundary as they are now
  c->ln_jobs.clear();
  c->wgrad_carry.nprob = 0;
  c->pending_nwg = 0;
  const pt_config& g = c->cfg;
  const Plan& p = c->plan;
  const int L = g.L, D = g.D, S = g.S, k = c->k, nb = c->nb, dt = c->dt;
  hipStream_t st = c->st;
  // forward through the active blocks, keeping what the backward pass reads
  const void* x = d_hk;
  // under a first-token head the top block runs on those tokens' rows behind its attention, both ways
  const bool top_first_rows = S >= 4 && (g.arch == PT_VIT_PRELN || g.head == PT_HEAD_CLS);
  for (int l = k; l < L; ++l) {
    if (l == L - 1 && top_first_rows) block_forward_first_rows(c, l, x, c->w(p.X[l + 1]), p.slot[l], nb);
    else block_forward(c, l, x, c->w(p.X[l + 1]), p.slot[l], nb, true);
    x = c->w(p.X[l + 1]);
  }
  GradBufs dcur{c->wf(p.sA), c->w(p.oA)};
  GradBufs dnext{c->wf(p.sB), c->w(p.oB)};
  // head, loss, head backward -> dcur = dL/dx_L
  if (g.arch == PT_VIT_PRELN) {
    const int C = g.n_out;
    const int hg = c->head(0), hb = c->head(1), hW = c->head(2), hbias = c->head(3);
    { prof_ln_fwd(c, dt, false, x, (int64_t)S * D, c->cp(hg), c->cp(hb), c->w(p.CFEAT), D, c->wf(p.MUF), c->wf(p.RSF), nb, D, g.ln_eps, st); }
    Gemm m;
    m.A = c->w(p.CFEAT); m.lda = D; m.B = c->cp(hW); m.ldb = C; m.C = c->w(p.LOGITS); m.ldc = C;
    m.M = nb; m.N = C; m.K = D; m.epi = EPI_BIAS; m.bias = c->cp(hbias); m.c_f32 = true;
    { ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K); gemm(dt, m, st); }
    ce_rows(dt, c->wf(p.LOGITS), d_labels, c->wf(p.LOSSROWS), c->w(p.DZ), nb, C, st);
    mean_reduce(c->wf(p.LOSSROWS), nb, c->wf(p.LOSS), st);
    Gemm wg;
    wg.A = c->w(p.CFEAT); wg.lda = D; wg.ta = true; wg.B = c->w(p.DZ); wg.ldb = C; wg.C = c->gp(hW); wg.ldc = C;
    wg.M = D; wg.N = C; wg.K = nb; wg.c_f32 = true;
    wg.ws = c->wf(p.GEMMWS); wg.ws_floats = p.gemmws_floats; wg.colsum_out = c->gp(hbias);
    { ProfScope ps_(c, gemm_cat(dt, wg), 2.0 * wg.M * wg.N * wg.K); gemm(dt, wg, st); }
    Gemm dg;
    dg.A = c->w(p.DZ); dg.lda = C; dg.B = c->cp(hW); dg.ldb = C; dg.tb = true; dg.C = c->w(p.DC); dg.ldc = D;
    dg.M = nb; dg.N = D; dg.K = C;
    { ProfScope ps_(c, gemm_cat(dt, dg), 2.0 * dg.M * dg.N * dg.K); gemm(dt, dg, st); }
    // only the CLS rows of dL/dx_L are non-zero: when the top block's backward runs on those rows (below) they
    // go, dense, straight into its row buffers; otherwise into a zero-filled full-size gradient
    if (top_first_rows && k < L) {
      { prof_ln_bwd(c, dt, false, false, c->w(p.DC), D, x, (int64_t)S * D, c->wf(p.MUF), c->wf(p.RSF), c->cp(hg), nullptr, 0,
                    c->wf(p.rS0), c->w(p.rDO), D, c->gp(hg), c->gp(hb), c->gp(c->blk(L - 1, B2)), nb, D, st); }
    } else {
      fill_zero(dcur.s, (size_t)nb * S * D * 4, st);
      fill_zero(dcur.o, (size_t)nb * S * D * c->esz, st);
      { prof_ln_bwd(c, dt, false, false, c->w(p.DC), D, x, (int64_t)S * D, c->wf(p.MUF), c->wf(p.RSF), c->cp(hg), nullptr, 0, dcur.s,
                    dcur.o, (int64_t)S * D, c->gp(hg), c->gp(hb), k < L ? c->gp(c->blk(L - 1, B2)) : nullptr,
                    nb, D, st); }
    }
  } else if (g.head == PT_HEAD_CLS) {
    // sequence classification: the first token's final activation -> linear classifier -> cross-entropy
    const int C = g.n_out;
    const int hW = c->head(0), hbias = c->head(1);
    const int64_t SD = (int64_t)S * D;
    Gemm m;
    m.A = x; m.lda = SD; m.B = c->cp(hW); m.ldb = C; m.C = c->w(p.LOGITS); m.ldc = C;
    m.M = nb; m.N = C; m.K = D; m.epi = EPI_BIAS; m.bias = c->cp(hbias); m.c_f32 = true;
    { ProfScope ps_(c, gemm_cat(dt, m), 2.0 * m.M * m.N * m.K); gemm(dt, m, st); }
    ce_rows(dt, c->wf(p.LOGITS), d_labels, c->wf(p.LOSSROWS), c->w(p.DZ), nb, C, st);
    mean_reduce(c->wf(p.LOSSROWS), nb, c->wf(p.LOSS), st);
    Gemm wg;
    wg.A = x; wg.lda = SD; wg.ta = true; wg.B = c->w(p.DZ); wg.ldb = C; wg.C = c->gp(hW); wg.ldc = C;
    wg.M = D; wg.N = C; wg.K = nb; wg.c_f32 = true;
    wg.ws = c->wf(p.GEMMWS); wg.ws_floats = p.gemmws_floats; wg.colsum_out = c->gp(hbias);
    { ProfScope ps_(c, gemm_cat(dt, wg), 2.0 * wg.M * wg.N * wg.K); gemm(dt, wg, st); }
    // dL/dx_L is zero except in the first token's rows, which the input-gradient product writes in place
    fill_zero(dcur.s, (size_t)nb * S * D * 4, st);
    Gemm dg;
    dg.A = c->w(p.DZ); dg.lda = C; dg.B = c->cp(hW); dg.ldb = C; dg.tb = true; dg.C = dcur.s; dg.ldc = SD;
    dg.M = nb; dg.N = D; dg.K = C; dg.c_f32 = true;
    { ProfScope ps_(c, gemm_cat(dt, dg), 2.0 * dg.M * dg.N * dg.K); gemm(dt, dg, st); }
  } else {
    const int hW = c->head(0), hbias = c->head(1);
    qa_logits(dt, x, c->cp(hW), c->cp(hbias), c->wf(p.LOGITS), nb * S, D, st);
    qa_ce(dt, c->wf(p.LOGITS), d_labels, c->wf(p.LOSSROWS), c->wf(p.DZ), nb, S, st);
    mean_reduce(c->wf(p.LOSSROWS), nb, c->wf(p.LOSS), st);
    qa_head_bwd(dt, x, c->cp(hW), c->wf(p.DZ), dcur.s, c->gp(hW), c->gp(hbias), c->wf(p.QAPART), nb * S, D, st);
  }
  // backward through the active blocks; stops at the boundary (Sec. 3.2.1)
  for (int l = L - 1; l >= k; --l) {
    const void* xin = (l == k) ? d_hk : c->w(p.X[l]);
    const bool need_dx = (l > k) || (k == 0);
    float* lower_b2 = (g.arch == PT_VIT_PRELN && l > k) ? c->gp(c->blk(l - 1, B2)) : nullptr;
    // under a first-token head only those tokens' rows of dL/dx_L are non-zero
    const bool first_rows = l == L - 1 && top_first_rows;
    if (first_rows) block_backward_first_rows(c, l, xin, p.slot[l], dcur, dnext, nb, need_dx, lower_b2);
    else block_backward(c, l, xin, p.slot[l], dcur, dnext, nb, need_dx, lower_b2);
    std::swap(dcur, dnext);
  }
  launch_pending_wgrads(c, nullptr);
  flush_wgrad_carry(c);   // in front of the front end's products, which use the same workspace
  if (k == 0) front_backward(c, dcur.s, nb);
  flush_ln_reductions(c);
  c->last_dhk = dcur.s;
  HIP_TRY(c, hipGetLastError());
  c->phase = 2;
  if (loss_out) return pt_last_loss(c, loss_out);
  return PT_OK;
}

pt_status pt_last_loss(pt_ctx* c, float* loss_out) {
  if (!c || !loss_out) return PT_EINVAL;
  if (c->phase < 2) return fail(c, PT_ESTATE, "no loss has been computed");
  // through the pinned buffer (its slot behind the norms): a copy into pageable memory takes several times as long
  float* h = c->h_norms + c->cfg.L + 2;
  HIP_TRY(c, hipMemcpyAsync(h, c->w(c->plan.LOSS), 4, hipMemcpyDeviceToHost, c->st));
  HIP_TRY(c, hipStreamSynchronize(c->st));
  *loss_out = *h;
  return PT_OK;
}

namespace {
// the norm kernels over the active chunks; with_sumsq = false when the chunk sums are already there
pt_status enqueue_norms(pt_ctx* c, bool with_sumsq) {
  const auto& gf = c->plan.group_first_chunk;
  const int G = c->cfg.L + 2, k = c->k;
  const int64_t first = k == 0 ? 0 : gf[k + 1], total = gf[G];
  if (with_sumsq) { ProfScope ps_(c, PT_PROF_NORMS, 4.0 * (total - first) * kChunk); sumsq_chunks(c->grads, c->wf(c->plan.CHUNKSQ), first, total - first, c->st); }
  // the last kernel writes the L + 2 norms straight into pinned host memory: the only thing between the GPU
  // finishing and the caller going on is the wait itself (a copy command into pageable memory cost 15-25 us)
  if (with_sumsq) {
    finalize_norms(c->wf(c->plan.CHUNKSQ), reinterpret_cast<const int64_t*>(c->w(c->plan.GROUPFIRST)), G, k + 1, k == 0,
                   c->h_norms, c->st);
  } else {   // the pass over the gradient was the update's: only this kernel is booked under the norms
    ProfScope ps_(c, PT_PROF_NORMS, 0.0);
    finalize_norms(c->wf(c->plan.CHUNKSQ), reinterpret_cast<const int64_t*>(c->w(c->plan.GROUPFIRST)), G, k + 1, k == 0,
                   c->h_norms, c->st);
  }
  HIP_TRY(c, hipEventRecord(c->norms_ev, c->st));
  return PT_OK;
}

}  // namespace

// The begin half only notes the request.  If the update comes next, it reads the gradient anyway and leaves
// the per-chunk sums of squares as a by-product (one pass over the gradient instead of two); otherwise the
// end half, or whatever else would change the gradient or the boundary first, enqueues the norm pass itself.
pt_status pt_layer_grad_norms_begin(pt_ctx* c) {
  if (!c) return PT_EINVAL;
  if (c->phase != 2) return fail(c, PT_ESTATE, "gradient norms need a completed pt_active_fwd_bwd");
  if (c->norms_pending) return fail(c, PT_ESTATE, "the norms of an earlier pt_layer_grad_norms_begin have not been fetched");
  c->norms_pending = true;
  c->norms_deferred = true;
  return PT_OK;
}

namespace {
// called by every entry point that is about to change the gradients or the boundary while norms are deferred
pt_status flush_deferred_norms(pt_ctx* c) {
  if (!c->norms_pending || !c->norms_deferred) return PT_OK;
  c->norms_deferred = false;
  return enqueue_norms(c, true);
}
}  // namespace

pt_status pt_layer_grad_norms_end(pt_ctx* c, float* norms_out) {
  if (!c || !norms_out) return PT_EINVAL;
  if (!c->norms_pending) return fail(c, PT_ESTATE, "pt_layer_grad_norms_begin has not run");
  const pt_status s = flush_deferred_norms(c);
  if (s != PT_OK) return s;
  HIP_TRY(c, hipEventSynchronize(c->norms_ev));
  std::memcpy(norms_out, c->h_norms, (size_t)(c->cfg.L + 2) * 4);
  c->norms_pending = false;
  return PT_OK;
}

pt_status pt_layer_grad_norms(pt_ctx* c, float* norms_out) {
  if (!c || !norms_out) return PT_EINVAL;
  const pt_status s = pt_layer_grad_norms_begin(c);
  return s == PT_OK ? pt_layer_grad_norms_end(c, norms_out) : s;
}

// pt_layer_grad_norms for callers that may not allocate and have no workspace to lend: the per-chunk sums go
// to the library's static array on this GPU (address resolved in pt_create).  Nothing has to be cleared: the
// first kernel overwrites the sum of every active chunk and the second reads active chunks only.
pt_status pt_layer_grad_norms_static(pt_ctx* c, float* norms_out) {
  if (!c || !norms_out) return PT_EINVAL;
  if (c->phase != 2) return fail(c, PT_ESTATE, "gradient norms need a completed pt_active_fwd_bwd");
  if (c->norms_pending) return fail(c, PT_ESTATE, "the norms of an earlier pt_layer_grad_norms_begin have not been fetched");
  const auto& gf = c->plan.group_first_chunk;
  const int G = c->cfg.L + 2, k = c->k;
  const int64_t first = k == 0 ? 0 : gf[k + 1], total = gf[G];
  if (total > static_chunk_capacity())
    return fail(c, PT_EINVAL, "model too large for pt_layer_grad_norms_static: " + std::to_string(total) + " chunks of 1024 parameters, the static array holds " + std::to_string(static_chunk_capacity()));
  if (!c->static_sq) return fail(c, PT_EDEVICE, "the static array's address is unknown");
  sumsq_chunks(c->grads, c->static_sq, first, total - first, c->st);   // no timing scope here: it may create events
  finalize_norms(c->static_sq, reinterpret_cast<const int64_t*>(c->w(c->plan.GROUPFIRST)), G, k + 1, k == 0, c->h_norms, c->st);
  HIP_TRY(c, hipGetLastError());
  HIP_TRY(c, hipEventRecord(c->norms_ev, c->st));
  HIP_TRY(c, hipEventSynchronize(c->norms_ev));
  std::memcpy(norms_out, c->h_norms, (size_t)(c->cfg.L + 2) * 4);
  return PT_OK;
}

pt_status pt_optimizer_step(pt_ctx* c, const pt_opt_hparams* hp) {
  if (!c || !hp) return PT_EINVAL;
  if (c->phase != 2) return fail(c, PT_ESTATE, "the optimizer needs a completed pt_active_fwd_bwd");
  const auto& gf = c->plan.group_first_chunk;
  const int G = c->cfg.L + 2, k = c->k;
  const int64_t first = k == 0 ? 0 : gf[k + 1], total = gf[G];
  const int64_t t = c->step + 1;
  OptArgs a;
  a.lr = hp->lr; a.momentum = hp->momentum; a.beta1 = hp->beta1; a.beta2 = hp->beta2; a.eps = hp->eps;
  a.weight_decay = hp->weight_decay;
  a.bias_c1 = (float)(1.0 - std::pow((double)hp->beta1, (double)t));
  a.bias_c2 = (float)(1.0 - std::pow((double)hp->beta2, (double)t));
  const uint8_t* decay = reinterpret_cast<const uint8_t*>(c->w(c->plan.CHUNKDECAY));
  // norms asked for and not yet enqueued: this pass over the gradient also leaves the per-chunk sums of squares
  const bool take_norms = c->norms_pending && c->norms_deferred;
  float* chunk_sq = take_norms ? c->wf(c->plan.CHUNKSQ) : nullptr;
  if (c->cfg.optimizer == PT_ADAMW)
    { ProfScope ps_(c, PT_PROF_OPT, (c->shadow ? 30.0 : 28.0) * (total - first) * kChunk); adamw_chunks(c->master, c->grads, c->mom1, c->mom2, c->shadow, decay, first, total - first, a, chunk_sq, c->st); }
  else
    { ProfScope ps_(c, PT_PROF_OPT, (c->shadow ? 22.0 : 20.0) * (total - first) * kChunk); sgdm_chunks(c->master, c->grads, c->mom1, c->shadow, decay, first, total - first, a, chunk_sq, c->st); }
  HIP_TRY(c, hipGetLastError());
  if (take_norms) {
    c->norms_deferred = false;
    const pt_status ns = enqueue_norms(c, false);
    if (ns != PT_OK) return ns;
  }
  c->step = t;
  c->phase = 0;
  if (c->prof_on) prof_collect(c);
  return PT_OK;
}

pt_status pt_accumulate_grads(pt_ctx* c, int32_t first) {
  if (!c) return PT_EINVAL;
  if (!c->gacc) return fail(c, PT_ESTATE, "the configuration has grad_accum = 0");
  if (c->phase != 2) return fail(c, PT_ESTATE, "accumulation needs a completed pt_active_fwd_bwd");
  if (!first && c->acc_samples == 0) return fail(c, PT_ESTATE, "no accumulation in progress: pass first = 1");
  const auto& gf = c->plan.group_first_chunk;
  const int G = c->cfg.L + 2, k = c->k;
  const int64_t lo = k == 0 ? 0 : gf[k + 1], total = gf[G];
  { ProfScope ps_(c, PT_PROF_OPT, 12.0 * (total - lo) * kChunk);
    grad_accumulate_chunks(c->gacc, c->grads, lo, total - lo, (float)c->nb, first != 0, c->wf(c->plan.LOSS),
                           c->wf(c->plan.LOSSACC), c->st); }
  HIP_TRY(c, hipGetLastError());
  c->acc_samples = (first ? 0 : c->acc_samples) + c->nb;
  c->phase = 0;
  return PT_OK;
}

pt_status pt_finish_accumulation(pt_ctx* c, float* mean_loss_out) {
  if (!c) return PT_EINVAL;
  if (!c->gacc || c->acc_samples == 0) return fail(c, PT_ESTATE, "no accumulation in progress");
  if (c->phase != 0) return fail(c, PT_ESTATE, "a micro-batch is in flight: accumulate it first");
  { const pt_status fs = flush_deferred_norms(c); if (fs != PT_OK) return fs; }   // pending norms are of the gradients and boundary as they are now
  const auto& gf = c->plan.group_first_chunk;
  const int G = c->cfg.L + 2, k = c->k;
  const int64_t lo = k == 0 ? 0 : gf[k + 1], total = gf[G];
  { ProfScope ps_(c, PT_PROF_OPT, 8.0 * (total - lo) * kChunk);
    grad_average_chunks(c->grads, c->gacc, lo, total - lo, 1.0f / (float)c->acc_samples, c->wf(c->plan.LOSS),
                        c->wf(c->plan.LOSSACC), c->st); }
  HIP_TRY(c, hipGetLastError());
  c->acc_samples = 0;
  c->phase = 2;
  if (mean_loss_out) return pt_last_loss(c, mean_loss_out);
  return PT_OK;
}

pt_status pt_next_boundary(const float* norms, int32_t L, int32_t k_prev, double alpha, int32_t* k_next) {
  if (!norms || !k_next || L < 1 || k_prev < 0 || k_prev > L || !(alpha > 0.0 && alpha < 1.0)) return PT_EINVAL;
  if (k_prev == L) { *k_next = L; return PT_OK; }
  const int bound = (int)std::floor((double)k_prev + alpha * (double)(L - k_prev));
  int arg = k_prev;
  for (int l = k_prev + 1; l < L; ++l)
    if (norms[1 + l] < norms[1 + arg]) arg = l;
  *k_next = std::max(k_prev, std::min(bound, arg));
  return PT_OK;
}

// ---- tensor table ---------------------------------------------------------
pt_status pt_num_tensors(const pt_ctx* c, int32_t* n) {
  if (!c || !n) return PT_EINVAL;
  *n = (int32_t)c->plan.tensors.size();
  return PT_OK;
}

pt_status pt_tensor_info(const pt_ctx* c, int32_t id, char* name, size_t name_cap, int64_t* numel, int32_t* rows,
                         int32_t* cols, int32_t* group, int32_t* decayed) {
  if (!c || id < 0 || id >= (int)c->plan.tensors.size()) return PT_EINVAL;
  const TensorDesc& t = c->plan.tensors[id];
  if (name && name_cap) { std::strncpy(name, t.name.c_str(), name_cap - 1); name[name_cap - 1] = 0; }
  if (numel) *numel = t.numel;
  if (rows) *rows = t.rows;
  if (cols) *cols = t.cols;
  if (group) *group = t.group;
  if (decayed) *decayed = t.decayed;
  return PT_OK;
}

static float* kind_base(pt_ctx* c, int kind) {
  switch (kind) {
    case PT_KIND_PARAM: return c->master;
    case PT_KIND_GRAD: return c->grads;
    case PT_KIND_MOMENT1: return c->mom1;
    case PT_KIND_MOMENT2: return c->mom2;
    default: return nullptr;
  }
}

pt_status pt_write_tensor(pt_ctx* c, int32_t id, int32_t kind, const float* src) {
  if (!c || !src || id < 0 || id >= (int)c->plan.tensors.size()) return PT_EINVAL;
  float* base = kind_base(c, kind);
  if (!base) return fail(c, PT_EINVAL, "tensor kind not writable in this configuration");
  const TensorDesc& t = c->plan.tensors[id];
  if (kind != PT_KIND_PARAM && t.offset < c->plan.state_lo) return fail(c, PT_EINVAL, "the tensor lies below k_min: it has no gradient or optimizer state");
  if (kind == PT_KIND_GRAD) { const pt_status fs = flush_deferred_norms(c); if (fs != PT_OK) return fs; }
  HIP_TRY(c, hipMemcpyAsync(base + t.offset, src, (size_t)t.numel * 4, hipMemcpyHostToDevice, c->st));
  if (kind == PT_KIND_PARAM && c->shadow) f32_to_bf16(c->master + t.offset, c->shadow + t.offset * 2, (size_t)t.numel, c->st);
  HIP_TRY(c, hipStreamSynchronize(c->st));
  return PT_OK;
}

pt_status pt_read_tensor(pt_ctx* c, int32_t id, int32_t kind, float* dst) {
  if (!c || !dst || id < 0 || id >= (int)c->plan.tensors.size()) return PT_EINVAL;
  const TensorDesc& t = c->plan.tensors[id];
  if (kind == PT_KIND_SHADOW) {
    if (!c->shadow) return fail(c, PT_EINVAL, "no bf16 shadow in fp32 mode");
    bf16_to_f32(c->shadow + t.offset * 2, c->wf(c->plan.STAGE), (size_t)t.numel, c->st);
    HIP_TRY(c, hipMemcpyAsync(dst, c->w(c->plan.STAGE), (size_t)t.numel * 4, hipMemcpyDeviceToHost, c->st));
  } else {
    float* base = kind_base(c, kind);
    if (!base) return fail(c, PT_EINVAL, "tensor kind not present in this configuration");
    if (kind != PT_KIND_PARAM && t.offset < c->plan.state_lo) {   // below k_min: no storage, the value is zero by definition
      std::memset(dst, 0, (size_t)t.numel * 4);
      return PT_OK;
    }
    HIP_TRY(c, hipMemcpyAsync(dst, base + t.offset, (size_t)t.numel * 4, hipMemcpyDeviceToHost, c->st));
  }
  HIP_TRY(c, hipStreamSynchronize(c->st));
  return PT_OK;
}

pt_status pt_get_step_count(const pt_ctx* c, int64_t* t) {
  if (!c || !t) return PT_EINVAL;
  *t = c->step;
  return PT_OK;
}
pt_status pt_set_step_count(pt_ctx* c, int64_t t) {
  if (!c || t < 0) return PT_EINVAL;
  c->step = t;
  return PT_OK;
}

pt_status pt_read_activation(pt_ctx* c, int32_t which, float* dst, size_t numel) {
  if (!c || !dst) return PT_EINVAL;
  const pt_config& g = c->cfg;
  const size_t act = (size_t)c->nb * g.S * g.D;
  const void* src = nullptr;
  size_t n = 0;
  bool is_f32 = c->dt == 0;
  switch (which) {
    case PT_ACT_HK: if (c->phase < 1) return fail(c, PT_ESTATE, "no boundary activation yet"); src = c->last_hk; n = act; break;
    case PT_ACT_HL: if (c->phase < 2) return fail(c, PT_ESTATE, "no forward pass yet"); src = c->k == g.L ? c->last_hk : c->w(c->plan.X[g.L]); n = act; break;
    case PT_ACT_LOGITS: if (c->phase < 2) return fail(c, PT_ESTATE, "no forward pass yet"); src = c->w(c->plan.LOGITS);
      n = (g.arch == PT_VIT_PRELN || g.head == PT_HEAD_CLS) ? (size_t)c->nb * g.n_out : (size_t)c->nb * g.S * 2; is_f32 = true; break;
    case PT_ACT_DHK: if (c->phase < 2) return fail(c, PT_ESTATE, "no backward pass yet"); src = c->last_dhk; n = act; is_f32 = true; break;
    default: return fail(c, PT_EINVAL, "unknown activation");
  }
  if (numel != n) return fail(c, PT_EINVAL, "activation size mismatch");
  if (is_f32) {
    HIP_TRY(c, hipMemcpyAsync(dst, src, n * 4, hipMemcpyDeviceToHost, c->st));
  } else {
    bf16_to_f32(src, c->wf(c->plan.STAGE), n, c->st);
    HIP_TRY(c, hipMemcpyAsync(dst, c->w(c->plan.STAGE), n * 4, hipMemcpyDeviceToHost, c->st));
  }
  HIP_TRY(c, hipStreamSynchronize(c->st));
  return PT_OK;
}

pt_status pt_cache_row(pt_ctx* c, int64_t sample_id, void* dst, size_t dst_bytes, int32_t* written_at_k) {
  if (!c || !dst) return PT_EINVAL;
  if (sample_id < 0 || sample_id >= c->cfg.cache_slots + c->cfg.host_slots) return fail(c, PT_EINVAL, "sample id outside the cache");
  const size_t row_bytes = (size_t)c->cfg.S * c->cfg.D * c->esz;
  if (dst_bytes != row_bytes) return fail(c, PT_EINVAL, "row size mismatch");
  if (c->slot_k[(size_t)sample_id] < 0) return PT_ECACHE_MISS;
  if (sample_id >= c->cfg.cache_slots) {
    if (!c->host_rows) return fail(c, PT_ESTATE, "no host tier is attached");
    HIP_TRY(c, hipStreamSynchronize(c->st));
    HIP_TRY(c, hipStreamSynchronize(c->copy_st));
    std::memcpy(dst, host_row(c, sample_id), row_bytes);
    if (written_at_k) *written_at_k = c->slot_k[(size_t)sample_id];
    return PT_OK;
  }
  HIP_TRY(c, hipMemcpyAsync(dst, c->cache + (size_t)sample_id * row_bytes, row_bytes, hipMemcpyDeviceToHost, c->st));
  HIP_TRY(c, hipStreamSynchronize(c->st));
  if (written_at_k) *written_at_k = c->slot_k[(size_t)sample_id];
  return PT_OK;
}

pt_status pt_cache_stats(const pt_ctx* c, int64_t* hits, int64_t* advances, int64_t* misses, int64_t* block_runs) {
  if (!c) return PT_EINVAL;
  if (hits) *hits = c->n_hit;
  if (advances) *advances = c->n_adv;
  if (misses) *misses = c->n_miss;
  if (block_runs) *block_runs = c->n_runs;
  return PT_OK;
}

pt_status pt_profile_enable(pt_ctx* c, int32_t on) {
  if (!c) return PT_EINVAL;
  if (!on) prof_collect(c);
  c->prof_on = on != 0;
  return PT_OK;
}

pt_status pt_profile_reset(pt_ctx* c) {
  if (!c) return PT_EINVAL;
  prof_collect(c);
  for (int i = 0; i < PT_PROF_COUNT; ++i) { c->prof_ms[i] = 0; c->prof_work[i] = 0; c->prof_n[i] = 0; }
  return PT_OK;
}

pt_status pt_profile_read(pt_ctx* c, int32_t category, double* total_ms, int64_t* launches, double* work) {
  if (!c || category < 0 || category >= PT_PROF_COUNT) return PT_EINVAL;
  prof_collect(c);
  if (total_ms) *total_ms = c->prof_ms[category];
  if (launches) *launches = c->prof_n[category];
  if (work) *work = c->prof_work[category];
  return PT_OK;
}
