// C ABI of libbsr_hip (see include/bsr.h): context, workspace plan and the kernel sequence of one
// Block Selective Reprogramming step.  Everything is enqueued on the caller's stream; nothing here
// allocates device memory or waits for the device.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/bsr.h"
#include "bsr_internal.h"

using namespace bsr;

namespace {

thread_local char g_err[512] = "";

struct Schedule {
  int T0 = 0;                       // tokens entering block 0 (CLS included)
  int keep_k[BSR_MAX_BLOCKS] = {};  // per drop
  int Ta[BSR_MAX_BLOCKS] = {};      // tokens seen by MHSA of block l
  int Tm[BSR_MAX_BLOCKS] = {};      // tokens seen by FFN of block l
  int drop_of[BSR_MAX_BLOCKS];      // drop index of block l, or -1
  int fused[BSR_MAX_BLOCKS] = {};   // per drop: 1 when the dropped tokens are fused into one more token
  int T_last = 0;
  int ft = 0;                       // first trainable block: blocks before it are the frozen prefix
  bool trainable[BSR_MAX_BLOCKS] = {};  // block l is trained (others at or after ft: frozen, in the gradient path)
  bool moe[BSR_MAX_BLOCKS] = {};    // block l has a mixture-of-experts FFN
  int moe_row0[BSR_MAX_BLOCKS] = {};// per image: tokens of the mixture blocks before l (routing I/O layout)
  // frozen prefix, bf16: LN1 / LN2 of block l is folded into the qkv / fc1 product behind it (no launch, no
  // normalised copy): that product takes the row statistics itself, the folded weights are built once
  bool fold1[BSR_MAX_BLOCKS] = {}, fold2[BSR_MAX_BLOCKS] = {};
};

struct MoeBuf {      // routing and the expert-ordered tensors of one mixture-of-experts FFN
  float *logits, *gates, *dsel;
  int32_t *experts, *pos, *perm_tok, *off;
  char *xg;          // gathered tokens [M*K, D] (u and g live in the block's u / g)
  float *y;          // expert outputs [M*K, D], fp32: they are rounded once, after the weighted sum
};

struct SavedBlock {  // what a trainable block keeps for its backward pass (Sec. 3.2 of the paper)
  float *mean1, *rstd1, *mean2, *rstd2, *lse;
  char *h1, *qkv, *o, *xmid_full, *xmid, *h2, *u, *g, *xout;
  int32_t* idx;
  float* fw;         // [B, Ta-1] weights of the fused token (drop locations with fusion)
  MoeBuf moe;        // used when the block's FFN is a mixture of experts (u, g then have K rows per token)
};

struct Shadow {  // bf16 copies of a block's matrices: transposed [out,in] and, if trained, straight [in,out]
  bf16 *t_qkv, *t_proj, *t_fc1, *t_fc2;     // (a mixture-of-experts block: E matrices each, expert-major)
  bf16 *s_qkv, *s_proj, *s_fc1, *s_fc2;
  bf16 *t_router;                           // [E,D], mixture-of-experts blocks only
  // folded LayerNorm (then t_qkv / t_fc1 hold W diag(gamma)): column sums of that matrix, b + W beta
  float *cs_qkv, *fb_qkv, *cs_fc1, *fb_fc1;
};

struct Buffers {
  bf16* t_patch = nullptr;
  Shadow sh[BSR_MAX_BLOCKS] = {};
  char *patches = nullptr, *x0 = nullptr, *x1 = nullptr, *h = nullptr, *qkv = nullptr, *o = nullptr, *g = nullptr;
  float *clsp = nullptr, *scores = nullptr, *fw = nullptr;   // fw: fusion weights of a frozen drop location
  // Scratch of the trainable part that is not kept for backward.  It has buffers of its own because the
  // frozen prefix of the next batch may run beside it on another stream.
  float *clsp_t = nullptr, *scores_t = nullptr;
  char *h_t = nullptr, *o_t = nullptr, *g_t = nullptr;
  int32_t* idx_tmp = nullptr;
  SavedBlock sv[BSR_MAX_BLOCKS] = {};
  MoeBuf moe = {};                      // frozen mixture blocks share this one
  char *moe_u = nullptr;                // their GELU outputs [M*K, F]
  char *moe_dy = nullptr, *moe_dxg = nullptr;   // backward scratch
  float* moe_rw_partial = nullptr;              // chunk sums of the router weight gradient
  char *dxa = nullptr, *dxb = nullptr, *dgu = nullptr, *dh = nullptr, *dqkv = nullptr;
  float *delta = nullptr, *partial = nullptr, *splitk = nullptr;
  float *ln_partial = nullptr;          // one slot per LayerNorm of the trained blocks (deferred dgamma / dbeta sums)
  size_t splitk_floats = 0;
  float *xc = nullptr, *z = nullptr, *dz = nullptr, *dxc = nullptr, *meanf = nullptr, *rstdf = nullptr;
  float *logits = nullptr, *dlogits = nullptr, *loss_rows = nullptr;
};

}  // namespace

struct ProfRec {
  hipEvent_t start, stop;
  int cls;
  double flops;
};

// Tile choice per NT GEMM launch, measured on the context's own launches (bsr_autotune).  A launch is
// identified by the entry point it belongs to and its position in that call's launch order.
struct TunePick { int M, N, K, tile; float us; };   // us: the chosen shape's measured time (0: not measured)
struct TuneRec { int kind, cand; size_t site; int M, N, K; hipEvent_t start, stop; };
struct Tune {
  int batch = 0;                       // the picks hold for this batch size (0: none)
  std::vector<TunePick> pick[2];       // [0] bsr_forward_frozen, [1] bsr_train_blocks_fwd_bwd
  int kind = 0;                        // entry point running now
  size_t site = 0;                     // NT launches it has issued so far
  int cur_batch = 0;
  int cand = -1;                       // >= 0 while tuning: index of the shape every launch is forced to
  int cand_train = -1;                 // >= 0: the trainable part is forced to this shape instead (two-stream tuning)
  std::vector<TuneRec> recs;
};

struct bsr_ctx {
  Tune tune;
  TnChain tn_chain;            // split-K reduction of the latest weight gradient, folded into the next one's launch
  std::vector<ProfRec> prof;   // event pairs of the profiling mode (bsr_profile_begin / _end)
  // bsr_pipeline_step: per x buffer, "the frozen prefix has filled it" and "the trainable part has read it"
  struct PipeSlot { const void* x; hipEvent_t ready, free; bool has_ready, has_free; };
  std::vector<PipeSlot> pipe;
  size_t prof_used = 0;
  bool prof_on = false;
  bsr_config cfg;
  bsr_params p;
  Schedule sc;
  Buffers b;
  bool f32;
  size_t esz;
  float eps;
  char* ws;
  size_t ws_bytes;
  int deferred = BSR_OK;                     // an error met by a helper that cannot return it (see defer_fail)
  const int32_t* forced_experts = nullptr;   // bsr_moe_routing_io
  int32_t* experts_out = nullptr;
  float* router_logits_out = nullptr;
  char err[512];
};

namespace {

int fail(bsr_ctx* c, int code, const char* fmt, ...) {
  char* dst = c ? c->err : g_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 512, fmt, ap);
  va_end(ap);
  if (c) snprintf(g_err, sizeof(g_err), "%s", dst);
  return code;
}

bool aligned16(const void* p) { return p && (((uintptr_t)p) & 15) == 0; }

// An error found inside a launch helper that returns nothing (a product that no kernel takes): the launch is
// skipped, the text is kept, and the entry point that is running returns the code from check_hip instead of
// BSR_OK (what it enqueued after the skipped launch read a tensor nobody wrote).
void defer_fail(bsr_ctx* c, int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(c->err, sizeof(c->err), fmt, ap);
  va_end(ap);
  snprintf(g_err, sizeof(g_err), "%s", c->err);
  if (c->deferred == BSR_OK) c->deferred = code;
}

int check_hip(bsr_ctx* c, const char* where) {
  hipError_t e = hipGetLastError();
  if (c && c->deferred != BSR_OK) {
    const int code = c->deferred;
    c->deferred = BSR_OK;
    return code;                     // (the text is already in place)
  }
  if (e != hipSuccess) return fail(c, BSR_ERR_HIP, "%s: %s", where, hipGetErrorString(e));
  return BSR_OK;
}

// Validates the configuration and derives the token schedule: K = floor(keep_ratio * n + 1e-9)
// on the current patch count when keep_k is not given (Sec. 4.1, Sec. 4.3 Discussion 3).
int make_schedule(const bsr_config* c, Schedule* s, char* why, size_t whyn) {
#define BAD(...) do { snprintf(why, whyn, __VA_ARGS__); return BSR_ERR_BAD_CONFIG; } while (0)
  if (c->dim <= 0 || c->heads <= 0 || c->dim % c->heads) BAD("dim %d must be a positive multiple of heads %d", c->dim, c->heads);
  if (c->dim % 8) BAD("dim %d must be a multiple of 8", c->dim);
  if (c->dim / c->heads > 256) BAD("head size %d exceeds 256", c->dim / c->heads);
  if (c->mlp_hidden <= 0 || c->mlp_hidden % 8) BAD("mlp_hidden %d must be a positive multiple of 8", c->mlp_hidden);
  if (c->depth <= 0 || c->depth > BSR_MAX_BLOCKS) BAD("depth %d out of range 1..%d", c->depth, BSR_MAX_BLOCKS);
  if (c->max_batch <= 0) BAD("max_batch %d must be positive", c->max_batch);
  if (c->first_trainable_block < 0 || c->first_trainable_block > c->depth) BAD("first_trainable_block %d out of range", c->first_trainable_block);
  if (c->dtype != BSR_BF16 && c->dtype != BSR_FP32) BAD("unknown dtype %d", c->dtype);
  if (c->loss != BSR_LOSS_CE && c->loss != BSR_LOSS_MEAN_SQ) BAD("unknown loss %d", c->loss);
  if (c->loss == BSR_LOSS_CE && c->num_classes <= 0) BAD("cross-entropy needs num_classes > 0");
  if (c->loss == BSR_LOSS_MEAN_SQ && c->num_classes != 0) BAD("mean-square loss is defined for num_classes == 0");
  if (c->num_classes < 0) BAD("num_classes %d is negative", c->num_classes);
  if (c->image_size > 0) {
    if (c->patch_size <= 0 || c->in_chans <= 0 || c->image_size % c->patch_size) BAD("image %d / patch %d / channels %d inconsistent", c->image_size, c->patch_size, c->in_chans);
    if ((c->in_chans * c->patch_size * c->patch_size) % 8) BAD("patch vector length must be a multiple of 8");
    int g = c->image_size / c->patch_size;
    s->T0 = g * g + 1;
  } else if (c->image_size == 0) {
    if (c->tokens_in < 1) BAD("tokens_in %d must be >= 1 when image_size == 0", c->tokens_in);
    s->T0 = c->tokens_in;
  } else {
    BAD("image_size %d is negative", c->image_size);
  }
  if (s->T0 > 1024) BAD("%d tokens exceed the limit of 1024", s->T0);
  if (c->n_drop < 0 || c->n_drop > BSR_MAX_BLOCKS) BAD("n_drop %d out of range", c->n_drop);
  bool given = false;
  for (int i = 0; i < c->n_drop; ++i) given |= c->keep_k[i] != 0;
  if (!given && c->n_drop > 0 && !(c->keep_ratio > 0.f && c->keep_ratio <= 1.f)) BAD("keep_ratio %g must lie in (0, 1]", (double)c->keep_ratio);
  for (int l = 0; l < BSR_MAX_BLOCKS; ++l) s->drop_of[l] = -1;
  int n = s->T0 - 1;
  for (int i = 0; i < c->n_drop; ++i) {
    int blk = c->drop_blocks[i];
    if (blk < 0 || blk >= c->depth) BAD("drop_blocks[%d] = %d out of range", i, blk);
    if (i && blk <= c->drop_blocks[i - 1]) BAD("drop_blocks must be strictly ascending");
    int k = given ? c->keep_k[i] : (int)floor((double)c->keep_ratio * (double)n + 1e-9);
    if (k < 0 || k > n) BAD("keep_k[%d] = %d must lie in 0..%d", i, k, n);
    s->keep_k[i] = k;
    s->drop_of[blk] = i;
    s->fused[i] = (c->fuse_dropped && n - k > 0) ? 1 : 0;
    n = k + s->fused[i];        // the fused token is a patch token of the following blocks
  }
  int T = s->T0;
  for (int l = 0; l < c->depth; ++l) {
    s->Ta[l] = T;
    if (s->drop_of[l] >= 0) T = s->keep_k[s->drop_of[l]] + 1 + s->fused[s->drop_of[l]];
    s->Tm[l] = T;
  }
  s->T_last = T;
  if (c->n_trainable < 0 || c->n_trainable > BSR_MAX_BLOCKS) BAD("n_trainable %d out of range", c->n_trainable);
  if (c->n_trainable == 0) {
    s->ft = c->first_trainable_block;
    for (int l = s->ft; l < c->depth; ++l) s->trainable[l] = true;
  } else {
    for (int i = 0; i < c->n_trainable; ++i) {
      const int blk = c->trainable_blocks[i];
      if (blk < 0 || blk >= c->depth) BAD("trainable_blocks[%d] = %d out of range", i, blk);
      if (i && blk <= c->trainable_blocks[i - 1]) BAD("trainable_blocks must be strictly ascending");
      s->trainable[blk] = true;
    }
    s->ft = c->trainable_blocks[0];
  }
  if (c->n_moe < 0 || c->n_moe > BSR_MAX_BLOCKS) BAD("n_moe %d out of range", c->n_moe);
  if (c->n_moe > 0) {
    if (c->dtype != BSR_BF16) BAD("mixture-of-experts blocks need dtype bf16");
    if (c->n_experts < 1 || c->n_experts > MOE_MAX_EXPERTS) BAD("n_experts %d must lie in 1..%d", c->n_experts, MOE_MAX_EXPERTS);
    if (c->moe_top_k < 1 || c->moe_top_k > MOE_MAX_TOPK || c->moe_top_k > c->n_experts)
      BAD("moe_top_k %d must lie in 1..min(%d, n_experts)", c->moe_top_k, MOE_MAX_TOPK);
    for (int i = 0; i < c->n_moe; ++i) {
      const int blk = c->moe_blocks[i];
      if (blk < 0 || blk >= c->depth) BAD("moe_blocks[%d] = %d out of range", i, blk);
      if (i && blk <= c->moe_blocks[i - 1]) BAD("moe_blocks must be strictly ascending");
      s->moe[blk] = true;
    }
    int rows = 0;
    for (int l = 0; l < c->depth; ++l) {
      s->moe_row0[l] = rows;
      if (s->moe[l]) rows += s->Tm[l];
    }
  }
  // A LayerNorm of the frozen prefix can be folded when its output goes into a dense product only (after a
  // token drop the LayerNorm kernel also does the gather; a mixture block routes on the normalised tokens).
  // The fold trades launches (a fixed cost) for 8 - 15 % more time in the products that carry it, which run in
  // the register-staged kernel: it is the caller's choice (measured on ViT-B/16: 1.5 % faster step at 6304
  // token rows before the direct-to-LDS products existed, 1 % slower with them; 2.8 % slower at 25216 rows).
  if (c->fold_frozen_layernorm != 0 && c->fold_frozen_layernorm != 1) BAD("fold_frozen_layernorm must be 0 or 1");
  if (c->fold_frozen_layernorm && c->dtype != BSR_BF16) BAD("fold_frozen_layernorm needs dtype bf16");
  if (c->fold_frozen_layernorm && c->dim % 64 == 0)
    for (int l = 0; l < s->ft && l < c->depth; ++l) {
      s->fold1[l] = true;
      s->fold2[l] = s->drop_of[l] < 0 && !s->moe[l];
    }
  return BSR_OK;
#undef BAD
}

struct Carver {
  char* base;
  size_t off = 0;
  template <typename T>
  T* take(size_t count, uint64_t* tally = nullptr) {   // tally: unpadded bytes, for the saved-activation report
    if (tally) *tally += count * sizeof(T);
    size_t bytes = (count * sizeof(T) + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += bytes;
    return p;
  }
};

// One function lays out the workspace; with base == nullptr it only measures.
size_t carve(const bsr_config& c, const Schedule& s, char* base, Buffers* out, bsr_saved_bytes* saved = nullptr) {
  Carver w{base};
  Buffers b;
  const bool f32 = c.dtype == BSR_FP32;
  const size_t E = f32 ? 4 : 2;
  const size_t B = c.max_batch, D = c.dim, F = c.mlp_hidden, H = c.heads, T0 = s.T0;
  const int ft = s.ft, L = c.depth;
  const size_t Kp = (size_t)c.in_chans * c.patch_size * c.patch_size;
  if (!f32) {
    if (c.image_size) b.t_patch = w.take<bf16>(D * Kp);
    for (int l = 0; l < L; ++l) {
      const size_t ne = s.moe[l] ? (size_t)c.n_experts : 1;    // FFN matrices per block
      b.sh[l].t_qkv = w.take<bf16>(3 * D * D);
      b.sh[l].t_proj = w.take<bf16>(D * D);
      b.sh[l].t_fc1 = w.take<bf16>(ne * D * F);
      b.sh[l].t_fc2 = w.take<bf16>(ne * D * F);
      if (s.moe[l]) b.sh[l].t_router = w.take<bf16>((size_t)c.n_experts * D);
      if (s.fold1[l]) { b.sh[l].cs_qkv = w.take<float>(3 * D); b.sh[l].fb_qkv = w.take<float>(3 * D); }
      if (s.fold2[l]) { b.sh[l].cs_fc1 = w.take<float>(F); b.sh[l].fb_fc1 = w.take<float>(F); }
      if (l >= ft) {
        b.sh[l].s_qkv = w.take<bf16>(3 * D * D);
        b.sh[l].s_proj = w.take<bf16>(D * D);
        b.sh[l].s_fc1 = w.take<bf16>(ne * D * F);
        b.sh[l].s_fc2 = w.take<bf16>(ne * D * F);
      }
    }
  }
  if (c.image_size) b.patches = w.take<char>(B * (T0 - 1) * Kp * E);
  b.x0 = w.take<char>(B * T0 * D * E);
  b.x1 = w.take<char>(B * T0 * D * E);
  b.h = w.take<char>(B * T0 * D * E);
  b.qkv = w.take<char>(B * T0 * 3 * D * E);
  b.o = w.take<char>(B * T0 * D * E);
  b.g = w.take<char>(B * T0 * F * E);
  b.clsp = w.take<float>(B * H * T0);
  b.scores = w.take<float>(B * T0);
  b.clsp_t = w.take<float>(B * H * T0);
  b.scores_t = w.take<float>(B * T0);
  b.fw = w.take<float>(B * T0);
  b.idx_tmp = w.take<int32_t>(B * T0);
  const size_t KE = c.n_moe > 0 ? (size_t)c.moe_top_k : 1, NE = c.n_moe > 0 ? (size_t)c.n_experts : 0;
  auto take_moe = [&](MoeBuf& m, size_t rows, uint64_t* t = nullptr) {      // rows = tokens of the FFN
    m.logits = w.take<float>(rows * NE, t);
    m.gates = w.take<float>(rows * KE, t);
    m.dsel = w.take<float>(rows * KE, t);
    m.experts = w.take<int32_t>(rows * KE, t);
    m.pos = w.take<int32_t>(rows * KE, t);
    m.perm_tok = w.take<int32_t>(rows * KE, t);
    m.off = w.take<int32_t>(NE + 1, t);
    m.xg = w.take<char>(rows * KE * D * E, t);
    m.y = w.take<float>(rows * KE * D, t);
  };
  bool frozen_moe = false;
  for (int l = 0; l < ft && l < L; ++l) frozen_moe |= s.moe[l];
  if (frozen_moe) {
    take_moe(b.moe, B * T0);
    b.moe_u = w.take<char>(B * T0 * KE * F * E);
  }
  size_t Tmax = s.T_last;
  bool any_drop = false, any_dgrad_only = false;
  for (int l = ft; l < L; ++l) {
    any_drop |= s.drop_of[l] >= 0;
    any_dgrad_only |= !(s.trainable[l] || s.moe[l]);
  }
  if (any_drop) b.o_t = w.take<char>(B * T0 * D * E);
  if (any_dgrad_only) {
    b.h_t = w.take<char>(B * T0 * D * E);
    b.g_t = w.take<char>(B * T0 * F * E);
  }
  for (int l = ft; l < L; ++l) {
    const size_t Ta = s.Ta[l], Tm = s.Tm[l];
    Tmax = std::max(Tmax, Ta);
    SavedBlock& v = b.sv[l];
    bsr_saved_bytes none = {};
    bsr_saved_bytes& r = saved ? saved[l] : none;
    v.mean1 = w.take<float>(B * Ta, &r.stats);
    v.rstd1 = w.take<float>(B * Ta, &r.stats);
    v.mean2 = w.take<float>(B * Tm, &r.stats);
    v.rstd2 = w.take<float>(B * Tm, &r.stats);
    v.lse = w.take<float>(B * H * Ta, &r.softmax);
    const bool keep_lin = s.trainable[l] || s.moe[l];   // inputs of the linear layers: only Eq. 4 needs them
    v.h1 = keep_lin ? w.take<char>(B * Ta * D * E, &r.linear_in) : b.h_t;
    v.qkv = w.take<char>(B * Ta * 3 * D * E, &r.qkv);
    v.o = w.take<char>(B * Ta * D * E, &r.attn_out);
    // x after MHSA: at a drop location only its gathered rows are read again, the full tensor is scratch
    const bool drop = s.drop_of[l] >= 0;
    v.xmid_full = drop ? b.o_t : w.take<char>(B * Ta * D * E, &r.residual);
    v.xmid = drop ? w.take<char>(B * Tm * D * E, &r.residual) : v.xmid_full;
    v.h2 = keep_lin ? w.take<char>(B * Tm * D * E, &r.linear_in) : b.h_t;
    const size_t kf = s.moe[l] ? KE : 1;               // a mixture block keeps u and g per (token, slot)
    v.u = w.take<char>(B * Tm * kf * F * E, &r.gelu_in);
    v.g = keep_lin ? w.take<char>(B * Tm * kf * F * E, &r.linear_in) : b.g_t;
    if (s.moe[l]) take_moe(v.moe, B * Tm, &r.moe);
    v.xout = w.take<char>(B * Tm * D * E, &r.residual);
    v.idx = w.take<int32_t>(drop ? B * Tm : 0, &r.stats);
    v.fw = (drop && s.fused[s.drop_of[l]]) ? w.take<float>(B * Ta, &r.stats) : nullptr;
    r.total = r.qkv + r.softmax + r.attn_out + r.gelu_in + r.linear_in + r.residual + r.stats + r.moe;
  }
  b.dxa = w.take<char>(B * Tmax * D * E);
  b.dxb = w.take<char>(B * Tmax * D * E);
  bool train_moe = false;
  for (int l = ft; l < L; ++l) train_moe |= s.moe[l];
  b.dgu = w.take<char>(B * Tmax * (train_moe ? KE : 1) * F * E);
  if (train_moe) {
    b.moe_dy = w.take<char>(B * Tmax * KE * D * E);
    b.moe_dxg = w.take<char>(B * Tmax * KE * D * E);
    b.moe_rw_partial = w.take<float>(moe_router_wgrad_partial_floats((int)D, (int)NE));
  }
  b.dh = w.take<char>(B * Tmax * D * E);
  b.dqkv = w.take<char>(B * Tmax * 3 * D * E);
  b.delta = w.take<float>(B * H * Tmax);
  b.partial = w.take<float>(std::max(colsum_partial_floats(0, (int)std::max(3 * D, F)), mean_sq_partial_floats()));
  int n_ln = 0;
  for (int l = ft; l < L; ++l) n_ln += s.trainable[l] ? 2 : 0;
  if (!f32 && n_ln > 0 && n_ln <= LN_DEFER_MAX) b.ln_partial = w.take<float>((size_t)n_ln * ln_deferred_partial_floats((int)D));
  b.splitk_floats = f32 ? 0 : gemm_splitk_ws_floats((int)D, (int)F);
  if (ft < L && b.splitk_floats) b.splitk = w.take<float>(b.splitk_floats);
  const size_t C = std::max(c.num_classes, 1);
  b.xc = w.take<float>(B * D);
  b.z = w.take<float>(B * D);
  b.dz = w.take<float>(B * D);
  b.dxc = w.take<float>(B * D);
  b.meanf = w.take<float>(B);
  b.rstdf = w.take<float>(B);
  b.logits = w.take<float>(B * C);
  b.dlogits = w.take<float>(B * C);
  b.loss_rows = w.take<float>(B);
  if (out) *out = b;
  return w.off;
}

// ---- GEMM descriptions of the three uses of a linear layer ------------------------------------

// y[M,out] = x[M,in] . W        (forward; W from the fp32 master [in,out] or the bf16 copy [out,in])
GemmDesc fwd_desc(const bsr_ctx* c, const void* x, int M, int in, int out, const void* w_master,
                  const bf16* w_t, void* y) {
  GemmDesc g;
  g.A = x; g.a_rs = in; g.a_cs = 1;
  if (c->f32) { g.B = w_master; g.b_rs = out; g.b_cs = 1; }
  else        { g.B = w_t;      g.b_rs = 1;   g.b_cs = in; }
  g.C = y; g.ldc = out; g.M = M; g.N = out; g.K = in;
  g.in_f32 = c->f32; g.out_f32 = c->f32;
  return g;
}

// dx[M,in] = dy[M,out] . W^T    (Eq. 2 of the paper)
GemmDesc dgrad_desc(const bsr_ctx* c, const void* dy, int M, int in, int out, const void* w_master,
                    const bf16* w_s, void* dx) {
  GemmDesc g;
  g.A = dy; g.a_rs = out; g.a_cs = 1;
  g.B = c->f32 ? w_master : (const void*)w_s; g.b_rs = 1; g.b_cs = out;   // B(k=o, n=i) = W[i*out + o]
  g.C = dx; g.ldc = in; g.M = M; g.N = in; g.K = out;
  g.in_f32 = c->f32; g.out_f32 = c->f32;
  return g;
}

// dW[in,out] = x^T . dy  (Eq. 4), fp32 result summed over all M tokens
GemmDesc wgrad_desc(const bsr_ctx* c, const void* x, const void* dy, int M, int in, int out, void* dw) {
  GemmDesc g;
  g.A = x;  g.a_rs = 1;   g.a_cs = in;    // A(m=i, k=token)
  g.B = dy; g.b_rs = out; g.b_cs = 1;     // B(k=token, n=o)
  g.C = dw; g.ldc = out; g.M = in; g.N = out; g.K = M;
  g.in_f32 = c->f32; g.out_f32 = true;
  return g;
}

// Profiling mode: an event pair around one launch (or a short launch group) of a kernel class.
struct ProfScope {
  bsr_ctx* c;
  hipStream_t s;
  ProfRec* r = nullptr;
  ProfScope(bsr_ctx* c_, int cls, double flops, hipStream_t s_) : c(c_), s(s_) {
    if (!c->prof_on) return;
    if (c->prof_used == c->prof.size()) {
      ProfRec n{};
      if (hipEventCreate(&n.start) != hipSuccess || hipEventCreate(&n.stop) != hipSuccess) return;
      c->prof.push_back(n);
    }
    r = &c->prof[c->prof_used++];
    r->cls = cls;
    r->flops = flops;
    (void)hipEventRecord(r->start, s);
  }
  ~ProfScope() {
    if (r) (void)hipEventRecord(r->stop, s);
  }
};

// Tile shape for the NT launch at this position of the running call: the shape under test while tuning
// (the launch is then bracketed by events), the measured choice for this batch size, or 0 (cost model).
struct TileChoice {
  int tile = 0;
  bool timing = false;
  TuneRec rec{};
};
TileChoice choose_tile(bsr_ctx* c, const GemmDesc& g, hipStream_t s) {
  TileChoice ch;
  if (!gemm_nt_tile_is_free(g)) return ch;
  Tune& t = c->tune;
  const size_t site = t.site++;
  if (t.cand >= 0) {
    const int cand = (t.kind == 1 && t.cand_train >= 0) ? t.cand_train : t.cand;
    ch.tile = gemm_nt_tile_id(cand);
    ch.rec = TuneRec{t.kind, cand, site, g.M, g.N, g.K, nullptr, nullptr};
    ch.timing = hipEventCreate(&ch.rec.start) == hipSuccess && hipEventCreate(&ch.rec.stop) == hipSuccess;
    if (ch.timing) (void)hipEventRecord(ch.rec.start, s);
  } else if (t.batch == t.cur_batch && site < t.pick[t.kind].size()) {
    const TunePick& p = t.pick[t.kind][site];
    if (p.M == g.M && p.N == g.N && p.K == g.K) ch.tile = p.tile;
  }
  return ch;
}
void tile_done(bsr_ctx* c, TileChoice& ch, hipStream_t s) {
  if (!ch.timing) return;
  (void)hipEventRecord(ch.rec.stop, s);
  c->tune.recs.push_back(ch.rec);
}

void gemm(bsr_ctx* c, const GemmDesc& g, hipStream_t s) {
  if (g.ln_colsum && (g.K % 64 || g.grp_off || !gemm_mfma_supported(g))) {
    defer_fail(c, BSR_ERR_BAD_CONFIG, "folded LayerNorm on a product of %d x %d x %d that cannot carry it", g.M, g.N, g.K);
    return;
  }
  ProfScope ps(c, BSR_PROF_GEMM, 2.0 * g.M * g.N * g.K, s);
  if (gemm_mfma_supported(g)) {
    TileChoice ch = choose_tile(c, g, s);
    gemm_mfma(g, c->b.splitk, c->b.splitk_floats, s, ch.tile, &c->tn_chain);
    tile_done(c, ch, s);
  }
  else if (g.grp_off) defer_fail(c, BSR_ERR_BAD_CONFIG, "grouped GEMM %d x %d x %d is not an MFMA shape", g.M, g.N, g.K);
  else gemm_generic(g, s);
}

// Eq. 4 for one linear layer: dW = x^T dy and db = column sums of dy.  The MFMA kernel produces db
// alongside dW; other shapes (and fp32 mode) take the separate column-sum kernels.
void wgrad(bsr_ctx* c, const void* x, const void* dy, int M, int in, int out, void* dw, void* db, hipStream_t s) {
  GemmDesc g = wgrad_desc(c, x, dy, M, in, out, dw);
  if (gemm_mfma_supported(g)) {
    g.bsum = (float*)db;
    gemm(c, g, s);
  } else {
    gemm(c, g, s);
    colsum(dy, M, out, out, c->f32, c->b.partial, (float*)db, s);
  }
}

// Input gradient (Eq. 2, described by dg) and weight gradient (Eq. 4) of one linear layer: both read dy and
// neither reads what the other writes, so on the MFMA path they go out together (one launch when the tile
// shape of the input gradient allows it).
void dgrad_wgrad(bsr_ctx* c, const GemmDesc& dg, const void* x, const void* dy, int M, int in, int out, void* dw, void* db,
                 hipStream_t s) {
  GemmDesc wg = wgrad_desc(c, x, dy, M, in, out, dw);
  if (!(gemm_nt_tile_is_free(dg) && gemm_mfma_supported(wg)) || wg.grp_off) {
    gemm(c, dg, s);
    wgrad(c, x, dy, M, in, out, dw, db, s);
    return;
  }
  wg.bsum = (float*)db;
  ProfScope ps(c, BSR_PROF_GEMM, 2.0 * dg.M * dg.N * dg.K + 2.0 * wg.M * wg.N * wg.K, s);
  TileChoice ch = choose_tile(c, dg, s);
  gemm_mfma_pair(dg, wg, c->b.splitk, c->b.splitk_floats, s, ch.tile, &c->tn_chain);
  tile_done(c, ch, s);
}

// Mixture-of-experts FFN of block l on M2 tokens (Sec. 5.3):  x_out = x_res + sum_s gate_s FFN_{e_s}(h),
// h = LN2(x_res).  Routing, stable sort of the (token, slot) pairs by expert, gather, two grouped
// GEMMs over the expert ranges (fc1 + GELU, fc2), weighted un-permute.  u (pre-GELU, may be null)
// and g are [M2*K, F] in expert order.
void moe_ffn_forward(bsr_ctx* c, int l, int B, const void* h, const void* x_res, int M2, MoeBuf& m, void* u,
                     void* gbuf, void* x_out, hipStream_t s) {
  const bsr_config& cf = c->cfg;
  const int D = cf.dim, F = cf.mlp_hidden, E = cf.n_experts, K = cf.moe_top_k;
  const bsr_block_params& w = c->p.blocks[l];
  const Shadow& sh = c->b.sh[l];
  const size_t row0 = (size_t)B * c->sc.moe_row0[l];       // rows of the earlier mixture blocks in the routing I/O
  GemmDesc gl = fwd_desc(c, h, M2, D, E, nullptr, sh.t_router, m.logits);       // router logits, fp32
  gl.out_f32 = true;
  gemm(c, gl, s);
  moe_topk(m.logits, M2, E, K, c->forced_experts ? c->forced_experts + row0 * K : nullptr, m.experts, m.gates, s);
  if (c->experts_out)
    (void)hipMemcpyAsync(c->experts_out + row0 * K, m.experts, sizeof(int32_t) * (size_t)M2 * K, hipMemcpyDeviceToDevice, s);
  if (c->router_logits_out)
    (void)hipMemcpyAsync(c->router_logits_out + row0 * E, m.logits, sizeof(float) * (size_t)M2 * E, hipMemcpyDeviceToDevice, s);
  moe_sort(m.experts, M2, E, K, m.off, m.pos, m.perm_tok, s);
  moe_gather_rows(h, m.perm_tok, (int64_t)M2 * K, D, m.xg, s);
  GemmDesc g1 = fwd_desc(c, m.xg, M2 * K, D, F, nullptr, sh.t_fc1, gbuf);
  g1.bias = (const float*)w.b_fc1; g1.act = ACT_GELU; g1.aux = u;
  g1.grp_off = m.off; g1.groups = E; g1.b_gs = (int64_t)D * F; g1.bias_gs = F;
  gemm(c, g1, s);
  GemmDesc g2 = fwd_desc(c, gbuf, M2 * K, F, D, nullptr, sh.t_fc2, m.y);
  g2.bias = (const float*)w.b_fc2;
  g2.out_f32 = true;
  g2.grp_off = m.off; g2.groups = E; g2.b_gs = (int64_t)D * F; g2.bias_gs = D;
  gemm(c, g2, s);
  moe_combine(m.y, m.pos, m.gates, x_res, M2, D, K, x_out, s);
}

// Backward of moe_ffn_forward for a trainable block: dx is the gradient at the block output [M2, D];
// dh receives the gradient at h = LN2(x_mid).  The expert choice is a constant; the gates are
// differentiated through the softmax over the selected logits.  Expert weights get Eq. 4 over the
// rows routed to them (grouped wgrad), the router gets dW_r = h^T dlogits.
void moe_ffn_backward(bsr_ctx* c, int l, const void* dx, int M2, SavedBlock& v, const bsr_block_params& gw, void* dh,
                      bool train, hipStream_t s) {
  const bsr_config& cf = c->cfg;
  Buffers& b = c->b;
  const int D = cf.dim, F = cf.mlp_hidden, E = cf.n_experts, K = cf.moe_top_k;
  const bsr_block_params& w = c->p.blocks[l];
  const Shadow& sh = b.sh[l];
  MoeBuf& m = v.moe;
  const int R = M2 * K;
  moe_combine_bwd(dx, m.y, m.pos, m.experts, m.gates, M2, D, E, K, b.moe_dy, m.dsel, s);
  GemmDesc d1 = dgrad_desc(c, b.moe_dy, R, F, D, nullptr, sh.s_fc2, b.dgu);      // du = (dy W2^T) * GELU'(u)
  d1.act = ACT_GELU_BWD; d1.aux = v.u;
  d1.grp_off = m.off; d1.groups = E; d1.b_gs = (int64_t)D * F;
  gemm(c, d1, s);
  if (train) {
    GemmDesc w2 = wgrad_desc(c, v.g, b.moe_dy, R, F, D, gw.w_fc2);
    w2.bsum = (float*)gw.b_fc2;
    w2.grp_off = m.off; w2.groups = E; w2.c_gs = (int64_t)F * D; w2.bsum_gs = D;
    gemm(c, w2, s);
  }
  GemmDesc d2 = dgrad_desc(c, b.dgu, R, D, F, nullptr, sh.s_fc1, b.moe_dxg);     // gradient at the gathered tokens
  d2.grp_off = m.off; d2.groups = E; d2.b_gs = (int64_t)D * F;
  gemm(c, d2, s);
  if (train) {
    GemmDesc w1 = wgrad_desc(c, m.xg, b.dgu, R, D, F, gw.w_fc1);
    w1.bsum = (float*)gw.b_fc1;
    w1.grp_off = m.off; w1.groups = E; w1.c_gs = (int64_t)D * F; w1.bsum_gs = F;
    gemm(c, w1, s);
  }
  moe_unpermute_bwd(b.moe_dxg, m.pos, m.experts, m.dsel, (const float*)w.w_router, M2, D, E, K, dh, s);
  if (train)   // dW_r = h^T dlogits, the logit gradients in fp32
    moe_router_wgrad(v.h2, m.experts, m.dsel, M2, D, E, K, b.moe_rw_partial, (float*)gw.w_router, s);
}

void attention_fwd(bsr_ctx* c, const void* qkv, int B, int T, void* out, float* lse, float* clsp,
                   hipStream_t s) {
  const int H = c->cfg.heads, d = c->cfg.dim / H;
  ProfScope ps(c, BSR_PROF_ATTN_FWD, 4.0 * B * H * (double)T * T * d, s);
  if (!c->f32 && attn_mfma_supported(T, d)) attn_fwd_mfma(qkv, B, T, H, out, lse, clsp, s);
  else attn_fwd_generic(qkv, B, T, H, d, c->f32, out, lse, clsp, s);
}

void attention_bwd(bsr_ctx* c, const void* qkv, const void* out, const void* dout, const float* lse,
                   int B, int T, void* dqkv, hipStream_t s) {
  const int H = c->cfg.heads, d = c->cfg.dim / H;
  ProfScope ps(c, BSR_PROF_ATTN_BWD, 10.0 * B * H * (double)T * T * d, s);
  if (!c->f32 && attn_mfma_supported(T, d)) attn_bwd_mfma(qkv, out, dout, lse, B, T, H, c->b.delta, dqkv, s);
  else attn_bwd_generic(qkv, out, dout, lse, B, T, H, d, c->f32, c->b.delta, dqkv, s);
}

// Rank the patch tokens of a drop location and hand CLS + the K best to the FFN (Sec. 4.1).
// Returns the device pointer holding the kept indices.
// fw != null: the dropped tokens are fused into one more token (row k+1 of x_kept, pitch k+2) and
// fw receives the fusion weights.
// LayerNorm that follows the token drop (LN2 of the drop location): when given, and when the one-pass kernel
// takes the shape, gather and LayerNorm are one launch and done is set.
struct LnAfterDrop {
  const float *gamma, *beta;
  void* y;
  float *mean, *rstd;
  bool done;
};

const int32_t* drop_tokens(bsr_ctx* c, int B, int T, int k, const void* x_full, void* x_kept,
                           int32_t* idx_own, const int32_t* forced, int32_t* idx_out, float* scores_out,
                           float* fw, hipStream_t s, LnAfterDrop* ln = nullptr, bool trainable_part = false) {
  const int H = c->cfg.heads, D = c->cfg.dim;
  const float* clsp = trainable_part ? c->b.clsp_t : c->b.clsp;
  float* scores = scores_out ? scores_out : (trainable_part ? c->b.scores_t : c->b.scores);
  const int32_t* idx = forced;
  if (!forced) {
    topk_select_from_cls(clsp, B, H, T, k, scores, idx_own, s);
    idx = idx_own;
  } else if (scores_out || fw) {
    cls_head_mean(clsp, B, H, T, scores, s);
  }
  if (idx_out && k > 0)
    (void)hipMemcpyAsync(idx_out, idx, sizeof(int32_t) * (size_t)B * k, hipMemcpyDeviceToDevice, s);
  if (ln && !fw) {
    ln->done = gather_layernorm_fwd(x_full, idx, B, T, k, D, ln->gamma, ln->beta, c->eps, c->f32, x_kept, ln->y, ln->mean,
                                    ln->rstd, s);
    if (ln->done) return idx;
  }
  gather_tokens(x_full, idx, B, T, k, D, c->f32, x_kept, s, fw ? k + 2 : k + 1);
  if (fw) fuse_dropped(x_full, scores, idx, B, T, k, D, c->f32, fw, x_kept, s);
  return idx;
}

void build_shadows(bsr_ctx* c, int first_block, hipStream_t s) {
  if (c->f32) return;
  const bsr_config& cf = c->cfg;
  const int D = cf.dim, F = cf.mlp_hidden;
  MatTable tab;
  auto add = [&](const void* w, int rows, int cols, bf16* sp, bf16* tp) {
    matrix_table_add(tab, (float*)const_cast<void*>(w), nullptr, nullptr, nullptr, rows, cols, sp, tp);
    if (tab.count == MAT_TABLE_MAX) { matrix_table_run(tab, false, OptArgs(), s); tab = MatTable(); }
  };
  if (first_block == 0 && cf.image_size)
    add(c->p.w_patch, cf.in_chans * cf.patch_size * cf.patch_size, D, nullptr, c->b.t_patch);
  for (int l = first_block; l < cf.depth; ++l) {
    const bsr_block_params& w = c->p.blocks[l];
    Shadow& sh = c->b.sh[l];
    if (c->sc.fold1[l])
      ln_fold_weights((const float*)w.w_qkv, (const float*)w.b_qkv, (const float*)w.ln1_g, (const float*)w.ln1_b, D, 3 * D,
                      sh.t_qkv, sh.cs_qkv, sh.fb_qkv, s);
    else
      add(w.w_qkv, D, 3 * D, sh.s_qkv, sh.t_qkv);
    add(w.w_proj, D, D, sh.s_proj, sh.t_proj);
    if (c->sc.moe[l]) {   // one entry per expert matrix
      for (int e = 0; e < cf.n_experts; ++e) {
        const size_t o = (size_t)e * D * F;
        add((const float*)w.w_fc1 + o, D, F, sh.s_fc1 ? sh.s_fc1 + o : nullptr, sh.t_fc1 + o);
        add((const float*)w.w_fc2 + o, F, D, sh.s_fc2 ? sh.s_fc2 + o : nullptr, sh.t_fc2 + o);
      }
      continue;
    }
    if (c->sc.fold2[l])
      ln_fold_weights((const float*)w.w_fc1, (const float*)w.b_fc1, (const float*)w.ln2_g, (const float*)w.ln2_b, D, F,
                      sh.t_fc1, sh.cs_fc1, sh.fb_fc1, s);
    else
      add(w.w_fc1, D, F, sh.s_fc1, sh.t_fc1);
    add(w.w_fc2, F, D, sh.s_fc2, sh.t_fc2);
  }
  matrix_table_run(tab, false, OptArgs(), s);
  for (int l = first_block; l < cf.depth; ++l)
    if (c->sc.moe[l]) moe_router_copy((const float*)c->p.blocks[l].w_router, D, cf.n_experts, c->b.sh[l].t_router, s);
}

// only_trainable: a table of gradients or momenta (entries of frozen blocks are not read)
int check_params(const bsr_config& cf, const bsr_params* p, int first_block, bool need_stem, const char** which,
                 const Schedule* only_trainable = nullptr) {
#define NEED(ptr, name) if (!aligned16(ptr)) { *which = name; return BSR_ERR_INVALID_ARG; }
  if (need_stem && cf.image_size) { NEED(p->w_patch, "w_patch"); NEED(p->b_patch, "b_patch"); NEED(p->cls, "cls"); NEED(p->pos, "pos"); }
  for (int l = first_block; l < cf.depth; ++l) {
    if (only_trainable && !only_trainable->trainable[l]) continue;
    const bsr_block_params& w = p->blocks[l];
    NEED(w.ln1_g, "ln1_g"); NEED(w.ln1_b, "ln1_b"); NEED(w.w_qkv, "w_qkv"); NEED(w.b_qkv, "b_qkv");
    NEED(w.w_proj, "w_proj"); NEED(w.b_proj, "b_proj"); NEED(w.ln2_g, "ln2_g"); NEED(w.ln2_b, "ln2_b");
    NEED(w.w_fc1, "w_fc1"); NEED(w.b_fc1, "b_fc1"); NEED(w.w_fc2, "w_fc2"); NEED(w.b_fc2, "b_fc2");
    for (int i = 0; i < cf.n_moe; ++i)
      if (cf.moe_blocks[i] == l) NEED(w.w_router, "w_router");
  }
  if (cf.num_classes > 0) { NEED(p->lnf_g, "lnf_g"); NEED(p->lnf_b, "lnf_b"); NEED(p->w_head, "w_head"); NEED(p->b_head, "b_head"); }
#undef NEED
  return BSR_OK;
}

// Scratch of bsr_linear_wgrad_static: the split-K partial sums of one weight gradient, in device memory that
// belongs to the library's code object (every GPU the library runs on holds its own copy until the process ends).
constexpr size_t STATIC_SCRATCH_FLOATS = (size_t)6 << 20;          // 24 MiB
static __device__ __align__(256) float scratch[STATIC_SCRATCH_FLOATS];
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static float* g_scratch_ptr[STATIC_SCRATCH_MAX_DEVICES] = {};      // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

// Device address of the array on the current device (looked up once per device, with that device current).
// The array's name is only a host-side handle; kernels and copies get this pointer.
static int static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES) {
    (void)hipGetLastError();
    return fail(nullptr, BSR_ERR_HIP, "bsr_linear_wgrad_static: no current device (or more than %d devices)", STATIC_SCRATCH_MAX_DEVICES);
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      (void)hipGetLastError();
      return fail(nullptr, BSR_ERR_HIP, "bsr_linear_wgrad_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    }
    g_scratch_ptr[dev] = (float*)p;
  }
  *out = g_scratch_ptr[dev];
  return BSR_OK;
}

}  // namespace

// ================================================================================ C ABI

extern "C" {

int32_t bsr_token_schedule(const bsr_config* cfg, int32_t* keep_k_out, int32_t* tokens_attn,
                           int32_t* tokens_mlp) {
  if (!cfg) return fail(nullptr, BSR_ERR_INVALID_ARG, "cfg is NULL");
  Schedule s;
  char why[256];
  int rc = make_schedule(cfg, &s, why, sizeof(why));
  if (rc != BSR_OK) return fail(nullptr, rc, "%s", why);
  for (int i = 0; i < cfg->n_drop && keep_k_out; ++i) keep_k_out[i] = s.keep_k[i];
  for (int l = 0; l < cfg->depth; ++l) {
    if (tokens_attn) tokens_attn[l] = s.Ta[l];
    if (tokens_mlp) tokens_mlp[l] = s.Tm[l];
  }
  return BSR_OK;
}

int32_t bsr_workspace_bytes(const bsr_config* cfg, size_t* bytes_out) {
  if (!cfg || !bytes_out) return fail(nullptr, BSR_ERR_INVALID_ARG, "cfg or bytes_out is NULL");
  Schedule s;
  char why[256];
  int rc = make_schedule(cfg, &s, why, sizeof(why));
  if (rc != BSR_OK) return fail(nullptr, rc, "%s", why);
  *bytes_out = carve(*cfg, s, nullptr, nullptr);
  return BSR_OK;
}

int32_t bsr_saved_activation_bytes(const bsr_config* cfg, int32_t batch, bsr_saved_bytes* per_block,
                                   bsr_saved_bytes* sum) {
  if (!cfg) return fail(nullptr, BSR_ERR_INVALID_ARG, "cfg is NULL");
  Schedule s;
  char why[256];
  int rc = make_schedule(cfg, &s, why, sizeof(why));
  if (rc != BSR_OK) return fail(nullptr, rc, "%s", why);
  if (batch < 1 || batch > cfg->max_batch) return fail(nullptr, BSR_ERR_INVALID_ARG, "batch %d outside 1..max_batch %d", batch, cfg->max_batch);
  bsr_config c = *cfg;
  c.max_batch = batch;
  bsr_saved_bytes rep[BSR_MAX_BLOCKS] = {};
  carve(c, s, nullptr, nullptr, rep);
  bsr_saved_bytes t = {};
  for (int l = 0; l < cfg->depth; ++l) {
    if (per_block) per_block[l] = rep[l];
    t.qkv += rep[l].qkv; t.softmax += rep[l].softmax; t.attn_out += rep[l].attn_out; t.gelu_in += rep[l].gelu_in;
    t.linear_in += rep[l].linear_in; t.residual += rep[l].residual; t.stats += rep[l].stats; t.moe += rep[l].moe;
    t.total += rep[l].total;
  }
  if (sum) *sum = t;
  return BSR_OK;
}

int32_t bsr_init(const bsr_config* cfg, const bsr_params* params, void* workspace,
                 size_t workspace_bytes, void* stream, bsr_ctx** ctx_out) {
  if (!cfg || !params || !ctx_out) return fail(nullptr, BSR_ERR_INVALID_ARG, "cfg, params or ctx_out is NULL");
  *ctx_out = nullptr;
  Schedule s;
  char why[256];
  int rc = make_schedule(cfg, &s, why, sizeof(why));
  if (rc != BSR_OK) return fail(nullptr, rc, "%s", why);
  if (!workspace || (((uintptr_t)workspace) & 255)) return fail(nullptr, BSR_ERR_INVALID_ARG, "workspace must be a 256-byte aligned device pointer");
  const size_t need = carve(*cfg, s, nullptr, nullptr);
  if (workspace_bytes < need) return fail(nullptr, BSR_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  const char* which = "";
  if (check_params(*cfg, params, 0, true, &which) != BSR_OK) return fail(nullptr, BSR_ERR_INVALID_ARG, "parameter %s is NULL or not 16-byte aligned", which);
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
    (void)hipGetLastError();
    return fail(nullptr, BSR_ERR_HIP, "no usable HIP device");
  }
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return fail(nullptr, BSR_ERR_UNSUPPORTED_ARCH, "device is %s, this library is built for gfx950", prop.gcnArchName);
  bsr_ctx* c = new (std::nothrow) bsr_ctx();
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "out of host memory");
  c->cfg = *cfg;
  c->cfg.first_trainable_block = s.ft;      // (from trainable_blocks[0] when a list is given)
  c->p = *params;
  c->sc = s;
  c->f32 = cfg->dtype == BSR_FP32;
  c->esz = c->f32 ? 4 : 2;
  c->eps = cfg->ln_eps > 0.f ? cfg->ln_eps : 1e-6f;
  c->ws = (char*)workspace;
  c->ws_bytes = workspace_bytes;
  c->err[0] = 0;
  carve(*cfg, s, c->ws, &c->b);
  build_shadows(c, 0, (hipStream_t)stream);
  rc = check_hip(c, "bsr_init");
  if (rc != BSR_OK) { snprintf(g_err, sizeof(g_err), "%s", c->err); delete c; return rc; }
  *ctx_out = c;
  return BSR_OK;
}

int32_t bsr_refresh_weights(bsr_ctx* c, void* stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  build_shadows(c, 0, (hipStream_t)stream);
  return check_hip(c, "bsr_refresh_weights");
}

int32_t bsr_forward_frozen(bsr_ctx* c, const void* input, int32_t B, void* x_out,
                           int32_t* kept_idx_out, float* scores_out, const int32_t* forced_idx,
                           void* stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if (!aligned16(input) || !aligned16(x_out)) return fail(c, BSR_ERR_INVALID_ARG, "input / x_out is NULL or not 16-byte aligned");
  if (B < 1 || B > c->cfg.max_batch) return fail(c, BSR_ERR_INVALID_ARG, "B = %d outside 1..max_batch (%d)", B, c->cfg.max_batch);
  c->tune.kind = 0; c->tune.site = 0; c->tune.cur_batch = B;
  hipStream_t s = (hipStream_t)stream;
  const bsr_config& cf = c->cfg;
  const Schedule& sc = c->sc;
  Buffers& b = c->b;
  const int D = cf.dim, F = cf.mlp_hidden, ft = cf.first_trainable_block;
  const bool f32 = c->f32;
  const size_t E = c->esz;

  // stem (Sec. 3.1): patch embedding, CLS token, positional embedding
  char* x = (ft == 0) ? (char*)x_out : b.x0;
  char* xalt = b.x1;
  if (cf.image_size) {
    const int np = sc.T0 - 1, Kp = cf.in_chans * cf.patch_size * cf.patch_size;
    patchify(input, B, cf.in_chans, cf.image_size, cf.patch_size, f32, b.patches, s, (const float*)c->p.cls,
             (const float*)c->p.pos, sc.T0, D, x);
    GemmDesc g = fwd_desc(c, b.patches, B * np, Kp, D, c->p.w_patch, b.t_patch, x);
    g.bias = (const float*)c->p.b_patch;
    g.remap_np = np;
    g.pos = (const float*)c->p.pos;
    gemm(c, g, s);
  } else {
    (void)hipMemcpyAsync(x, input, (size_t)B * sc.T0 * D * E, hipMemcpyDeviceToDevice, s);
  }

  size_t idx_off = 0, sc_off = 0;
  for (int l = 0; l < ft; ++l) {
    const bsr_block_params& w = c->p.blocks[l];
    const Shadow& sh = b.sh[l];
    const int Ta = sc.Ta[l], Tm = sc.Tm[l], M = B * Ta, M2 = B * Tm;
    const int di = sc.drop_of[l];
    // MHSA: x <- x + proj(Attention(LN1(x)))
    const bool f1 = sc.fold1[l], f2 = sc.fold2[l];
    if (!f1) layernorm_fwd(x, M, D, (const float*)w.ln1_g, (const float*)w.ln1_b, c->eps, f32, b.h, nullptr, nullptr, s);
    GemmDesc g1 = fwd_desc(c, f1 ? x : b.h, M, D, 3 * D, w.w_qkv, sh.t_qkv, b.qkv);
    g1.bias = f1 ? sh.fb_qkv : (const float*)w.b_qkv;
    if (f1) { g1.ln_colsum = sh.cs_qkv; g1.ln_eps = c->eps; }
    gemm(c, g1, s);
    attention_fwd(c, b.qkv, B, Ta, b.o, nullptr, di >= 0 ? b.clsp : nullptr, s);
    GemmDesc g2 = fwd_desc(c, b.o, M, D, D, w.w_proj, sh.t_proj, x);
    g2.bias = (const float*)w.b_proj;
    g2.res = x;
    gemm(c, g2, s);
    LnAfterDrop ln2{(const float*)w.ln2_g, (const float*)w.ln2_b, b.h, nullptr, nullptr, false};
    if (di >= 0) {
      const int k = sc.keep_k[di];
      drop_tokens(c, B, Ta, k, x, xalt, b.idx_tmp, forced_idx ? forced_idx + idx_off : nullptr,
                  kept_idx_out ? kept_idx_out + idx_off : nullptr, scores_out ? scores_out + sc_off : nullptr,
                  sc.fused[di] ? b.fw : nullptr, s, &ln2);
      std::swap(x, xalt);
      idx_off += (size_t)B * k;
      sc_off += (size_t)B * (Ta - 1);
    }
    // FFN: x <- x + fc2(GELU(fc1(LN2(x)))), or the mixture of expert FFNs
    if (!ln2.done && !f2)
      layernorm_fwd(x, M2, D, (const float*)w.ln2_g, (const float*)w.ln2_b, c->eps, f32, b.h, nullptr, nullptr, s);
    char* dest = (l == ft - 1) ? (char*)x_out : x;
    if (sc.moe[l]) {
      moe_ffn_forward(c, l, B, b.h, x, M2, b.moe, nullptr, b.moe_u, dest, s);
      continue;
    }
    GemmDesc g3 = fwd_desc(c, f2 ? x : b.h, M2, D, F, w.w_fc1, sh.t_fc1, b.g);
    g3.bias = f2 ? sh.fb_fc1 : (const float*)w.b_fc1;
    g3.act = ACT_GELU;
    if (f2) { g3.ln_colsum = sh.cs_fc1; g3.ln_eps = c->eps; }
    gemm(c, g3, s);
    GemmDesc g4 = fwd_desc(c, b.g, M2, F, D, w.w_fc2, sh.t_fc2, dest);
    g4.bias = (const float*)w.b_fc2;
    g4.res = x;
    gemm(c, g4, s);
  }
  return check_hip(c, "bsr_forward_frozen");
}

int32_t bsr_select_tokens(bsr_ctx* c, const float* cls_attn, const void* x_in, int32_t B, int32_t n,
                          int32_t k, int32_t* idx_out, void* x_out, void* stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if (!aligned16(cls_attn) || !aligned16(idx_out)) return fail(c, BSR_ERR_INVALID_ARG, "cls_attn / idx_out is NULL or not 16-byte aligned");
  if ((x_in == nullptr) != (x_out == nullptr)) return fail(c, BSR_ERR_INVALID_ARG, "x_in and x_out must both be given or both be NULL");
  if (x_in && (!aligned16(x_in) || !aligned16(x_out))) return fail(c, BSR_ERR_INVALID_ARG, "x_in / x_out not 16-byte aligned");
  if (B < 1 || n < 0 || n > 1024 || k < 0 || k > n) return fail(c, BSR_ERR_INVALID_ARG, "need B >= 1 and 0 <= k <= n <= 1024 (B=%d n=%d k=%d)", B, n, k);
  hipStream_t s = (hipStream_t)stream;
  topk_select(cls_attn, B, n, k, idx_out, s);
  if (x_in) gather_tokens(x_in, idx_out, B, n + 1, k, c->cfg.dim, c->f32, x_out, s);
  return check_hip(c, "bsr_select_tokens");
}

int32_t bsr_train_blocks_fwd_bwd(bsr_ctx* c, const void* x_in, const int32_t* labels, int32_t B,
                                 float* loss_out, float* logits_out, void* x_final_out,
                                 const bsr_params* grads, int32_t* kept_idx_out, float* scores_out,
                                 const int32_t* forced_idx, void* stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  const bsr_config& cf = c->cfg;
  if (!aligned16(x_in) || !loss_out || !grads) return fail(c, BSR_ERR_INVALID_ARG, "x_in, loss_out or grads is NULL / misaligned");
  if (cf.loss == BSR_LOSS_CE && !labels) return fail(c, BSR_ERR_INVALID_ARG, "labels are required for the cross-entropy loss");
  if (B < 1 || B > cf.max_batch) return fail(c, BSR_ERR_INVALID_ARG, "B = %d outside 1..max_batch (%d)", B, cf.max_batch);
  const char* which = "";
  if (check_params(cf, grads, cf.first_trainable_block, false, &which, &c->sc) != BSR_OK)
    return fail(c, BSR_ERR_INVALID_ARG, "gradient tensor %s is NULL or not 16-byte aligned", which);
  c->tune.kind = 1; c->tune.site = 0; c->tune.cur_batch = B;
  hipStream_t s = (hipStream_t)stream;
  const Schedule& sc = c->sc;
  Buffers& b = c->b;
  const int D = cf.dim, F = cf.mlp_hidden, ft = cf.first_trainable_block, L = cf.depth;
  const bool f32 = c->f32;
  const size_t E = c->esz;
  const int32_t* idx_used[BSR_MAX_BLOCKS] = {};

  // ---------------------------------------------------------------- forward, keeping activations
  const char* x = (const char*)x_in;
  size_t idx_off = 0, sc_off = 0;
  for (int l = ft; l < L; ++l) {
    const bsr_block_params& w = c->p.blocks[l];
    const Shadow& sh = b.sh[l];
    SavedBlock& v = b.sv[l];
    const int Ta = sc.Ta[l], Tm = sc.Tm[l], M = B * Ta, M2 = B * Tm;
    const int di = sc.drop_of[l];
    layernorm_fwd(x, M, D, (const float*)w.ln1_g, (const float*)w.ln1_b, c->eps, f32, v.h1, v.mean1, v.rstd1, s);
    GemmDesc g1 = fwd_desc(c, v.h1, M, D, 3 * D, w.w_qkv, sh.t_qkv, v.qkv);
    g1.bias = (const float*)w.b_qkv;
    gemm(c, g1, s);
    attention_fwd(c, v.qkv, B, Ta, v.o, v.lse, di >= 0 ? b.clsp_t : nullptr, s);
    GemmDesc g2 = fwd_desc(c, v.o, M, D, D, w.w_proj, sh.t_proj, v.xmid_full);
    g2.bias = (const float*)w.b_proj;
    g2.res = x;
    gemm(c, g2, s);
    LnAfterDrop ln2{(const float*)w.ln2_g, (const float*)w.ln2_b, v.h2, v.mean2, v.rstd2, false};
    if (di >= 0) {
      const int k = sc.keep_k[di];
      idx_used[l] = drop_tokens(c, B, Ta, k, v.xmid_full, v.xmid, v.idx, forced_idx ? forced_idx + idx_off : nullptr,
                                kept_idx_out ? kept_idx_out + idx_off : nullptr,
                                scores_out ? scores_out + sc_off : nullptr, sc.fused[di] ? v.fw : nullptr, s, &ln2, true);
      idx_off += (size_t)B * k;
      sc_off += (size_t)B * (Ta - 1);
    }
    if (!ln2.done)
      layernorm_fwd(v.xmid, M2, D, (const float*)w.ln2_g, (const float*)w.ln2_b, c->eps, f32, v.h2, v.mean2, v.rstd2, s);
    if (sc.moe[l]) {
      moe_ffn_forward(c, l, B, v.h2, v.xmid, M2, v.moe, v.u, v.g, v.xout, s);
    } else {
      GemmDesc g3 = fwd_desc(c, v.h2, M2, D, F, w.w_fc1, sh.t_fc1, v.g);
      g3.bias = (const float*)w.b_fc1;
      g3.act = ACT_GELU;
      g3.aux = v.u;
      gemm(c, g3, s);
      GemmDesc g4 = fwd_desc(c, v.g, M2, F, D, w.w_fc2, sh.t_fc2, v.xout);
      g4.bias = (const float*)w.b_fc2;
      g4.res = v.xmid;
      gemm(c, g4, s);
    }
    x = v.xout;
  }
  const int Tl = sc.T_last;
  if (x_final_out) (void)hipMemcpyAsync(x_final_out, x, (size_t)B * Tl * D * E, hipMemcpyDeviceToDevice, s);

  // ---------------------------------------------------------------- head, loss, dLoss/dx_last
  char* dx = b.dxa;
  char* dx_other = b.dxb;
  if (cf.loss == BSR_LOSS_CE) {
    const int C = cf.num_classes;
    if (head_lds_bytes(D, C) <= 64 * 1024) {
      head_fwd_bwd(x, B, Tl, D, C, f32, (const float*)c->p.lnf_g, (const float*)c->p.lnf_b, c->eps, (const float*)c->p.w_head,
                   (const float*)c->p.b_head, labels, b.xc, b.z, b.logits, b.dlogits, b.dz, b.loss_rows, dx,
                   (float*)grads->w_head, (float*)grads->b_head, (float*)grads->lnf_g, (float*)grads->lnf_b, loss_out, s);
      if (logits_out) (void)hipMemcpyAsync(logits_out, b.logits, sizeof(float) * (size_t)B * C, hipMemcpyDeviceToDevice, s);
    } else {
    extract_cls(x, B, Tl, D, f32, b.xc, s);
    layernorm_fwd(b.xc, B, D, (const float*)c->p.lnf_g, (const float*)c->p.lnf_b, c->eps, true, b.z, b.meanf, b.rstdf, s);
    GemmDesc gl;   // logits = z . W_h + b_h (fp32)
    gl.A = b.z; gl.a_rs = D; gl.a_cs = 1; gl.B = c->p.w_head; gl.b_rs = C; gl.b_cs = 1;
    gl.C = b.logits; gl.ldc = C; gl.M = B; gl.N = C; gl.K = D; gl.in_f32 = gl.out_f32 = true;
    gl.bias = (const float*)c->p.b_head;
    gemm_small_f32(gl, s);
    cross_entropy(b.logits, labels, B, C, b.loss_rows, b.dlogits, loss_out, s);
    if (logits_out) (void)hipMemcpyAsync(logits_out, b.logits, sizeof(float) * (size_t)B * C, hipMemcpyDeviceToDevice, s);
    GemmDesc gz;   // dz = dlogits . W_h^T
    gz.A = b.dlogits; gz.a_rs = C; gz.a_cs = 1; gz.B = c->p.w_head; gz.b_rs = 1; gz.b_cs = C;
    gz.C = b.dz; gz.ldc = D; gz.M = B; gz.N = D; gz.K = C; gz.in_f32 = gz.out_f32 = true;
    gemm_small_f32(gz, s);
    GemmDesc gw;   // dW_h = z^T . dlogits
    gw.A = b.z; gw.a_rs = 1; gw.a_cs = D; gw.B = b.dlogits; gw.b_rs = C; gw.b_cs = 1;
    gw.C = grads->w_head; gw.ldc = C; gw.M = D; gw.N = C; gw.K = B; gw.in_f32 = gw.out_f32 = true;
    gemm_small_f32(gw, s);
    colsum(b.dlogits, B, C, C, true, b.partial, (float*)grads->b_head, s);
    layernorm_bwd_params(b.dz, b.xc, b.meanf, b.rstdf, B, D, true, b.partial, (float*)grads->lnf_g, (float*)grads->lnf_b, s);
    layernorm_bwd_dx(b.dz, b.xc, b.meanf, b.rstdf, (const float*)c->p.lnf_g, nullptr, B, D, true, b.dxc, s);
    place_cls_grad(b.dxc, B, Tl, D, f32, dx, s);
    }
  } else {
    mean_sq_loss(x, (int64_t)B * Tl * D, f32, b.partial, loss_out, dx, s);
  }

  // ---------------------------------------------------------------- backward (Eq. 2-5), last block first
  LnDeferTable ln_tab;          // dgamma / dbeta of all trained LayerNorms are summed in one launch at the end
  int ln_slot = 0;
  for (int l = L - 1; l >= ft; --l) {
    const bsr_block_params& w = c->p.blocks[l];
    const bsr_block_params& gw = grads->blocks[l];
    const Shadow& sh = b.sh[l];
    SavedBlock& v = b.sv[l];
    const int Ta = sc.Ta[l], Tm = sc.Tm[l], M = B * Ta, M2 = B * Tm;
    const int di = sc.drop_of[l];
    const char* xin = (l == ft) ? (const char*)x_in : b.sv[l - 1].xout;

    // A frozen block in the gradient path (tr == false) only passes the input gradient on (Eq. 2, 3).
    const bool tr = sc.trainable[l];
    // FFN branch.  du = (dx . W2^T) * GELU'(u); dW2 = g^T dx; dh2 = du . W1^T; dW1 = h2^T du
    if (sc.moe[l]) {
      moe_ffn_backward(c, l, dx, M2, v, gw, b.dh, tr, s);
    } else {
      GemmDesc d1 = dgrad_desc(c, dx, M2, F, D, w.w_fc2, sh.s_fc2, b.dgu);
      d1.act = ACT_GELU_BWD;
      d1.aux = v.u;
      if (tr) dgrad_wgrad(c, d1, v.g, dx, M2, F, D, gw.w_fc2, gw.b_fc2, s);
      else gemm(c, d1, s);
      const GemmDesc d2 = dgrad_desc(c, b.dgu, M2, D, F, w.w_fc1, sh.s_fc1, b.dh);
      if (tr) dgrad_wgrad(c, d2, v.h2, b.dgu, M2, D, F, gw.w_fc1, gw.b_fc1, s);
      else gemm(c, d2, s);
    }
    if (tr) {
      float* slot = b.ln_partial ? b.ln_partial + (size_t)(ln_slot++) * ln_deferred_partial_floats(D) : nullptr;
      if (!layernorm_bwd_deferred(b.dh, v.xmid, v.mean2, v.rstd2, (const float*)w.ln2_g, dx, M2, D, f32, dx_other, slot,
                                  (float*)gw.ln2_g, (float*)gw.ln2_b, ln_tab, s))
        layernorm_bwd(b.dh, v.xmid, v.mean2, v.rstd2, (const float*)w.ln2_g, dx, M2, D, f32, dx_other, b.partial,
                      (float*)gw.ln2_g, (float*)gw.ln2_b, s);
    }
    else
      layernorm_bwd_dx(b.dh, v.xmid, v.mean2, v.rstd2, (const float*)w.ln2_g, dx, M2, D, f32, dx_other, s);
    std::swap(dx, dx_other);   // dx: gradient at x_mid (kept tokens)

    // adjoint of the token drop: dropped tokens receive nothing from the FFN side
    if (di >= 0) {
      scatter_tokens(dx, idx_used[l], B, Ta, sc.keep_k[di], D, f32, dx_other, s, sc.fused[di] ? v.fw : nullptr);
      std::swap(dx, dx_other);
    }

    // MHSA branch.  dO = dx . Wproj^T; dWproj = o^T dx; attention backward; dWqkv = h1^T dqkv
    const GemmDesc d3 = dgrad_desc(c, dx, M, D, D, w.w_proj, sh.s_proj, b.dh);
    if (tr) dgrad_wgrad(c, d3, v.o, dx, M, D, D, gw.w_proj, gw.b_proj, s);
    else gemm(c, d3, s);
    attention_bwd(c, v.qkv, v.o, b.dh, v.lse, B, Ta, b.dqkv, s);
    const GemmDesc d4 = dgrad_desc(c, b.dqkv, M, D, 3 * D, w.w_qkv, sh.s_qkv, b.dh);
    if (tr) dgrad_wgrad(c, d4, v.h1, b.dqkv, M, D, 3 * D, gw.w_qkv, gw.b_qkv, s);
    else gemm(c, d4, s);
    // the gradient is not carried below the earliest trainable block (Fig. 2): no dx there
    if (tr) {
      float* slot = b.ln_partial ? b.ln_partial + (size_t)(ln_slot++) * ln_deferred_partial_floats(D) : nullptr;
      if (!layernorm_bwd_deferred(b.dh, xin, v.mean1, v.rstd1, (const float*)w.ln1_g, dx, M, D, f32,
                                  l > ft ? dx_other : nullptr, slot, (float*)gw.ln1_g, (float*)gw.ln1_b, ln_tab, s))
        layernorm_bwd(b.dh, xin, v.mean1, v.rstd1, (const float*)w.ln1_g, dx, M, D, f32, l > ft ? dx_other : nullptr,
                      b.partial, (float*)gw.ln1_g, (float*)gw.ln1_b, s);
    }
    else
      layernorm_bwd_dx(b.dh, xin, v.mean1, v.rstd1, (const float*)w.ln1_g, dx, M, D, f32, dx_other, s);
    if (l > ft) std::swap(dx, dx_other);
  }
  ln_deferred_finish(ln_tab, s);
  gemm_tn_flush(&c->tn_chain, s);
  return check_hip(c, "bsr_train_blocks_fwd_bwd");
}

int32_t bsr_moe_routing_io(bsr_ctx* c, const int32_t* forced_experts, int32_t* experts_out,
                           float* router_logits_out) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if ((forced_experts && !aligned16(forced_experts)) || (experts_out && !aligned16(experts_out)) ||
      (router_logits_out && !aligned16(router_logits_out)))
    return fail(c, BSR_ERR_INVALID_ARG, "bsr_moe_routing_io: pointer not 16-byte aligned");
  c->forced_experts = forced_experts;
  c->experts_out = experts_out;
  c->router_logits_out = router_logits_out;
  return BSR_OK;
}

// One optimiser step over the trainable tensors: vectors through sgd_table, matrices through the
// matrix table (which also rewrites their bf16 copies).  m1 / m2: first / second moment tables (null
// when the rule does not use them).
static int32_t optimizer_step(bsr_ctx* c, const bsr_params* grads, const bsr_params* m1, const bsr_params* m2,
                              const OptArgs& o, hipStream_t s, const char* where) {
  const bsr_config& cf = c->cfg;
  const int D = cf.dim, F = cf.mlp_hidden;
  SgdTable tab;
  int ntab = 0;
  auto vec = [&](void* w, const void* g, void* a, void* b2, int64_t n) {
    tab.e[ntab++] = SgdEntry{(float*)w, (const float*)g, m1 ? (float*)a : nullptr, m2 ? (float*)b2 : nullptr, n};
    if (ntab == SGD_TABLE_MAX) { sgd_table(tab, ntab, o, s); ntab = 0; }
  };
  MatTable mats;
  auto mat = [&](void* w, const void* g, void* a, void* b2, size_t off, int rows, int cols, bf16* sp, bf16* tp) {
    float* wp = (float*)w + off;
    const float* gp = (const float*)g + off;
    float* ap = m1 ? (float*)a + off : nullptr;
    float* bp = m2 ? (float*)b2 + off : nullptr;
    matrix_table_add(mats, wp, gp, ap, bp, rows, cols, sp, tp);
    if (mats.count == MAT_TABLE_MAX) { matrix_table_run(mats, true, o, s); mats = MatTable(); }
  };
  for (int l = cf.first_trainable_block; l < cf.depth; ++l) {
    if (!c->sc.trainable[l]) continue;
    const bsr_block_params& W = c->p.blocks[l];
    const bsr_block_params& G = grads->blocks[l];
    const bsr_block_params& A = m1 ? m1->blocks[l] : grads->blocks[l];
    const bsr_block_params& V = m2 ? m2->blocks[l] : grads->blocks[l];
    const Shadow& sh = c->b.sh[l];
    vec(W.ln1_g, G.ln1_g, A.ln1_g, V.ln1_g, D); vec(W.ln1_b, G.ln1_b, A.ln1_b, V.ln1_b, D);
    vec(W.b_qkv, G.b_qkv, A.b_qkv, V.b_qkv, 3 * D); vec(W.b_proj, G.b_proj, A.b_proj, V.b_proj, D);
    vec(W.ln2_g, G.ln2_g, A.ln2_g, V.ln2_g, D); vec(W.ln2_b, G.ln2_b, A.ln2_b, V.ln2_b, D);
    mat(W.w_qkv, G.w_qkv, A.w_qkv, V.w_qkv, 0, D, 3 * D, sh.s_qkv, sh.t_qkv);
    mat(W.w_proj, G.w_proj, A.w_proj, V.w_proj, 0, D, D, sh.s_proj, sh.t_proj);
    if (c->sc.moe[l]) {   // router, E bias vectors each, E matrices each
      const int E = cf.n_experts;
      vec(W.w_router, G.w_router, A.w_router, V.w_router, (int64_t)D * E);
      vec(W.b_fc1, G.b_fc1, A.b_fc1, V.b_fc1, (int64_t)E * F); vec(W.b_fc2, G.b_fc2, A.b_fc2, V.b_fc2, (int64_t)E * D);
      for (int e = 0; e < E; ++e) {
        const size_t off = (size_t)e * D * F;
        mat(W.w_fc1, G.w_fc1, A.w_fc1, V.w_fc1, off, D, F, sh.s_fc1 + off, sh.t_fc1 + off);
        mat(W.w_fc2, G.w_fc2, A.w_fc2, V.w_fc2, off, F, D, sh.s_fc2 + off, sh.t_fc2 + off);
      }
      continue;
    }
    vec(W.b_fc1, G.b_fc1, A.b_fc1, V.b_fc1, F); vec(W.b_fc2, G.b_fc2, A.b_fc2, V.b_fc2, D);
    mat(W.w_fc1, G.w_fc1, A.w_fc1, V.w_fc1, 0, D, F, sh.s_fc1, sh.t_fc1);
    mat(W.w_fc2, G.w_fc2, A.w_fc2, V.w_fc2, 0, F, D, sh.s_fc2, sh.t_fc2);
  }
  if (cf.num_classes > 0) {
    const bsr_params& W = c->p;
    const bsr_params& G = *grads;
    const bsr_params& A = m1 ? *m1 : *grads;
    const bsr_params& V = m2 ? *m2 : *grads;
    vec(W.lnf_g, G.lnf_g, A.lnf_g, V.lnf_g, D); vec(W.lnf_b, G.lnf_b, A.lnf_b, V.lnf_b, D);
    vec(W.w_head, G.w_head, A.w_head, V.w_head, (int64_t)D * cf.num_classes);
    vec(W.b_head, G.b_head, A.b_head, V.b_head, cf.num_classes);
  }
  sgd_table(tab, ntab, o, s);
  matrix_table_run(mats, true, o, s);
  for (int l = cf.first_trainable_block; l < cf.depth; ++l)      // the routers were updated as vectors
    if (c->sc.moe[l] && c->sc.trainable[l])
      moe_router_copy((const float*)c->p.blocks[l].w_router, D, cf.n_experts, c->b.sh[l].t_router, s);
  return check_hip(c, where);
}

// The two-stream schedule is not tuned launch by launch.  Side by side, a launch cannot be judged by its own
// time: a shape whose workgroup fills the LDS of a CU is quick by itself and stalls whatever runs on the other
// stream, and with the GPU always full it is the work per CU-second that counts, not how evenly one launch
// alone fills the chip.  (Measured on a ViT-B/16 step, batch 32: the per-launch best of all shapes timed alone gives
// 2.13 ms pipelined, 192 x 128 forced everywhere 2.03 ms; per-launch event times taken side by side chose
// worse than that, too.)  So the choice is one shape for all launches, among the shapes that leave room for a
// second workgroup on a CU (two tile buffers of at most 80 KB; the shape id is [prefetch depth] BM BN in
// decimal), and what is timed is a whole side-by-side pass.
static bool shares_a_cu(int tile_id) { return gemm_nt_tile_lds_bytes(tile_id) <= 80 * 1024; }

static int32_t autotune_overlapped(bsr_ctx* c, const void* input, const int32_t* labels, int32_t B, void* x_frozen,
                                   void* x_side, float* loss_out, const bsr_params* grads, int32_t* launches_out,
                                   int32_t* changed_out, void* stream, void* side) {
  hipStream_t s = (hipStream_t)stream, s2 = (hipStream_t)side;
  Tune& t = c->tune;
  t.batch = 0;
  t.pick[0].clear();
  t.pick[1].clear();
  const int n = gemm_nt_tile_count();
  hipEvent_t e0 = nullptr, e1 = nullptr, ej = nullptr, ready[2] = {nullptr, nullptr}, done[2] = {nullptr, nullptr};
  bool ok = hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess &&
            hipEventCreateWithFlags(&ej, hipEventDisableTiming) == hipSuccess;
  for (int i = 0; i < 2 && ok; ++i)
    ok = hipEventCreateWithFlags(&ready[i], hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&done[i], hipEventDisableTiming) == hipSuccess;
  auto drop_events = [&]() {
    for (hipEvent_t e : {e0, e1, ej, ready[0], ready[1], done[0], done[1]})
      if (e) (void)hipEventDestroy(e);
  };
  if (!ok) { drop_events(); return fail(c, BSR_ERR_HIP, "bsr_autotune_overlapped: cannot create events"); }
  int rc = BSR_OK;
  // One pass.  f < 0: the two calls one after the other on `stream`, untimed.  Otherwise a short run of the
  // pipeline itself with every launch forced to its shape: the frozen prefix (shape f) of iteration k+1 on s
  // beside the trainable part (shape tr) of iteration k on s2, ordered as bsr_pipeline_step orders them with
  // two x buffers (the prefix may run one iteration ahead), and in place of the optimizer step, which a
  // tuning pass must not take, the rebuild of the trainable blocks' bf16 weight copies: the same matrices
  // read and rewritten, bound by memory like the update.  The prefix writes x_side every time; the trainable
  // part reads x_frozen, which the untimed pass has left.
  constexpr int ITER = 6;
  auto pass = [&](int f, int tr, float* ms) {
    t.cand = f;
    t.cand_train = tr;
    if (f < 0) {
      rc = bsr_forward_frozen(c, input, B, x_frozen, nullptr, nullptr, nullptr, stream);
      if (rc == BSR_OK)
        rc = bsr_train_blocks_fwd_bwd(c, x_frozen, labels, B, loss_out, nullptr, nullptr, grads, nullptr, nullptr, nullptr, stream);
      return;
    }
    (void)hipEventRecord(e0, s);
    (void)hipStreamWaitEvent(s2, e0, 0);
    rc = bsr_forward_frozen(c, input, B, x_side, nullptr, nullptr, nullptr, stream);           // iteration 0's prefix
    (void)hipEventRecord(ready[0], s);
    for (int k = 0; k < ITER && rc == BSR_OK; ++k) {
      if (k + 1 < ITER) {
        if (k >= 1) (void)hipStreamWaitEvent(s, done[(k + 1) % 2], 0);     // the reader of that buffer, two iterations back
        rc = bsr_forward_frozen(c, input, B, x_side, nullptr, nullptr, nullptr, stream);
        (void)hipEventRecord(ready[(k + 1) % 2], s);
        if (rc != BSR_OK) break;
      }
      (void)hipStreamWaitEvent(s2, ready[k % 2], 0);
      rc = bsr_train_blocks_fwd_bwd(c, x_frozen, labels, B, loss_out, nullptr, nullptr, grads, nullptr, nullptr, nullptr, side);
      build_shadows(c, c->sc.ft, s2);
      (void)hipEventRecord(done[k % 2], s2);
    }
    if (rc != BSR_OK) return;
    (void)hipEventRecord(ej, s2);
    (void)hipStreamWaitEvent(s, ej, 0);
    (void)hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(ms, e0, e1) != hipSuccess) rc = BSR_ERR_HIP;
  };
  float dummy = 0.f;
  pass(-1, -1, &dummy);                                   // set-up; leaves a valid x_frozen
  (void)hipStreamSynchronize(s);
  std::vector<int> cands;
  for (int j = 0; j < n; ++j)
    if (shares_a_cu(gemm_nt_tile_id(j))) cands.push_back(j);
  // the shape with the shortest pass, three tries each.  (Refining it into one shape for the prefix and another
  // for the trainable part was tried: the passes differ by less than they scatter, and the refined pairs ran
  // 4 - 6 % slower in the pipeline than the single shape.)
  int both = -1;
  float best = 0.f;
  for (int round = 0; round < 3 && rc == BSR_OK; ++round)
    for (int j : cands) {
      float ms = 0.f;
      pass(j, j, &ms);
      if (rc != BSR_OK) break;
      if (both < 0 || ms < best) { both = j; best = ms; }
    }
  const int fz = both, tr = both;
  t.cand = -1;
  t.cand_train = -1;
  const bool synced = hipStreamSynchronize(s) == hipSuccess && hipStreamSynchronize(s2) == hipSuccess;
  drop_events();
  int launches = 0;
  if (rc == BSR_OK && synced && fz >= 0 && tr >= 0) {
    // the launch sites and their dimensions come from the records of the passes; their times are not used
    size_t sites[2] = {0, 0};
    for (const TuneRec& r : t.recs) sites[r.kind] = std::max(sites[r.kind], r.site + 1);
    for (int k = 0; k < 2; ++k) {
      t.pick[k].assign(sites[k], TunePick{0, 0, 0, 0, 0.f});
      for (const TuneRec& r : t.recs) {
        if (r.kind != k) continue;
        TunePick& p = t.pick[k][r.site];
        p.M = r.M; p.N = r.N; p.K = r.K;
        p.tile = gemm_nt_tile_id(k == 0 ? fz : tr);
      }
      launches += (int)sites[k];
    }
    t.batch = B;
  }
  for (TuneRec& r : t.recs) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  t.recs.clear();
  if (rc != BSR_OK) return rc == BSR_ERR_HIP ? fail(c, BSR_ERR_HIP, "bsr_autotune_overlapped: event timing failed") : rc;
  if (!synced) return fail(c, BSR_ERR_HIP, "bsr_autotune_overlapped: stream synchronisation failed");
  if (launches_out) *launches_out = launches;
  if (changed_out) {
    int diff = 0;
    for (int k = 0; k < 2; ++k)
      for (const TunePick& p : t.pick[k]) diff += p.tile != 0 && p.tile != gemm_nt_model_tile(p.M, p.N, p.K);
    *changed_out = diff;
  }
  return check_hip(c, "bsr_autotune_overlapped");
}

// Measured tile choice, launch by launch: the two calls follow each other on `stream`, once per shape (twice
// over), every NT launch bracketed by events in its place in the step.
static int32_t autotune(bsr_ctx* c, const void* input, const int32_t* labels, int32_t B, void* x_frozen,
                        float* loss_out, const bsr_params* grads, int32_t* launches_out, int32_t* changed_out,
                        void* stream) {
  hipStream_t s = (hipStream_t)stream;
  Tune& t = c->tune;
  t.batch = 0;
  t.pick[0].clear();
  t.pick[1].clear();
  const int n = gemm_nt_tile_count();
  constexpr int ROUNDS = 2;
  int rc = BSR_OK;
  // pass -1 is untimed (first-use set-up of the kernels); then every shape, ROUNDS times
  for (int pass = -1; pass < ROUNDS * n && rc == BSR_OK; ++pass) {
    t.cand = pass < 0 ? -1 : pass % n;
    rc = bsr_forward_frozen(c, input, B, x_frozen, nullptr, nullptr, nullptr, stream);
    if (rc == BSR_OK) rc = bsr_train_blocks_fwd_bwd(c, x_frozen, labels, B, loss_out, nullptr, nullptr, grads, nullptr, nullptr, nullptr, stream);
  }
  t.cand = -1;
  const bool synced = hipStreamSynchronize(s) == hipSuccess;
  int launches = 0;
  if (rc == BSR_OK && synced) {
    size_t sites[2] = {0, 0};
    for (const TuneRec& r : t.recs) sites[r.kind] = std::max(sites[r.kind], r.site + 1);
    for (int k = 0; k < 2; ++k) {
      std::vector<float> best(sites[k] * n, -1.f);          // min over the rounds, per (site, shape)
      t.pick[k].assign(sites[k], TunePick{0, 0, 0, 0, 0.f});
      for (const TuneRec& r : t.recs) {
        if (r.kind != k) continue;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) continue;
        float& b = best[r.site * n + r.cand];
        if (b < 0.f || ms < b) b = ms;
        TunePick& p = t.pick[k][r.site];
        p.M = r.M; p.N = r.N; p.K = r.K;
      }
      for (size_t i = 0; i < sites[k]; ++i) {
        int arg = -1;
        for (int j = 0; j < n; ++j)
          if (best[i * n + j] >= 0.f && (arg < 0 || best[i * n + j] < best[i * n + arg])) arg = j;
        t.pick[k][i].tile = arg < 0 ? 0 : gemm_nt_tile_id(arg);
        t.pick[k][i].us = arg < 0 ? 0.f : best[i * n + arg] * 1e3f;
        ++launches;
      }
    }
    t.batch = B;
  }
  for (TuneRec& r : t.recs) {
    (void)hipEventDestroy(r.start);
    (void)hipEventDestroy(r.stop);
  }
  t.recs.clear();
  if (rc != BSR_OK) return rc;
  if (!synced) return fail(c, BSR_ERR_HIP, "bsr_autotune: stream synchronisation failed");
  if (launches_out) *launches_out = launches;
  if (changed_out) {
    // how many launches now take another shape than the built-in model would give them
    int diff = 0;
    for (int k = 0; k < 2; ++k)
      for (const TunePick& p : t.pick[k]) diff += p.tile != 0 && p.tile != gemm_nt_model_tile(p.M, p.N, p.K);
    *changed_out = diff;
  }
  return check_hip(c, "bsr_autotune");
}

int32_t bsr_autotune(bsr_ctx* c, const void* input, const int32_t* labels, int32_t B, void* x_frozen,
                     float* loss_out, const bsr_params* grads, int32_t* launches_out, int32_t* changed_out,
                     void* stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  return autotune(c, input, labels, B, x_frozen, loss_out, grads, launches_out, changed_out, stream);
}

int32_t bsr_tile_choices(const bsr_ctx* c, int32_t part, bsr_tile_choice* out, int32_t max) {
  if (!c || part < 0 || part > 1) return 0;
  const std::vector<TunePick>& v = c->tune.pick[part];
  for (size_t i = 0; out && i < v.size() && (int32_t)i < max; ++i) {
    out[i].rows = v[i].M; out[i].out = v[i].N; out[i].in = v[i].K; out[i].tile = v[i].tile; out[i].microseconds = v[i].us;
  }
  return (int32_t)v.size();
}

int32_t bsr_autotune_overlapped(bsr_ctx* c, const void* input, const int32_t* labels, int32_t B, void* x_frozen,
                                void* x_side, float* loss_out, const bsr_params* grads, int32_t* launches_out,
                                int32_t* changed_out, void* stream, void* side_stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if (!aligned16(x_side) || x_side == x_frozen) return fail(c, BSR_ERR_INVALID_ARG, "x_side is NULL, misaligned or x_frozen itself");
  if (!side_stream || side_stream == stream) return fail(c, BSR_ERR_INVALID_ARG, "side_stream must be a second stream");
  if (c->sc.ft == 0)
    return fail(c, BSR_ERR_BAD_CONFIG, "there is no frozen prefix to run beside the trainable part");
  return autotune_overlapped(c, input, labels, B, x_frozen, x_side, loss_out, grads, launches_out, changed_out, stream, side_stream);
}

int32_t bsr_sgd_step(bsr_ctx* c, const bsr_params* grads, const bsr_params* momenta, float lr,
                     float momentum, float weight_decay, void* stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if (!grads) return fail(c, BSR_ERR_INVALID_ARG, "grads is NULL");
  if (momentum < 0.f) return fail(c, BSR_ERR_INVALID_ARG, "momentum must be >= 0");
  if (momentum > 0.f && !momenta) return fail(c, BSR_ERR_INVALID_ARG, "momenta is NULL but momentum > 0");
  const bsr_config& cf = c->cfg;
  const char* which = "";
  if (check_params(cf, grads, cf.first_trainable_block, false, &which, &c->sc) != BSR_OK)
    return fail(c, BSR_ERR_INVALID_ARG, "gradient tensor %s is NULL or not 16-byte aligned", which);
  if (momentum > 0.f && check_params(cf, momenta, cf.first_trainable_block, false, &which, &c->sc) != BSR_OK)
    return fail(c, BSR_ERR_INVALID_ARG, "momentum tensor %s is NULL or not 16-byte aligned", which);
  OptArgs o;
  o.kind = OPT_SGD; o.lr = lr; o.mu = momentum; o.wd = weight_decay;
  return optimizer_step(c, grads, momentum > 0.f ? momenta : nullptr, nullptr, o, (hipStream_t)stream, "bsr_sgd_step");
}

// One step of the two-stream pipeline (the rule on concurrent calls in the header): the frozen prefix of the
// next batch on stream_frozen, the trainable part and the SGD step of the current batch on stream_train, and
// the events that order the producer and the consumer of every x buffer.
int32_t bsr_pipeline_step(bsr_ctx* c, const void* input_next, void* x_next, const void* x_cur, const int32_t* labels_cur,
                          int32_t B, float* loss_out, const bsr_params* grads, const bsr_params* momenta, float lr,
                          float momentum, float weight_decay, void* stream_frozen, void* stream_train) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if ((input_next == nullptr) != (x_next == nullptr)) return fail(c, BSR_ERR_INVALID_ARG, "input_next and x_next go together");
  if (!x_next && !x_cur) return fail(c, BSR_ERR_INVALID_ARG, "nothing to do: neither a next batch nor a current one");
  if (x_next && x_next == x_cur) return fail(c, BSR_ERR_INVALID_ARG, "x_next and x_cur must be two buffers");
  if (stream_frozen == stream_train) return fail(c, BSR_ERR_INVALID_ARG, "the pipeline needs two streams");
  if (c->sc.ft == 0) return fail(c, BSR_ERR_BAD_CONFIG, "there is no frozen prefix to run ahead");
  auto slot_of = [&](const void* x) -> bsr_ctx::PipeSlot* {
    for (auto& p : c->pipe)
      if (p.x == x) return &p;
    if (c->pipe.size() >= 8) return nullptr;
    bsr_ctx::PipeSlot p{x, nullptr, nullptr, false, false};
    if (hipEventCreateWithFlags(&p.ready, hipEventDisableTiming) != hipSuccess) return nullptr;
    if (hipEventCreateWithFlags(&p.free, hipEventDisableTiming) != hipSuccess) { (void)hipEventDestroy(p.ready); return nullptr; }
    c->pipe.push_back(p);
    return &c->pipe.back();
  };
  hipStream_t sf = (hipStream_t)stream_frozen, st = (hipStream_t)stream_train;
  bsr_ctx::PipeSlot* cur = nullptr;
  if (x_cur) {
    for (auto& p : c->pipe)
      if (p.x == x_cur) cur = &p;
    if (!cur || !cur->has_ready) return fail(c, BSR_ERR_INVALID_ARG, "x_cur has not been filled by an earlier bsr_pipeline_step");
  }
  int32_t rc = BSR_OK;
  if (x_next) {
    const size_t cur_index = cur ? (size_t)(cur - c->pipe.data()) : 0;
    bsr_ctx::PipeSlot* nx = slot_of(x_next);
    if (!nx) return fail(c, BSR_ERR_HIP, "bsr_pipeline_step: more than 8 x buffers, or no event to be had");
    if (cur) cur = &c->pipe[cur_index];                   // the table may have moved
    if (nx->has_free) (void)hipStreamWaitEvent(sf, nx->free, 0);     // its previous reader is done
    rc = bsr_forward_frozen(c, input_next, B, x_next, nullptr, nullptr, nullptr, stream_frozen);
    if (rc != BSR_OK) return rc;
    (void)hipEventRecord(nx->ready, sf);
    nx->has_ready = true;
    nx->has_free = false;
  }
  if (cur) {
    (void)hipStreamWaitEvent(st, cur->ready, 0);
    rc = bsr_train_blocks_fwd_bwd(c, x_cur, labels_cur, B, loss_out, nullptr, nullptr, grads, nullptr, nullptr, nullptr, stream_train);
    if (rc == BSR_OK) rc = bsr_sgd_step(c, grads, momenta, lr, momentum, weight_decay, stream_train);
    if (rc != BSR_OK) return rc;
    (void)hipEventRecord(cur->free, st);
    cur->has_free = true;
    cur->has_ready = false;
  }
  return check_hip(c, "bsr_pipeline_step");
}

int32_t bsr_adamw_step(bsr_ctx* c, const bsr_params* grads, const bsr_params* exp_avg, const bsr_params* exp_avg_sq,
                       float lr, float beta1, float beta2, float eps, float weight_decay, int32_t step,
                       void* stream) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if (!grads || !exp_avg || !exp_avg_sq) return fail(c, BSR_ERR_INVALID_ARG, "grads, exp_avg or exp_avg_sq is NULL");
  if (step < 1) return fail(c, BSR_ERR_INVALID_ARG, "step counts from 1");
  if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f && eps > 0.f))
    return fail(c, BSR_ERR_INVALID_ARG, "need 0 <= beta1, beta2 < 1 and eps > 0");
  const bsr_config& cf = c->cfg;
  const char* which = "";
  for (const bsr_params* t : {grads, exp_avg, exp_avg_sq})
    if (check_params(cf, t, cf.first_trainable_block, false, &which, &c->sc) != BSR_OK)
      return fail(c, BSR_ERR_INVALID_ARG, "tensor %s of a table is NULL or not 16-byte aligned", which);
  OptArgs o;
  o.kind = OPT_ADAMW; o.lr = lr; o.wd = weight_decay; o.b1 = beta1; o.b2 = beta2; o.eps = eps;
  o.bc1 = (float)(1.0 - pow((double)beta1, (double)step));
  o.bc2 = (float)(1.0 - pow((double)beta2, (double)step));
  return optimizer_step(c, grads, exp_avg, exp_avg_sq, o, (hipStream_t)stream, "bsr_adamw_step");
}

static bool known_tile(int tile) {
  bool known = tile == 0;
  for (int i = 0; i < gemm_nt_tile_count(); ++i) known |= gemm_nt_tile_id(i) == tile;
  return known;
}

static int32_t run_layer(const GemmDesc& g, int32_t* used_mfma, void* stream, const char* where,
                         float* ws = nullptr, size_t ws_floats = 0, int tile = 0) {
  const bool mfma = gemm_mfma_supported(g);
  if (used_mfma) *used_mfma = mfma ? 1 : 0;
  if (mfma) gemm_mfma(g, ws, ws_floats, (hipStream_t)stream, tile);
  else gemm_generic(g, (hipStream_t)stream);
  return check_hip(nullptr, where);
}

int32_t bsr_linear_forward(const void* x, int32_t M, int32_t in, int32_t out, const void* w_t,
                           const float* bias, int32_t act, void* u_out, const void* res, void* y,
                           int32_t tile, int32_t* used_mfma, void* stream) {
  if (!aligned16(x) || !aligned16(w_t) || !aligned16(y) || M < 1 || in < 1 || out < 1 || (act != 0 && act != 1) ||
      (bias && !aligned16(bias)) || (u_out && !aligned16(u_out)) || (res && !aligned16(res)))
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_forward: bad argument");
  if (!known_tile(tile)) return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_forward: %d is not a tile shape id", tile);
  GemmDesc g;
  g.A = x; g.a_rs = in; g.a_cs = 1; g.B = w_t; g.b_rs = 1; g.b_cs = in;
  g.C = y; g.ldc = out; g.M = M; g.N = out; g.K = in;
  g.bias = bias; g.act = act ? ACT_GELU : ACT_NONE; g.aux = act ? u_out : nullptr; g.res = res;
  return run_layer(g, used_mfma, stream, "bsr_linear_forward", nullptr, 0, tile);
}

int32_t bsr_gemm_tile_shapes(int32_t* ids, int32_t max) {
  const int n = gemm_nt_tile_count();
  for (int i = 0; ids && i < n && i < max; ++i) ids[i] = gemm_nt_tile_id(i);
  return n;
}

int32_t bsr_ln_linear_fold(const float* w, const float* bias, const float* gamma, const float* beta, int32_t in,
                           int32_t out, void* w_folded, float* colsum, float* bias_folded, void* stream) {
  if (!aligned16(w) || !aligned16(bias) || !aligned16(gamma) || !aligned16(beta) || !aligned16(w_folded) ||
      !aligned16(colsum) || !aligned16(bias_folded) || in < 8 || in % 8 || out < 1)
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_ln_linear_fold: bad argument");
  ln_fold_weights(w, bias, gamma, beta, in, out, (bf16*)w_folded, colsum, bias_folded, (hipStream_t)stream);
  return check_hip(nullptr, "bsr_ln_linear_fold");
}

int32_t bsr_ln_linear_forward(const void* x, int32_t M, int32_t in, int32_t out, const void* w_folded,
                              const float* colsum, const float* bias_folded, float eps, int32_t act, void* y,
                              int32_t tile, void* stream) {
  if (!aligned16(x) || !aligned16(w_folded) || !aligned16(colsum) || !aligned16(bias_folded) || !aligned16(y) || M < 1 ||
      in < 64 || in % 64 || out < 8 || out % 8 || (act != 0 && act != 1))
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_ln_linear_forward: bad argument");
  if (!known_tile(tile)) return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_ln_linear_forward: %d is not a tile shape id", tile);
  GemmDesc g;
  g.A = x; g.a_rs = in; g.a_cs = 1; g.B = w_folded; g.b_rs = 1; g.b_cs = in;
  g.C = y; g.ldc = out; g.M = M; g.N = out; g.K = in;
  g.bias = bias_folded; g.act = act ? ACT_GELU : ACT_NONE;
  g.ln_colsum = colsum; g.ln_eps = eps;
  if (!gemm_mfma_supported(g)) return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_ln_linear_forward: shape not taken by the MFMA kernel");
  gemm_mfma(g, nullptr, 0, (hipStream_t)stream, tile);
  return check_hip(nullptr, "bsr_ln_linear_forward");
}

int32_t bsr_linear_dgrad(const void* dy, int32_t M, int32_t in, int32_t out, const void* w_s,
                         const void* u, void* dx, int32_t tile, int32_t* used_mfma, void* stream) {
  if (!aligned16(dy) || !aligned16(w_s) || !aligned16(dx) || M < 1 || in < 1 || out < 1)
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_dgrad: bad argument");
  if (!known_tile(tile)) return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_dgrad: %d is not a tile shape id", tile);
  GemmDesc g;
  g.A = dy; g.a_rs = out; g.a_cs = 1; g.B = w_s; g.b_rs = 1; g.b_cs = out;
  g.C = dx; g.ldc = in; g.M = M; g.N = in; g.K = out;
  if (u) { g.act = ACT_GELU_BWD; g.aux = const_cast<void*>(u); }
  return run_layer(g, used_mfma, stream, "bsr_linear_dgrad", nullptr, 0, tile);
}

int32_t bsr_linear_wgrad(const void* x, const void* dy, int32_t M, int32_t in, int32_t out, float* dw,
                         float* db, float* workspace, size_t workspace_floats, int32_t* used_mfma, void* stream) {
  if (!aligned16(x) || !aligned16(dy) || !aligned16(dw) || M < 1 || in < 1 || out < 1)
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_wgrad: bad argument");
  GemmDesc g;
  g.A = x; g.a_rs = 1; g.a_cs = in; g.B = dy; g.b_rs = out; g.b_cs = 1;
  g.C = dw; g.ldc = out; g.M = in; g.N = out; g.K = M; g.out_f32 = true;
  if (workspace && !aligned16(workspace)) return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_wgrad: workspace misaligned");
  if (db && gemm_mfma_supported(g)) {
    g.bsum = db;
  } else if (db) {   // shapes the MFMA kernel does not take: separate column sums, staged in the workspace
    if (!workspace || workspace_floats < colsum_partial_floats(M, out))
      return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_wgrad: db for this shape needs a workspace of %zu floats",
                  colsum_partial_floats(M, out));
    colsum(dy, M, out, out, false, workspace, db, (hipStream_t)stream);
  }
  return run_layer(g, used_mfma, stream, "bsr_linear_wgrad", workspace, workspace_floats);
}

int32_t bsr_linear_wgrad_static(const void* x, const void* dy, int32_t M, int32_t in, int32_t out, float* dw, float* db,
                                int32_t* used_mfma, void* stream) {
  if (!aligned16(x) || !aligned16(dy) || !aligned16(dw) || M < 1 || in < 1 || out < 1)
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_linear_wgrad_static: bad argument");
  // the smallest split (two partial copies of dw and of db) has to fit, and so do the column-sum partials of a
  // shape the MFMA kernel does not take: larger layers are refused rather than run without their scratch
  const size_t need = (size_t)2 * ((size_t)in + 1) * (size_t)out;
  if (need > STATIC_SCRATCH_FLOATS || colsum_partial_floats(M, out) > STATIC_SCRATCH_FLOATS)
    return fail(nullptr, BSR_ERR_INVALID_ARG,
                "bsr_linear_wgrad_static: a layer of %d x %d needs %zu floats of scratch, the built-in array holds %zu "
                "(2 (in + 1) out must not exceed it)", in, out, need, STATIC_SCRATCH_FLOATS);
  float* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc != BSR_OK) return rc;
  // every partial sum that is read has been written by this call: nothing in the array has to start at zero
  return bsr_linear_wgrad(x, dy, M, in, out, dw, db, ws, STATIC_SCRATCH_FLOATS, used_mfma, stream);
}

int32_t bsr_attention_forward(const void* qkv, int32_t B, int32_t T, int32_t H, int32_t d, void* out,
                              float* lse, float* cls_prob, int32_t* used_mfma, void* stream) {
  if (!aligned16(qkv) || !aligned16(out) || B < 1 || T < 1 || T > 1024 || H < 1 || d < 1 || d > 256 || (H * d) % 8)
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_attention_forward: bad argument");
  const bool mfma = attn_mfma_supported(T, d);
  if (used_mfma) *used_mfma = mfma ? 1 : 0;
  if (mfma) attn_fwd_mfma(qkv, B, T, H, out, lse, cls_prob, (hipStream_t)stream);
  else attn_fwd_generic(qkv, B, T, H, d, false, out, lse, cls_prob, (hipStream_t)stream);
  return check_hip(nullptr, "bsr_attention_forward");
}

int32_t bsr_attention_backward(const void* qkv, const void* out, const void* dout, const float* lse,
                               int32_t B, int32_t T, int32_t H, int32_t d, float* delta, void* dqkv,
                               int32_t* used_mfma, void* stream) {
  if (!aligned16(qkv) || !aligned16(out) || !aligned16(dout) || !aligned16(dqkv) || !lse || !delta || B < 1 ||
      T < 1 || T > 1024 || H < 1 || d < 1 || d > 256 || (H * d) % 8)
    return fail(nullptr, BSR_ERR_INVALID_ARG, "bsr_attention_backward: bad argument");
  const bool mfma = attn_mfma_supported(T, d);
  if (used_mfma) *used_mfma = mfma ? 1 : 0;
  if (mfma) attn_bwd_mfma(qkv, out, dout, lse, B, T, H, delta, dqkv, (hipStream_t)stream);
  else attn_bwd_generic(qkv, out, dout, lse, B, T, H, d, false, delta, dqkv, (hipStream_t)stream);
  return check_hip(nullptr, "bsr_attention_backward");
}

int32_t bsr_profile_begin(bsr_ctx* c) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  c->prof_used = 0;
  c->prof_on = true;
  return BSR_OK;
}

int32_t bsr_profile_end(bsr_ctx* c, double* ms, double* flops, int32_t* launches) {
  if (!c) return fail(nullptr, BSR_ERR_INVALID_ARG, "ctx is NULL");
  if (!ms || !flops || !launches) return fail(c, BSR_ERR_INVALID_ARG, "output arrays are NULL");
  c->prof_on = false;
  for (int k = 0; k < BSR_PROF_CLASSES; ++k) { ms[k] = 0; flops[k] = 0; launches[k] = 0; }
  for (size_t i = 0; i < c->prof_used; ++i) {
    ProfRec& r = c->prof[i];
    float t = 0.f;
    if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&t, r.start, r.stop) != hipSuccess)
      return fail(c, BSR_ERR_HIP, "bsr_profile_end: %s", hipGetErrorString(hipGetLastError()));
    ms[r.cls] += t;
    flops[r.cls] += r.flops;
    launches[r.cls] += 1;
  }
  c->prof_used = 0;
  return BSR_OK;
}

int32_t bsr_destroy(bsr_ctx* c) {
  if (c) {
    for (ProfRec& r : c->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    for (auto& p : c->pipe) { (void)hipEventDestroy(p.ready); (void)hipEventDestroy(p.free); }
  }
  delete c;
  return BSR_OK;
}

const char* bsr_last_error(const bsr_ctx* c) { return c ? c->err : g_err; }

}  // extern "C"
