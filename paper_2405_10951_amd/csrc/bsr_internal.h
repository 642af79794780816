// Internal declarations shared by the translation units of libbsr_hip: kernel launchers take raw
// device pointers and a stream, never allocate and never synchronise.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bsr {

typedef __bf16 bf16;

enum Act { ACT_NONE = 0, ACT_GELU = 1, ACT_GELU_BWD = 2 };

// C(m,n) = epilogue( sum_k A(m,k) * B(k,n) ), operands addressed through element strides so that
// one description covers X.W (forward), dY.W^T (Eq. 2) and X^T.dY (Eq. 4).
struct GemmDesc {
  const void* A = nullptr; int64_t a_rs = 0, a_cs = 0;   // A(m,k) = A[m*a_rs + k*a_cs]
  const void* B = nullptr; int64_t b_rs = 0, b_cs = 0;   // B(k,n) = B[k*b_rs + n*b_cs]
  void* C = nullptr;       int64_t ldc = 0;              // C(m,n) = C[row(m)*ldc + n]
  int M = 0, N = 0, K = 0;
  bool in_f32 = false;                                   // A and B are fp32 (else bf16)
  bool out_f32 = false;                                  // C is fp32 (else bf16)
  const float* bias = nullptr;                           // [N], added before the activation
  int act = ACT_NONE;
  void* aux = nullptr;       // ACT_GELU: if set, receives the pre-activation u (dtype of C, ld = ldc)
                             // ACT_GELU_BWD: the stored u; C = acc * GELU'(u)
  const void* res = nullptr; // residual added last (dtype of C, ld = ldc, same row mapping)
  int remap_np = 0;          // > 0 (patch embedding): row(m) = m + m / np + 1, and pos[(m % np + 1), n]
  const float* pos = nullptr;//   is added; rows of CLS tokens are left untouched
  float* bsum = nullptr;     // weight-gradient form only (A^T and B share the token index k): if set,
                             //   receives sum_k B(k,n), the bias gradient of the same layer
  // Grouped form (expert FFNs over routed tokens): the token rows are cut into `groups` consecutive
  // ranges, range e = [grp_off[e], grp_off[e+1]) (device array), each with its own weight matrix.
  //   forward / dgrad: rows of A and C in range e use B + e*b_gs and bias + e*bias_gs
  //   wgrad:           the contraction runs over range e only and fills C + e*c_gs, bsum + e*bsum_gs
  const int32_t* grp_off = nullptr;
  int groups = 0;
  int64_t b_gs = 0, bias_gs = 0, c_gs = 0, bsum_gs = 0;
  // LayerNorm folded into the linear layer that follows it (frozen weights; NT form, K a multiple of 64):
  //   LN(x) W^T + b = rstd (x W'^T - mean colsum(W')) + b',   W' = W diag(gamma),  b' = b + W beta.
  // With ln_colsum set ([N], sum_k W'(n,k)), A is the raw x, B is W', bias is b'; the kernel takes mean and
  // 1/std of every row of A from the tiles it streams anyway and applies the formula in its epilogue.
  const float* ln_colsum = nullptr;
  float ln_eps = 0.f;
};

// ---- generic (any shape, fp32 or bf16 storage, fp32 arithmetic) ---------------------------------
void gemm_generic(const GemmDesc& g, hipStream_t s);
void attn_fwd_generic(const void* qkv, int B, int T, int H, int d, bool f32, void* out, float* lse,
                      float* cls_prob, hipStream_t s);
void attn_bwd_generic(const void* qkv, const void* out, const void* dout, const float* lse, int B,
                      int T, int H, int d, bool f32, float* delta, void* dqkv, hipStream_t s);

// W'(n,k) = bf16(w[k,n] gamma[k]) as [out][in], colsum[n] = sum_k W'(n,k), bias_out[n] = bias[n] + sum_k beta[k] w[k,n]
// (w is the fp32 master matrix [in][out]; in a multiple of 8)
void ln_fold_weights(const float* w, const float* bias, const float* gamma, const float* beta, int in, int out,
                     bf16* w_t, float* colsum, float* bias_out, hipStream_t s);

// ---- bf16 MFMA paths --------------------------------------------------------------------------
bool gemm_mfma_supported(const GemmDesc& g);
// splitk_ws: fp32 scratch for the partial sums of split-K weight gradients (may be null: no split)
// A split-K weight gradient leaves fp32 partials that one more pass has to add up.  With a chain, that
// pass does not get a launch of its own: it rides as extra workgroups on the NEXT weight-gradient launch
// (which works on the other half of the workspace), and gemm_tn_flush runs the last one.  The sums and
// their order are the same either way.
struct TnReduce {
  const float* partial = nullptr;   // [splits][n]
  int64_t n = 0;
  int splits = 0;
  float* out = nullptr;
  const float* bpartial = nullptr;  // [splits][nb] column sums (bias gradient), may be null
  int nb = 0;
  float* bout = nullptr;
};
struct TnChain {
  TnReduce pending;                 // pending.splits > 0: a reduction is waiting
  int slot = 0;                     // workspace half the next split launch writes
};
// tile: one of gemm_nt_tile_id() for the NT kernel (ignored by the others), 0 = the built-in model chooses
void gemm_mfma(const GemmDesc& g, float* splitk_ws, size_t splitk_ws_floats, hipStream_t s, int tile = 0,
               TnChain* chain = nullptr);
void gemm_tn_flush(TnChain* chain, hipStream_t s);
// input gradient (NT) + weight gradient (TN) of one layer, in one launch when the NT tile shape allows it
void gemm_mfma_pair(const GemmDesc& nt, const GemmDesc& tn, float* splitk_ws, size_t splitk_ws_floats, hipStream_t s,
                    int tile = 0, TnChain* chain = nullptr);
// the block-tile shapes the NT kernel is instantiated for, and whether a GEMM is free to take any of them
int gemm_nt_tile_count();
int gemm_nt_model_tile(int M, int N, int K);   // the built-in model's choice
int gemm_nt_tile_id(int i);
size_t gemm_nt_tile_lds_bytes(int id);          // dynamic LDS a workgroup of that shape holds
bool gemm_nt_tile_is_free(const GemmDesc& g);
size_t gemm_splitk_ws_floats(int dim, int mlp_hidden);

bool attn_mfma_supported(int T, int d);
void attn_fwd_mfma(const void* qkv, int B, int T, int H, void* out, float* lse, float* cls_prob, hipStream_t s);
void attn_bwd_mfma(const void* qkv, const void* out, const void* dout, const float* lse, int B, int T, int H,
                   float* delta, void* dqkv, hipStream_t s);

// ---- row-wise / element-wise kernels ------------------------------------------------------------
void layernorm_fwd(const void* x, int64_t M, int D, const float* gamma, const float* beta, float eps,
                   bool f32, void* y, float* mean, float* rstd, hipStream_t s);
// dx = res + LN'(dy) (res may be null; dx may be null to skip it)
// Token gather (x_kept[b,0] = x[b,0], x_kept[b,1+i] = x[b,1+idx[b,i]]; x is [B,T,D]) and the LayerNorm of the
// gathered rows in one pass.  Returns false (nothing done) for shapes the one-pass kernel does not take.
bool gather_layernorm_fwd(const void* x, const int32_t* idx, int B, int T, int k, int D, const float* gamma,
                          const float* beta, float eps, bool f32, void* x_kept, void* y, float* mean, float* rstd,
                          hipStream_t s);
void layernorm_bwd_dx(const void* dy, const void* x, const float* mean, const float* rstd,
                      const float* gamma, const void* res, int64_t M, int D, bool f32, void* dx,
                      hipStream_t s);
// dgamma[j] = sum_m dy*xhat, dbeta[j] = sum_m dy ; partial is scratch of colsum_partial_floats()
void layernorm_bwd_params(const void* dy, const void* x, const float* mean, const float* rstd,
                          int64_t M, int D, bool f32, float* partial, float* dgamma, float* dbeta,
                          hipStream_t s);
// both of the above; one pass over dy and x on the bf16 path
void layernorm_bwd(const void* dy, const void* x, const float* mean, const float* rstd, const float* gamma,
                   const void* res, int64_t M, int D, bool f32, void* dx, float* partial, float* dgamma,
                   float* dbeta, hipStream_t s);
// out[j] = sum_m a[m*ld + j]
void colsum(const void* a, int64_t M, int N, int64_t ld, bool f32, float* partial, float* out,
            hipStream_t s);
size_t colsum_partial_floats(int64_t M, int N);
// The LayerNorm backward of several layers with one final reduction for all of them: each call of
// layernorm_bwd_deferred writes dx and its workgroup partials of dgamma / dbeta into `partial` (its own
// buffer of ln_deferred_partial_floats(D) floats, kept until the reduction) and adds an entry to the
// table; ln_deferred_finish adds the partials of every entry in one launch.  Returns false (nothing
// done) when the shape is not one the one-pass kernel takes: then use layernorm_bwd.
constexpr int LN_DEFER_MAX = 32;
struct LnDeferEntry { const float* partial; float* dgamma; float* dbeta; int blocks; };
struct LnDeferTable { LnDeferEntry e[LN_DEFER_MAX]; int count = 0; int D = 0; };
size_t ln_deferred_partial_floats(int D);
bool layernorm_bwd_deferred(const void* dy, const void* x, const float* mean, const float* rstd, const float* gamma,
                            const void* res, int64_t M, int D, bool f32, void* dx, float* partial, float* dgamma,
                            float* dbeta, LnDeferTable& t, hipStream_t s);
void ln_deferred_finish(LnDeferTable& t, hipStream_t s);

// cls given: also writes the class-token rows x[b, 0, :] = cls + pos[0] of the token tensor x [B, T, D] (same launch
// on the 16-byte path)
void patchify(const void* img, int B, int C, int S, int P, bool f32, void* out, hipStream_t s,
              const float* cls = nullptr, const float* pos = nullptr, int T = 0, int D = 0, void* x = nullptr);
void write_cls_rows(const float* cls, const float* pos, int B, int T, int D, bool f32, void* x,
                    hipStream_t s);
void cls_head_mean(const float* cls_prob, int B, int H, int T, float* scores, hipStream_t s);
void topk_select(const float* scores, int B, int n, int k, int32_t* idx, hipStream_t s);
// head mean of the CLS softmax rows [B,H,T] -> scores [B,T-1], then the selection, in one launch
void topk_select_from_cls(const float* cls_prob, int B, int H, int T, int k, float* scores, int32_t* idx,
                          hipStream_t s);
// y rows [CLS; kept] per image; T_out: rows per image of y (0: k + 1)
void gather_tokens(const void* x, const int32_t* idx, int B, int T, int k, int D, bool f32, void* y,
                   hipStream_t s, int T_out = 0);
// Sec. 4.1: row k+1 of y (pitch k+2) = importance-weighted average of the dropped tokens; fw [B,T-1]
// receives the weights (0 for kept tokens)
void fuse_dropped(const void* x, const float* scores, const int32_t* idx, int B, int T, int k, int D, bool f32,
                  float* fw, void* y, hipStream_t s);
// fw != null: dy has rows [CLS; kept; fused] and dropped tokens get fw times the fused token's gradient
void scatter_tokens(const void* dy, const int32_t* idx, int B, int T, int k, int D, bool f32,
                    void* dx, hipStream_t s, const float* fw = nullptr);
// Classification head, forward and backward, in two launches (class-token LayerNorm, logits, mean
// cross-entropy, and the gradients of the head, of the final LayerNorm and of the last block's output
// dx [B,Tl,D], whose non-class rows are set to zero).  xhat, z, dz: [B,D] fp32 scratch; logits, dlogits:
// [B,C] fp32; loss_rows [B].  Needs head_lds_bytes(D, C) of LDS per workgroup (caller checks <= 64 KB).
size_t head_lds_bytes(int D, int C);
void head_fwd_bwd(const void* x, int B, int Tl, int D, int C, bool f32, const float* gamma, const float* beta, float eps,
                  const float* w_head, const float* b_head, const int32_t* labels, float* xhat, float* z, float* logits,
                  float* dlogits, float* dz, float* loss_rows, void* dx, float* dw, float* db, float* dgamma, float* dbeta,
                  float* loss, hipStream_t s);
void extract_cls(const void* x, int B, int T, int D, bool f32, float* out, hipStream_t s);
void place_cls_grad(const float* dxc, int B, int T, int D, bool f32, void* dx, hipStream_t s);
void cross_entropy(const float* logits, const int32_t* labels, int B, int C, float* loss_rows,
                   float* dlogits, float* loss, hipStream_t s);
void mean_sq_loss(const void* x, int64_t n, bool f32, float* partial, float* loss, void* dx,
                  hipStream_t s);
size_t mean_sq_partial_floats();

// ---- mixture-of-experts FFN (bf16) ----------------------------------------------------------------
constexpr int MOE_MAX_EXPERTS = 32, MOE_MAX_TOPK = 4;
// from the router logits [M,E]: the K largest (ties: lower index) in descending order, or the forced
// choice; gates = softmax over the K selected logits
void moe_topk(const float* logits, int64_t M, int E, int K, const int32_t* forced, int32_t* experts, float* gates,
              hipStream_t s);
// bf16 copy of w_router [D,E] stored [E,D]
void moe_router_copy(const float* w_router, int D, int E, void* t_router, hipStream_t s);
// stable counting sort of the (token, slot) pairs by expert: off[E+1], pos[t*K+s] = row of the pair
// in expert order, perm_tok[row] = t
void moe_sort(const int32_t* experts, int64_t M, int E, int K, int32_t* off, int32_t* pos, int32_t* perm_tok,
              hipStream_t s);
// y[r,:] = x[src[r],:]   (rows of D bf16, D % 8 == 0)
void moe_gather_rows(const void* x, const int32_t* src, int64_t rows, int D, void* y, hipStream_t s);
// x_out[t,:] = res[t,:] + sum_s gates[t,s] * y[pos[t,s],:]   (y: fp32 expert outputs)
void moe_combine(const void* y, const int32_t* pos, const float* gates, const void* res, int64_t M, int D, int K,
                 void* x_out, hipStream_t s);
// backward of moe_combine w.r.t. y and the gates: dy[pos[t,s],:] = gates[t,s] * dx[t,:];
// dgate_s = <dx[t], y[pos[t,s]]>; dsel[t,s] = gates_s (dgate_s - sum_j gates_j dgate_j) (fp32): the gradient at
// the K selected router logits of token t (the other logits get none)
void moe_combine_bwd(const void* dx, const void* y, const int32_t* pos, const int32_t* experts, const float* gates,
                     int64_t M, int D, int E, int K, void* dy, float* dsel, hipStream_t s);
// dW_r[D,E] (fp32) = h^T dlogits with dlogits[t, experts[t,s]] = dsel[t,s] kept in fp32; partial: scratch of
// moe_router_wgrad_partial_floats(D, E) floats; sums in a fixed order
size_t moe_router_wgrad_partial_floats(int D, int E);
void moe_router_wgrad(const void* h, const int32_t* experts, const float* dsel, int64_t M, int D, int E, int K,
                      float* partial, float* dw, hipStream_t s);
// dh[t,:] = sum_s dxg[pos[t,s],:] + sum_s dsel[t,s] * w_router[:, experts[t,s]]
void moe_unpermute_bwd(const void* dxg, const int32_t* pos, const int32_t* experts, const float* dsel,
                       const float* w_router, int64_t M, int D, int E, int K, void* dh, hipStream_t s);

// Update rule of the optimiser kernels.  SGD: g' = g + wd w; mu > 0: m = mu m + g', w -= lr m; else
// w -= lr g'.  AdamW: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2; w -= lr ((m/bc1) / (sqrt(v/bc2) + eps)
// + wd w) with bc = 1 - b^t computed on the host.
enum { OPT_SGD = 0, OPT_ADAMW = 1 };
struct OptArgs { int kind = OPT_SGD; float lr = 0.f, mu = 0.f, wd = 0.f, b1 = 0.f, b2 = 0.f, eps = 0.f, bc1 = 1.f, bc2 = 1.f; };

// A table of weight matrices handled by one launch: bf16 copies (straight and / or transposed) of
// each, optionally after an optimiser update.  The table travels as a kernel argument (< 4 KB).
constexpr int MAT_TABLE_MAX = 56;
struct MatEntry { float* w; const float* g; float* m; float* v2; bf16* s; bf16* t; int rows, cols, tile_start; };
struct MatTable { MatEntry e[MAT_TABLE_MAX]; int count = 0; int total_tiles = 0; };
void matrix_table_add(MatTable& t, float* w, const float* g, float* m, float* v2, int rows, int cols, bf16* straight,
                      bf16* transposed);
void matrix_table_run(const MatTable& t, bool update, const OptArgs& o, hipStream_t s);

// The same update on up to SGD_TABLE_MAX tensors without bf16 copies in one launch
constexpr int SGD_TABLE_MAX = 96;
struct SgdEntry { float* w; const float* g; float* m; float* v2; int64_t n; };
struct SgdTable { SgdEntry e[SGD_TABLE_MAX]; };
void sgd_table(const SgdTable& t, int count, const OptArgs& o, hipStream_t s);
// fp32 C[M,N] = A.B (+bias) for tiny problems (the classification head)
void gemm_small_f32(const GemmDesc& g, hipStream_t s);

}  // namespace bsr
