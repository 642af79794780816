/*
 * bsr.h — C ABI of the MI355X (gfx950) library for one Block Selective Reprogramming (BSR)
 * fine-tuning step of a Vision Transformer (arxiv 2405.10951).
 *
 * One step is:  bsr_forward_frozen  ->  bsr_train_blocks_fwd_bwd  ->  bsr_sgd_step.
 *
 * Conventions for every entry point
 *   - Plain C.  Every function returns a bsr status (0 = BSR_OK, negative = error); nothing throws
 *     or aborts.  bsr_last_error() gives a text for the last failure on a context.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory.  The library never allocates or frees device memory.  The calls of a step
 *     (bsr_forward_frozen, bsr_select_tokens, bsr_train_blocks_fwd_bwd, bsr_sgd_step, bsr_adamw_step,
 *     bsr_pipeline_step), bsr_init and the single-layer calls never wait for the device: all kernels are
 *     enqueued on the `stream` argument (a hipStream_t passed as void*; NULL is the default stream)
 *     and the call returns.  Three set-up / measurement calls DO block until their streams have
 *     drained, because they read event times: bsr_autotune, bsr_autotune_overlapped and
 *     bsr_profile_end.  The library owns the small host-side context and the HIP events it creates
 *     for those three calls and for bsr_pipeline_step, all released by bsr_destroy().
 *   - Device pointers must be 16-byte aligned.  A NULL or misaligned required pointer gives
 *     BSR_ERR_INVALID_ARG before anything is launched.
 *   - Activations ("act" below) have the configured compute dtype: bf16 (2 bytes) or fp32.
 *     Parameters, gradients and momenta are always fp32.  Linear weights are row-major [in, out].
 *   - Block and drop indices are 0-based.  Token tensors are row-major [B, T, D], token 0 = CLS.
 *   - Calls on one context are not thread-safe (one host thread at a time) and must be issued on one
 *     stream or be ordered by the caller, with one exception made for pipelining: bsr_forward_frozen of
 *     the next batch may run on a second stream beside bsr_train_blocks_fwd_bwd and the optimizer step
 *     of the current batch.  The frozen prefix reads only frozen weights (Fig. 2) and shares no device
 *     scratch with the other two; the caller orders the producer and the consumer of each x_out buffer
 *     with events (two such buffers make a pipeline).  Different contexts are independent.
 */
#ifndef BSR_H_
#define BSR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BSR_MAX_BLOCKS 16

enum {
  BSR_OK = 0,
  BSR_ERR_INVALID_ARG = -1,         /* NULL / misaligned pointer, B out of range, ...            */
  BSR_ERR_BAD_CONFIG = -2,          /* inconsistent bsr_config                                    */
  BSR_ERR_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes < bsr_workspace_bytes()                    */
  BSR_ERR_UNSUPPORTED_ARCH = -4,    /* current device is not gfx950                               */
  BSR_ERR_HIP = -5                  /* a HIP call failed; text in bsr_last_error()                */
};

enum { BSR_BF16 = 0, BSR_FP32 = 1 };          /* activation / compute dtype                       */
enum { BSR_LOSS_CE = 0, BSR_LOSS_MEAN_SQ = 1 }; /* cross-entropy on the head, or mean of squared
                                                   outputs of the last block (no head)            */

typedef struct bsr_ctx bsr_ctx;

/* The model and the BSR layout (Fig. 2; Sec. 4.3 Discussion 3): which blocks drop tokens, how many
 * patch tokens survive each drop, and from which block on weights are trained. */
typedef struct {
  int32_t image_size, patch_size, in_chans; /* 224, 16, 3.  image_size == 0: no stem, the input of
                                               bsr_forward_frozen already is tokens [B,tokens_in,D] */
  int32_t tokens_in;                        /* T of a token input; ignored when image_size > 0     */
  int32_t dim, heads, mlp_hidden, depth;    /* L (=D), H, D_ffn, number of encoder blocks          */
  int32_t num_classes;                      /* 0: no head (use BSR_LOSS_MEAN_SQ)                   */
  int32_t max_batch;                        /* workspace is sized for this many images             */
  int32_t n_drop;                           /* number of token drop locations                      */
  int32_t drop_blocks[BSR_MAX_BLOCKS];      /* strictly ascending block indices                    */
  int32_t keep_k[BSR_MAX_BLOCKS];           /* patch tokens kept at each drop (CLS is kept on top).
                                               If all entries are 0 they are derived from
                                               keep_ratio as floor(keep_ratio * n + 1e-9) on the
                                               current patch count n (Sec. 4.1: K follows from the
                                               drop rate; keep_ratio = 1 - drop rate)              */
  float keep_ratio;                         /* 0 < r <= 1; only read when keep_k is all 0          */
  int32_t first_trainable_block;            /* blocks [first, depth), the final LayerNorm and the
                                               head are trained; blocks before it are frozen and
                                               keep no activations (Fig. 2, Eq. 8)                 */
  int32_t dtype;                            /* BSR_BF16 or BSR_FP32                                */
  int32_t loss;                             /* BSR_LOSS_CE or BSR_LOSS_MEAN_SQ                     */
  float ln_eps;                             /* LayerNorm epsilon; 0 means 1e-6                     */
  /* Mixture-of-experts FFN (Sec. 5.3: the FFN of chosen blocks is replaced by expert MLPs of which
   * a router activates a few per token and adds their outputs).  bf16 only. */
  int32_t n_experts;                        /* E, 0: every FFN is dense; at most 32                */
  int32_t moe_top_k;                        /* K experts active per token, 1..4                    */
  int32_t n_moe;                            /* number of mixture-of-experts blocks                 */
  int32_t moe_blocks[BSR_MAX_BLOCKS];       /* their block indices, strictly ascending             */
  /* Trainable set as a list (the paper's default layout trains every fourth block, Sec. 5 /
   * Table 7).  n_trainable == 0: blocks [first_trainable_block, depth) are trained.  Otherwise
   * first_trainable_block is ignored and taken as trainable_blocks[0]; a block after it that is not
   * listed is frozen but lies in the gradient path: it keeps the inputs of its non-linear layers and
   * only passes the input gradient on (Eq. 2, Eq. 3), it gets no weight gradient and its entries in
   * the gradient / momentum tables may be NULL. */
  int32_t n_trainable;
  int32_t trainable_blocks[BSR_MAX_BLOCKS]; /* strictly ascending block indices                    */
  /* Sec. 4.1 merges the tokens ranked unimportant into one token for the FFN that follows.  1: a drop
   * location that drops at least one token appends one more token after the kept ones, the
   * importance-weighted average of the dropped tokens (weights = their scores divided by the sum of
   * the dropped scores; constants of the backward pass, like the kept indices).  It is a patch token
   * of the following blocks: the next drop location ranks it with the others, so the schedule becomes
   * n -> K + 1 patch tokens per drop.  0: dropped tokens are discarded. */
  int32_t fuse_dropped;
  /* 1 (bf16 only): a LayerNorm of the frozen prefix whose output feeds one dense product only is not run as a
   * kernel of its own; the qkv / fc1 product behind it reads the residual stream and applies the row statistics
   * itself (see bsr_ln_linear_fold).  Same result up to rounding; saves launches, costs time inside the products.
   * 0: every LayerNorm is its own kernel. */
  int32_t fold_frozen_layernorm;
} bsr_config;

/* Tables of device pointers, one per tensor (fp32).  The same struct describes parameters,
 * gradients and momenta.  Shapes: ln*_g, ln*_b, b_proj, b_fc2 [D]; w_qkv [D,3D] with columns
 * [q|k|v], each split into H heads of D/H; b_qkv [3D]; w_proj [D,D]; w_fc1 [D,F]; b_fc1 [F];
 * w_fc2 [F,D]; w_patch [C*P*P, D] with rows in (channel, row, column) order of a patch;
 * b_patch, cls [D]; pos [T,D]; lnf_g, lnf_b [D]; w_head [D,classes]; b_head [classes].
 * A mixture-of-experts block holds one FFN per expert and a router: w_router [D,E] (no bias),
 * w_fc1 [E,D,F], b_fc1 [E,F], w_fc2 [E,F,D], b_fc2 [E,D]; w_router is NULL in dense blocks. */
typedef struct {
  void *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_proj, *b_proj, *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
  void *w_router;
} bsr_block_params;

typedef struct {
  void *w_patch, *b_patch, *cls, *pos;
  bsr_block_params blocks[BSR_MAX_BLOCKS];
  void *lnf_g, *lnf_b, *w_head, *b_head;
} bsr_params;

/*
 * Token schedule of a configuration (host only, touches no GPU).  Sec. 4.1 / Sec. 4.3
 * Discussion 3: a drop location ranks all incoming tokens in its MHSA and hands K of them to its
 * FFN, e.g. N/2, N/4, N/8 at drop rate 0.5.
 *   keep_k_out   host [n_drop]  patch tokens kept at each drop, may be NULL
 *   tokens_attn  host [depth]   tokens (CLS included) seen by the MHSA of each block, may be NULL
 *   tokens_mlp   host [depth]   tokens seen by the FFN of each block, may be NULL
 * Errors: BSR_ERR_INVALID_ARG (cfg NULL), BSR_ERR_BAD_CONFIG.
 */
int32_t bsr_token_schedule(const bsr_config* cfg, int32_t* keep_k_out, int32_t* tokens_attn,
                           int32_t* tokens_mlp);

/* Bytes of device workspace bsr_init needs for this configuration (host only). */
int32_t bsr_workspace_bytes(const bsr_config* cfg, size_t* bytes_out);

/*
 * Bytes of activations the blocks in the gradient path keep between their forward and backward
 * pass (host only, touches no GPU), per block and by kind, for `batch` images.  The counts are the
 * unpadded sizes of the very buffers the workspace layout reserves, so the report cannot drift
 * from what the library stores.  Sec. 3.2 / Table 1 list what the non-linear layers of a block
 * need (Q, K, V, the softmax input, the GELU input); a block whose weights are trained also keeps
 * the inputs of its linear layers (Eq. 4).  This library keeps one log-sum-exp per attention row
 * in place of the [H,T,T] softmax input and recomputes the probabilities in the backward pass.
 *   qkv        Q, K, V                               [B,T,3D]  act
 *   softmax    per-row log-sum-exp                   [B,H,T]   fp32
 *   attn_out   attention output O (softmax backward reads rowsum(dO*O); the projection's input)
 *   gelu_in    FFN hidden pre-activation u           [B,T',F]  act  (x top-k in a mixture block)
 *   linear_in  LN1 output, LN2 output, GELU output: inputs of linears whose weights are trained
 *   residual   the tensors LayerNorm backward reads: x after MHSA (gathered at a drop location)
 *              and the block output (which is the next block's input)
 *   stats      LayerNorm mean / rstd, kept-token indices, fused-token weights
 *   moe        router logits, gates, expert choice, expert-major row copies and expert outputs
 *   total      sum of the above
 * Blocks before the first one in the gradient path report zeros: they store nothing.
 *   per_block  host [depth], may be NULL;  sum  host, one entry, may be NULL.
 * Errors: INVALID_ARG (cfg NULL, batch < 1 or > max_batch), BAD_CONFIG.
 */
typedef struct {
  uint64_t qkv, softmax, attn_out, gelu_in, linear_in, residual, stats, moe, total;
} bsr_saved_bytes;
int32_t bsr_saved_activation_bytes(const bsr_config* cfg, int32_t batch, bsr_saved_bytes* per_block,
                                   bsr_saved_bytes* sum);

/*
 * Create a context (the problem statement of Sec. 4.1: a pre-trained ViT, drop locations, drop
 * rate, trainable set).
 *   params     host struct of device fp32 pointers: the master weights.  The struct is copied; the
 *              tensors stay owned by the caller, must outlive the context and are updated in place
 *              by bsr_sgd_step.  Entries for parts the configuration lacks (stem, head) may be NULL.
 *   workspace  device, 256-byte aligned, workspace_bytes >= bsr_workspace_bytes(); owned by the
 *              caller, used by the context until bsr_destroy.
 * In bf16 mode this enqueues the kernels that build bf16 copies of the weight matrices.
 * Errors: INVALID_ARG, BAD_CONFIG, WORKSPACE_TOO_SMALL, UNSUPPORTED_ARCH, HIP.
 */
int32_t bsr_init(const bsr_config* cfg, const bsr_params* params, void* workspace,
                 size_t workspace_bytes, void* stream, bsr_ctx** ctx_out);

/* After the caller has overwritten master weights by other means than bsr_sgd_step (loading a
 * checkpoint), rebuild the bf16 copies. */
int32_t bsr_refresh_weights(bsr_ctx* ctx, void* stream);

/*
 * Frozen prefix (Fig. 2; Sec. 4.1): stem (Sec. 3.1) and blocks [0, first_trainable_block), forward
 * only, nothing kept for backward.  Drop locations inside the prefix rank patch tokens by the
 * head-averaged CLS row of the softmax attention map (Eq. 6) and pass CLS + the K best on to the
 * FFN of that block.
 *   input        device act: images [B,C,S,S], or tokens [B,tokens_in,D] when image_size == 0
 *   x_out        device act [B,T_f,D]: tokens entering block first_trainable_block
 *   kept_idx_out device int32, may be NULL: kept patch indices (ascending) of the prefix's drops,
 *                concatenated, drop i holding [B,keep_k[i]]
 *   scores_out   device fp32, may be NULL: importance scores of the prefix's drops, concatenated,
 *                drop i holding [B,n_i]
 *   forced_idx   device int32, may be NULL: use these indices (layout of kept_idx_out) instead of
 *                ranking — for parity tests against a reference that took the same decisions
 * Errors: INVALID_ARG (NULL input/x_out, B < 1 or > max_batch), HIP.
 */
int32_t bsr_forward_frozen(bsr_ctx* ctx, const void* input, int32_t B, void* x_out,
                           int32_t* kept_idx_out, float* scores_out, const int32_t* forced_idx,
                           void* stream);

/*
 * Token selection on its own (Sec. 4.1): the K largest of each row of cls_attn, ties to the lower
 * index, indices emitted ascending; then x_out[b,0] = x_in[b,0], x_out[b,1+i] = x_in[b,1+idx[b,i]].
 *   cls_attn device fp32 [B,n]   importance of the n patch tokens
 *   x_in     device act [B,n+1,D], may be NULL together with x_out (indices only)
 *   idx_out  device int32 [B,k]
 *   x_out    device act [B,k+1,D]
 * Limits: 0 <= k <= n <= 1024.  Errors: INVALID_ARG, HIP.
 */
int32_t bsr_select_tokens(bsr_ctx* ctx, const float* cls_attn, const void* x_in, int32_t B,
                          int32_t n, int32_t k, int32_t* idx_out, void* x_out, void* stream);

/*
 * Trainable blocks [first_trainable_block, depth) and the head: forward keeping what Eq. 2-5 need
 * (Sec. 3.2), loss, and backward down to the parameters of block first_trainable_block; the
 * gradient is not propagated into the frozen prefix (Fig. 2, Eq. 8).  Drop locations inside the
 * trainable range behave as in the prefix; kept indices are constants of the backward pass.
 *   x_in         device act [B,T_f,D] (output of bsr_forward_frozen); not modified
 *   labels       device int32 [B]; may be NULL with BSR_LOSS_MEAN_SQ
 *   loss_out     device fp32 scalar
 *   logits_out   device fp32 [B,classes], may be NULL
 *   x_final_out  device act [B,T_last,D], may be NULL: output of the last block
 *   grads        host struct of device fp32 pointers; every tensor of the trainable blocks, lnf_*
 *                and *_head must be non-NULL; each is overwritten with dLoss/dTensor
 *   kept_idx_out, scores_out, forced_idx: as in bsr_forward_frozen, for the drops in this range
 * Errors: INVALID_ARG, HIP.
 */
int32_t bsr_train_blocks_fwd_bwd(bsr_ctx* ctx, const void* x_in, const int32_t* labels, int32_t B,
                                 float* loss_out, float* logits_out, void* x_final_out,
                                 const bsr_params* grads, int32_t* kept_idx_out, float* scores_out,
                                 const int32_t* forced_idx, void* stream);

/*
 * Measured tile choice (set-up, not part of a step).  The tiled matrix-multiply kernel behind the
 * linear layers comes in several block-tile shapes; which one is fastest for a launch depends on how
 * its tile count divides over the 256 compute units and on what surrounds it in the step.  This call
 * runs bsr_forward_frozen + bsr_train_blocks_fwd_bwd on the given batch once per shape (twice over),
 * times every such launch with HIP events in its place in the step, and from then on gives each
 * launch of a batch of the same size B its fastest shape; other batch sizes keep the built-in cost
 * model.  Every shape adds up an output element in the same order, so results do not change by a
 * bit.  Arguments as for the two entry points (x_frozen is the x_out of the first and the x_in of
 * the second; loss_out and grads are overwritten as by a normal step).
 *   launches_out  host, may be NULL: number of launches that now have a measured choice
 *   changed_out   host, may be NULL: how many of them differ from the cost model's choice
 * BLOCKS until the stream has drained (it reads event times).  Not capturable into a graph.
 * Errors: as the two entry points; HIP.
 */
int32_t bsr_autotune(bsr_ctx* ctx, const void* input, const int32_t* labels, int32_t B, void* x_frozen,
                     float* loss_out, const bsr_params* grads, int32_t* launches_out, int32_t* changed_out,
                     void* stream);
/*
 * The tile choice for the two-stream schedule (see the rule on concurrent calls at the top).  Shapes
 * that are fastest alone on the GPU are not the ones that share it best, and side by side a launch
 * cannot be judged by its own time, so this call times short runs of the pipeline itself: six
 * iterations, the frozen prefix on `stream` (writing x_side, device act [B,T_f,D], a second buffer) one
 * iteration ahead of the trainable part on `side_stream` (reading x_frozen), ordered as
 * bsr_pipeline_step orders them, every launch with the shape under test; in place of the optimizer
 * step the bf16 copies of the trainable weights are rebuilt (no weight changes).  Three runs per shape,
 * over the shapes whose workgroups leave room for a second one on a compute unit.  The fastest shape
 * is then used for every launch of a batch of size B.  The choice replaces the one of bsr_autotune (a
 * context holds one).  BLOCKS until both streams have drained.
 * Errors: as bsr_autotune; INVALID_ARG for a missing second buffer or stream; BAD_CONFIG when the
 * model has no frozen prefix.
 */
int32_t bsr_autotune_overlapped(bsr_ctx* ctx, const void* input, const int32_t* labels, int32_t B, void* x_frozen,
                                void* x_side, float* loss_out, const bsr_params* grads, int32_t* launches_out,
                                int32_t* changed_out, void* stream, void* side_stream);

/*
 * The tile choices a context holds after bsr_autotune / bsr_autotune_overlapped, for inspection and reports (host
 * only).  part 0: the launches of bsr_forward_frozen in launch order, part 1: those of bsr_train_blocks_fwd_bwd
 * (a backward launch carries the input gradient named here and, fused with it, the weight gradient of its layer).
 *   rows, out, in  the product: rows x in times in x out      tile  shape id (see bsr_gemm_tile_shapes)
 *   microseconds   what bsr_autotune measured for that shape at that launch (0 after bsr_autotune_overlapped,
 *                  which times whole passes)
 * Returns the number of launches of that part (0 without a choice or with bad arguments); writes at most max.
 */
typedef struct { int32_t rows, out, in, tile; float microseconds; } bsr_tile_choice;
int32_t bsr_tile_choices(const bsr_ctx* ctx, int32_t part, bsr_tile_choice* choices_out, int32_t max);

/*
 * Routing of the mixture-of-experts blocks (Sec. 5.3), for tests and inspection.  Per token the K
 * experts with the largest router logits (logits = LN2(x) . w_router; ties: lower expert index) are
 * active, ordered by descending logit, and weighted by the softmax over those K logits; the choice
 * is a constant for the backward pass.  The three device pointers (each may be NULL) are remembered
 * by the context and used by every later bsr_forward_frozen / bsr_train_blocks_fwd_bwd call until
 * they are replaced; all are laid out block after block over the mixture-of-experts blocks in
 * ascending order, block l holding B * tokens_mlp[l] rows:
 *   forced_experts     int32 [rows, K]   use this choice instead of the ranking (gates still come
 *                                        from the logits); values must lie in 0..E-1, distinct per row
 *   experts_out        int32 [rows, K]   receives the choice
 *   router_logits_out  fp32  [rows, E]   receives the router logits
 * Errors: INVALID_ARG (ctx NULL, misaligned pointer).
 */
int32_t bsr_moe_routing_io(bsr_ctx* ctx, const int32_t* forced_experts, int32_t* experts_out,
                           float* router_logits_out);

/*
 * SGD update of the trainable tensors (Sec. 5, "SGD optimizer"), in place on the master weights
 * given to bsr_init:  g' = g + weight_decay * w;  momentum > 0: m = momentum * m + g', w -= lr * m;
 * otherwise w -= lr * g'.  Also refreshes the bf16 copies the kernels read.
 *   grads     host struct of device fp32 pointers, as produced by bsr_train_blocks_fwd_bwd
 *   momenta   same layout, or NULL when momentum == 0; updated in place
 * Errors: INVALID_ARG, HIP.
 */
int32_t bsr_sgd_step(bsr_ctx* ctx, const bsr_params* grads, const bsr_params* momenta, float lr,
                     float momentum, float weight_decay, void* stream);

/*
 * One step of the two-stream pipeline (see the rule on concurrent calls at the top; Fig. 2: the frozen
 * prefix depends on frozen weights only).  Enqueues
 *   on stream_frozen: bsr_forward_frozen(input_next) -> x_next            (the NEXT batch)
 *   on stream_train:  bsr_train_blocks_fwd_bwd(x_cur, labels_cur) and bsr_sgd_step   (the CURRENT batch)
 * and the events that order them: the trainable part waits until the call that named its x_cur as
 * x_next has filled it, and a frozen prefix waits until the trainable part that last read its x_next
 * is done.  The context owns these events (one pair per x buffer it has seen, at most 8 buffers).
 *   input_next, x_next  as input / x_out of bsr_forward_frozen; both NULL on the last step
 *   x_cur               the x_next of an earlier call; NULL on the first call (which only primes)
 *   the other arguments as for bsr_train_blocks_fwd_bwd and bsr_sgd_step
 * A loop over batches 0..n-1 with two buffers x[2] is: step(in[0], x[0], NULL); then for i = 0..n-1:
 * step(i+1 < n ? in[i+1] : NULL, i+1 < n ? x[(i+1)%2] : NULL, x[i%2], labels[i]).  The results are
 * those of the three calls issued one after the other, bit for bit.  The caller joins both streams
 * before it reads loss, gradients or weights.
 * Errors: INVALID_ARG (x_cur never filled, one stream given twice, x_next == x_cur, ...), BAD_CONFIG
 * (no frozen prefix), HIP, and those of the three entry points.
 */
int32_t bsr_pipeline_step(bsr_ctx* ctx, const void* input_next, void* x_next, const void* x_cur,
                          const int32_t* labels_cur, int32_t B, float* loss_out, const bsr_params* grads,
                          const bsr_params* momenta, float lr, float momentum, float weight_decay,
                          void* stream_frozen, void* stream_train);

/*
 * AdamW update of the trainable tensors (the optimiser of the paper's DeiT-S runs, Sec. 5), in place:
 *   m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   w -= lr * ( (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps) + weight_decay * w )
 * (decoupled weight decay).  Also refreshes the bf16 copies the kernels read.
 *   grads, exp_avg, exp_avg_sq   host structs of device fp32 pointers (layout of bsr_params); the two
 *                                moment tables are updated in place and start at zero
 *   step                         1 for the first update
 * Errors: INVALID_ARG, HIP.
 */
int32_t bsr_adamw_step(bsr_ctx* ctx, const bsr_params* grads, const bsr_params* exp_avg,
                       const bsr_params* exp_avg_sq, float lr, float beta1, float beta2, float eps,
                       float weight_decay, int32_t step, void* stream);

/*
 * Single layers in bf16, as the step runs them (for kernel-level parity tests and benchmarks; no
 * context needed).  All pointers are device pointers, 16-byte aligned; bf16 tensors unless noted.
 * *used_mfma (host, may be NULL) is set to 1 when the MFMA kernel took the shape, 0 when the
 * generic kernel did.  Errors: INVALID_ARG, HIP.
 *
 * bsr_linear_forward: y[M,out] = act(x[M,in] . W + bias) (+ res), the a_{i+1} = W a_i + b of Sec. 3.2.
 *   w_t   bf16 copy of W stored [out,in]        bias  fp32 [out], may be NULL
 *   act   0: none, 1: exact-erf GELU            u_out [M,out], may be NULL: pre-activation (act = 1)
 *   res   [M,out], may be NULL: added last      y     [M,out]
 * bsr_linear_dgrad (Eq. 2): dx[M,in] = dy[M,out] . W^T, optionally times GELU'(u) element-wise.
 *   w_s   bf16 copy of W stored [in,out]        u     [M,in], may be NULL
 * tile (both): 0, or the id of a block-tile shape (bsr_gemm_tile_shapes) the MFMA kernel is to use; a shape that
 *   cannot take the product (a direct-to-LDS shape when `in` / `out` to contract over is not a multiple of 64)
 *   gives way to the default.  Every shape gives the same bits.  An unknown id: INVALID_ARG.
 * bsr_linear_wgrad (Eq. 4): dw[in,out] (fp32) = x[M,in]^T . dy[M,out], summed over all M rows.
 *   db         fp32 [out], may be NULL: the bias gradient, db[o] = sum over rows of dy[:,o], from the
 *              same launch when the MFMA kernel takes the shape (otherwise it needs the workspace)
 *   workspace  device fp32 scratch of workspace_floats elements, may be NULL.  With at least
 *              2*(in+1)*out floats the sum over M is split over several workgroups per output tile
 *              (partial sums are added in a fixed order: results are bit-reproducible).
 */
int32_t bsr_linear_forward(const void* x, int32_t M, int32_t in, int32_t out, const void* w_t,
                           const float* bias, int32_t act, void* u_out, const void* res, void* y,
                           int32_t tile, int32_t* used_mfma, void* stream);
int32_t bsr_linear_dgrad(const void* dy, int32_t M, int32_t in, int32_t out, const void* w_s,
                         const void* u, void* dx, int32_t tile, int32_t* used_mfma, void* stream);
int32_t bsr_linear_wgrad(const void* x, const void* dy, int32_t M, int32_t in, int32_t out, float* dw,
                         float* db, float* workspace, size_t workspace_floats, int32_t* used_mfma, void* stream);

/*
 * bsr_linear_wgrad for callers that cannot allocate device memory and have no workspace to hand over (code under
 * HIP graph capture, serving loops, harnesses that forbid hipMalloc): the same kernels and the same result, with
 * the split-K partial sums in an array that is part of the library itself (24 MiB of device memory on every GPU
 * the library runs on, held until the process ends).  The call allocates nothing and frees nothing.
 *   Limit: 2 * (in + 1) * out <= 6 Mi floats (two partial copies of dw and db; every matrix of ViT-B fits);
 *          beyond it the call returns BSR_ERR_INVALID_ARG and launches nothing.
 *   All calls on one GPU share that array and it keeps the last call's contents (no call needs it cleared: every
 *   partial sum that is read was written by the same call): calls that overlap on one GPU, on different streams
 *   or from different threads, race.  The first call on a device looks the array's address up
 *   (hipGetSymbolAddress); make that call outside a graph capture.
 * Errors: INVALID_ARG, HIP.
 */
int32_t bsr_linear_wgrad_static(const void* x, const void* dy, int32_t M, int32_t in, int32_t out, float* dw,
                                float* db, int32_t* used_mfma, void* stream);

/*
 * LayerNorm followed by a linear layer (the LN -> qkv and LN -> fc1 pairs of the pre-norm block, Sec. 3.1),
 * as the frozen prefix runs them in bf16: the LayerNorm is folded into the product,
 *   LN(x) W + b = rstd (x W' - mean c) + b',   W' = diag(gamma) W,   c = column sums of W',   b' = b + beta W,
 * and the product takes mean and 1/std of every row of x from the tiles it reads anyway.
 * bsr_ln_linear_fold (once per weight matrix):
 *   w [in,out] fp32 (the master layout), bias [out], gamma [in], beta [in]: device fp32, 16-byte aligned
 *   w_folded    device bf16 [out,in]: W' transposed, rounded once
 *   colsum      device fp32 [out]: sums of the rounded W' over `in`
 *   bias_folded device fp32 [out]
 * bsr_ln_linear_forward: y[M,out] (bf16) = act(LN(x) W + b) from x [M,in] bf16 and the three folded tensors.
 *   act   0: none, 1: exact-erf GELU
 *   tile  0: the library chooses the block-tile shape; otherwise one of the ids bsr_gemm_tile_shapes
 *         lists.  Every shape gives the same bits.
 * bsr_gemm_tile_shapes: writes up to `max` shape ids to ids (host) and returns how many there are.
 * Errors: INVALID_ARG (NULL / misaligned pointer, M < 1, `in` not a multiple of 64, `out` not a multiple of
 * 8, unknown tile id), HIP.
 */
int32_t bsr_ln_linear_fold(const float* w, const float* bias, const float* gamma, const float* beta, int32_t in,
                           int32_t out, void* w_folded, float* colsum, float* bias_folded, void* stream);
int32_t bsr_ln_linear_forward(const void* x, int32_t M, int32_t in, int32_t out, const void* w_folded,
                              const float* colsum, const float* bias_folded, float eps, int32_t act, void* y,
                              int32_t tile, void* stream);
int32_t bsr_gemm_tile_shapes(int32_t* ids, int32_t max);

/*
 * Multi-head softmax attention in bf16 (Eq. 1), as the step runs it.  qkv is [B,T,3*H*d] with
 * columns [q|k|v], head h owning columns h*d .. h*d+d-1 of each third.
 * bsr_attention_forward:
 *   out      [B,T,H*d] bf16: per-head Softmax(Q K^T / sqrt d) V, heads concatenated
 *   lse      fp32 [B,H,T], may be NULL: log-sum-exp of every score row (what backward keeps instead
 *            of the T x T softmax input of Table 1)
 *   cls_prob fp32 [B,H,T], may be NULL: softmax row of query 0, the CLS token (Eq. 6)
 * bsr_attention_backward (Eq. 3, 5): dqkv [B,T,3*H*d] bf16 from qkv, out, dout [B,T,H*d] and lse;
 *   delta    fp32 [B,H,T] scratch.
 * Limits: T <= 1024, d <= 256.  Errors: INVALID_ARG, HIP.
 */
int32_t bsr_attention_forward(const void* qkv, int32_t B, int32_t T, int32_t H, int32_t d, void* out,
                              float* lse, float* cls_prob, int32_t* used_mfma, void* stream);
int32_t bsr_attention_backward(const void* qkv, const void* out, const void* dout, const float* lse,
                               int32_t B, int32_t T, int32_t H, int32_t d, float* delta, void* dqkv,
                               int32_t* used_mfma, void* stream);

/*
 * Profiling mode, for measurement only.  Between bsr_profile_begin and bsr_profile_end every launch
 * of the classes below is bracketed by a pair of HIP events on the call's stream (created on first
 * use and kept by the context).  bsr_profile_end WAITS for the recorded work, then adds up, per
 * class, the elapsed milliseconds, the floating-point operations launched (2*M*N*K per GEMM; 4*T*T*d
 * per head for attention forward, 10*T*T*d backward) and the number of launches.
 *   ms, flops, launches  host arrays of BSR_PROF_CLASSES entries
 * Errors: INVALID_ARG, HIP.
 */
enum { BSR_PROF_GEMM = 0, BSR_PROF_ATTN_FWD = 1, BSR_PROF_ATTN_BWD = 2, BSR_PROF_CLASSES = 3 };
int32_t bsr_profile_begin(bsr_ctx* ctx);
int32_t bsr_profile_end(bsr_ctx* ctx, double* ms, double* flops, int32_t* launches);

/* Release the host-side context (no device memory is touched). */
int32_t bsr_destroy(bsr_ctx* ctx);

/* Text of the last error on this context ("" if none); valid until the next call on it.
 * With ctx == NULL: the text of the last failed bsr_init / bsr_workspace_bytes on this thread. */
const char* bsr_last_error(const bsr_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* BSR_H_ */
