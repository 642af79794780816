/*
 * CPU oracle for one Block Selective Reprogramming (BSR) fine-tuning step of a ViT.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is checked
 * against.  It shares no code, header, table or helper with the HIP path and must never be called
 * from it.  Compile twice: -DREAL=double (gradient checks, parity reference) and -DREAL=float.
 *
 * What it follows (arxiv 2405.10951):
 *   Sec. 3.1        ViT tokenisation, MHSA, Eq. 1 softmax attention, 2-layer GELU FFN
 *   Sec. 3.2        Eq. 2-5: input- and weight-gradients of linear and non-linear layers
 *   Sec. 4.1        Eq. 6 token importance = CLS row of the attention map; top-K kept at the
 *                   token drop locations, applied between MHSA and FFN (Sec. 4.3, Discussion 3)
 *   Fig. 2, Eq. 8   only the chosen blocks and the head are trained; no gradient flows beyond
 *                   the earliest trainable block
 *   Sec. 5          SGD update
 *   Sec. 5.3        mixture-of-experts FFN: a router activates a few of the expert MLPs per token
 *                   and their outputs are added (here: top-K by router logit, weighted by the
 *                   softmax over the K selected logits, as the workload definition states it)
 * Readings taken where the paper is silent: pre-norm blocks with biases; exact erf GELU; the
 * importance of a patch token is the mean over heads of the post-softmax CLS row; CLS is always
 * kept; ties go to the lower index; kept tokens stay in ascending original order; dropped tokens
 * are discarded; kept indices are constants for the backward pass.
 *
 * Every loop is the textbook definition of its operation.  Threads split rows (or images) only;
 * each output element is produced by one thread in a fixed order, so results do not depend on the
 * thread count.
 *
 * Pins: every function here is pinned by tests/test_oracle_*.py against numpy / torch-CPU library
 * routines, brute force, closed forms and finite differences.  Accuracy figures of the paper's
 * tables are "parity unpinned" (datasets and pre-trained weights are not available).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL double
#endif
typedef REAL real;

#define ORC_MAX_BLOCKS 16
#define ORC_LOSS_CE 0
#define ORC_LOSS_MEAN_SQ 1

typedef struct {
  int32_t image_size, patch_size, in_chans; /* image_size == 0: the input already is tokens      */
  int32_t tokens_in;                        /* T of a token input (used when image_size == 0)    */
  int32_t dim, heads, mlp_hidden, depth;
  int32_t num_classes;                      /* 0: no head, loss = mean of squared block outputs  */
  int32_t n_drop;
  int32_t drop_blocks[ORC_MAX_BLOCKS];      /* 0-based, ascending                                */
  int32_t keep_k[ORC_MAX_BLOCKS];           /* patch tokens kept at each drop location           */
  int32_t first_trainable;                  /* blocks [first_trainable, depth) + head are trained */
  int32_t loss;
  double ln_eps;
  int32_t n_experts, moe_top_k;             /* mixture-of-experts FFN: E experts, K active per token */
  int32_t moe_block[ORC_MAX_BLOCKS];        /* 1: the FFN of this block is a mixture of experts     */
  int32_t fuse_dropped;                     /* 1: the dropped tokens of a drop location are fused into
                                               one extra token instead of being discarded (Sec. 4.1) */
} orc_config;

typedef struct {
  real *ln1_g, *ln1_b, *w_qkv, *b_qkv, *w_proj, *b_proj, *ln2_g, *ln2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
  real* w_router; /* [D,E]; in a mixture-of-experts block w_fc1 [E,D,F], b_fc1 [E,F], w_fc2 [E,F,D], b_fc2 [E,D] */
} orc_block;

typedef struct {
  real *w_patch, *b_patch, *cls, *pos;
  orc_block blocks[ORC_MAX_BLOCKS];
  real *lnf_g, *lnf_b, *w_head, *b_head;
} orc_params;

int32_t orc_sizeof_real(void) { return (int32_t)sizeof(real); }

static real* ralloc(int64_t n) { return (real*)malloc(sizeof(real) * (size_t)(n > 0 ? n : 1)); }

/* ---------------------------------------------------------------- elementary layers (forward) */

/* LayerNorm over the last axis: y = (x - mean) / sqrt(var + eps) * gamma + beta, biased variance.
 * xhat and rstd are kept because the backward pass needs them (Eq. 5: non-linear layers' gradients
 * depend on their input). */
void orc_layernorm(const real* x, int64_t M, int32_t D, const real* gamma, const real* beta,
                   double eps, real* y, real* xhat, real* rstd) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    const real* xr = x + m * D;
    real mean = 0;
    for (int32_t j = 0; j < D; ++j) mean += xr[j];
    mean /= (real)D;
    real var = 0;
    for (int32_t j = 0; j < D; ++j) var += (xr[j] - mean) * (xr[j] - mean);
    var /= (real)D;
    real rs = (real)1 / (real)sqrt((double)var + eps);
    if (rstd) rstd[m] = rs;
    for (int32_t j = 0; j < D; ++j) {
      real xh = (xr[j] - mean) * rs;
      if (xhat) xhat[m * D + j] = xh;
      y[m * D + j] = xh * gamma[j] + beta[j];
    }
  }
}

/* y[M,N] = x[M,K] . w[K,N] + bias[N]   (a_{i+1} = W a_i + b of Sec. 3.2, weights stored [in,out]) */
void orc_linear(const real* x, int64_t M, int32_t K, const real* w, const real* bias, int32_t N,
                real* y) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m) {
    real* yr = y + m * N;
    for (int32_t n = 0; n < N; ++n) yr[n] = bias ? bias[n] : (real)0;
    for (int32_t k = 0; k < K; ++k) {
      real a = x[m * K + k];
      const real* wr = w + (int64_t)k * N;
      for (int32_t n = 0; n < N; ++n) yr[n] += a * wr[n];
    }
  }
}

/* Multi-head softmax attention, Eq. 1.  qkv is [B,T,3D] with columns [q|k|v], head h owning
 * columns h*d..h*d+d-1 of each third.  P[B,H,T,T] receives Softmax(Q K^T / sqrt(d)); out[B,T,D]
 * the per-head P V, heads concatenated. */
void orc_attention(const real* qkv, int32_t B, int32_t T, int32_t H, int32_t d, real* P, real* out) {
  const int32_t D = H * d;
  const real scale = (real)(1.0 / sqrt((double)d));
#pragma omp parallel for collapse(2) schedule(static)
  for (int32_t b = 0; b < B; ++b)
    for (int32_t h = 0; h < H; ++h) {
      const real* base = qkv + (int64_t)b * T * 3 * D;
      real* Pbh = P + ((int64_t)b * H + h) * T * T;
      for (int32_t i = 0; i < T; ++i) {
        const real* q = base + (int64_t)i * 3 * D + h * d;
        real* row = Pbh + (int64_t)i * T;
        real mx = -INFINITY;
        for (int32_t j = 0; j < T; ++j) {
          const real* k = base + (int64_t)j * 3 * D + D + h * d;
          real s = 0;
          for (int32_t e = 0; e < d; ++e) s += q[e] * k[e];
          s *= scale;
          row[j] = s;
          if (s > mx) mx = s;
        }
        real sum = 0;
        for (int32_t j = 0; j < T; ++j) {
          row[j] = (real)exp((double)(row[j] - mx));
          sum += row[j];
        }
        for (int32_t j = 0; j < T; ++j) row[j] /= sum;
        real* o = out + ((int64_t)b * T + i) * D + h * d;
        for (int32_t e = 0; e < d; ++e) o[e] = 0;
        for (int32_t j = 0; j < T; ++j) {
          const real* v = base + (int64_t)j * 3 * D + 2 * D + h * d;
          real p = row[j];
          for (int32_t e = 0; e < d; ++e) o[e] += p * v[e];
        }
      }
    }
}

/* GELU(u) = u/2 * (1 + erf(u / sqrt 2)) */
void orc_gelu(const real* u, int64_t n, real* g) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i)
    g[i] = (real)(0.5 * (double)u[i] * (1.0 + erf((double)u[i] * 0.70710678118654752440)));
}

/* Token importance (Eq. 6 read as the CLS row of the softmax map, averaged over heads):
 * a[b,j] = (1/H) sum_h P[b,h,0,1+j] for the n = T-1 patch tokens; the CLS column is not ranked. */
void orc_cls_scores(const real* P, int32_t B, int32_t H, int32_t T, real* a) {
  const int32_t n = T - 1;
  for (int32_t b = 0; b < B; ++b)
    for (int32_t j = 0; j < n; ++j) {
      real s = 0;
      for (int32_t h = 0; h < H; ++h) s += P[(((int64_t)b * H + h) * T + 0) * T + 1 + j];
      a[(int64_t)b * n + j] = s / (real)H;
    }
}

/* Indices of the k largest of a[0..n), ties to the lower index, returned in ascending order.
 * Token j is kept when fewer than k tokens precede it in the order (larger score, then lower
 * index). */
void orc_topk(const real* a, int32_t n, int32_t k, int32_t* idx) {
  int32_t out = 0;
  for (int32_t j = 0; j < n; ++j) {
    int32_t ahead = 0;
    for (int32_t i = 0; i < n; ++i)
      if (a[i] > a[j] || (a[i] == a[j] && i < j)) ++ahead;
    if (ahead < k) idx[out++] = j;
  }
}

/* y[b,0] = x[b,0];  y[b,1+i] = x[b,1+idx[b,i]]   (CLS kept, k patch tokens kept) */
void orc_gather(const real* x, int32_t B, int32_t T, int32_t D, const int32_t* idx, int32_t k,
                real* y) {
  for (int32_t b = 0; b < B; ++b) {
    memcpy(y + (int64_t)b * (k + 1) * D, x + (int64_t)b * T * D, sizeof(real) * D);
    for (int32_t i = 0; i < k; ++i)
      memcpy(y + ((int64_t)b * (k + 1) + 1 + i) * D,
             x + ((int64_t)b * T + 1 + idx[(int64_t)b * k + i]) * D, sizeof(real) * D);
  }
}

/* Fusion of the dropped tokens (Sec. 4.1: the unimportant tokens "are fused and passed onto the
 * subsequent FFN layer"; the rule is the importance-weighted average of the method the paper follows):
 *   f[b] = sum_{j not kept} a[b,j] x[b,1+j] / sum_{j not kept} a[b,j],   a = importance scores [B,n].
 * wts [B,n] receives the normalised weight of every dropped token (0 for kept ones); the weights are
 * constants of the backward pass, like the kept indices. */
void orc_fuse_dropped(const real* x, const real* a, int32_t B, int32_t T, int32_t D, const int32_t* idx,
                      int32_t k, real* wts, real* f) {
  const int32_t n = T - 1;
  for (int32_t b = 0; b < B; ++b) {
    real* w = wts + (int64_t)b * n;
    for (int32_t j = 0; j < n; ++j) w[j] = a[(int64_t)b * n + j];
    for (int32_t i = 0; i < k; ++i) w[idx[(int64_t)b * k + i]] = 0;
    real sum = 0;
    for (int32_t j = 0; j < n; ++j) sum += w[j];
    for (int32_t j = 0; j < n; ++j) w[j] /= sum;
    for (int32_t c = 0; c < D; ++c) {
      real v = 0;
      for (int32_t j = 0; j < n; ++j) v += w[j] * x[((int64_t)b * T + 1 + j) * D + c];
      f[(int64_t)b * D + c] = v;
    }
  }
}

/* Patch embedding + CLS + positional embedding (Sec. 3.1).  img [B,C,S,S]; patch p = row-major
 * grid index; a patch is flattened in (channel, row, column) order. */
void orc_stem(const real* img, int32_t B, int32_t C, int32_t S, int32_t Pp, int32_t D,
              const real* w_patch, const real* b_patch, const real* cls, const real* pos, real* x) {
  const int32_t G = S / Pp, N = G * G, T = N + 1, Kp = C * Pp * Pp;
#pragma omp parallel for schedule(static)
  for (int32_t b = 0; b < B; ++b) {
    real* flat = (real*)malloc(sizeof(real) * Kp);
    real* xb = x + (int64_t)b * T * D;
    for (int32_t j = 0; j < D; ++j) xb[j] = cls[j] + pos[j];
    for (int32_t gy = 0; gy < G; ++gy)
      for (int32_t gx = 0; gx < G; ++gx) {
        int32_t p = gy * G + gx;
        for (int32_t c = 0; c < C; ++c)
          for (int32_t r = 0; r < Pp; ++r)
            for (int32_t q = 0; q < Pp; ++q)
              flat[(c * Pp + r) * Pp + q] =
                  img[(((int64_t)b * C + c) * S + gy * Pp + r) * S + gx * Pp + q];
        real* xr = xb + (int64_t)(1 + p) * D;
        for (int32_t j = 0; j < D; ++j) xr[j] = b_patch[j];
        for (int32_t kk = 0; kk < Kp; ++kk) {
          real a = flat[kk];
          const real* wr = w_patch + (int64_t)kk * D;
          for (int32_t j = 0; j < D; ++j) xr[j] += a * wr[j];
        }
        for (int32_t j = 0; j < D; ++j) xr[j] += pos[(int64_t)(1 + p) * D + j];
      }
    free(flat);
  }
}

/* ---------------------------------------------------------------- elementary layers (backward) */

/* Eq. 2: dx = dy . w^T   (dx[M,K], dy[M,N], w[K,N]) */
void orc_linear_dgrad(const real* dy, int64_t M, int32_t N, const real* w, int32_t K, real* dx) {
#pragma omp parallel for schedule(static)
  for (int64_t m = 0; m < M; ++m)
    for (int32_t k = 0; k < K; ++k) {
      const real* dyr = dy + m * N;
      const real* wr = w + (int64_t)k * N;
      real s = 0;
#pragma omp simd reduction(+ : s)
      for (int32_t n = 0; n < N; ++n) s += dyr[n] * wr[n];
      dx[m * K + k] = s;
    }
}

/* Eq. 4: dw = x^T . dy (summed over all tokens of all images), db = column sums of dy */
void orc_linear_wgrad(const real* x, const real* dy, int64_t M, int32_t K, int32_t N, real* dw,
                      real* db) {
  if (dw) {
#pragma omp parallel for schedule(static)
    for (int32_t k = 0; k < K; ++k) {
      real* dwr = dw + (int64_t)k * N;
      for (int32_t n = 0; n < N; ++n) dwr[n] = 0;
      for (int64_t m = 0; m < M; ++m) {
        real a = x[m * K + k];
        const real* dyr = dy + m * N;
        for (int32_t n = 0; n < N; ++n) dwr[n] += a * dyr[n];
      }
    }
  }
  if (db) {
    for (int32_t n = 0; n < N; ++n) db[n] = 0;
    for (int64_t m = 0; m < M; ++m)
      for (int32_t n = 0; n < N; ++n) db[n] += dy[m * N + n];
  }
}

/* LayerNorm backward.  With g = dy*gamma:  dx = rstd * (g - mean(g) - xhat * mean(g*xhat));
 * dgamma = sum_rows dy*xhat;  dbeta = sum_rows dy.  dx / dgamma / dbeta may be NULL. */
void orc_layernorm_bwd(const real* dy, const real* xhat, const real* rstd, const real* gamma,
                       int64_t M, int32_t D, real* dx, real* dgamma, real* dbeta) {
  if (dx) {
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
      const real* dyr = dy + m * D;
      const real* xh = xhat + m * D;
      real m1 = 0, m2 = 0;
      for (int32_t j = 0; j < D; ++j) {
        real g = dyr[j] * gamma[j];
        m1 += g;
        m2 += g * xh[j];
      }
      m1 /= (real)D;
      m2 /= (real)D;
      for (int32_t j = 0; j < D; ++j) {
        real g = dyr[j] * gamma[j];
        dx[m * D + j] = rstd[m] * (g - m1 - xh[j] * m2);
      }
    }
  }
  if (dgamma || dbeta) {
    for (int32_t j = 0; j < D; ++j) {
      real sg = 0, sb = 0;
      for (int64_t m = 0; m < M; ++m) {
        sg += dy[m * D + j] * xhat[m * D + j];
        sb += dy[m * D + j];
      }
      if (dgamma) dgamma[j] = sg;
      if (dbeta) dbeta[j] = sb;
    }
  }
}

/* GELU'(u) = Phi(u) + u * phi(u);  du = dg * GELU'(u) */
void orc_gelu_bwd(const real* dg, const real* u, int64_t n, real* du) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    double v = (double)u[i];
    double cdf = 0.5 * (1.0 + erf(v * 0.70710678118654752440));
    double pdf = exp(-0.5 * v * v) * 0.39894228040143267794;
    du[i] = (real)((double)dg[i] * (cdf + v * pdf));
  }
}

/* Backward of Eq. 1 per head, from the stored q,k,v and P (Eq. 3, 5: softmax and attention need
 * their inputs).  dV = P^T dO; dP = dO V^T; dS = P * (dP - rowsum(dP*P)); dQ = dS K / sqrt(d);
 * dK = dS^T Q / sqrt(d).  dqkv has the layout of qkv. */
void orc_attention_bwd(const real* qkv, const real* P, const real* dout, int32_t B, int32_t T,
                       int32_t H, int32_t d, real* dqkv) {
  const int32_t D = H * d;
  const real scale = (real)(1.0 / sqrt((double)d));
#pragma omp parallel for collapse(2) schedule(static)
  for (int32_t b = 0; b < B; ++b)
    for (int32_t h = 0; h < H; ++h) {
      const real* base = qkv + (int64_t)b * T * 3 * D;
      real* dbase = dqkv + (int64_t)b * T * 3 * D;
      const real* Pbh = P + ((int64_t)b * H + h) * T * T;
      real* dS = (real*)malloc(sizeof(real) * T);
      for (int32_t t = 0; t < T; ++t)
        for (int32_t e = 0; e < d; ++e) {
          dbase[(int64_t)t * 3 * D + h * d + e] = 0;         /* dq */
          dbase[(int64_t)t * 3 * D + D + h * d + e] = 0;     /* dk */
          dbase[(int64_t)t * 3 * D + 2 * D + h * d + e] = 0; /* dv */
        }
      for (int32_t i = 0; i < T; ++i) {
        const real* dO = dout + ((int64_t)b * T + i) * D + h * d;
        const real* q = base + (int64_t)i * 3 * D + h * d;
        const real* row = Pbh + (int64_t)i * T;
        real dot = 0;
        for (int32_t j = 0; j < T; ++j) {
          const real* v = base + (int64_t)j * 3 * D + 2 * D + h * d;
          real* dv = dbase + (int64_t)j * 3 * D + 2 * D + h * d;
          real dp = 0;
          for (int32_t e = 0; e < d; ++e) {
            dp += dO[e] * v[e];
            dv[e] += row[j] * dO[e];
          }
          dS[j] = dp;
          dot += dp * row[j];
        }
        real* dq = dbase + (int64_t)i * 3 * D + h * d;
        for (int32_t j = 0; j < T; ++j) {
          real ds = row[j] * (dS[j] - dot) * scale;
          const real* k = base + (int64_t)j * 3 * D + D + h * d;
          real* dk = dbase + (int64_t)j * 3 * D + D + h * d;
          for (int32_t e = 0; e < d; ++e) {
            dq[e] += ds * k[e];
            dk[e] += ds * q[e];
          }
        }
      }
      free(dS);
    }
}

/* Adjoint of orc_gather: dx = 0; dx[b,0] = dy[b,0]; dx[b,1+idx[b,i]] = dy[b,1+i]. */
void orc_gather_bwd(const real* dy, int32_t B, int32_t T, int32_t D, const int32_t* idx, int32_t k,
                    real* dx) {
  memset(dx, 0, sizeof(real) * (size_t)B * T * D);
  for (int32_t b = 0; b < B; ++b) {
    memcpy(dx + (int64_t)b * T * D, dy + (int64_t)b * (k + 1) * D, sizeof(real) * D);
    for (int32_t i = 0; i < k; ++i)
      memcpy(dx + ((int64_t)b * T + 1 + idx[(int64_t)b * k + i]) * D,
             dy + ((int64_t)b * (k + 1) + 1 + i) * D, sizeof(real) * D);
  }
}

/* Mean cross-entropy over the batch and its gradient: dlogits = (softmax - onehot) / B. */
real orc_cross_entropy(const real* logits, const int32_t* labels, int32_t B, int32_t C,
                       real* dlogits) {
  real loss = 0;
  for (int32_t b = 0; b < B; ++b) {
    const real* z = logits + (int64_t)b * C;
    real mx = z[0];
    for (int32_t c = 1; c < C; ++c)
      if (z[c] > mx) mx = z[c];
    real sum = 0;
    for (int32_t c = 0; c < C; ++c) sum += (real)exp((double)(z[c] - mx));
    real lse = mx + (real)log((double)sum);
    loss += lse - z[labels[b]];
    if (dlogits)
      for (int32_t c = 0; c < C; ++c)
        dlogits[(int64_t)b * C + c] =
            ((real)exp((double)(z[c] - lse)) - (c == labels[b] ? (real)1 : (real)0)) / (real)B;
  }
  return loss / (real)B;
}

/* SGD (Sec. 5): g' = g + wd*w;  mu > 0: m = mu*m + g', w -= lr*m;  else w -= lr*g'. */
void orc_sgd(real* w, const real* g, real* m, int64_t n, double lr, double mu, double wd) {
  for (int64_t i = 0; i < n; ++i) {
    real gp = g[i] + (real)wd * w[i];
    if (mu > 0) {
      m[i] = (real)mu * m[i] + gp;
      w[i] -= (real)lr * m[i];
    } else {
      w[i] -= (real)lr * gp;
    }
  }
}

/* AdamW (the optimiser of the paper's DeiT-S runs, Sec. 5), step t = 1, 2, ...:
 *   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;  mhat = m / (1-b1^t);  vhat = v / (1-b2^t);
 *   w = w - lr (mhat / (sqrt(vhat) + eps) + wd w)          (decoupled weight decay) */
void orc_adamw(real* w, const real* g, real* m, real* v, int64_t n, double lr, double b1, double b2,
               double eps, double wd, int32_t t) {
  const double c1 = 1.0 - pow(b1, (double)t), c2 = 1.0 - pow(b2, (double)t);
  for (int64_t i = 0; i < n; ++i) {
    const double gi = (double)g[i];
    const double mi = b1 * (double)m[i] + (1.0 - b1) * gi;
    const double vi = b2 * (double)v[i] + (1.0 - b2) * gi * gi;
    m[i] = (real)mi;
    v[i] = (real)vi;
    w[i] = (real)((double)w[i] - lr * ((mi / c1) / (sqrt(vi / c2) + eps) + wd * (double)w[i]));
  }
}

/* ---------------------------------------------------------------- mixture-of-experts FFN (Sec. 5.3) */

/* Routing of one token: the K experts with the largest router logits (ties: lower expert index
 * first), in descending order of logit, and their gate weights = softmax over those K logits.
 * forced (may be NULL) replaces the ranking; the gates still come from the logits. */
void orc_moe_route(const real* logits, int64_t M, int32_t E, int32_t K, const int32_t* forced,
                   int32_t* experts, real* gates) {
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < M; ++t) {
    const real* lg = logits + t * E;
    int32_t* ex = experts + t * K;
    if (forced) {
      for (int32_t s = 0; s < K; ++s) ex[s] = forced[t * K + s];
    } else {
      for (int32_t s = 0; s < K; ++s) {
        int32_t best = -1;
        for (int32_t e = 0; e < E; ++e) {
          int32_t taken = 0;
          for (int32_t j = 0; j < s; ++j) taken |= (ex[j] == e);
          if (taken) continue;
          if (best < 0 || lg[e] > lg[best]) best = e; /* strict >: a tie keeps the lower index */
        }
        ex[s] = best;
      }
    }
    real mx = lg[ex[0]];
    for (int32_t s = 1; s < K; ++s) if (lg[ex[s]] > mx) mx = lg[ex[s]];
    real sum = 0;
    for (int32_t s = 0; s < K; ++s) { gates[t * K + s] = (real)exp((double)(lg[ex[s]] - mx)); sum += gates[t * K + s]; }
    for (int32_t s = 0; s < K; ++s) gates[t * K + s] /= sum;
  }
}

/* y[t] = sum_s gate[t,s] * FFN_{e(t,s)}(h[t]),  FFN_e(h) = GELU(h W1_e + b1_e) W2_e + b2_e.
 * Kept for the backward pass: logits [M,E], experts [M,K], gates [M,K], u and g [M,K,F] (input and
 * output of GELU per active expert), ye [M,K,D] (each active expert's output). */
void orc_moe_ffn(const real* h, int64_t M, int32_t D, int32_t F, int32_t E, int32_t K,
                 const real* w_router, const real* w1, const real* b1, const real* w2, const real* b2,
                 const int32_t* forced, real* logits, int32_t* experts, real* gates, real* u, real* g,
                 real* ye, real* y) {
  orc_linear(h, M, D, w_router, NULL, E, logits);
  orc_moe_route(logits, M, E, K, forced, experts, gates);
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < M; ++t) {
    for (int32_t j = 0; j < D; ++j) y[t * D + j] = 0;
    for (int32_t s = 0; s < K; ++s) {
      const int32_t e = experts[t * K + s];
      real* ur = u + (t * K + s) * F;
      real* gr = g + (t * K + s) * F;
      real* yr = ye + (t * K + s) * D;
      orc_linear(h + t * D, 1, D, w1 + (int64_t)e * D * F, b1 + (int64_t)e * F, F, ur);
      orc_gelu(ur, F, gr);
      orc_linear(gr, 1, F, w2 + (int64_t)e * F * D, b2 + (int64_t)e * D, D, yr);
      for (int32_t j = 0; j < D; ++j) y[t * D + j] += gates[t * K + s] * yr[j];
    }
  }
}

/* Backward of orc_moe_ffn.  The expert choice is a constant; the gates are differentiated through
 * the softmax over the selected logits:  dgate_s = <dy, ye_s>,  dlogit_{e_s} = gate_s (dgate_s -
 * sum_j gate_j dgate_j).  Expert weights receive Eq. 4 over the tokens routed to them (ascending
 * token order), the router receives dW_r = h^T dlogits.  dh [M,D] is overwritten. */
void orc_moe_ffn_bwd(const real* dy, const real* h, int64_t M, int32_t D, int32_t F, int32_t E, int32_t K,
                     const real* w_router, const real* w1, const real* w2, const int32_t* experts,
                     const real* gates, const real* u, const real* g, const real* ye, real* dh,
                     real* dw_router, real* dw1, real* db1, real* dw2, real* db2) {
  real* du = ralloc(M * K * F);     /* gradient at the GELU input of every (token, slot) */
  real* dye = ralloc(M * K * D);    /* gradient at every active expert's output         */
  real* dlog = ralloc(M * E);
#pragma omp parallel for schedule(static)
  for (int64_t t = 0; t < M; ++t) {
    real dgate[16];
    real mix = 0;
    for (int32_t s = 0; s < K; ++s) {
      real a = 0;
      for (int32_t j = 0; j < D; ++j) a += dy[t * D + j] * ye[(t * K + s) * D + j];
      dgate[s] = a;
      mix += gates[t * K + s] * a;
    }
    for (int32_t e = 0; e < E; ++e) dlog[t * E + e] = 0;
    for (int32_t j = 0; j < D; ++j) dh[t * D + j] = 0;
    for (int32_t s = 0; s < K; ++s) {
      const int32_t e = experts[t * K + s];
      dlog[t * E + e] = gates[t * K + s] * (dgate[s] - mix);
      real* dyr = dye + (t * K + s) * D;
      for (int32_t j = 0; j < D; ++j) dyr[j] = gates[t * K + s] * dy[t * D + j];
      real* dg = ralloc(F);
      orc_linear_dgrad(dyr, 1, D, w2 + (int64_t)e * F * D, F, dg);                 /* Eq. 2 */
      orc_gelu_bwd(dg, u + (t * K + s) * F, F, du + (t * K + s) * F);
      free(dg);
      real* dhe = ralloc(D);
      orc_linear_dgrad(du + (t * K + s) * F, 1, F, w1 + (int64_t)e * D * F, D, dhe);
      for (int32_t j = 0; j < D; ++j) dh[t * D + j] += dhe[j];
      free(dhe);
    }
    /* router path: dh += dlogits W_r^T */
    for (int32_t j = 0; j < D; ++j) {
      real a = 0;
      for (int32_t e = 0; e < E; ++e) a += dlog[t * E + e] * w_router[(int64_t)j * E + e];
      dh[t * D + j] += a;
    }
  }
  if (dw_router) orc_linear_wgrad(h, dlog, M, D, E, dw_router, NULL);
  /* expert weights: one expert per thread, its tokens in ascending order */
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t e = 0; e < E; ++e) {
    real* a1 = dw1 ? dw1 + (int64_t)e * D * F : NULL;
    real* c1 = db1 ? db1 + (int64_t)e * F : NULL;
    real* a2 = dw2 ? dw2 + (int64_t)e * F * D : NULL;
    real* c2 = db2 ? db2 + (int64_t)e * D : NULL;
    if (a1) for (int64_t i = 0; i < (int64_t)D * F; ++i) a1[i] = 0;
    if (c1) for (int32_t i = 0; i < F; ++i) c1[i] = 0;
    if (a2) for (int64_t i = 0; i < (int64_t)F * D; ++i) a2[i] = 0;
    if (c2) for (int32_t i = 0; i < D; ++i) c2[i] = 0;
    for (int64_t t = 0; t < M; ++t)
      for (int32_t s = 0; s < K; ++s) {
        if (experts[t * K + s] != e) continue;
        const real* dur = du + (t * K + s) * F;
        const real* dyr = dye + (t * K + s) * D;
        const real* gr = g + (t * K + s) * F;
        if (a1) for (int32_t i = 0; i < D; ++i) for (int32_t f = 0; f < F; ++f) a1[(int64_t)i * F + f] += h[t * D + i] * dur[f];
        if (c1) for (int32_t f = 0; f < F; ++f) c1[f] += dur[f];
        if (a2) for (int32_t f = 0; f < F; ++f) for (int32_t j = 0; j < D; ++j) a2[(int64_t)f * D + j] += gr[f] * dyr[j];
        if (c2) for (int32_t j = 0; j < D; ++j) c2[j] += dyr[j];
      }
  }
  free(du); free(dye); free(dlog);
}

/* ---------------------------------------------------------------- the whole step */

typedef struct {         /* what a trainable block keeps for its backward pass (Sec. 3.2) */
  int32_t Ta, Tm;        /* tokens seen by MHSA / by the FFN                               */
  int32_t dropped, k;    /* is a drop location; patch tokens kept                          */
  real *xhat1, *rstd1, *h1, *qkv, *P, *o;
  real *xhat2, *rstd2, *h2, *u, *g;
  int32_t* idx;
  real* fw;              /* [B, Ta-1] weights of the fused token (NULL: nothing was fused) */
  /* mixture-of-experts FFN: u and g are [M,K,F]; router logits, chosen experts, gates, expert outputs */
  real *rlogits, *gates, *ye;
  int32_t* experts;
} saved_block;

static void free_saved(saved_block* s) {
  free(s->xhat1); free(s->rstd1); free(s->h1); free(s->qkv); free(s->P); free(s->o);
  free(s->xhat2); free(s->rstd2); free(s->h2); free(s->u); free(s->g); free(s->idx);
  free(s->rlogits); free(s->gates); free(s->ye); free(s->experts); free(s->fw);
  memset(s, 0, sizeof(*s));
}

/*
 * One BSR step: frozen prefix forward (nothing kept), token drops at the drop locations, forward
 * and backward through blocks >= first_trainable and the head.
 *
 * input        images [B,C,S,S], or tokens [B,tokens_in,D] when image_size == 0
 * forced_idx   NULL, or kept indices to use instead of the ranking (concatenated over drops,
 *              drop i holding [B, keep_k[i]])
 * x_trainable  out, may be NULL: the token tensor entering block first_trainable [B,T,D]
 * kept_idx     out, may be NULL: concatenated kept indices, as forced_idx
 * cls_scores   out, may be NULL: concatenated importance scores, drop i holding [B, n_i]
 * x_final      out, may be NULL: output of the last block [B,T_last,D]
 * logits       out, may be NULL: [B,num_classes]
 * loss         out: scalar
 * grads        NULL (forward only) or a table whose non-NULL entries receive dL/dparam of the
 *              trainable tensors (overwritten).  A block at or after first_trainable whose entries
 *              are all NULL is frozen but in the gradient path (the paper's default layout trains
 *              every fourth block): it keeps its activations and only passes the input gradient
 *              on (Eq. 2, Eq. 3), no weight gradient is formed for it
 * dx_trainable out, may be NULL: dL/d(x_trainable), computed only on request (tests); the method
 *              itself never propagates this far (Fig. 2)
 * forced_experts  NULL, or the expert choice to use in the mixture-of-experts blocks (concatenated
 *              over those blocks in ascending order, block l holding [B*T_l, K])
 * experts_out  out, may be NULL: the expert choice, laid out as forced_experts
 * router_out   out, may be NULL: router logits, block l holding [B*T_l, E]
 * Returns 0, or a negative number for an inconsistent configuration.
 */
int32_t orc_step_moe(const orc_config* c, const orc_params* p, const real* input, const int32_t* labels,
                     int32_t B, const int32_t* forced_idx, real* x_trainable, int32_t* kept_idx,
                     real* cls_scores, real* x_final, real* logits, real* loss, const orc_params* grads,
                     real* dx_trainable, const int32_t* forced_experts, int32_t* experts_out,
                     real* router_out) {
  const int32_t D = c->dim, H = c->heads, F = c->mlp_hidden, L = c->depth, C = c->num_classes;
  if (D <= 0 || H <= 0 || D % H || L <= 0 || L > ORC_MAX_BLOCKS || B <= 0) return -1;
  if (c->first_trainable < 0 || c->first_trainable > L) return -1;
  const int32_t E = c->n_experts, K = c->moe_top_k;
  for (int32_t l = 0; l < L; ++l)
    if (c->moe_block[l] && (E < 1 || K < 1 || K > E || K > 16)) return -3;
  int64_t ex_off = 0, rl_off = 0;
  const int32_t d = D / H;
  int32_t T = c->image_size ? (c->image_size / c->patch_size) * (c->image_size / c->patch_size) + 1
                            : c->tokens_in;
  if (T < 1) return -1;
  {
    int32_t n = T - 1;
    for (int32_t i = 0; i < c->n_drop; ++i) {
      if (c->drop_blocks[i] < 0 || c->drop_blocks[i] >= L) return -2;
      if (i && c->drop_blocks[i] <= c->drop_blocks[i - 1]) return -2;
      if (c->keep_k[i] < 0 || c->keep_k[i] > n) return -2;
      n = c->keep_k[i] + ((c->fuse_dropped && n - c->keep_k[i] > 0) ? 1 : 0); /* the fused token is a patch token from here on */
    }
  }

  real* x = ralloc((int64_t)B * T * D);
  if (c->image_size)
    orc_stem(input, B, c->in_chans, c->image_size, c->patch_size, D, p->w_patch, p->b_patch, p->cls,
             p->pos, x);
  else
    memcpy(x, input, sizeof(real) * (size_t)B * T * D);

  saved_block saved[ORC_MAX_BLOCKS];
  memset(saved, 0, sizeof(saved));
  int32_t drop_i = 0;
  int64_t idx_off = 0, score_off = 0;

  /* ------------------------------------------------ forward through the blocks */
  for (int32_t l = 0; l < L; ++l) {
    const orc_block* w = &p->blocks[l];
    const int32_t trainable = (l >= c->first_trainable) && grads != NULL;
    if (l == c->first_trainable && x_trainable)
      memcpy(x_trainable, x, sizeof(real) * (size_t)B * T * D);
    const int64_t M = (int64_t)B * T;
    saved_block s;
    memset(&s, 0, sizeof(s));
    s.Ta = T;

    /* MHSA: x <- x + proj(Attention(LN1(x))) */
    s.xhat1 = ralloc(M * D); s.rstd1 = ralloc(M); s.h1 = ralloc(M * D);
    orc_layernorm(x, M, D, w->ln1_g, w->ln1_b, c->ln_eps, s.h1, s.xhat1, s.rstd1);
    s.qkv = ralloc(M * 3 * D);
    orc_linear(s.h1, M, D, w->w_qkv, w->b_qkv, 3 * D, s.qkv);
    s.P = ralloc((int64_t)B * H * T * T);
    s.o = ralloc(M * D);
    orc_attention(s.qkv, B, T, H, d, s.P, s.o);
    real* y = ralloc(M * D);
    orc_linear(s.o, M, D, w->w_proj, w->b_proj, D, y);
    for (int64_t i = 0; i < M * D; ++i) x[i] += y[i];
    free(y);

    /* token drop between MHSA and FFN of a drop location (Sec. 4.1; Sec. 4.3 Discussion 3) */
    if (drop_i < c->n_drop && c->drop_blocks[drop_i] == l) {
      const int32_t n = T - 1, k = c->keep_k[drop_i];
      real* a = ralloc((int64_t)B * n);
      orc_cls_scores(s.P, B, H, T, a);
      if (cls_scores) memcpy(cls_scores + score_off, a, sizeof(real) * (size_t)B * n);
      s.idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)(B * k > 0 ? B * k : 1));
      if (forced_idx)
        memcpy(s.idx, forced_idx + idx_off, sizeof(int32_t) * (size_t)B * k);
      else
        for (int32_t b = 0; b < B; ++b) orc_topk(a + (int64_t)b * n, n, k, s.idx + (int64_t)b * k);
      if (kept_idx) memcpy(kept_idx + idx_off, s.idx, sizeof(int32_t) * (size_t)B * k);
      const int32_t fused = (c->fuse_dropped && n - k > 0) ? 1 : 0;
      real* xk = ralloc((int64_t)B * (k + 1) * D);
      orc_gather(x, B, T, D, s.idx, k, xk);
      if (fused) {   /* [CLS; kept tokens; fused token] */
        real* f = ralloc((int64_t)B * D);
        s.fw = ralloc((int64_t)B * n);
        orc_fuse_dropped(x, a, B, T, D, s.idx, k, s.fw, f);
        real* xf = ralloc((int64_t)B * (k + 2) * D);
        for (int32_t b = 0; b < B; ++b) {
          memcpy(xf + (int64_t)b * (k + 2) * D, xk + (int64_t)b * (k + 1) * D, sizeof(real) * (size_t)(k + 1) * D);
          memcpy(xf + ((int64_t)b * (k + 2) + k + 1) * D, f + (int64_t)b * D, sizeof(real) * D);
        }
        free(f); free(xk);
        xk = xf;
      }
      free(a);
      free(x);
      x = xk;
      s.dropped = 1;
      s.k = k;
      T = k + 1 + fused;
      idx_off += (int64_t)B * k;
      score_off += (int64_t)B * n;
      ++drop_i;
    }
    s.Tm = T;

    /* FFN: x <- x + fc2(GELU(fc1(LN2(x)))) */
    const int64_t M2 = (int64_t)B * T;
    s.xhat2 = ralloc(M2 * D); s.rstd2 = ralloc(M2); s.h2 = ralloc(M2 * D);
    orc_layernorm(x, M2, D, w->ln2_g, w->ln2_b, c->ln_eps, s.h2, s.xhat2, s.rstd2);
    y = ralloc(M2 * D);
    if (c->moe_block[l]) {   /* mixture of experts in place of the FFN (Sec. 5.3) */
      s.u = ralloc(M2 * K * F); s.g = ralloc(M2 * K * F); s.ye = ralloc(M2 * K * D);
      s.rlogits = ralloc(M2 * E); s.gates = ralloc(M2 * K);
      s.experts = (int32_t*)malloc(sizeof(int32_t) * (size_t)(M2 * K));
      orc_moe_ffn(s.h2, M2, D, F, E, K, w->w_router, w->w_fc1, w->b_fc1, w->w_fc2, w->b_fc2,
                  forced_experts ? forced_experts + ex_off : NULL, s.rlogits, s.experts, s.gates, s.u, s.g,
                  s.ye, y);
      if (experts_out) memcpy(experts_out + ex_off, s.experts, sizeof(int32_t) * (size_t)(M2 * K));
      if (router_out) memcpy(router_out + rl_off, s.rlogits, sizeof(real) * (size_t)(M2 * E));
      ex_off += M2 * K;
      rl_off += M2 * E;
    } else {
      s.u = ralloc(M2 * F);
      orc_linear(s.h2, M2, D, w->w_fc1, w->b_fc1, F, s.u);
      s.g = ralloc(M2 * F);
      orc_gelu(s.u, M2 * F, s.g);
      orc_linear(s.g, M2, F, w->w_fc2, w->b_fc2, D, y);
    }
    for (int64_t i = 0; i < M2 * D; ++i) x[i] += y[i];
    free(y);

    if (trainable) saved[l] = s;   /* a trainable block keeps its activations */
    else free_saved(&s);           /* a frozen block before the trainable ones keeps nothing */
  }
  if (c->first_trainable == L && x_trainable)
    memcpy(x_trainable, x, sizeof(real) * (size_t)B * T * D);
  if (x_final) memcpy(x_final, x, sizeof(real) * (size_t)B * T * D);

  /* ------------------------------------------------ head and loss */
  const int64_t Mf = (int64_t)B * T;
  real* dx = ralloc(Mf * D); /* dL/dx at the output of the last block */
  memset(dx, 0, sizeof(real) * (size_t)Mf * D);
  if (C > 0) {
    /* z = LN_f(x[:,0]); logits = z W_h + b_h; cross-entropy */
    real* xc = ralloc((int64_t)B * D);
    for (int32_t b = 0; b < B; ++b) memcpy(xc + (int64_t)b * D, x + (int64_t)b * T * D, sizeof(real) * D);
    real* z = ralloc((int64_t)B * D); real* zhat = ralloc((int64_t)B * D); real* zr = ralloc(B);
    orc_layernorm(xc, B, D, p->lnf_g, p->lnf_b, c->ln_eps, z, zhat, zr);
    real* lg = ralloc((int64_t)B * C);
    orc_linear(z, B, D, p->w_head, p->b_head, C, lg);
    if (logits) memcpy(logits, lg, sizeof(real) * (size_t)B * C);
    real* dlg = ralloc((int64_t)B * C);
    *loss = orc_cross_entropy(lg, labels, B, C, dlg);
    if (grads) {
      real* dz = ralloc((int64_t)B * D);
      orc_linear_dgrad(dlg, B, C, p->w_head, D, dz);
      orc_linear_wgrad(z, dlg, B, D, C, grads->w_head, grads->b_head);
      real* dxc = ralloc((int64_t)B * D);
      orc_layernorm_bwd(dz, zhat, zr, p->lnf_g, B, D, dxc, grads->lnf_g, grads->lnf_b);
      for (int32_t b = 0; b < B; ++b) memcpy(dx + (int64_t)b * T * D, dxc + (int64_t)b * D, sizeof(real) * D);
      free(dz); free(dxc);
    }
    free(xc); free(z); free(zhat); free(zr); free(lg); free(dlg);
  } else {
    /* loss = mean over all output elements of x^2 */
    real s = 0;
    for (int64_t i = 0; i < Mf * D; ++i) s += x[i] * x[i];
    *loss = s / (real)(Mf * D);
    for (int64_t i = 0; i < Mf * D; ++i) dx[i] = (real)2 * x[i] / (real)(Mf * D);
  }
  free(x);

  /* ------------------------------------------------ backward through the trainable blocks */
  if (grads) {
    for (int32_t l = L - 1; l >= c->first_trainable; --l) {
      const orc_block* w = &p->blocks[l];
      const orc_block* g = &grads->blocks[l];
      saved_block* s = &saved[l];
      const int64_t M2 = (int64_t)B * s->Tm, M = (int64_t)B * s->Ta;

      /* FFN branch: x_out = x_mid + fc2(GELU(fc1(LN2(x_mid)))) */
      real* dh2 = ralloc(M2 * D);
      if (c->moe_block[l]) {
        orc_moe_ffn_bwd(dx, s->h2, M2, D, F, E, K, w->w_router, w->w_fc1, w->w_fc2, s->experts, s->gates,
                        s->u, s->g, s->ye, dh2, g->w_router, g->w_fc1, g->b_fc1, g->w_fc2, g->b_fc2);
      } else {
        real* dg = ralloc(M2 * F);
        orc_linear_dgrad(dx, M2, D, w->w_fc2, F, dg);
        orc_linear_wgrad(s->g, dx, M2, F, D, g->w_fc2, g->b_fc2);
        real* du = ralloc(M2 * F);
        orc_gelu_bwd(dg, s->u, M2 * F, du);
        free(dg);
        orc_linear_dgrad(du, M2, F, w->w_fc1, D, dh2);
        orc_linear_wgrad(s->h2, du, M2, D, F, g->w_fc1, g->b_fc1);
        free(du);
      }
      real* dxm = ralloc(M2 * D);
      orc_layernorm_bwd(dh2, s->xhat2, s->rstd2, w->ln2_g, M2, D, dxm, g->ln2_g, g->ln2_b);
      free(dh2);
      for (int64_t i = 0; i < M2 * D; ++i) dxm[i] += dx[i]; /* residual */
      free(dx);

      /* adjoint of the token drop: dropped tokens get no gradient from the FFN side */
      if (s->dropped) {
        real* full = ralloc(M * D);
        if (s->fw) {   /* rows [CLS; kept; fused]: the fused token's gradient goes to the dropped tokens by weight */
          const int32_t k = s->k, n = s->Ta - 1;
          real* dk = ralloc((int64_t)B * (k + 1) * D);
          for (int32_t b = 0; b < B; ++b)
            memcpy(dk + (int64_t)b * (k + 1) * D, dxm + (int64_t)b * (k + 2) * D, sizeof(real) * (size_t)(k + 1) * D);
          orc_gather_bwd(dk, B, s->Ta, D, s->idx, k, full);
          free(dk);
          for (int32_t b = 0; b < B; ++b)
            for (int32_t j = 0; j < n; ++j) {
              const real wj = s->fw[(int64_t)b * n + j];
              if (wj == 0) continue;
              for (int32_t cc = 0; cc < D; ++cc)
                full[((int64_t)b * s->Ta + 1 + j) * D + cc] += wj * dxm[((int64_t)b * (k + 2) + k + 1) * D + cc];
            }
        } else {
          orc_gather_bwd(dxm, B, s->Ta, D, s->idx, s->k, full);
        }
        free(dxm);
        dxm = full;
      }

      /* MHSA branch: x_mid = x_in + proj(Attention(LN1(x_in))) */
      real* dO = ralloc(M * D);
      orc_linear_dgrad(dxm, M, D, w->w_proj, D, dO);
      orc_linear_wgrad(s->o, dxm, M, D, D, g->w_proj, g->b_proj);
      real* dqkv = ralloc(M * 3 * D);
      orc_attention_bwd(s->qkv, s->P, dO, B, s->Ta, H, d, dqkv);
      free(dO);
      real* dh1 = ralloc(M * D);
      orc_linear_dgrad(dqkv, M, 3 * D, w->w_qkv, D, dh1);
      orc_linear_wgrad(s->h1, dqkv, M, D, 3 * D, g->w_qkv, g->b_qkv);
      free(dqkv);
      const int32_t need_dx = (l > c->first_trainable) || dx_trainable != NULL;
      real* dxin = need_dx ? ralloc(M * D) : NULL;
      orc_layernorm_bwd(dh1, s->xhat1, s->rstd1, w->ln1_g, M, D, dxin, g->ln1_g, g->ln1_b);
      free(dh1);
      if (need_dx)
        for (int64_t i = 0; i < M * D; ++i) dxin[i] += dxm[i]; /* residual */
      free(dxm);
      dx = dxin; /* NULL once the earliest trainable block is done: gradient flow stops (Fig. 2) */
      if (l == c->first_trainable && dx_trainable)
        memcpy(dx_trainable, dx, sizeof(real) * (size_t)M * D);
      free_saved(s);
    }
    if (c->first_trainable == L && dx_trainable)
      memcpy(dx_trainable, dx, sizeof(real) * (size_t)Mf * D);
  }
  free(dx);
  return 0;
}

/* The step without any mixture-of-experts arguments. */
int32_t orc_step(const orc_config* c, const orc_params* p, const real* input, const int32_t* labels,
                 int32_t B, const int32_t* forced_idx, real* x_trainable, int32_t* kept_idx,
                 real* cls_scores, real* x_final, real* logits, real* loss, const orc_params* grads,
                 real* dx_trainable) {
  return orc_step_moe(c, p, input, labels, B, forced_idx, x_trainable, kept_idx, cls_scores, x_final, logits,
                      loss, grads, dx_trainable, NULL, NULL, NULL);
}
