// Row-wise and element-wise kernels of the BSR step: LayerNorm forward / backward, column sums
// (bias and LayerNorm parameter gradients), patch extraction, CLS-attention ranking (Eq. 6 of the
// paper), token gather / scatter, losses, SGD and weight casts.  All are HBM-bound; reductions are
// two-pass with a fixed order, so results are bit-reproducible run to run.
#include <algorithm>

#include "bsr_internal.h"

namespace bsr {

namespace {

constexpr int WAVE = 64;
constexpr int COLSUM_R = 64;  // row chunks of the two-pass column reductions

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// ---------------------------------------------------------------- LayerNorm
// One wavefront per token row; mean and biased variance in fp32, two passes over the row.
template <typename T>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ x, int64_t M, int D,
                                                     const float* __restrict__ gamma,
                                                     const float* __restrict__ beta, float eps,
                                                     T* __restrict__ y, float* __restrict__ mean,
                                                     float* __restrict__ rstd) {
  const int lane = threadIdx.x % WAVE;
  const int64_t m = (int64_t)blockIdx.x * (blockDim.x / WAVE) + threadIdx.x / WAVE;
  if (m >= M) return;
  const T* xr = x + m * D;
  float s = 0.f;
  for (int j = lane; j < D; j += WAVE) s += (float)xr[j];
  const float mu = wave_sum(s) / (float)D;
  float v = 0.f;
  for (int j = lane; j < D; j += WAVE) {
    float c = (float)xr[j] - mu;
    v += c * c;
  }
  const float rs = rsqrtf(wave_sum(v) / (float)D + eps);
  if (lane == 0) {
    if (mean) mean[m] = mu;
    if (rstd) rstd[m] = rs;
  }
  T* yr = y + m * D;
  for (int j = lane; j < D; j += WAVE) yr[j] = (T)(((float)xr[j] - mu) * rs * gamma[j] + beta[j]);
}

// dx = res + rstd * (g - mean(g) - xhat * mean(g * xhat)),  g = dy * gamma
template <typename T>
__global__ __launch_bounds__(256) void ln_bwd_dx_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                        const float* __restrict__ mean,
                                                        const float* __restrict__ rstd,
                                                        const float* __restrict__ gamma,
                                                        const T* __restrict__ res, int64_t M, int D,
                                                        T* __restrict__ dx) {
  const int lane = threadIdx.x % WAVE;
  const int64_t m = (int64_t)blockIdx.x * (blockDim.x / WAVE) + threadIdx.x / WAVE;
  if (m >= M) return;
  const float mu = mean[m], rs = rstd[m];
  const T* dyr = dy + m * D;
  const T* xr = x + m * D;
  float s1 = 0.f, s2 = 0.f;
  for (int j = lane; j < D; j += WAVE) {
    float g = (float)dyr[j] * gamma[j];
    s1 += g;
    s2 += g * ((float)xr[j] - mu) * rs;
  }
  const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
  for (int j = lane; j < D; j += WAVE) {
    float g = (float)dyr[j] * gamma[j];
    float xh = ((float)xr[j] - mu) * rs;
    float v = rs * (g - m1 - xh * m2);
    if (res) v += (float)res[m * D + j];
    dx[m * D + j] = (T)v;
  }
}

// bf16 rows whose length is a multiple of 8 and at most 2048: one wavefront per row, the row is read
// once with 16-byte loads and stays in registers (up to 4 chunks of 8 per lane).
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
constexpr int LN_MAXC = 4;

// With idx (token selection fused in, Sec. 4.1): output row m = b * (k + 1) + i reads token 0 (i == 0) or
// token 1 + idx[b, i - 1] of image b of x [B, T_in, D], and the row itself is also copied to xcopy[m].
__global__ __launch_bounds__(256) void ln_fwd_vec_kernel(const bf16* __restrict__ x, int64_t M, int D,
                                                         const float* __restrict__ gamma,
                                                         const float* __restrict__ beta, float eps,
                                                         bf16* __restrict__ y, float* __restrict__ mean,
                                                         float* __restrict__ rstd, const int32_t* __restrict__ idx,
                                                         int T_in, int k, bf16* __restrict__ xcopy) {
  const int lane = threadIdx.x % WAVE;
  const int64_t m = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
  if (m >= M) return;
  const int nch = D / 8;
  int64_t src = m;
  if (idx) {
    const int64_t b = m / (k + 1);
    const int i = (int)(m % (k + 1));
    src = b * T_in + (i == 0 ? 0 : 1 + idx[b * k + i - 1]);
  }
  const bf16x8_t* xr = (const bf16x8_t*)(x + src * D);
  bf16x8_t* cr = xcopy ? (bf16x8_t*)(xcopy + m * D) : nullptr;
  float v[LN_MAXC][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + i * WAVE;
    if (c < nch) {
      const bf16x8_t t = xr[c];
      if (cr) cr[c] = t;
#pragma unroll
      for (int e = 0; e < 8; ++e) { v[i][e] = (float)t[e]; s += v[i][e]; }
    }
  }
  const float mu = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i)
    if (lane + i * WAVE < nch)
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d0 = v[i][e] - mu; q += d0 * d0; }
  const float rs = rsqrtf(wave_sum(q) / (float)D + eps);
  if (lane == 0) {
    if (mean) mean[m] = mu;
    if (rstd) rstd[m] = rs;
  }
  bf16x8_t* yr = (bf16x8_t*)(y + m * D);
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + i * WAVE;
    if (c < nch) {
      const float4 g0 = *(const float4*)(gamma + c * 8), g1 = *(const float4*)(gamma + c * 8 + 4);
      const float4 b0 = *(const float4*)(beta + c * 8), b1 = *(const float4*)(beta + c * 8 + 4);
      const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      const float bb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
      bf16x8_t o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (bf16)((v[i][e] - mu) * rs * gg[e] + bb[e]);
      yr[c] = o;
    }
  }
}

// dx = res + rstd * (g - mean(g) - xhat * mean(g * xhat)),  g = dy * gamma   (same row layout)
__global__ __launch_bounds__(256) void ln_bwd_dx_vec_kernel(const bf16* __restrict__ dy, const bf16* __restrict__ x,
                                                            const float* __restrict__ mean,
                                                            const float* __restrict__ rstd,
                                                            const float* __restrict__ gamma,
                                                            const bf16* __restrict__ res, int64_t M, int D,
                                                            bf16* __restrict__ dx) {
  const int lane = threadIdx.x % WAVE;
  const int64_t m = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
  if (m >= M) return;
  const int nch = D / 8;
  const float mu = mean[m], rs = rstd[m];
  const bf16x8_t* dyr = (const bf16x8_t*)(dy + m * D);
  const bf16x8_t* xr = (const bf16x8_t*)(x + m * D);
  float g[LN_MAXC][8], xh[LN_MAXC][8];
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + i * WAVE;
    if (c < nch) {
      const bf16x8_t a = dyr[c], t = xr[c];
      const float4 g0 = *(const float4*)(gamma + c * 8), g1 = *(const float4*)(gamma + c * 8 + 4);
      const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        g[i][e] = (float)a[e] * gg[e];
        xh[i][e] = ((float)t[e] - mu) * rs;
        s1 += g[i][e];
        s2 += g[i][e] * xh[i][e];
      }
    }
  }
  const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
  const bf16x8_t* rr = res ? (const bf16x8_t*)(res + m * D) : nullptr;
  bf16x8_t* dxr = (bf16x8_t*)(dx + m * D);
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + i * WAVE;
    if (c < nch) {
      bf16x8_t o;
      bf16x8_t r8;
      if (rr) r8 = rr[c];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float t = rs * (g[i][e] - m1 - xh[i][e] * m2);
        if (rr) t += (float)r8[e];
        o[e] = (bf16)t;
      }
      dxr[c] = o;
    }
  }
}

// LayerNorm backward in one pass over dy and x: dx as above (skipped when dx is null) and, per
// workgroup, the partial sums over its rows of dy * xhat (dgamma) and dy (dbeta).  A wavefront walks
// rows blockIdx.x * 4 + wave + k * 4 * gridDim.x with the next row's loads in flight; the four wave
// partials are added in wave order and land in partial[blockIdx.x] (dgamma) and
// partial[LN_BWD_BLOCKS + blockIdx.x] (dbeta); colsum_final_kernel adds the workgroups.
constexpr int LN_BWD_BLOCKS = 256;

__global__ __launch_bounds__(256) void ln_bwd_fused_vec_kernel(const bf16* __restrict__ dy, const bf16* __restrict__ x,
                                                               const float* __restrict__ mean,
                                                               const float* __restrict__ rstd,
                                                               const float* __restrict__ gamma,
                                                               const bf16* __restrict__ res, int64_t M, int D,
                                                               bf16* __restrict__ dx, float* __restrict__ partial) {
  __shared__ float red[3][8 * WAVE * LN_MAXC];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int nch = D / 8;
  const int64_t stride = (int64_t)gridDim.x * 4;
  float gg[LN_MAXC][8];
  float dg[LN_MAXC][8], db[LN_MAXC][8];
#pragma unroll
  for (int i = 0; i < LN_MAXC; ++i) {
    const int c = lane + i * WAVE;
#pragma unroll
    for (int e = 0; e < 8; ++e) { dg[i][e] = 0.f; db[i][e] = 0.f; gg[i][e] = 0.f; }
    if (c < nch) {
      const float4 g0 = *(const float4*)(gamma + c * 8), g1 = *(const float4*)(gamma + c * 8 + 4);
      gg[i][0] = g0.x; gg[i][1] = g0.y; gg[i][2] = g0.z; gg[i][3] = g0.w;
      gg[i][4] = g1.x; gg[i][5] = g1.y; gg[i][6] = g1.z; gg[i][7] = g1.w;
    }
  }
  bf16x8_t na[LN_MAXC], nt[LN_MAXC];     // the next row, already loading
  float nmu = 0.f, nrs = 0.f;
  auto prefetch = [&](int64_t m) {
    if (m >= M) return;
    const bf16x8_t* dyr = (const bf16x8_t*)(dy + m * D);
    const bf16x8_t* xr = (const bf16x8_t*)(x + m * D);
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
      const int c = lane + i * WAVE;
      if (c < nch) { na[i] = dyr[c]; nt[i] = xr[c]; }
    }
    nmu = mean[m]; nrs = rstd[m];
  };
  int64_t m = (int64_t)blockIdx.x * 4 + w;
  prefetch(m);
  for (; m < M; m += stride) {
    bf16x8_t a[LN_MAXC], t[LN_MAXC];
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) { a[i] = na[i]; t[i] = nt[i]; }
    const float mu = nmu, rs = nrs;
    prefetch(m + stride);
    float g[LN_MAXC][8], xh[LN_MAXC][8];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXC; ++i) {
      if (lane + i * WAVE < nch) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float d0 = (float)a[i][e];
          xh[i][e] = ((float)t[i][e] - mu) * rs;
          g[i][e] = d0 * gg[i][e];
          dg[i][e] += d0 * xh[i][e];
          db[i][e] += d0;
          s1 += g[i][e];
          s2 += g[i][e] * xh[i][e];
        }
      }
    }
    if (dx) {
      const float m1 = wave_sum(s1) / (float)D, m2 = wave_sum(s2) / (float)D;
      const bf16x8_t* rr = res ? (const bf16x8_t*)(res + m * D) : nullptr;
      bf16x8_t* dxr = (bf16x8_t*)(dx + m * D);
#pragma unroll
      for (int i = 0; i < LN_MAXC; ++i) {
        const int c = lane + i * WAVE;
        if (c < nch) {
          bf16x8_t o;
          bf16x8_t r8;
          if (rr) r8 = rr[c];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float v = rs * (g[i][e] - m1 - xh[i][e] * m2);
            if (rr) v += (float)r8[e];
            o[e] = (bf16)v;
          }
          dxr[c] = o;
        }
      }
    }
  }
  // workgroup partials: waves 1..3 park their sums in LDS, wave 0 adds them in wave order
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    if (pass) __syncthreads();
    if (w > 0) {
#pragma unroll
      for (int i = 0; i < LN_MAXC; ++i)
        if (lane + i * WAVE < nch)
#pragma unroll
          for (int e = 0; e < 8; ++e) red[w - 1][(lane + i * WAVE) * 8 + e] = pass ? db[i][e] : dg[i][e];
    }
    __syncthreads();
    if (w == 0) {
      float* dst = partial + ((int64_t)pass * LN_BWD_BLOCKS + blockIdx.x) * D;
#pragma unroll
      for (int i = 0; i < LN_MAXC; ++i) {
        const int c = lane + i * WAVE;
        if (c < nch) {
          float o[8];
#pragma unroll
          for (int e = 0; e < 8; ++e)
            o[e] = (((pass ? db[i][e] : dg[i][e]) + red[0][c * 8 + e]) + red[1][c * 8 + e]) + red[2][c * 8 + e];
          *(float4*)(dst + c * 8) = make_float4(o[0], o[1], o[2], o[3]);
          *(float4*)(dst + c * 8 + 4) = make_float4(o[4], o[5], o[6], o[7]);
        }
      }
    }
  }
}

// Pass 1 of a column reduction over M rows: block (cx, r) sums rows of chunk r for 64 columns.
// WITH_XHAT: two sums, dy*xhat (slot 0) and dy (slot 1); otherwise the plain column sum (slot 0).
template <typename T, bool WITH_XHAT>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ a, int64_t ld,
                                                             const T* __restrict__ x,
                                                             const float* __restrict__ mean,
                                                             const float* __restrict__ rstd, int64_t M,
                                                             int N, int rows_per_chunk,
                                                             float* __restrict__ partial) {
  __shared__ float red[2][4][WAVE];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int col = blockIdx.x * WAVE + lane;
  const int64_t r0 = (int64_t)blockIdx.y * rows_per_chunk;
  const int64_t r1 = min(r0 + (int64_t)rows_per_chunk, M);
  float s0 = 0.f, s1 = 0.f;
  if (col < N) {
    for (int64_t m = r0 + w; m < r1; m += 4) {
      float v = (float)a[m * ld + col];
      if (WITH_XHAT) {
        s0 += v * ((float)x[m * ld + col] - mean[m]) * rstd[m];
        s1 += v;
      } else {
        s0 += v;
      }
    }
  }
  red[0][w][lane] = s0;
  red[1][w][lane] = s1;
  __syncthreads();
  if (w == 0 && col < N) {
    partial[(int64_t)blockIdx.y * N + col] = red[0][0][lane] + red[0][1][lane] + red[0][2][lane] + red[0][3][lane];
    if (WITH_XHAT)
      partial[(int64_t)(COLSUM_R + blockIdx.y) * N + col] =
          red[1][0][lane] + red[1][1][lane] + red[1][2][lane] + red[1][3][lane];
  }
}

// Pass 2: out[col] = sum over chunks.  Wave w of the block adds chunks w, w+16, ... in ascending
// order, then the wave sums are added in wave order: a fixed order, bit-reproducible.  The second
// sum (if out1) starts `second` rows into the partial buffer.
constexpr int FINAL_WAVES = 16;
__global__ __launch_bounds__(FINAL_WAVES * WAVE) void colsum_final_kernel(const float* __restrict__ partial, int N,
                                                                          int chunks, int second,
                                                                          float* __restrict__ out0,
                                                                          float* __restrict__ out1) {
  __shared__ float red[2][FINAL_WAVES][WAVE];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int col = blockIdx.x * WAVE + lane;
  float s = 0.f, t = 0.f;
  if (col < N) {
#pragma unroll 4
    for (int r = w; r < chunks; r += FINAL_WAVES) {
      s += partial[(int64_t)r * N + col];
      if (out1) t += partial[(int64_t)(second + r) * N + col];
    }
  }
  red[0][w][lane] = s;
  red[1][w][lane] = t;
  __syncthreads();
  if (w == 0 && col < N) {
    float a0 = red[0][0][lane], a1 = red[1][0][lane];
#pragma unroll
    for (int i = 1; i < FINAL_WAVES; ++i) { a0 += red[0][i][lane]; a1 += red[1][i][lane]; }
    out0[col] = a0;
    if (out1) out1[col] = a1;
  }
}

// the same reduction for a table of LayerNorm backward passes: blockIdx.y picks the entry
__global__ __launch_bounds__(FINAL_WAVES * WAVE) void ln_deferred_final_kernel(LnDeferTable t) {
  __shared__ float red[2][FINAL_WAVES][WAVE];
  const LnDeferEntry e = t.e[blockIdx.y];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE, N = t.D;
  const int col = blockIdx.x * WAVE + lane;
  float s = 0.f, u = 0.f;
  if (col < N) {
#pragma unroll 4
    for (int r = w; r < e.blocks; r += FINAL_WAVES) {
      s += e.partial[(int64_t)r * N + col];
      u += e.partial[(int64_t)(LN_BWD_BLOCKS + r) * N + col];
    }
  }
  red[0][w][lane] = s;
  red[1][w][lane] = u;
  __syncthreads();
  if (w == 0 && col < N) {
    float a0 = red[0][0][lane], a1 = red[1][0][lane];
#pragma unroll
    for (int i = 1; i < FINAL_WAVES; ++i) { a0 += red[0][i][lane]; a1 += red[1][i][lane]; }
    e.dgamma[col] = a0;
    e.dbeta[col] = a1;
  }
}

// ---------------------------------------------------------------- stem helpers
// out[(b*N + p), (c*P + r)*P + q] = img[b, c, gy*P + r, gx*P + q],  p = gy*G + gx
template <typename T>
__global__ void patchify_kernel(const T* __restrict__ img, int B, int C, int S, int P,
                                T* __restrict__ out) {
  const int G = S / P, Kp = C * P * P;
  const int64_t total = (int64_t)B * G * G * Kp;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * blockDim.x) {
    int kk = (int)(i % Kp);
    int64_t bp = i / Kp;
    int p = (int)(bp % (G * G));
    int b = (int)(bp / (G * G));
    int q = kk % P, r = (kk / P) % P, c = kk / (P * P);
    int gy = p / G, gx = p % G;
    out[i] = img[(((int64_t)b * C + c) * S + gy * P + r) * S + gx * P + q];
  }
}

// the same copy in 16-byte pieces: V elements of one patch row at a time (P % V == 0, 16-byte aligned rows)
// Workgroups past the copy (cls_blocks of them, one per image) write the class-token rows of the token tensor,
// x[b, 0, :] = cls + pos[0] (Sec. 3.1): the same launch, since nothing else has to run before the embedding product.
template <typename T, int V>
__global__ void patchify_vec_kernel(const T* __restrict__ img, int B, int C, int S, int P, T* __restrict__ out,
                                    int copy_blocks, const float* __restrict__ cls, const float* __restrict__ pos,
                                    int T_, int D, T* __restrict__ x) {
  if ((int)blockIdx.x >= copy_blocks) {
    const int b = blockIdx.x - copy_blocks;
    for (int j = threadIdx.x; j < D; j += blockDim.x) x[(int64_t)b * T_ * D + j] = (T)(cls[j] + pos[j]);
    return;
  }
  const int G = S / P, PV = P / V;                      // pieces per patch row
  const int64_t total = (int64_t)B * G * G * C * P * PV;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  const int qv = (int)(i % PV);
  int64_t t = i / PV;
  const int r = (int)(t % P); t /= P;
  const int c = (int)(t % C); t /= C;
  const int p = (int)(t % (G * G));
  const int b = (int)(t / (G * G));
  const int gy = p / G, gx = p % G;
  const uint4 v = *(const uint4*)(img + (((int64_t)b * C + c) * S + gy * P + r) * S + gx * P + qv * V);
  *(uint4*)(out + i * V) = v;                           // out index = ((b*N + p) * C*P*P + (c*P + r)*P + qv*V)
}

template <typename T>
__global__ void write_cls_rows_kernel(const float* __restrict__ cls, const float* __restrict__ pos,
                                      int B, int T_, int D, T* __restrict__ x) {
  const int b = blockIdx.x;
  for (int j = threadIdx.x; j < D; j += blockDim.x) x[(int64_t)b * T_ * D + j] = (T)(cls[j] + pos[j]);
}

// ---------------------------------------------------------------- token importance and selection
// scores[b, j] = (sum_h cls_prob[b, h, 1 + j]) / H, heads added in ascending order (Eq. 6 read as
// the head mean of the post-softmax CLS row; the CLS column itself is not ranked).
__global__ void cls_head_mean_kernel(const float* __restrict__ cls_prob, int B, int H, int T_,
                                     float* __restrict__ scores) {
  const int n = T_ - 1;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)B * n) return;
  const int b = (int)(i / n), j = (int)(i % n);
  float s = 0.f;
  for (int h = 0; h < H; ++h) s += cls_prob[((int64_t)b * H + h) * T_ + 1 + j];
  scores[i] = s / (float)H;
}

// One workgroup of 4 wavefronts per image.  Token j is kept when fewer than k tokens beat it (larger
// score, or the same score and a lower index).  Each thread ranks one token per pass of 256; kept
// indices are written in ascending order through ballot prefixes within a wave and a running
// offset across waves and passes.
// With cls_prob given, the scores are first formed here as the head mean of the CLS softmax rows
// (heads added in ascending order, then divided by H, as in cls_head_mean_kernel) and stored.
__global__ __launch_bounds__(256) void topk_select_kernel(float* __restrict__ scores, int n, int k,
                                                          int32_t* __restrict__ idx,
                                                          const float* __restrict__ cls_prob, int H) {
  __shared__ float sc[1024];
  __shared__ int wave_count[4];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid % WAVE, w = tid / WAVE;
  for (int j = tid; j < n; j += 256) {
    float v;
    if (cls_prob) {
      v = 0.f;
      for (int h = 0; h < H; ++h) v += cls_prob[((int64_t)b * H + h) * (n + 1) + 1 + j];
      v /= (float)H;
      scores[(int64_t)b * n + j] = v;
    } else {
      v = scores[(int64_t)b * n + j];
    }
    // a NaN score (a diverged step) compares false with everything: ranked as it stands it would be "ahead of
    // nobody and behind nobody" and more than k tokens would be kept.  It ranks last instead (the order stays total).
    sc[j] = (v == v) ? v : -INFINITY;
  }
  __syncthreads();
  int base = 0;
  for (int c0 = 0; c0 < n; c0 += 256) {
    const int j = c0 + tid;
    bool keep = false;
    if (j < n) {
      const float mine = sc[j];
      int ahead = 0;
#pragma unroll 8
      for (int i = 0; i < n; ++i) {
        const float o = sc[i];
        ahead += (o > mine || (o == mine && i < j)) ? 1 : 0;
      }
      keep = ahead < k;
    }
    const unsigned long long mask = __ballot(keep);
    if (lane == 0) wave_count[w] = __popcll(mask);
    __syncthreads();
    int before = base;
    for (int v = 0; v < w; ++v) before += wave_count[v];
    const int slot = before + __popcll(mask & ((1ull << lane) - 1ull));
    if (keep && slot < k) idx[(int64_t)b * k + slot] = j;
    base += wave_count[0] + wave_count[1] + wave_count[2] + wave_count[3];
    __syncthreads();
  }
}

// y[b,0] = x[b,0]; y[b,1+i] = x[b,1+idx[b,i]].  One block per output row, 16-byte accesses.
__global__ void gather_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ idx,
                                   int T_, int k, int T_out, int row_vecs, uint4* __restrict__ y) {
  const int i = blockIdx.x, b = blockIdx.y;
  const int src = (i == 0) ? 0 : 1 + idx[(int64_t)b * k + i - 1];
  const uint4* s = x + ((int64_t)b * T_ + src) * row_vecs;
  uint4* d = y + ((int64_t)b * T_out + i) * row_vecs;
  for (int v = threadIdx.x; v < row_vecs; v += blockDim.x) d[v] = s[v];
}

// Fusion of the dropped tokens of one image (Sec. 4.1): the importance-weighted average
// f = sum_j w_j x[1+j], w_j = a_j / sum over the dropped j of a_j, written as row k+1 of y (pitch k+2).
// fw [B,n] receives the weights (0 for kept tokens), the backward pass reuses them as constants.
// One workgroup per image; every thread owns columns and adds the tokens in ascending order.
template <typename T>
__global__ __launch_bounds__(256) void fuse_dropped_kernel(const T* __restrict__ x, const float* __restrict__ scores,
                                                           const int32_t* __restrict__ idx, int T_, int k, int D,
                                                           float* __restrict__ fw, T* __restrict__ y) {
  __shared__ float w[1024];
  __shared__ float red[256];
  const int b = blockIdx.x, n = T_ - 1, tid = threadIdx.x;
  for (int j = tid; j < n; j += 256) w[j] = scores[(int64_t)b * n + j];
  __syncthreads();
  for (int i = tid; i < k; i += 256) w[idx[(int64_t)b * k + i]] = 0.f;
  __syncthreads();
  float part = 0.f;
  for (int j = tid; j < n; j += 256) part += w[j];
  red[tid] = part;
  __syncthreads();
  if (tid == 0) {
    float tot = 0.f;
    for (int i = 0; i < 256; ++i) tot += red[i];     // fixed order
    red[0] = 1.0f / tot;
  }
  __syncthreads();
  const float inv = red[0];
  for (int j = tid; j < n; j += 256) {
    const float v = w[j] * inv;
    fw[(int64_t)b * n + j] = v;
  }
  const T* xb = x + ((int64_t)b * T_ + 1) * D;
  for (int c = tid; c < D; c += 256) {
    float acc = 0.f;
    for (int j = 0; j < n; ++j) {
      const float wj = w[j];
      if (wj != 0.f) acc = fmaf(wj * inv, (float)xb[(int64_t)j * D + c], acc);
    }
    y[((int64_t)b * (k + 2) + k + 1) * D + c] = (T)acc;
  }
}

// Adjoint of gather + fusion: rows [CLS; kept; fused] of dy (pitch k+2) -> dx [B,T,D]; a dropped
// token j receives fw[j] times the gradient of the fused token.  Every row is written exactly once.
template <typename T>
__global__ void scatter_fused_kernel(const T* __restrict__ dy, const int32_t* __restrict__ idx,
                                     const float* __restrict__ fw, int T_, int k, int D, T* __restrict__ dx) {
  const int t = blockIdx.x, b = blockIdx.y;
  int src = -1;
  if (t == 0) {
    src = 0;
  } else {
    const int32_t* row = idx + (int64_t)b * k;
    int lo = 0, hi = k - 1;
    while (lo <= hi) {
      int mid = (lo + hi) >> 1;
      int v = row[mid];
      if (v == t - 1) { src = 1 + mid; break; }
      if (v < t - 1) lo = mid + 1; else hi = mid - 1;
    }
  }
  T* d = dx + ((int64_t)b * T_ + t) * D;
  if (src >= 0) {
    const T* s = dy + ((int64_t)b * (k + 2) + src) * D;
    for (int c = threadIdx.x; c < D; c += blockDim.x) d[c] = s[c];
  } else {
    const float wj = fw[(int64_t)b * (T_ - 1) + t - 1];
    const T* s = dy + ((int64_t)b * (k + 2) + k + 1) * D;
    for (int c = threadIdx.x; c < D; c += blockDim.x) d[c] = (T)(wj * (float)s[c]);
  }
}

// Adjoint of the gather: every row of dx is written exactly once (kept rows copied, dropped rows
// zero), found by a binary search of the ascending kept list — no atomics, no separate memset.
__global__ void scatter_rows_kernel(const uint4* __restrict__ dy, const int32_t* __restrict__ idx,
                                    int T_, int k, int row_vecs, uint4* __restrict__ dx) {
  const int t = blockIdx.x, b = blockIdx.y;
  int src = -1;
  if (t == 0) {
    src = 0;
  } else {
    const int32_t* row = idx + (int64_t)b * k;
    int lo = 0, hi = k - 1;
    while (lo <= hi) {
      int mid = (lo + hi) >> 1;
      int v = row[mid];
      if (v == t - 1) { src = 1 + mid; break; }
      if (v < t - 1) lo = mid + 1; else hi = mid - 1;
    }
  }
  uint4* d = dx + ((int64_t)b * T_ + t) * row_vecs;
  if (src < 0) {
    for (int v = threadIdx.x; v < row_vecs; v += blockDim.x) d[v] = make_uint4(0, 0, 0, 0);
  } else {
    const uint4* s = dy + ((int64_t)b * (k + 1) + src) * row_vecs;
    for (int v = threadIdx.x; v < row_vecs; v += blockDim.x) d[v] = s[v];
  }
}

// ---------------------------------------------------------------- head helpers
template <typename T>
__global__ void extract_cls_kernel(const T* __restrict__ x, int T_, int D, float* __restrict__ out) {
  const int b = blockIdx.x;
  for (int j = threadIdx.x; j < D; j += blockDim.x) out[(int64_t)b * D + j] = (float)x[(int64_t)b * T_ * D + j];
}

template <typename T>
__global__ void place_cls_grad_kernel(const float* __restrict__ dxc, int T_, int D, T* __restrict__ dx) {
  const int t = blockIdx.x, b = blockIdx.y;
  T* d = dx + ((int64_t)b * T_ + t) * D;
  for (int j = threadIdx.x; j < D; j += blockDim.x) d[j] = (t == 0) ? (T)dxc[(int64_t)b * D + j] : (T)0.f;
}

// One wavefront per image: loss_b = logsumexp(z) - z[y]; dlogits = (softmax(z) - onehot) / B.
__global__ __launch_bounds__(WAVE) void cross_entropy_kernel(const float* __restrict__ logits,
                                                             const int32_t* __restrict__ labels, int B,
                                                             int C, float* __restrict__ loss_rows,
                                                             float* __restrict__ dlogits) {
  const int b = blockIdx.x, lane = threadIdx.x;
  const float* z = logits + (int64_t)b * C;
  float mx = -INFINITY;
  for (int c = lane; c < C; c += WAVE) mx = fmaxf(mx, z[c]);
  mx = wave_max(mx);
  float s = 0.f;
  for (int c = lane; c < C; c += WAVE) s += expf(z[c] - mx);
  const float lse = mx + logf(wave_sum(s));
  const int y = labels[b];
  if (lane == 0) loss_rows[b] = lse - ((y >= 0 && y < C) ? z[y] : 0.f);
  for (int c = lane; c < C; c += WAVE)
    dlogits[(int64_t)b * C + c] = (expf(z[c] - lse) - (c == y ? 1.f : 0.f)) / (float)B;
}

__global__ void mean_of_rows_kernel(const float* __restrict__ v, int n, float scale, float* __restrict__ out) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    float s = 0.f;
    for (int i = 0; i < n; ++i) s += v[i];
    *out = s * scale;
  }
}

constexpr int MSQ_BLOCKS = 256;
template <typename T>
__global__ __launch_bounds__(256) void mean_sq_kernel(const T* __restrict__ x, int64_t n,
                                                      float* __restrict__ partial, T* __restrict__ dx) {
  __shared__ float red[4];
  const int64_t per = (n + MSQ_BLOCKS - 1) / MSQ_BLOCKS;
  const int64_t i0 = (int64_t)blockIdx.x * per, i1 = min(i0 + per, n);
  const float g = 2.0f / (float)n;
  float s = 0.f;
  for (int64_t i = i0 + threadIdx.x; i < i1; i += blockDim.x) {
    float v = (float)x[i];
    s += v * v;
    if (dx) dx[i] = (T)(v * g);
  }
  s = wave_sum(s);
  if (threadIdx.x % WAVE == 0) red[threadIdx.x / WAVE] = s;
  __syncthreads();
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

// ---------------------------------------------------------------- weights: casts and SGD
// A table of matrices in one launch.  64x64 tiles, 16-byte accesses; the tile goes through LDS so
// that both the straight [rows,cols] and the transposed [cols,rows] bf16 copies are written with
// contiguous rows.  With UPDATE the tile is first updated by SGD (Sec. 5 of the paper):
//   g' = g + wd*w;  mu > 0: m = mu*m + g', w -= lr*m;  else w -= lr*g'.
// rows and cols are multiples of 4.
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));

// one element of the optimiser update; m / v2 are the element's moments, used and rewritten only by
// the rules that have them
__device__ inline float opt_update(const OptArgs& o, float w, float g, float& m, float& v2) {
  if (o.kind == OPT_ADAMW) {
    m = o.b1 * m + (1.0f - o.b1) * g;
    v2 = o.b2 * v2 + (1.0f - o.b2) * g * g;
    return w - o.lr * ((m / o.bc1) / (sqrtf(v2 / o.bc2) + o.eps) + o.wd * w);
  }
  float gp = g + o.wd * w;
  if (o.mu > 0.f) {
    gp = o.mu * m + gp;
    m = gp;
  }
  return w - o.lr * gp;
}

// four consecutive elements at offset off (16-byte accesses)
__device__ inline float4 opt_update4(const OptArgs& o, float4 w, float4 g, float* m, float* v2, int64_t off) {
  const bool use_m = o.kind == OPT_ADAMW || o.mu > 0.f, use_v = o.kind == OPT_ADAMW;
  float4 mm = use_m ? *(const float4*)(m + off) : make_float4(0.f, 0.f, 0.f, 0.f);
  float4 vv = use_v ? *(const float4*)(v2 + off) : make_float4(0.f, 0.f, 0.f, 0.f);
  w.x = opt_update(o, w.x, g.x, mm.x, vv.x);
  w.y = opt_update(o, w.y, g.y, mm.y, vv.y);
  w.z = opt_update(o, w.z, g.z, mm.z, vv.z);
  w.w = opt_update(o, w.w, g.w, mm.w, vv.w);
  if (use_m) *(float4*)(m + off) = mm;
  if (use_v) *(float4*)(v2 + off) = vv;
  return w;
}

template <bool UPDATE>
__global__ __launch_bounds__(256) void matrix_table_kernel(MatTable t, OptArgs o) {
  __shared__ float tile[64][65];
  int ei = 0;
  while (ei + 1 < t.count && (int)blockIdx.x >= t.e[ei + 1].tile_start) ++ei;
  const MatEntry e = t.e[ei];
  const int local = blockIdx.x - e.tile_start, tiles_x = (e.cols + 63) / 64;
  const int c0 = (local % tiles_x) * 64, r0 = (local / tiles_x) * 64;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int lr_ = ty + 16 * i, r = r0 + lr_, c = c0 + 4 * tx;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r < e.rows && c < e.cols) {
      const int64_t off = (int64_t)r * e.cols + c;
      v = *(const float4*)(e.w + off);
      if (UPDATE) {
        const float4 g = *(const float4*)(e.g + off);
        v = opt_update4(o, v, g, e.m, e.v2, off);
        *(float4*)(e.w + off) = v;
      }
      if (e.s) {
        bf16x4_t o;
        o[0] = (bf16)v.x; o[1] = (bf16)v.y; o[2] = (bf16)v.z; o[3] = (bf16)v.w;
        *(bf16x4_t*)(e.s + off) = o;
      }
    }
    tile[lr_][4 * tx + 0] = v.x; tile[lr_][4 * tx + 1] = v.y; tile[lr_][4 * tx + 2] = v.z; tile[lr_][4 * tx + 3] = v.w;
  }
  __syncthreads();
  if (e.t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int cc = ty + 16 * i, c = c0 + cc, r = r0 + 4 * tx;
      if (c < e.cols && r < e.rows) {
        bf16x4_t o;
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = (bf16)tile[4 * tx + j][cc];
        *(bf16x4_t*)(e.t + (int64_t)c * e.rows + r) = o;
      }
    }
  }
}

// SGD on a table of small tensors (biases, LayerNorm parameters, the head) in one launch:
// blockIdx.y picks the tensor, blockIdx.x a slice of 1024 elements.
__global__ __launch_bounds__(256) void sgd_table_kernel(SgdTable t, OptArgs o) {
  const SgdEntry e = t.e[blockIdx.y];
  const int64_t i0 = (int64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int64_t i = i0 + 256 * j;
    if (i >= e.n) break;
    const bool use_m = o.kind == OPT_ADAMW || o.mu > 0.f, use_v = o.kind == OPT_ADAMW;
    float mm = use_m ? e.m[i] : 0.f, vv = use_v ? e.v2[i] : 0.f;
    e.w[i] = opt_update(o, e.w[i], e.g[i], mm, vv);
    if (use_m) e.m[i] = mm;
    if (use_v) e.v2[i] = vv;
  }
}

inline int rows_per_chunk(int64_t M) { return (int)((M + COLSUM_R - 1) / COLSUM_R); }
inline int chunks_of(int64_t M) {
  int rpc = rows_per_chunk(M);
  return (int)((M + rpc - 1) / rpc);
}

// LayerNorm folded into the frozen linear layer behind it: one thread per output column n walks k in
// ascending order, so the column sum is the sum of exactly the rounded values the matrix cores will see.
__global__ __launch_bounds__(128) void ln_fold_kernel(const float* __restrict__ w, const float* __restrict__ bias,
                                                     const float* __restrict__ gamma, const float* __restrict__ beta,
                                                     int in, int out, bf16* __restrict__ w_t, float* __restrict__ colsum,
                                                     float* __restrict__ bias_out) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= out) return;
  float cs = 0.f, bb = bias[n];
  for (int k0 = 0; k0 < in; k0 += 8) {
    bf16x8_t o;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float wv = w[(int64_t)(k0 + j) * out + n];
      const bf16 r = (bf16)(wv * gamma[k0 + j]);
      o[j] = r;
      cs += (float)r;
      bb = fmaf(beta[k0 + j], wv, bb);
    }
    *(bf16x8_t*)(w_t + (int64_t)n * in + k0) = o;
  }
  colsum[n] = cs;
  bias_out[n] = bb;
}

}  // namespace

// ---------------------------------------------------------------- launchers

void layernorm_fwd(const void* x, int64_t M, int D, const float* gamma, const float* beta, float eps,
                   bool f32, void* y, float* mean, float* rstd, hipStream_t s) {
  if (M <= 0) return;
  dim3 grid((unsigned)((M + 3) / 4));
  if (f32) ln_fwd_kernel<float><<<grid, 256, 0, s>>>((const float*)x, M, D, gamma, beta, eps, (float*)y, mean, rstd);
  else if (D % 8 == 0 && D <= 8 * WAVE * LN_MAXC)
    ln_fwd_vec_kernel<<<grid, 256, 0, s>>>((const bf16*)x, M, D, gamma, beta, eps, (bf16*)y, mean, rstd, nullptr, 0, 0, nullptr);
  else ln_fwd_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)x, M, D, gamma, beta, eps, (bf16*)y, mean, rstd);
}

bool gather_layernorm_fwd(const void* x, const int32_t* idx, int B, int T, int k, int D, const float* gamma,
                          const float* beta, float eps, bool f32, void* x_kept, void* y, float* mean, float* rstd,
                          hipStream_t s) {
  if (f32 || D % 8 != 0 || D > 8 * WAVE * LN_MAXC || B <= 0) return false;
  const int64_t M = (int64_t)B * (k + 1);
  // k == 0: only the class tokens; the kernel then never reads idx, which may be null: give it any non-null value
  const int32_t* ip = idx ? idx : (const int32_t*)x;
  ln_fwd_vec_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const bf16*)x, M, D, gamma, beta, eps, (bf16*)y, mean, rstd, ip, T, k,
                                                           (bf16*)x_kept);
  return true;
}

void layernorm_bwd_dx(const void* dy, const void* x, const float* mean, const float* rstd,
                      const float* gamma, const void* res, int64_t M, int D, bool f32, void* dx,
                      hipStream_t s) {
  if (M <= 0 || !dx) return;
  dim3 grid((unsigned)((M + 3) / 4));
  if (f32)
    ln_bwd_dx_kernel<float><<<grid, 256, 0, s>>>((const float*)dy, (const float*)x, mean, rstd, gamma,
                                                  (const float*)res, M, D, (float*)dx);
  else if (D % 8 == 0 && D <= 8 * WAVE * LN_MAXC)
    ln_bwd_dx_vec_kernel<<<grid, 256, 0, s>>>((const bf16*)dy, (const bf16*)x, mean, rstd, gamma,
                                              (const bf16*)res, M, D, (bf16*)dx);
  else
    ln_bwd_dx_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)dy, (const bf16*)x, mean, rstd, gamma,
                                                 (const bf16*)res, M, D, (bf16*)dx);
}

void layernorm_bwd(const void* dy, const void* x, const float* mean, const float* rstd, const float* gamma,
                   const void* res, int64_t M, int D, bool f32, void* dx, float* partial, float* dgamma,
                   float* dbeta, hipStream_t s) {
  if (M <= 0) return;
  if (!f32 && D % 8 == 0 && D <= 8 * WAVE * LN_MAXC) {
    const int blocks = (int)std::min<int64_t>(LN_BWD_BLOCKS, (M + 3) / 4);
    ln_bwd_fused_vec_kernel<<<blocks, 256, 0, s>>>((const bf16*)dy, (const bf16*)x, mean, rstd, gamma,
                                                   (const bf16*)res, M, D, (bf16*)dx, partial);
    colsum_final_kernel<<<(D + WAVE - 1) / WAVE, FINAL_WAVES * WAVE, 0, s>>>(partial, D, blocks, LN_BWD_BLOCKS,
                                                                           dgamma, dbeta);
    return;
  }
  layernorm_bwd_params(dy, x, mean, rstd, M, D, f32, partial, dgamma, dbeta, s);
  layernorm_bwd_dx(dy, x, mean, rstd, gamma, res, M, D, f32, dx, s);
}

size_t ln_deferred_partial_floats(int D) { return (size_t)2 * LN_BWD_BLOCKS * (size_t)D; }

bool layernorm_bwd_deferred(const void* dy, const void* x, const float* mean, const float* rstd, const float* gamma,
                            const void* res, int64_t M, int D, bool f32, void* dx, float* partial, float* dgamma,
                            float* dbeta, LnDeferTable& t, hipStream_t s) {
  if (M <= 0 || f32 || D % 8 != 0 || D > 8 * WAVE * LN_MAXC || !partial || t.count >= LN_DEFER_MAX ||
      (t.count > 0 && t.D != D))
    return false;
  const int blocks = (int)std::min<int64_t>(LN_BWD_BLOCKS, (M + 3) / 4);
  ln_bwd_fused_vec_kernel<<<blocks, 256, 0, s>>>((const bf16*)dy, (const bf16*)x, mean, rstd, gamma,
                                                 (const bf16*)res, M, D, (bf16*)dx, partial);
  t.D = D;
  t.e[t.count++] = LnDeferEntry{partial, dgamma, dbeta, blocks};
  return true;
}

void ln_deferred_finish(LnDeferTable& t, hipStream_t s) {
  if (t.count == 0) return;
  ln_deferred_final_kernel<<<dim3((t.D + WAVE - 1) / WAVE, t.count), FINAL_WAVES * WAVE, 0, s>>>(t);
  t.count = 0;
}

size_t colsum_partial_floats(int64_t, int N) { return (size_t)2 * std::max(COLSUM_R, LN_BWD_BLOCKS) * (size_t)N; }

void layernorm_bwd_params(const void* dy, const void* x, const float* mean, const float* rstd,
                          int64_t M, int D, bool f32, float* partial, float* dgamma, float* dbeta,
                          hipStream_t s) {
  if (M <= 0) return;
  const int rpc = rows_per_chunk(M), ch = chunks_of(M);
  dim3 grid((D + WAVE - 1) / WAVE, ch);
  if (f32)
    colsum_partial_kernel<float, true><<<grid, 256, 0, s>>>((const float*)dy, D, (const float*)x, mean, rstd, M, D, rpc, partial);
  else
    colsum_partial_kernel<bf16, true><<<grid, 256, 0, s>>>((const bf16*)dy, D, (const bf16*)x, mean, rstd, M, D, rpc, partial);
  colsum_final_kernel<<<(D + WAVE - 1) / WAVE, FINAL_WAVES * WAVE, 0, s>>>(partial, D, ch, COLSUM_R, dgamma, dbeta);
}

void colsum(const void* a, int64_t M, int N, int64_t ld, bool f32, float* partial, float* out,
            hipStream_t s) {
  if (M <= 0) return;
  const int rpc = rows_per_chunk(M), ch = chunks_of(M);
  dim3 grid((N + WAVE - 1) / WAVE, ch);
  if (f32)
    colsum_partial_kernel<float, false><<<grid, 256, 0, s>>>((const float*)a, ld, nullptr, nullptr, nullptr, M, N, rpc, partial);
  else
    colsum_partial_kernel<bf16, false><<<grid, 256, 0, s>>>((const bf16*)a, ld, nullptr, nullptr, nullptr, M, N, rpc, partial);
  colsum_final_kernel<<<(N + WAVE - 1) / WAVE, FINAL_WAVES * WAVE, 0, s>>>(partial, N, ch, 0, out, nullptr);
}

void patchify(const void* img, int B, int C, int S, int P, bool f32, void* out, hipStream_t s, const float* cls,
              const float* pos, int T, int D, void* x) {
  const int64_t total = (int64_t)B * C * S * S;
  const int V = f32 ? 4 : 8;                             // elements per 16 bytes
  if (P % V == 0 && S % V == 0 && (((uintptr_t)img | (uintptr_t)out) & 15) == 0) {
    const unsigned vgrid = (unsigned)((total / V + 255) / 256), extra = cls ? (unsigned)B : 0u;
    if (f32) patchify_vec_kernel<float, 4><<<vgrid + extra, 256, 0, s>>>((const float*)img, B, C, S, P, (float*)out, (int)vgrid, cls, pos, T, D, (float*)x);
    else patchify_vec_kernel<bf16, 8><<<vgrid + extra, 256, 0, s>>>((const bf16*)img, B, C, S, P, (bf16*)out, (int)vgrid, cls, pos, T, D, (bf16*)x);
    return;
  }
  const unsigned grid = (unsigned)std::min<int64_t>((total + 255) / 256, 65536);
  if (f32) patchify_kernel<float><<<grid, 256, 0, s>>>((const float*)img, B, C, S, P, (float*)out);
  else patchify_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)img, B, C, S, P, (bf16*)out);
  if (cls) write_cls_rows(cls, pos, B, T, D, f32, x, s);
}

void write_cls_rows(const float* cls, const float* pos, int B, int T, int D, bool f32, void* x,
                    hipStream_t s) {
  if (f32) write_cls_rows_kernel<float><<<B, 256, 0, s>>>(cls, pos, B, T, D, (float*)x);
  else write_cls_rows_kernel<bf16><<<B, 256, 0, s>>>(cls, pos, B, T, D, (bf16*)x);
}

void cls_head_mean(const float* cls_prob, int B, int H, int T, float* scores, hipStream_t s) {
  const int64_t total = (int64_t)B * (T - 1);
  if (total <= 0) return;
  cls_head_mean_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(cls_prob, B, H, T, scores);
}

void topk_select(const float* scores, int B, int n, int k, int32_t* idx, hipStream_t s) {
  if (B <= 0 || k <= 0) return;
  topk_select_kernel<<<B, 256, 0, s>>>(const_cast<float*>(scores), n, k, idx, nullptr, 0);
}

void topk_select_from_cls(const float* cls_prob, int B, int H, int T, int k, float* scores, int32_t* idx,
                          hipStream_t s) {
  if (B <= 0) return;
  topk_select_kernel<<<B, 256, 0, s>>>(scores, T - 1, k, idx, cls_prob, H);
}

void gather_tokens(const void* x, const int32_t* idx, int B, int T, int k, int D, bool f32, void* y,
                   hipStream_t s, int T_out) {
  const int row_vecs = D * (f32 ? 4 : 2) / 16;
  gather_rows_kernel<<<dim3(k + 1, B), 64, 0, s>>>((const uint4*)x, idx, T, k, T_out > 0 ? T_out : k + 1, row_vecs,
                                                  (uint4*)y);
}

void fuse_dropped(const void* x, const float* scores, const int32_t* idx, int B, int T, int k, int D, bool f32,
                  float* fw, void* y, hipStream_t s) {
  if (f32) fuse_dropped_kernel<float><<<B, 256, 0, s>>>((const float*)x, scores, idx, T, k, D, fw, (float*)y);
  else fuse_dropped_kernel<bf16><<<B, 256, 0, s>>>((const bf16*)x, scores, idx, T, k, D, fw, (bf16*)y);
}

void scatter_tokens(const void* dy, const int32_t* idx, int B, int T, int k, int D, bool f32,
                    void* dx, hipStream_t s, const float* fw) {
  if (fw) {   // rows of dy are [CLS; kept; fused]
    if (f32) scatter_fused_kernel<float><<<dim3(T, B), 128, 0, s>>>((const float*)dy, idx, fw, T, k, D, (float*)dx);
    else scatter_fused_kernel<bf16><<<dim3(T, B), 128, 0, s>>>((const bf16*)dy, idx, fw, T, k, D, (bf16*)dx);
    return;
  }
  const int row_vecs = D * (f32 ? 4 : 2) / 16;
  scatter_rows_kernel<<<dim3(T, B), 64, 0, s>>>((const uint4*)dy, idx, T, k, row_vecs, (uint4*)dx);
}

void extract_cls(const void* x, int B, int T, int D, bool f32, float* out, hipStream_t s) {
  if (f32) extract_cls_kernel<float><<<B, 256, 0, s>>>((const float*)x, T, D, out);
  else extract_cls_kernel<bf16><<<B, 256, 0, s>>>((const bf16*)x, T, D, out);
}

void place_cls_grad(const float* dxc, int B, int T, int D, bool f32, void* dx, hipStream_t s) {
  if (f32) place_cls_grad_kernel<float><<<dim3(T, B), 128, 0, s>>>(dxc, T, D, (float*)dx);
  else place_cls_grad_kernel<bf16><<<dim3(T, B), 128, 0, s>>>(dxc, T, D, (bf16*)dx);
}

void cross_entropy(const float* logits, const int32_t* labels, int B, int C, float* loss_rows,
                   float* dlogits, float* loss, hipStream_t s) {
  cross_entropy_kernel<<<B, WAVE, 0, s>>>(logits, labels, B, C, loss_rows, dlogits);
  mean_of_rows_kernel<<<1, 64, 0, s>>>(loss_rows, B, 1.0f / (float)B, loss);
}

size_t mean_sq_partial_floats() { return MSQ_BLOCKS; }

void mean_sq_loss(const void* x, int64_t n, bool f32, float* partial, float* loss, void* dx,
                  hipStream_t s) {
  if (f32) mean_sq_kernel<float><<<MSQ_BLOCKS, 256, 0, s>>>((const float*)x, n, partial, (float*)dx);
  else mean_sq_kernel<bf16><<<MSQ_BLOCKS, 256, 0, s>>>((const bf16*)x, n, partial, (bf16*)dx);
  mean_of_rows_kernel<<<1, 64, 0, s>>>(partial, MSQ_BLOCKS, 1.0f / (float)n, loss);
}

void ln_fold_weights(const float* w, const float* bias, const float* gamma, const float* beta, int in, int out,
                     bf16* w_t, float* colsum, float* bias_out, hipStream_t s) {
  ln_fold_kernel<<<(out + 127) / 128, 128, 0, s>>>(w, bias, gamma, beta, in, out, w_t, colsum, bias_out);
}

void matrix_table_add(MatTable& t, float* w, const float* g, float* m, float* v2, int rows, int cols, bf16* straight,
                      bf16* transposed) {
  MatEntry& e = t.e[t.count];
  e.w = w; e.g = g; e.m = m; e.v2 = v2; e.s = straight; e.t = transposed; e.rows = rows; e.cols = cols;
  e.tile_start = t.total_tiles;
  t.total_tiles += ((rows + 63) / 64) * ((cols + 63) / 64);
  ++t.count;
}

void matrix_table_run(const MatTable& t, bool update, const OptArgs& o, hipStream_t s) {
  if (t.count == 0) return;
  if (update) matrix_table_kernel<true><<<t.total_tiles, 256, 0, s>>>(t, o);
  else matrix_table_kernel<false><<<t.total_tiles, 256, 0, s>>>(t, OptArgs());
}

void sgd_table(const SgdTable& t, int count, const OptArgs& o, hipStream_t s) {
  if (count <= 0) return;
  int64_t nmax = 0;
  for (int i = 0; i < count; ++i) nmax = std::max(nmax, t.e[i].n);
  sgd_table_kernel<<<dim3((unsigned)((nmax + 1023) / 1024), count), 256, 0, s>>>(t, o);
}

}  // namespace bsr
