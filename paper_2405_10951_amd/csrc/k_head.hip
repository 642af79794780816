// Classification head of the fine-tuning step in two launches (Sec. 3.1: the class token feeds the
// classifier; the loss is the batch mean of the cross-entropy):
//   head_rows_kernel   one workgroup per image: final LayerNorm of the class token, logits, loss of the
//                      image, dlogits = (softmax - onehot) / B, dz = dlogits . W_h^T, the LayerNorm
//                      backward of that row, and the gradient at the last block's output (the class
//                      row gets it, every other token row is zero);
//   head_batch_kernel  the sums over the batch: loss, dW_h = z^T dlogits, db_h, dgamma_f, dbeta_f,
//                      each added over the images in ascending order (bit-reproducible).
// All arithmetic is fp32 whatever the activation type.
#include "bsr_internal.h"

#include <stdint.h>

namespace bsr {
namespace {

constexpr int WAVE = 64, HT = 1024, HW = HT / WAVE;    // threads and wavefronts per workgroup of the row kernel
constexpr int NPART = 8;                               // d-ranges the logits are split over
constexpr int BT = 256;                                // threads per workgroup of the batch kernel
constexpr int RPP = 16;                                // rows of W_h a wavefront has in flight in the dz pass

__device__ inline float wave_sum_h(float v) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ inline float wave_max_h(float v) {
#pragma unroll
  for (int o = WAVE / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}
// sum (or max) over the workgroup; every thread gets the result; red: HW floats of LDS
__device__ inline float block_sum(float v, float* red) {
  v = wave_sum_h(v);
  __syncthreads();
  if (threadIdx.x % WAVE == 0) red[threadIdx.x / WAVE] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int i = 1; i < HW; ++i) s += red[i];
  return s;
}
__device__ inline float block_max(float v, float* red) {
  v = wave_max_h(v);
  __syncthreads();
  if (threadIdx.x % WAVE == 0) red[threadIdx.x / WAVE] = v;
  __syncthreads();
  float s = red[0];
#pragma unroll
  for (int i = 1; i < HW; ++i) s = fmaxf(s, red[i]);
  return s;
}

template <typename T>
__global__ __launch_bounds__(HT) void head_rows_kernel(const T* __restrict__ x, int Tl, int D, int C, int B,
                                                       const float* __restrict__ gamma, const float* __restrict__ beta,
                                                       float eps, const float* __restrict__ w_head,
                                                       const float* __restrict__ b_head, const int32_t* __restrict__ labels,
                                                       float* __restrict__ xhat_out, float* __restrict__ z_out,
                                                       float* __restrict__ logits_out, float* __restrict__ dlogits_out,
                                                       float* __restrict__ dz_out, float* __restrict__ loss_rows,
                                                       T* __restrict__ dx) {
  extern __shared__ float sm[];
  float* xh = sm;                 // [D] normalised class token
  float* zs = xh + D;             // [D] LayerNorm output
  float* lg = zs + D;             // [C] logits, then dlogits
  float* part = lg + C;           // [NPART][C] partial logits
  float* red = part + NPART * C;  // [HW]
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid % WAVE, w = tid / WAVE;
  const T* xr = x + (int64_t)b * Tl * D;
  // final LayerNorm of the class token (two passes over the row held in LDS)
  float s = 0.f;
  for (int d = tid; d < D; d += HT) { const float v = (float)xr[d]; xh[d] = v; s += v; }
  const float mean = block_sum(s, red) / (float)D;
  float q = 0.f;
  for (int d = tid; d < D; d += HT) { const float v = xh[d] - mean; q += v * v; }
  const float rstd = rsqrtf(block_sum(q, red) / (float)D + eps);
  for (int d = tid; d < D; d += HT) {
    const float h = (xh[d] - mean) * rstd, z = h * gamma[d] + beta[d];
    xh[d] = h; zs[d] = z;
    xhat_out[(int64_t)b * D + d] = h;
    z_out[(int64_t)b * D + d] = z;
  }
  __syncthreads();
  // logits: wavefront w covers the d-range of part w % NPART, its lanes walk the classes of the chunks
  // w / NPART, w / NPART + HW / NPART, ...; four independent accumulators keep loads in flight
  {
    const int pt = w % NPART;
    const int d0 = (int)((int64_t)pt * D / NPART), d1 = (int)((int64_t)(pt + 1) * D / NPART);
    for (int c0 = (w / NPART) * WAVE; c0 < C; c0 += (HW / NPART) * WAVE) {
      const int c = c0 + lane;
      if (c < C) {
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        const float* wc = w_head + c;
        int d = d0;
        for (; d + 31 < d1; d += 32) {          // 32 loads in flight
          float wv[32];
#pragma unroll
          for (int u = 0; u < 32; ++u) wv[u] = wc[(int64_t)(d + u) * C];
#pragma unroll
          for (int u = 0; u < 32; u += 4) {
            a0 = fmaf(zs[d + u], wv[u], a0);
            a1 = fmaf(zs[d + u + 1], wv[u + 1], a1);
            a2 = fmaf(zs[d + u + 2], wv[u + 2], a2);
            a3 = fmaf(zs[d + u + 3], wv[u + 3], a3);
          }
        }
        for (; d < d1; ++d) a0 = fmaf(zs[d], wc[(int64_t)d * C], a0);
        part[pt * C + c] = (a0 + a1) + (a2 + a3);
      }
    }
  }
  __syncthreads();
  for (int c = tid; c < C; c += HT) {
    float a = b_head ? b_head[c] : 0.f;
#pragma unroll
    for (int i = 0; i < NPART; ++i) a += part[i * C + c];
    lg[c] = a;
    logits_out[(int64_t)b * C + c] = a;
  }
  __syncthreads();
  // cross-entropy of this image and dlogits
  float mx = -INFINITY;
  for (int c = tid; c < C; c += HT) mx = fmaxf(mx, lg[c]);
  mx = block_max(mx, red);
  float se = 0.f;
  for (int c = tid; c < C; c += HT) se += expf(lg[c] - mx);
  const float lse = mx + logf(block_sum(se, red));
  const int y = labels[b];
  if (tid == 0) loss_rows[b] = lse - ((y >= 0 && y < C) ? lg[y] : 0.f);
  __syncthreads();
  for (int c = tid; c < C; c += HT) {
    const float g = (expf(lg[c] - lse) - (c == y ? 1.f : 0.f)) / (float)B;
    lg[c] = g;
    dlogits_out[(int64_t)b * C + c] = g;
  }
  __syncthreads();
  // dz = dlogits . W_h^T, then the LayerNorm backward of the row:
  //   dxhat = dz * gamma;  dx = rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat))
  // a wavefront per row d of W_h: lanes walk the classes (coalesced), then a wave sum
  for (int d = w; d < D; d += RPP * HW) {               // RPP rows per pass: their loads overlap
    float a[RPP];
#pragma unroll
    for (int u = 0; u < RPP; ++u) a[u] = 0.f;
    for (int c0 = 0; c0 < C; c0 += WAVE) {               // uniform trip count, lanes past C idle
      const int c = c0 + lane;
      const bool in = c < C;
      const float g = in ? lg[c] : 0.f;
#pragma unroll
      for (int u = 0; u < RPP; ++u) {
        const int dd = min(d + u * HW, D - 1);           // rows past D repeat the last one and are dropped below
        a[u] = fmaf(g, in ? w_head[(int64_t)dd * C + c] : 0.f, a[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < RPP; ++u) {
      const int dd = d + u * HW;
      const float t = wave_sum_h(a[u]);
      if (lane == 0 && dd < D) zs[dd] = t;               // raw dz (z is not needed any more)
    }
  }
  __syncthreads();
  float s1 = 0.f, s2 = 0.f;
  for (int d = tid; d < D; d += HT) {
    const float t = zs[d];
    dz_out[(int64_t)b * D + d] = t;
    const float dh = t * gamma[d];                       // dxhat
    zs[d] = dh;
    s1 += dh;
    s2 += dh * xh[d];
  }
  s1 = block_sum(s1, red) / (float)D;
  s2 = block_sum(s2, red) / (float)D;
  T* dr = dx + (int64_t)b * Tl * D;
  for (int d = tid; d < D; d += HT) dr[d] = (T)(rstd * (zs[d] - s1 - xh[d] * s2));
  // the other token rows of this image receive no gradient from the head
  const int64_t rest = (int64_t)(Tl - 1) * D;
  if ((((uintptr_t)(dr + D)) & 15) == 0 && (rest * sizeof(T)) % 16 == 0) {
    uint4* zr = (uint4*)(dr + D);
    const int64_t nv = rest * sizeof(T) / 16;
    for (int64_t i = tid; i < nv; i += HT) zr[i] = make_uint4(0u, 0u, 0u, 0u);
  } else {
    for (int64_t i = tid; i < rest; i += HT) dr[D + i] = (T)0.f;
  }
}

// item i < D*C: dW_h[d,c]; next C: db_h[c]; next D: dgamma_f[d], dbeta_f[d]; last: the loss
__global__ __launch_bounds__(BT) void head_batch_kernel(const float* __restrict__ z, const float* __restrict__ xhat,
                                                        const float* __restrict__ dlogits, const float* __restrict__ dz,
                                                        const float* __restrict__ loss_rows, int B, int D, int C,
                                                        float* __restrict__ dw, float* __restrict__ db,
                                                        float* __restrict__ dgamma, float* __restrict__ dbeta,
                                                        float* __restrict__ loss) {
  const int64_t i = (int64_t)blockIdx.x * BT + threadIdx.x, DC = (int64_t)D * C;
  if (i < DC) {
    const int d = (int)(i / C), c = (int)(i % C);
    float a = 0.f;
#pragma unroll 8
    for (int b = 0; b < B; ++b) a = fmaf(z[(int64_t)b * D + d], dlogits[(int64_t)b * C + c], a);
    dw[i] = a;
  } else if (i < DC + C) {
    const int c = (int)(i - DC);
    float a = 0.f;
    for (int b = 0; b < B; ++b) a += dlogits[(int64_t)b * C + c];
    if (db) db[c] = a;
  } else if (i < DC + C + D) {
    const int d = (int)(i - DC - C);
    float g = 0.f, bt = 0.f;
    for (int b = 0; b < B; ++b) {
      const float v = dz[(int64_t)b * D + d];
      g = fmaf(v, xhat[(int64_t)b * D + d], g);
      bt += v;
    }
    dgamma[d] = g;
    dbeta[d] = bt;
  } else if (i == DC + C + D) {
    float a = 0.f;
    for (int b = 0; b < B; ++b) a += loss_rows[b];
    *loss = a / (float)B;
  }
}

}  // namespace

size_t head_lds_bytes(int D, int C) { return sizeof(float) * ((size_t)2 * D + (size_t)C + (size_t)NPART * C + HW); }

void head_fwd_bwd(const void* x, int B, int Tl, int D, int C, bool f32, const float* gamma, const float* beta, float eps,
                  const float* w_head, const float* b_head, const int32_t* labels, float* xhat, float* z, float* logits,
                  float* dlogits, float* dz, float* loss_rows, void* dx, float* dw, float* db, float* dgamma, float* dbeta,
                  float* loss, hipStream_t s) {
  const size_t lds = head_lds_bytes(D, C);
  if (f32)
    head_rows_kernel<float><<<B, HT, lds, s>>>((const float*)x, Tl, D, C, B, gamma, beta, eps, w_head, b_head, labels, xhat, z,
                                               logits, dlogits, dz, loss_rows, (float*)dx);
  else
    head_rows_kernel<bf16><<<B, HT, lds, s>>>((const bf16*)x, Tl, D, C, B, gamma, beta, eps, w_head, b_head, labels, xhat, z,
                                              logits, dlogits, dz, loss_rows, (bf16*)dx);
  const int64_t items = (int64_t)D * C + C + D + 1;
  head_batch_kernel<<<(unsigned)((items + BT - 1) / BT), BT, 0, s>>>(z, xhat, dlogits, dz, loss_rows, B, D, C, dw, db, dgamma,
                                                                    dbeta, loss);
}

}  // namespace bsr
