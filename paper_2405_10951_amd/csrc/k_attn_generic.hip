// Generic softmax attention (Eq. 1 of the paper) forward and backward: one wavefront per query row
// (or per key row for dK / dV), fp32 arithmetic on fp32 or bf16 storage, any head size up to 256 and
// up to 1024 tokens.  It is the fp32-mode path and the fallback of the MFMA kernels.
//
// qkv is [B, T, 3D] with columns [q | k | v]; head h owns columns h*d .. h*d+d-1 of each third.
#include "bsr_internal.h"

namespace bsr {

namespace {

constexpr int WAVE = 64;
constexpr int MAX_T = 1024;
constexpr int MAX_D = 256;

__device__ inline float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ inline float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

// out[b,i,h*d+e] = sum_j softmax_j(q_i.k_j / sqrt d) v_j[e];  lse[b,h,i] = log sum_j exp(s_ij);
// cls_prob[b,h,j] = softmax row of query 0 (the CLS token), the by-product Eq. 6 ranks tokens by.
template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const T* __restrict__ qkv, int T_, int H, int d,
                                                       T* __restrict__ out, float* __restrict__ lse,
                                                       float* __restrict__ cls_prob) {
  __shared__ float p_s[4][MAX_T];
  __shared__ float q_s[4][MAX_D];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int i = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
  if (i >= T_) return;
  const int D = H * d;
  const T* base = qkv + (int64_t)b * T_ * 3 * D;
  const float scale = rsqrtf((float)d);
  for (int e = lane; e < d; e += WAVE) q_s[w][e] = (float)base[(int64_t)i * 3 * D + h * d + e];
  __builtin_amdgcn_wave_barrier();
  float mx = -INFINITY;
  for (int j = lane; j < T_; j += WAVE) {
    const T* kr = base + (int64_t)j * 3 * D + D + h * d;
    float s = 0.f;
    for (int e = 0; e < d; ++e) s = fmaf(q_s[w][e], (float)kr[e], s);
    s *= scale;
    p_s[w][j] = s;
    mx = fmaxf(mx, s);
  }
  mx = wmax(mx);
  float sum = 0.f;
  for (int j = lane; j < T_; j += WAVE) {
    float p = expf(p_s[w][j] - mx);
    p_s[w][j] = p;
    sum += p;
  }
  sum = wsum(sum);
  const float inv = 1.0f / sum;
  if (lse && lane == 0) lse[((int64_t)b * H + h) * T_ + i] = mx + logf(sum);
  __builtin_amdgcn_wave_barrier();
  if (cls_prob && i == 0)
    for (int j = lane; j < T_; j += WAVE) cls_prob[((int64_t)b * H + h) * T_ + j] = p_s[w][j] * inv;
  for (int e = lane; e < d; e += WAVE) {
    float o = 0.f;
    for (int j = 0; j < T_; ++j) o = fmaf(p_s[w][j], (float)base[(int64_t)j * 3 * D + 2 * D + h * d + e], o);
    out[((int64_t)b * T_ + i) * D + h * d + e] = (T)(o * inv);
  }
}

// Row pass of the backward: for query i, P_ij = exp(s_ij - lse_i), dP_ij = dO_i.v_j,
// delta_i = sum_j P_ij dP_ij, dS_ij = P_ij (dP_ij - delta_i) / sqrt d, dq_i = sum_j dS_ij k_j.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_q_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                         const float* __restrict__ lse, int T_, int H, int d,
                                                         float* __restrict__ delta, T* __restrict__ dqkv) {
  __shared__ float ds_s[4][MAX_T];
  __shared__ float dp_s[4][MAX_T];
  __shared__ float q_s[4][MAX_D];
  __shared__ float do_s[4][MAX_D];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int i = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
  if (i >= T_) return;
  const int D = H * d;
  const T* base = qkv + (int64_t)b * T_ * 3 * D;
  const float scale = rsqrtf((float)d);
  for (int e = lane; e < d; e += WAVE) {
    q_s[w][e] = (float)base[(int64_t)i * 3 * D + h * d + e];
    do_s[w][e] = (float)dout[((int64_t)b * T_ + i) * D + h * d + e];
  }
  __builtin_amdgcn_wave_barrier();
  const float l = lse[((int64_t)b * H + h) * T_ + i];
  float dot = 0.f;
  for (int j = lane; j < T_; j += WAVE) {
    const T* kr = base + (int64_t)j * 3 * D + D + h * d;
    const T* vr = kr + D;
    float s = 0.f, dp = 0.f;
    for (int e = 0; e < d; ++e) {
      s = fmaf(q_s[w][e], (float)kr[e], s);
      dp = fmaf(do_s[w][e], (float)vr[e], dp);
    }
    const float p = expf(s * scale - l);
    dot += p * dp;
    ds_s[w][j] = p;
    dp_s[w][j] = dp;
  }
  dot = wsum(dot);
  if (lane == 0) delta[((int64_t)b * H + h) * T_ + i] = dot;
  for (int j = lane; j < T_; j += WAVE) ds_s[w][j] = ds_s[w][j] * (dp_s[w][j] - dot) * scale;
  __builtin_amdgcn_wave_barrier();
  for (int e = lane; e < d; e += WAVE) {
    float a = 0.f;
    for (int j = 0; j < T_; ++j) a = fmaf(ds_s[w][j], (float)base[(int64_t)j * 3 * D + D + h * d + e], a);
    dqkv[((int64_t)b * T_ + i) * 3 * D + h * d + e] = (T)a;
  }
}

// Column pass: for key j, dv_j = sum_i P_ij dO_i, dk_j = sum_i dS_ij q_i.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_kv_kernel(const T* __restrict__ qkv, const T* __restrict__ dout,
                                                          const float* __restrict__ lse,
                                                          const float* __restrict__ delta, int T_, int H,
                                                          int d, T* __restrict__ dqkv) {
  __shared__ float p_s[4][MAX_T];
  __shared__ float ds_s[4][MAX_T];
  __shared__ float k_s[4][MAX_D];
  __shared__ float v_s[4][MAX_D];
  const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
  const int j = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
  if (j >= T_) return;
  const int D = H * d;
  const T* base = qkv + (int64_t)b * T_ * 3 * D;
  const T* dob = dout + (int64_t)b * T_ * D;
  const float scale = rsqrtf((float)d);
  for (int e = lane; e < d; e += WAVE) {
    k_s[w][e] = (float)base[(int64_t)j * 3 * D + D + h * d + e];
    v_s[w][e] = (float)base[(int64_t)j * 3 * D + 2 * D + h * d + e];
  }
  __builtin_amdgcn_wave_barrier();
  for (int i = lane; i < T_; i += WAVE) {
    const T* qr = base + (int64_t)i * 3 * D + h * d;
    const T* dor = dob + (int64_t)i * D + h * d;
    float s = 0.f, dp = 0.f;
    for (int e = 0; e < d; ++e) {
      s = fmaf((float)qr[e], k_s[w][e], s);
      dp = fmaf((float)dor[e], v_s[w][e], dp);
    }
    const int64_t r = ((int64_t)b * H + h) * T_ + i;
    float p = expf(s * scale - lse[r]);
    p_s[w][i] = p;
    ds_s[w][i] = p * (dp - delta[r]) * scale;
  }
  __builtin_amdgcn_wave_barrier();
  for (int e = lane; e < d; e += WAVE) {
    float dv = 0.f, dk = 0.f;
    for (int i = 0; i < T_; ++i) {
      dv = fmaf(p_s[w][i], (float)dob[(int64_t)i * D + h * d + e], dv);
      dk = fmaf(ds_s[w][i], (float)base[(int64_t)i * 3 * D + h * d + e], dk);
    }
    dqkv[((int64_t)b * T_ + j) * 3 * D + D + h * d + e] = (T)dk;
    dqkv[((int64_t)b * T_ + j) * 3 * D + 2 * D + h * d + e] = (T)dv;
  }
}

}  // namespace

void attn_fwd_generic(const void* qkv, int B, int T, int H, int d, bool f32, void* out, float* lse,
                      float* cls_prob, hipStream_t s) {
  dim3 grid((T + 3) / 4, H, B);
  if (f32) attn_fwd_kernel<float><<<grid, 256, 0, s>>>((const float*)qkv, T, H, d, (float*)out, lse, cls_prob);
  else attn_fwd_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)qkv, T, H, d, (bf16*)out, lse, cls_prob);
}

void attn_bwd_generic(const void* qkv, const void* /*out*/, const void* dout, const float* lse, int B,
                      int T, int H, int d, bool f32, float* delta, void* dqkv, hipStream_t s) {
  dim3 grid((T + 3) / 4, H, B);
  if (f32) {
    attn_bwd_q_kernel<float><<<grid, 256, 0, s>>>((const float*)qkv, (const float*)dout, lse, T, H, d, delta, (float*)dqkv);
    attn_bwd_kv_kernel<float><<<grid, 256, 0, s>>>((const float*)qkv, (const float*)dout, lse, delta, T, H, d, (float*)dqkv);
  } else {
    attn_bwd_q_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)qkv, (const bf16*)dout, lse, T, H, d, delta, (bf16*)dqkv);
    attn_bwd_kv_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)qkv, (const bf16*)dout, lse, delta, T, H, d, (bf16*)dqkv);
  }
}

}  // namespace bsr
