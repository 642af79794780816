// Generic strided GEMM with the fused epilogues of the BSR step.  fp32 arithmetic on fp32 or bf16
// storage, any shape.  It is the fp32-mode path and the fallback for shapes the MFMA kernels do
// not take; the hot bf16 shapes go through k_gemm_mfma.hip.
#include "bsr_internal.h"

namespace bsr {

namespace {

constexpr int TM = 64, TN = 64, TK = 16;

__device__ inline float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }
__device__ inline float gelu_grad_f(float u) {
  float cdf = 0.5f * (1.0f + erff(u * 0.70710678118654752f));
  float pdf = expf(-0.5f * u * u) * 0.39894228040143268f;
  return cdf + u * pdf;
}

template <typename TIn, typename TOut>
__global__ __launch_bounds__(256) void gemm_generic_kernel(GemmDesc g) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const TIn* __restrict__ A = (const TIn*)g.A;
  const TIn* __restrict__ Bm = (const TIn*)g.B;
  const int tid = threadIdx.x, tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  float acc[4][4] = {};
  const bool a_kfast = (g.a_cs == 1);   // contraction index contiguous in A
  const bool b_nfast = (g.b_cs == 1);   // output column contiguous in B
  for (int k0 = 0; k0 < g.K; k0 += TK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = tid + 256 * i;
      int m = a_kfast ? idx / TK : idx % TM;
      int k = a_kfast ? idx % TK : idx / TM;
      float v = 0.f;
      if (m0 + m < g.M && k0 + k < g.K) v = (float)A[(int64_t)(m0 + m) * g.a_rs + (int64_t)(k0 + k) * g.a_cs];
      As[k][m] = v;
      int kb = b_nfast ? idx / TN : idx % TK;
      int n = b_nfast ? idx % TN : idx / TK;
      float w = 0.f;
      if (n0 + n < g.N && k0 + kb < g.K) w = (float)Bm[(int64_t)(k0 + kb) * g.b_rs + (int64_t)(n0 + n) * g.b_cs];
      Bs[kb][n] = w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  TOut* __restrict__ C = (TOut*)g.C;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= g.M) continue;
    int64_t row = m;
    const float* posr = nullptr;
    if (g.remap_np > 0) {
      row = (int64_t)m + m / g.remap_np + 1;
      posr = g.pos + (int64_t)(m % g.remap_np + 1) * g.N;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= g.N) continue;
      float v = acc[i][j];
      if (g.bias) v += g.bias[n];
      int64_t off = row * g.ldc + n;
      if (g.act == ACT_GELU) {
        if (g.aux) ((TOut*)g.aux)[off] = (TOut)v;
        v = gelu_f(v);
      } else if (g.act == ACT_GELU_BWD) {
        v *= gelu_grad_f((float)((const TOut*)g.aux)[off]);
      }
      if (posr) v += posr[n];
      if (g.res) v += (float)((const TOut*)g.res)[off];
      C[off] = (TOut)v;
    }
  }
}

// One thread per output element; for the head's tiny fp32 products (at most a few 10^4 outputs) this
// beats a tiled kernel that would fill one or two workgroups.
__global__ __launch_bounds__(256) void gemm_small_f32_kernel(GemmDesc g) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (int64_t)g.M * g.N) return;
  const int m = (int)(idx / g.N), n = (int)(idx % g.N);
  const float* A = (const float*)g.A + (int64_t)m * g.a_rs;
  const float* B = (const float*)g.B + (int64_t)n * g.b_cs;
  float acc0 = 0.f, acc1 = 0.f, acc2 = 0.f, acc3 = 0.f;
  int k = 0;
  for (; k + 3 < g.K; k += 4) {
    acc0 = fmaf(A[(int64_t)k * g.a_cs], B[(int64_t)k * g.b_rs], acc0);
    acc1 = fmaf(A[(int64_t)(k + 1) * g.a_cs], B[(int64_t)(k + 1) * g.b_rs], acc1);
    acc2 = fmaf(A[(int64_t)(k + 2) * g.a_cs], B[(int64_t)(k + 2) * g.b_rs], acc2);
    acc3 = fmaf(A[(int64_t)(k + 3) * g.a_cs], B[(int64_t)(k + 3) * g.b_rs], acc3);
  }
  for (; k < g.K; ++k) acc0 = fmaf(A[(int64_t)k * g.a_cs], B[(int64_t)k * g.b_rs], acc0);
  float v = (acc0 + acc1) + (acc2 + acc3);
  if (g.bias) v += g.bias[n];
  ((float*)g.C)[(int64_t)m * g.ldc + n] = v;
}

// Long contractions (the logits: K = D): one wavefront per output element, lanes stride over k.
__global__ __launch_bounds__(256) void gemm_small_f32_wave_kernel(GemmDesc g) {
  const int64_t idx = (int64_t)blockIdx.x * 4 + threadIdx.x / 64;
  if (idx >= (int64_t)g.M * g.N) return;
  const int lane = threadIdx.x % 64;
  const int m = (int)(idx / g.N), n = (int)(idx % g.N);
  const float* A = (const float*)g.A + (int64_t)m * g.a_rs;
  const float* B = (const float*)g.B + (int64_t)n * g.b_cs;
  float acc = 0.f;
  for (int k = lane; k < g.K; k += 64) acc = fmaf(A[(int64_t)k * g.a_cs], B[(int64_t)k * g.b_rs], acc);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) ((float*)g.C)[(int64_t)m * g.ldc + n] = acc + (g.bias ? g.bias[n] : 0.f);
}

}  // namespace

void gemm_small_f32(const GemmDesc& g, hipStream_t s) {
  const int64_t total = (int64_t)g.M * g.N;
  if (total <= 0) return;
  if (g.K >= 256) gemm_small_f32_wave_kernel<<<(unsigned)((total + 3) / 4), 256, 0, s>>>(g);
  else gemm_small_f32_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(g);
}

void gemm_generic(const GemmDesc& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return;
  dim3 grid((g.N + TN - 1) / TN, (g.M + TM - 1) / TM);
  if (g.in_f32) {
    if (g.out_f32) gemm_generic_kernel<float, float><<<grid, 256, 0, s>>>(g);
    else gemm_generic_kernel<float, bf16><<<grid, 256, 0, s>>>(g);
  } else {
    if (g.out_f32) gemm_generic_kernel<bf16, float><<<grid, 256, 0, s>>>(g);
    else gemm_generic_kernel<bf16, bf16><<<grid, 256, 0, s>>>(g);
  }
}

}  // namespace bsr
