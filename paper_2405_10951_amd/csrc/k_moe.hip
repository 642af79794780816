// Mixture-of-experts FFN (Sec. 5.3 of the paper): the kernels around the grouped expert GEMMs.
// A router activates K of E expert MLPs per token and their outputs are added, weighted by the
// softmax over the K selected router logits.  The (token, slot) pairs are sorted by expert so that
// each expert sees a contiguous range of rows; the expert FFNs then run as grouped MFMA GEMMs.
#include "bsr_internal.h"

namespace bsr {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int WAVE = 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wavefront per token.  Lane j accumulates its slice of the D-long dot products for all E experts;
// the E sums are reduced over the wave and lane 0 ranks them.
__global__ __launch_bounds__(256) void moe_route_kernel(const bf16* __restrict__ h, int64_t M, int D,
                                                        const float* __restrict__ w_router, int E, int K,
                                                        const int32_t* __restrict__ forced,
                                                        float* __restrict__ logits, int32_t* __restrict__ experts,
                                                        float* __restrict__ gates) {
  const int lane = threadIdx.x % WAVE;
  const int64_t t = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
  if (t >= M) return;
  float acc[MOE_MAX_EXPERTS];
#pragma unroll
  for (int e = 0; e < MOE_MAX_EXPERTS; ++e) acc[e] = 0.f;
  for (int j = lane; j < D; j += WAVE) {
    const float x = (float)h[t * D + j];
    const float* wr = w_router + (int64_t)j * E;
#pragma unroll
    for (int e = 0; e < MOE_MAX_EXPERTS; ++e)
      if (e < E) acc[e] = fmaf(x, wr[e], acc[e]);
  }
#pragma unroll
  for (int e = 0; e < MOE_MAX_EXPERTS; ++e)
    if (e < E) acc[e] = wave_sum(acc[e]);
  if (lane != 0) return;
  if (logits)
    for (int e = 0; e < E; ++e) logits[t * E + e] = acc[e];
  int sel[MOE_MAX_TOPK];
  float lg[MOE_MAX_TOPK];
  for (int s = 0; s < K; ++s) {
    int best = -1;
    if (forced) {
      best = min(max(forced[t * K + s], 0), E - 1);   // a forced value outside 0..E-1 is clamped
    } else {
      for (int e = 0; e < E; ++e) {
        bool taken = false;
        for (int j = 0; j < s; ++j) taken |= (sel[j] == e);
        if (taken) continue;
        float ve = 0.f, vb = 0.f;
#pragma unroll
        for (int q = 0; q < MOE_MAX_EXPERTS; ++q) {   // register array: select by comparison, not by address
          if (q == e) ve = acc[q];
          if (q == best) vb = acc[q];
        }
        if (best < 0 || ve > vb) best = e;            // strict >: a tie keeps the lower index
      }
    }
    float v = 0.f;
#pragma unroll
    for (int q = 0; q < MOE_MAX_EXPERTS; ++q)
      if (q == best) v = acc[q];
    sel[s] = best;
    lg[s] = v;
  }
  float mx = lg[0];
  for (int s = 1; s < K; ++s) mx = fmaxf(mx, lg[s]);
  float sum = 0.f;
  for (int s = 0; s < K; ++s) { lg[s] = expf(lg[s] - mx); sum += lg[s]; }
  for (int s = 0; s < K; ++s) {
    experts[t * K + s] = sel[s];
    gates[t * K + s] = lg[s] / sum;
  }
}

// Stable counting sort by expert, one workgroup of 1024 threads.  Thread i owns the pairs
// a in [i*chunk, (i+1)*chunk) (a = t*K + s); for every expert in turn the per-thread counts are
// scanned over the workgroup, which gives each pair its row: pairs of one expert keep their order.
__global__ __launch_bounds__(1024) void moe_sort_kernel(const int32_t* __restrict__ experts, int64_t pairs, int E,
                                                        int K, int32_t* __restrict__ off, int32_t* __restrict__ pos,
                                                        int32_t* __restrict__ perm_tok) {
  __shared__ int wsum[16];
  __shared__ int total_s;
  const int tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
  const int64_t chunk = (pairs + 1023) / 1024;
  const int64_t a0 = min((int64_t)tid * chunk, pairs), a1 = min(a0 + chunk, pairs);
  int base = 0;                        // rows taken by the experts before e
  if (tid == 0) off[0] = 0;
  for (int e = 0; e < E; ++e) {
    int cnt = 0;
    for (int64_t a = a0; a < a1; ++a) cnt += (experts[a] == e);
    // inclusive scan over the wave, then over the 16 wave totals
    int incl = cnt;
#pragma unroll
    for (int o = 1; o < WAVE; o <<= 1) {
      const int v = __shfl_up(incl, o, 64);
      if (lane >= o) incl += v;
    }
    if (lane == WAVE - 1) wsum[wave] = incl;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    if (tid == 1023) total_s = before + incl;
    int row = base + before + incl - cnt;
    for (int64_t a = a0; a < a1; ++a)
      if (experts[a] == e) {
        pos[a] = row;
        perm_tok[row] = (int32_t)(a / K);
        ++row;
      }
    __syncthreads();
    base += total_s;
    if (tid == 0) off[e + 1] = base;
    __syncthreads();
  }
}

__global__ void moe_gather_rows_kernel(const uint4* __restrict__ x, const int32_t* __restrict__ src, int64_t rows,
                                       int chunks, uint4* __restrict__ y) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * chunks) return;
  const int64_t r = i / chunks;
  const int c = (int)(i % chunks);
  y[i] = x[(int64_t)src[r] * chunks + c];
}

// One wavefront per token, 8 columns per lane and pass.
__global__ __launch_bounds__(256) void moe_combine_kernel(const bf16* __restrict__ y, const int32_t* __restrict__ pos,
                                                          const float* __restrict__ gates,
                                                          const bf16* __restrict__ res, int64_t M, int D, int K,
                                                          bf16* __restrict__ out) {
  const int lane = threadIdx.x % WAVE;
  const int64_t t = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
  if (t >= M) return;
  for (int c = lane; c < D / 8; c += WAVE) {
    const bf16x8 r8 = *(const bf16x8*)(res + t * D + c * 8);
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (float)r8[e];
    for (int s = 0; s < K; ++s) {
      const float g = gates[t * K + s];
      const bf16x8 y8 = *(const bf16x8*)(y + (int64_t)pos[t * K + s] * D + c * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = fmaf(g, (float)y8[e], v[e]);
    }
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
    *(bf16x8*)(out + t * D + c * 8) = o;
  }
}

__global__ __launch_bounds__(256) void moe_combine_bwd_kernel(const bf16* __restrict__ dx, const bf16* __restrict__ y,
                                                              const int32_t* __restrict__ pos,
                                                              const int32_t* __restrict__ experts,
                                                              const float* __restrict__ gates, int64_t M, int D, int E,
                                                              int K, bf16* __restrict__ dy, float* __restrict__ dsel,
                                                              bf16* __restrict__ dlogits) {
  const int lane = threadIdx.x % WAVE;
  const int64_t t = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
  if (t >= M) return;
  float dgate[MOE_MAX_TOPK] = {0.f, 0.f, 0.f, 0.f};
  for (int c = lane; c < D / 8; c += WAVE) {
    const bf16x8 d8 = *(const bf16x8*)(dx + t * D + c * 8);
    for (int s = 0; s < K; ++s) {
      const int64_t row = pos[t * K + s];
      const float g = gates[t * K + s];
      const bf16x8 y8 = *(const bf16x8*)(y + row * D + c * 8);
      bf16x8 o;
      float a = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a = fmaf((float)d8[e], (float)y8[e], a);
        o[e] = (bf16)(g * (float)d8[e]);
      }
      *(bf16x8*)(dy + row * D + c * 8) = o;
#pragma unroll
      for (int q = 0; q < MOE_MAX_TOPK; ++q)
        if (q == s) dgate[q] += a;
    }
  }
  float mix = 0.f;
#pragma unroll
  for (int q = 0; q < MOE_MAX_TOPK; ++q) {
    dgate[q] = wave_sum(dgate[q]);
    if (q < K) mix = fmaf(gates[t * K + q], dgate[q], mix);
  }
  // dlogits row: zero, then the K selected entries (lane e owns column e; E <= 32)
  float mine = 0.f;
#pragma unroll
  for (int q = 0; q < MOE_MAX_TOPK; ++q)
    if (q < K) {
      const float d = gates[t * K + q] * (dgate[q] - mix);
      if (lane == 0) dsel[t * K + q] = d;
      if (experts[t * K + q] == lane) mine = d;
    }
  if (lane < E) dlogits[t * E + lane] = (bf16)mine;
}

__global__ __launch_bounds__(256) void moe_unpermute_bwd_kernel(const bf16* __restrict__ dxg,
                                                                const int32_t* __restrict__ pos,
                                                                const int32_t* __restrict__ experts,
                                                                const float* __restrict__ dsel,
                                                                const float* __restrict__ w_router, int64_t M, int D,
                                                                int E, int K, bf16* __restrict__ dh) {
  const int lane = threadIdx.x % WAVE;
  const int64_t t = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
  if (t >= M) return;
  for (int c = lane; c < D / 8; c += WAVE) {
    float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < K; ++s) {
      const bf16x8 g8 = *(const bf16x8*)(dxg + (int64_t)pos[t * K + s] * D + c * 8);
      const float d = dsel[t * K + s];
      const int ex = experts[t * K + s];
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += (float)g8[e] + d * w_router[(int64_t)(c * 8 + e) * E + ex];
    }
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
    *(bf16x8*)(dh + t * D + c * 8) = o;
  }
}

}  // namespace

void moe_route(const void* h, int64_t M, int D, const float* w_router, int E, int K, const int32_t* forced,
               float* logits, int32_t* experts, float* gates, hipStream_t s) {
  if (M <= 0) return;
  moe_route_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const bf16*)h, M, D, w_router, E, K, forced, logits, experts,
                                                         gates);
}

void moe_sort(const int32_t* experts, int64_t M, int E, int K, int32_t* off, int32_t* pos, int32_t* perm_tok,
              hipStream_t s) {
  moe_sort_kernel<<<1, 1024, 0, s>>>(experts, M * K, E, K, off, pos, perm_tok);
}

void moe_gather_rows(const void* x, const int32_t* src, int64_t rows, int D, void* y, hipStream_t s) {
  const int64_t total = rows * (D / 8);
  if (total <= 0) return;
  moe_gather_rows_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint4*)x, src, rows, D / 8, (uint4*)y);
}

void moe_combine(const void* y, const int32_t* pos, const float* gates, const void* res, int64_t M, int D, int K,
                 void* x_out, hipStream_t s) {
  if (M <= 0) return;
  moe_combine_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const bf16*)y, pos, gates, (const bf16*)res, M, D, K,
                                                           (bf16*)x_out);
}

void moe_combine_bwd(const void* dx, const void* y, const int32_t* pos, const int32_t* experts, const float* gates,
                     int64_t M, int D, int E, int K, void* dy, float* dsel, void* dlogits, hipStream_t s) {
  if (M <= 0) return;
  moe_combine_bwd_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const bf16*)dx, (const bf16*)y, pos, experts, gates, M,
                                                               D, E, K, (bf16*)dy, dsel, (bf16*)dlogits);
}

void moe_unpermute_bwd(const void* dxg, const int32_t* pos, const int32_t* experts, const float* dsel,
                       const float* w_router, int64_t M, int D, int E, int K, void* dh, hipStream_t s) {
  if (M <= 0) return;
  moe_unpermute_bwd_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const bf16*)dxg, pos, experts, dsel, w_router, M, D,
                                                                 E, K, (bf16*)dh);
}

}  // namespace bsr
