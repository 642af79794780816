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

// Expert choice of one token per thread, from the router logits [M,E] (a GEMM wrote them): the K
// largest logits (ties: lower index) in descending order, or the forced choice (clamped into
// 0..E-1); gates = softmax over the K selected logits.  The logits sit in registers and are picked by
// comparison, never by a computed register index.
template <int EMAX>
__global__ __launch_bounds__(256) void moe_topk_kernel(const float* __restrict__ logits, int64_t M, int E, int K,
                                                       const int32_t* __restrict__ forced,
                                                       int32_t* __restrict__ experts, float* __restrict__ gates) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= M) return;
  float v[EMAX];
#pragma unroll
  for (int e = 0; e < EMAX; ++e) v[e] = e < E ? logits[t * E + min(e, E - 1)] : -INFINITY;
  int sel[MOE_MAX_TOPK] = {0, 0, 0, 0};
  float lg[MOE_MAX_TOPK] = {0.f, 0.f, 0.f, 0.f};
  unsigned taken = 0;
#pragma unroll
  for (int s = 0; s < MOE_MAX_TOPK; ++s) {
    if (s >= K) break;
    int best = 0;
    float bv = -INFINITY;
    if (forced) {
      best = min(max(forced[t * K + s], 0), E - 1);
#pragma unroll
      for (int e = 0; e < EMAX; ++e)
        if (e == best) bv = v[e];
    } else {
      bool have = false;
#pragma unroll
      for (int e = 0; e < EMAX; ++e) {
        const bool ok = e < E && !((taken >> e) & 1u) && (!have || v[e] > bv);   // strict >: ties keep the lower index
        if (ok) { best = e; bv = v[e]; have = true; }
      }
    }
    taken |= 1u << best;
    sel[s] = best;
    lg[s] = bv;
  }
  float mx = lg[0];
#pragma unroll
  for (int s = 1; s < MOE_MAX_TOPK; ++s)
    if (s < K) mx = fmaxf(mx, lg[s]);
  float sum = 0.f;
#pragma unroll
  for (int s = 0; s < MOE_MAX_TOPK; ++s)
    if (s < K) { lg[s] = expf(lg[s] - mx); sum += lg[s]; }
#pragma unroll
  for (int s = 0; s < MOE_MAX_TOPK; ++s)
    if (s < K) {
      experts[t * K + s] = sel[s];
      gates[t * K + s] = lg[s] / sum;
    }
}

// bf16 copy of the router matrix [D,E] stored [E,D] (the layout the logits GEMM reads)
__global__ void moe_router_copy_kernel(const float* __restrict__ w, int D, int E, bf16* __restrict__ t) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= D * E) return;
  const int e = i / D, j = i % D;
  t[i] = (bf16)w[(int64_t)j * E + e];
}

// Stable counting sort by expert.  Workgroup e (1024 threads) handles expert e: thread i owns the pairs
// a in [i*chunk, (i+1)*chunk) (a = t*K + s), counts those of its expert and those of lower experts;
// the scan of the first over the workgroup gives each pair its row inside the expert's range, the
// sum of the second is where that range starts.  Pairs of one expert keep their (token, slot) order.
__global__ __launch_bounds__(1024) void moe_sort_kernel(const int32_t* __restrict__ experts, int64_t pairs, int E,
                                                        int K, int32_t* __restrict__ off, int32_t* __restrict__ pos,
                                                        int32_t* __restrict__ perm_tok) {
  __shared__ int w_eq[16], w_lt[16];
  const int e = blockIdx.x;
  const int tid = threadIdx.x, lane = tid % WAVE, wave = tid / WAVE;
  const int64_t chunk = (pairs + 1023) / 1024;
  const int64_t a0 = min((int64_t)tid * chunk, pairs), a1 = min(a0 + chunk, pairs);
  int eq = 0, lt = 0;
  for (int64_t a = a0; a < a1; ++a) {
    const int x = experts[a];
    eq += (x == e);
    lt += (x < e);
  }
  int incl = eq;                       // inclusive scan of eq over the wave
#pragma unroll
  for (int o = 1; o < WAVE; o <<= 1) {
    const int u = __shfl_up(incl, o, 64);
    if (lane >= o) incl += u;
  }
  int lts = lt;                        // wave total of lt
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) lts += __shfl_xor(lts, o, 64);
  if (lane == WAVE - 1) { w_eq[wave] = incl; w_lt[wave] = lts; }
  __syncthreads();
  int before = 0, base = 0, total = 0;
  for (int w = 0; w < 16; ++w) {
    if (w < wave) before += w_eq[w];
    total += w_eq[w];
    base += w_lt[w];
  }
  if (tid == 0) {
    off[e] = base;
    if (e == E - 1) off[E] = base + total;
  }
  int row = base + before + incl - eq;
  for (int64_t a = a0; a < a1; ++a)
    if (experts[a] == e) {
      pos[a] = row;
      perm_tok[row] = (int32_t)(a / K);
      ++row;
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
__global__ __launch_bounds__(256) void moe_combine_kernel(const float* __restrict__ y, const int32_t* __restrict__ pos,
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
      const float* yr = y + (int64_t)pos[t * K + s] * D + c * 8;
      const float4 y0 = *(const float4*)yr, y1 = *(const float4*)(yr + 4);
      const float y8[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = fmaf(g, y8[e], v[e]);
    }
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
    *(bf16x8*)(out + t * D + c * 8) = o;
  }
}

__global__ __launch_bounds__(256) void moe_combine_bwd_kernel(const bf16* __restrict__ dx, const float* __restrict__ y,
                                                              const int32_t* __restrict__ pos,
                                                              const int32_t* __restrict__ experts,
                                                              const float* __restrict__ gates, int64_t M, int D, int E,
                                                              int K, bf16* __restrict__ dy, float* __restrict__ dsel) {
  const int lane = threadIdx.x % WAVE;
  const int64_t t = (int64_t)blockIdx.x * 4 + threadIdx.x / WAVE;
  if (t >= M) return;
  float dgate[MOE_MAX_TOPK] = {0.f, 0.f, 0.f, 0.f};
  for (int c = lane; c < D / 8; c += WAVE) {
    const bf16x8 d8 = *(const bf16x8*)(dx + t * D + c * 8);
    for (int s = 0; s < K; ++s) {
      const int64_t row = pos[t * K + s];
      const float g = gates[t * K + s];
      const float* yr = y + row * D + c * 8;
      const float4 y0 = *(const float4*)yr, y1 = *(const float4*)(yr + 4);
      const float y8[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
      bf16x8 o;
      float a = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        a = fmaf((float)d8[e], y8[e], a);
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
  // gradient at the K selected logits (softmax over the selected ones); it stays in fp32
#pragma unroll
  for (int q = 0; q < MOE_MAX_TOPK; ++q)
    if (q < K && lane == 0) dsel[t * K + q] = gates[t * K + q] * (dgate[q] - mix);
}

// Router weight gradient dW_r[d, e] = sum_t h[t, d] dlogit[t, e], where row t of dlogit is zero except for
// dsel[t, s] at column experts[t, s]: all in fp32 (the operand h is the stored bf16 LayerNorm output), so that
// the router sees the same gradient precision as the classification head.  Workgroup (x, y): 64 columns d,
// token chunk y; its four wavefronts take every fourth token of the chunk and keep [E][64] sums in LDS, which
// are then added in wavefront order; the chunk sums go to partial[y][d][e] and a second launch adds the chunks
// in ascending order (no atomics: the result does not depend on timing).
constexpr int ROUTER_WGRAD_CHUNKS = 32;
__global__ __launch_bounds__(256) void moe_router_wgrad_kernel(const bf16* __restrict__ h, const int32_t* __restrict__ experts,
                                                               const float* __restrict__ dsel, int64_t M, int D, int E, int K,
                                                               float* __restrict__ partial) {
  __shared__ float acc[4][MOE_MAX_EXPERTS][WAVE];
  const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
  const int d = blockIdx.x * WAVE + lane;
  for (int e = 0; e < E; ++e) acc[wave][e][lane] = 0.f;
  const int64_t per = (M + gridDim.y - 1) / gridDim.y;
  const int64_t t0 = (int64_t)blockIdx.y * per, t1 = min(M, t0 + per);
  for (int64_t t = t0 + wave; t < t1; t += 4) {
    const float hv = d < D ? (float)h[t * D + d] : 0.f;
    for (int s = 0; s < K; ++s) {
      const int e = min(max(experts[t * K + s], 0), E - 1);      // (uniform over the wavefront)
      acc[wave][e][lane] = fmaf(hv, dsel[t * K + s], acc[wave][e][lane]);
    }
  }
  __syncthreads();
  if (d < D)
    for (int e = wave; e < E; e += 4)
      partial[((int64_t)blockIdx.y * D + d) * E + e] = ((acc[0][e][lane] + acc[1][e][lane]) + acc[2][e][lane]) + acc[3][e][lane];
}
__global__ __launch_bounds__(256) void moe_router_wgrad_sum_kernel(const float* __restrict__ partial, int n, int chunks,
                                                                   float* __restrict__ dw) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = partial[i];
  for (int c = 1; c < chunks; ++c) v += partial[(int64_t)c * n + i];
  dw[i] = v;
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

void moe_topk(const float* logits, int64_t M, int E, int K, const int32_t* forced, int32_t* experts, float* gates,
              hipStream_t s) {
  if (M <= 0) return;
  const unsigned grid = (unsigned)((M + 255) / 256);
  if (E <= 8) moe_topk_kernel<8><<<grid, 256, 0, s>>>(logits, M, E, K, forced, experts, gates);
  else if (E <= 16) moe_topk_kernel<16><<<grid, 256, 0, s>>>(logits, M, E, K, forced, experts, gates);
  else moe_topk_kernel<32><<<grid, 256, 0, s>>>(logits, M, E, K, forced, experts, gates);
}

void moe_router_copy(const float* w_router, int D, int E, void* t_router, hipStream_t s) {
  moe_router_copy_kernel<<<(D * E + 255) / 256, 256, 0, s>>>(w_router, D, E, (bf16*)t_router);
}

void moe_sort(const int32_t* experts, int64_t M, int E, int K, int32_t* off, int32_t* pos, int32_t* perm_tok,
              hipStream_t s) {
  moe_sort_kernel<<<E, 1024, 0, s>>>(experts, M * K, E, K, off, pos, perm_tok);
}

void moe_gather_rows(const void* x, const int32_t* src, int64_t rows, int D, void* y, hipStream_t s) {
  const int64_t total = rows * (D / 8);
  if (total <= 0) return;
  moe_gather_rows_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>((const uint4*)x, src, rows, D / 8, (uint4*)y);
}

void moe_combine(const void* y, const int32_t* pos, const float* gates, const void* res, int64_t M, int D, int K,
                 void* x_out, hipStream_t s) {
  if (M <= 0) return;
  moe_combine_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const float*)y, pos, gates, (const bf16*)res, M, D, K,
                                                           (bf16*)x_out);
}

void moe_combine_bwd(const void* dx, const void* y, const int32_t* pos, const int32_t* experts, const float* gates,
                     int64_t M, int D, int E, int K, void* dy, float* dsel, hipStream_t s) {
  if (M <= 0) return;
  moe_combine_bwd_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const bf16*)dx, (const float*)y, pos, experts, gates, M,
                                                               D, E, K, (bf16*)dy, dsel);
}

size_t moe_router_wgrad_partial_floats(int D, int E) { return (size_t)ROUTER_WGRAD_CHUNKS * D * E; }
void moe_router_wgrad(const void* h, const int32_t* experts, const float* dsel, int64_t M, int D, int E, int K,
                      float* partial, float* dw, hipStream_t s) {
  if (M <= 0) return;
  moe_router_wgrad_kernel<<<dim3((D + WAVE - 1) / WAVE, ROUTER_WGRAD_CHUNKS), 256, 0, s>>>((const bf16*)h, experts, dsel, M, D, E, K,
                                                                                          partial);
  moe_router_wgrad_sum_kernel<<<(D * E + 255) / 256, 256, 0, s>>>(partial, D * E, ROUTER_WGRAD_CHUNKS, dw);
}

void moe_unpermute_bwd(const void* dxg, const int32_t* pos, const int32_t* experts, const float* dsel,
                       const float* w_router, int64_t M, int D, int E, int K, void* dh, hipStream_t s) {
  if (M <= 0) return;
  moe_unpermute_bwd_kernel<<<(unsigned)((M + 3) / 4), 256, 0, s>>>((const bf16*)dxg, pos, experts, dsel, w_router, M, D,
                                                                 E, K, (bf16*)dh);
}

}  // namespace bsr
