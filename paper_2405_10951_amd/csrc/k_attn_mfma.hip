// bf16 MFMA softmax attention (Eq. 1 of the paper) for head size 64 and up to 256 tokens, the shape
// of every ViT-B/16 and DeiT-S block after token dropping.  The CLS row of the softmax map, which
// Eq. 6 ranks tokens by, leaves the forward kernel in fp32 as a by-product.
//
// Forward.  One workgroup = one (image, head): K and V of the head are staged once, and each of
// its ceil(T / 32) wavefronts owns 32 queries.  K and V sit in LDS row-major (swizzled 16-byte chunks);
// V^T fragments come from the LDS transpose read.  The wave computes S^T = K Q^T with 32x32x16 MFMAs, so that a
// lane owns one query and the softmax reductions over keys are in-register (plus one exchange between
// the two halves of the wave).  The normalised P^T accumulators are, as they lie in registers, an
// operand of the second product O^T = V^T P^T: MFMA contracts over a dummy index, so the key order
// that the accumulator layout dictates is simply applied to the V^T reads as well.  No T x T tensor
// ever leaves registers.
#include "bsr_internal.h"

namespace bsr {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int HD = 64;          // head size

// Chunk permutation of a row of 8 16-byte chunks (128 B, two rows per sweep of the 64 banks): chunk kc of
// row r sits at kc ^ swz(r).  It serves two access patterns without bank conflicts:
//   - row fragments (16 consecutive rows read the same logical chunk): the 8 rows of either parity get 8
//     different positions;
//   - transposed fragments (4 consecutive rows r..r+3, r % 4 == 0, 64 bytes each): bit 2 differs between
//     rows r and r+2 (and r+1, r+3), so the four rows hit the four 64-byte bank groups.
__device__ inline int swz(int row) { return (((row >> 1) & 1) << 2) | ((row >> 2) & 3); }

// key index of accumulator element r (of key block jb) held by a lane of wave half lh
__device__ inline int key_of(int jb, int r, int lh) { return jb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3); }

// K rows [T,64] of one head -> LDS chunks; rows >= T are zero.
__device__ inline void load_k(const bf16* base, int64_t row_stride, int T, int Tpad, u32x4* Ks, int tid,
                              int nthreads = 256) {
  // four loads in flight per thread before the first LDS write: one trip to memory instead of four
  const int total = Tpad * 8;
  for (int c0 = tid; c0 < total; c0 += 4 * nthreads) {
    u32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * nthreads, row = c >> 3, kc = c & 7;
      v[u] = u32x4{0u, 0u, 0u, 0u};
      if (c < total && row < T) v[u] = *(const u32x4*)(base + (int64_t)row * row_stride + kc * 8);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * nthreads, row = c >> 3, kc = c & 7;
      if (c < total) Ks[row * 8 + (kc ^ swz(row))] = v[u];
    }
  }
}

// Transposed fragment of a row-major LDS tile [rows][64 features] for the 32 features nb*32 .. +31:
// lane (feature nb*32 + lane % 32, half lh = lane / 32) receives rows 16 st + 4 lh + {0..3} and
// 16 st + 8 + 4 lh + {0..3}, the order in which a 32x32 accumulator holds its rows.  Two LDS
// transpose reads (ds_read_b64_tr_b16): within 16 lanes, lane 4e+q passes the address of 4 features of
// row e and lane j receives feature j of the four rows.
__device__ inline bf16x8 lds_frag_t(const u32x4* rows, int nb, int lane, int st) {
  const int j = lane & 15, cb = (lane >> 4) & 1, lh = lane >> 5;
  const int chunk = nb * 4 + cb * 2 + ((j & 3) >> 1), half = j & 1;
  const int r0 = 16 * st + 4 * lh + (j >> 2), r1 = r0 + 8;
  const unsigned char* p = (const unsigned char*)rows;
  union { bf16x8 v; s16x4 h[2]; } f;
  f.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p + (r0 * 8 + (chunk ^ swz(r0))) * 16 + half * 8));
  f.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (s16x4 __attribute__((address_space(3)))*)(p + (r1 * 8 + (chunk ^ swz(r1))) * 16 + half * 8));
  return f.v;
}

template <int NJ>
__global__ __launch_bounds__(NJ * 64) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv, int T, int H,
                                                               bf16* __restrict__ out, float* __restrict__ lse,
                                                               float* __restrict__ cls_prob) {
  constexpr int Tpad = NJ * 32, NTH = NJ * 64;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* Ks = (u32x4*)smem;                         // [Tpad][8 chunks]
  u32x4* Vs = Ks + Tpad * 8;                        // [Tpad][8 chunks]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  const int b = blockIdx.x / H, h = blockIdx.x % H;
  const int D = H * HD;
  const int64_t rs = 3 * (int64_t)D;
  const bf16* base = qkv + (int64_t)b * T * rs + h * HD;
  const int q0 = wave * 32;                         // wave w owns queries 32 w .. 32 w + 31 (q0 < T always)
  // Q fragments straight from global memory, requested before K and V are staged so that their
  // latency is hidden: lane (query lr, half lh) needs chunks 2 ks + lh
  bf16x8 qf[4];
  {
    const bf16* qrow = base + (int64_t)min(q0 + lr, T - 1) * rs;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const bf16x8*)(qrow + (2 * ks + lh) * 8);
  }
  load_k(base + D, rs, T, Tpad, Ks, tid, NTH);
  load_k(base + 2 * D, rs, T, Tpad, Vs, tid, NTH);
  __syncthreads();

  // S^T[key, query] = K Q^T
  f32x16 s[NJ];
  const int sw = swz(lr);
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) s[jb][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8 kf = *(const bf16x8*)(Ks + (jb * 32 + lr) * 8 + ((2 * ks + lh) ^ sw));
      s[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[jb], 0, 0, 0);
    }
  }
  // softmax over keys: this lane holds, for query q0 + lr, the keys key_of(jb, r, lh).  The probabilities
  // stay unnormalised (p = exp(s - max) in (0, 1]) on their way through the second product; 1 / sum is
  // applied to the 32 output values instead of the 32 NJ probabilities.
  const float c = 0.125f * 1.44269504088896341f;    // 1/sqrt(64) * log2(e)
  float mx = -INFINITY;
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
    if (jb * 32 + 32 > T) {                         // only the last key block can hold keys past T (uniform)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (key_of(jb, r, lh) >= T) s[jb][r] = -INFINITY;
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[jb][r]);
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float mc = mx * c;
  float sum = 0.f;
  bf16x8 pf[2 * NJ];
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = __builtin_amdgcn_exp2f(fmaf(s[jb][r], c, -mc));
      s[jb][r] = p;
      sum += p;
      pf[2 * jb + (r >> 3)][r & 7] = (bf16)p;
    }
  sum += __shfl_xor(sum, 32, 64);
  const float inv = 1.0f / sum;
  const int qi = q0 + lr;
  if (lse && lh == 0 && qi < T) lse[((int64_t)b * H + h) * T + qi] = mx * 0.125f + __logf(sum);
  if (cls_prob && qi == 0) {   // the CLS query: its softmax row in fp32 (Eq. 6)
    float* dst = cls_prob + ((int64_t)b * H + h) * T;
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = key_of(jb, r, lh);
        if (j < T) dst[j] = s[jb][r] * inv;
      }
  }
  // O^T = V^T P^T, contraction over keys in the order the accumulators hold them:
  // step st covers keys 16 st + {4 lh .. 4 lh + 3} and 16 st + 8 + {4 lh .. 4 lh + 3}.
  // With the features as rows, a lane ends up with 4 consecutive features of its own query per
  // accumulator quad: the output leaves in 8-byte stores.
  f32x16 o[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
    for (int r = 0; r < 16; ++r) o[nb][r] = 0.f;
#pragma unroll
    for (int st = 0; st < 2 * NJ; ++st)
      o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag_t(Vs, nb, lane, st), pf[st], o[nb], 0, 0, 0);
  }
  if (qi < T) {
    bf16* orow = out + ((int64_t)b * T + qi) * D + h * HD + 4 * lh;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16x4 v4;
#pragma unroll
        for (int e = 0; e < 4; ++e) v4[e] = (bf16)(o[nb][4 * rq + e] * inv);
        *(bf16x4*)(orow + nb * 32 + 8 * rq) = v4;
      }
  }
}

template <int NJ>
void launch_fwd(const bf16* qkv, int B, int T, int H, bf16* out, float* lse, float* cls_prob, hipStream_t s) {
  static bool attr_set = false;
  constexpr size_t lds = (size_t)2 * NJ * 32 * 128;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)attn_fwd_mfma_kernel<NJ>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_set = true;
  }
  attn_fwd_mfma_kernel<NJ><<<B * H, NJ * 64, lds, s>>>(qkv, T, H, out, lse, cls_prob);
}


// ------------------------------------------------------------------------------------------ backward
// Backward of Eq. 1 per head (the "non-linear layer" case of Eq. 3 / Eq. 5: it needs the stored
// q, k, v and the softmax statistics).  With P_ij = exp(s_ij / 8 - lse_i), dP_ij = dO_i . v_j,
// delta_i = dO_i . O_i (= sum_j P_ij dP_ij) and dS_ij = P_ij (dP_ij - delta_i) / 8:
//   dQ_i = sum_j dS_ij k_j      (kernel "dq":  a wave owns 32 queries, sweeps the key blocks)
//   dK_j = sum_i dS_ij q_i,  dV_j = sum_i P_ij dO_i   (kernel "dkv": a wave owns 32 keys, sweeps
//                                                      the query blocks)
// Both recompute S with MFMAs; nothing T x T is stored or exchanged between wavefronts, and no
// atomics are used.  As in the forward kernel the lane that owns the output row keeps the
// contraction index in accumulator order and the transposed operand in LDS is read in that order.

__device__ inline bf16x8 lds_frag(const u32x4* rows, int row, int chunk) {
  return *(const bf16x8*)(rows + row * 8 + (chunk ^ swz(row)));
}

template <int NJ>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ out,
                                                          const bf16* __restrict__ dout, const float* __restrict__ lse,
                                                          int T, int H, float* __restrict__ delta,
                                                          bf16* __restrict__ dqkv) {
  constexpr int Tpad = NJ * 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* Ks = (u32x4*)smem;
  u32x4* Vs = Ks + Tpad * 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int D = H * HD;
  const int64_t rs = 3 * (int64_t)D;
  const bf16* base = qkv + (int64_t)b * T * rs + h * HD;
  load_k(base + D, rs, T, Tpad, Ks, tid);
  load_k(base + 2 * D, rs, T, Tpad, Vs, tid);
  __syncthreads();
  const int q0 = blockIdx.x * 128 + wave * 32;
  if (q0 >= T) return;
  const int qi = q0 + lr, qc = min(qi, T - 1);
  bf16x8 qf[4], dof[4];
  float dl = 0.f;
  {
    const bf16* qrow = base + (int64_t)qc * rs;
    const bf16* dorow = dout + ((int64_t)b * T + qc) * D + h * HD;
    const bf16* orow = out + ((int64_t)b * T + qc) * D + h * HD;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qf[ks] = *(const bf16x8*)(qrow + (2 * ks + lh) * 8);
      dof[ks] = *(const bf16x8*)(dorow + (2 * ks + lh) * 8);
      const bf16x8 of = *(const bf16x8*)(orow + (2 * ks + lh) * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) dl += (float)dof[ks][e] * (float)of[e];
    }
  }
  dl += __shfl_xor(dl, 32, 64);
  const float l2 = lse[((int64_t)b * H + h) * T + qc] * 1.44269504088896341f;
  if (lh == 0 && qi < T) delta[((int64_t)b * H + h) * T + qi] = dl;
  const float c = 0.125f * 1.44269504088896341f;
  f32x16 o[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[nb][r] = 0.f;
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
    f32x16 sa, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { sa[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(Ks, jb * 32 + lr, 2 * ks + lh), qf[ks], sa, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(Vs, jb * 32 + lr, 2 * ks + lh), dof[ks], dp, 0, 0, 0);
    }
    bf16x8 dsf[2];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float pr = __builtin_amdgcn_exp2f(sa[r] * c - l2);
      if (key_of(jb, r, lh) >= T) pr = 0.f;
      dsf[r >> 3][r & 7] = (bf16)(pr * (dp[r] - dl) * 0.125f);
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
        o[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dsf[hf], lds_frag_t(Ks, nb, lane, 2 * jb + hf), o[nb], 0, 0, 0);
  }
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = q0 + 8 * (r >> 2) + 4 * lh + (r & 3);
      if (i < T) dqkv[((int64_t)b * T + i) * rs + h * HD + nb * 32 + lr] = (bf16)o[nb][r];
    }
}

template <int NJ>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dout,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           int T, int H, bf16* __restrict__ dqkv) {
  constexpr int Tpad = NJ * 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* Qs = (u32x4*)smem;
  u32x4* dOs = Qs + Tpad * 8;
  float* lse_s = (float*)(dOs + Tpad * 8);      // [Tpad], pre-multiplied by log2(e); +inf beyond T
  float* del_s = lse_s + Tpad;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  const int b = blockIdx.y / H, h = blockIdx.y % H;
  const int D = H * HD;
  const int64_t rs = 3 * (int64_t)D;
  const bf16* base = qkv + (int64_t)b * T * rs + h * HD;
  const bf16* dobase = dout + (int64_t)b * T * D + h * HD;
  load_k(base, rs, T, Tpad, Qs, tid);
  load_k(dobase, D, T, Tpad, dOs, tid);
  for (int i = tid; i < Tpad; i += 256) {
    lse_s[i] = (i < T) ? lse[((int64_t)b * H + h) * T + i] * 1.44269504088896341f : INFINITY;
    del_s[i] = (i < T) ? delta[((int64_t)b * H + h) * T + i] : 0.f;
  }
  __syncthreads();
  const int j0 = blockIdx.x * 128 + wave * 32;
  if (j0 >= T) return;
  const int jc = min(j0 + lr, T - 1);
  bf16x8 kf[4], vf[4];
  {
    const bf16* krow = base + (int64_t)jc * rs + D;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      kf[ks] = *(const bf16x8*)(krow + (2 * ks + lh) * 8);
      vf[ks] = *(const bf16x8*)(krow + D + (2 * ks + lh) * 8);
    }
  }
  const float c = 0.125f * 1.44269504088896341f;
  f32x16 ok[2], ov[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) { ok[nb][r] = 0.f; ov[nb][r] = 0.f; }
#pragma unroll
  for (int ib = 0; ib < NJ; ++ib) {
    f32x16 sa, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { sa[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(Qs, ib * 32 + lr, 2 * ks + lh), kf[ks], sa, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(dOs, ib * 32 + lr, 2 * ks + lh), vf[ks], dp, 0, 0, 0);
    }
    bf16x8 pf[2], dsf[2];
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {           // queries 32 ib + 8 g4 + 4 lh + {0..3}
      const float4 l4 = *(const float4*)(lse_s + ib * 32 + 8 * g4 + 4 * lh);
      const float4 d4 = *(const float4*)(del_s + ib * 32 + 8 * g4 + 4 * lh);
      const float lv[4] = {l4.x, l4.y, l4.z, l4.w};
      const float dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int r = g4 * 4 + e;
        const float pr = __builtin_amdgcn_exp2f(sa[r] * c - lv[e]);
        pf[r >> 3][r & 7] = (bf16)pr;
        dsf[r >> 3][r & 7] = (bf16)(pr * (dp[r] - dv[e]) * 0.125f);
      }
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        ov[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[hf], lds_frag_t(dOs, nb, lane, 2 * ib + hf), ov[nb], 0, 0, 0);
        ok[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dsf[hf], lds_frag_t(Qs, nb, lane, 2 * ib + hf), ok[nb], 0, 0, 0);
      }
  }
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = j0 + 8 * (r >> 2) + 4 * lh + (r & 3);
      if (j < T) {
        bf16* dst = dqkv + ((int64_t)b * T + j) * rs + h * HD + nb * 32 + lr;
        dst[D] = (bf16)ok[nb][r];
        dst[2 * D] = (bf16)ov[nb][r];
      }
    }
}

template <int NJ>
void launch_bwd(const bf16* qkv, const bf16* out, const bf16* dout, const float* lse, int B, int T, int H,
                float* delta, bf16* dqkv, hipStream_t s) {
  static bool attr_set = false;
  constexpr size_t lds_q = (size_t)2 * NJ * 32 * 128;
  constexpr size_t lds_kv = (size_t)2 * NJ * 32 * 128 + (size_t)2 * NJ * 32 * sizeof(float);
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)attn_bwd_dq_kernel<NJ>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_q);
    (void)hipFuncSetAttribute((const void*)attn_bwd_dkv_kernel<NJ>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_kv);
    attr_set = true;
  }
  const dim3 grid((T + 127) / 128, B * H);
  attn_bwd_dq_kernel<NJ><<<grid, 256, lds_q, s>>>(qkv, out, dout, lse, T, H, delta, dqkv);
  attn_bwd_dkv_kernel<NJ><<<grid, 256, lds_kv, s>>>(qkv, dout, lse, delta, T, H, dqkv);
}

}  // namespace

bool attn_mfma_supported(int T, int d) { return d == HD && T >= 1 && T <= 256; }

void attn_fwd_mfma(const void* qkv, int B, int T, int H, void* out, float* lse, float* cls_prob, hipStream_t s) {
  const bf16* q = (const bf16*)qkv;
  bf16* o = (bf16*)out;
  switch ((T + 31) / 32) {
    case 1: launch_fwd<1>(q, B, T, H, o, lse, cls_prob, s); break;
    case 2: launch_fwd<2>(q, B, T, H, o, lse, cls_prob, s); break;
    case 3: launch_fwd<3>(q, B, T, H, o, lse, cls_prob, s); break;
    case 4: launch_fwd<4>(q, B, T, H, o, lse, cls_prob, s); break;
    case 5: launch_fwd<5>(q, B, T, H, o, lse, cls_prob, s); break;
    case 6: launch_fwd<6>(q, B, T, H, o, lse, cls_prob, s); break;
    case 7: launch_fwd<7>(q, B, T, H, o, lse, cls_prob, s); break;
    default: launch_fwd<8>(q, B, T, H, o, lse, cls_prob, s); break;
  }
}

}  // namespace bsr

namespace bsr {

void attn_bwd_mfma(const void* qkv, const void* out, const void* dout, const float* lse, int B, int T, int H,
                   float* delta, void* dqkv, hipStream_t s) {
  const bf16* q = (const bf16*)qkv;
  const bf16* o = (const bf16*)out;
  const bf16* d = (const bf16*)dout;
  bf16* g = (bf16*)dqkv;
  switch ((T + 31) / 32) {
    case 1: launch_bwd<1>(q, o, d, lse, B, T, H, delta, g, s); break;
    case 2: launch_bwd<2>(q, o, d, lse, B, T, H, delta, g, s); break;
    case 3: launch_bwd<3>(q, o, d, lse, B, T, H, delta, g, s); break;
    case 4: launch_bwd<4>(q, o, d, lse, B, T, H, delta, g, s); break;
    case 5: launch_bwd<5>(q, o, d, lse, B, T, H, delta, g, s); break;
    case 6: launch_bwd<6>(q, o, d, lse, B, T, H, delta, g, s); break;
    case 7: launch_bwd<7>(q, o, d, lse, B, T, H, delta, g, s); break;
    default: launch_bwd<8>(q, o, d, lse, B, T, H, delta, g, s); break;
  }
}

}  // namespace bsr
