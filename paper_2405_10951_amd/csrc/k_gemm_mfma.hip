// bf16 MFMA GEMMs for gfx950 (CDNA4), the hot kernels of the BSR step.
//
// Two kernels, both C = epilogue(sum_k A(m,k) B(k,n)) with fp32 accumulation in
// v_mfma_f32_32x32x16_bf16 tiles staged through LDS:
//   NT: A[M,K] and B^T[N,K] both have the contraction index contiguous.  Covers the forward linears
//       (activations x bf16 weight copy stored [out,in]) and the input gradients of Eq. 2
//       (dY x weight copy stored [in,out]).
//   TN: A^T[K,M] and B[K,N] both have the contraction index strided (rows are tokens).  Covers the
//       weight gradients of Eq. 4, dW = X^T dY, contraction over all tokens of the batch.
//
// Block tile BM x BN x 64 shared by WM x WN wavefronts, each owning a wave tile of 32x32 MFMA tiles.
// LDS is double buffered; the next k-tile waits in registers while the current one feeds the
// matrix cores.  Workgroups are renumbered so that each XCD (the hardware deals consecutive
// workgroup ids round-robin over 8 XCDs) works on a contiguous range of tiles and its L2 sees whole
// operand panels.
#include <algorithm>
#include <utility>

#include "bsr_internal.h"

namespace bsr {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte chunk in registers

constexpr int BK = 64;        // k-tile: 64 bf16 = 8 chunks of 16 bytes per row
constexpr int NXCD = 8;

// GELU(u) = u Phi(u) and its derivative Phi(u) + u phi(u) with the exact (erf) Phi.  erf comes from
// the rational-exponential form of Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7 (below 1e-6 in
// fp32 arithmetic): far below the resolution of the bf16 values these epilogues write, at a fraction
// of the instructions of erff.  Its exp(-x^2) with x = u / sqrt(2) is the Gaussian that phi(u) needs
// as well.
__device__ inline float erf_as(float x, float& gauss) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(1.061405429f, t, -1.453152027f);
  p = fmaf(p, t, 1.421413741f);
  p = fmaf(p, t, -0.284496736f);
  p = fmaf(p, t, 0.254829592f);
  gauss = __expf(-ax * ax);
  return copysignf(fmaf(-p * t, gauss, 1.0f), x);
}
__device__ inline float gelu_f(float u) {
  float gauss;
  return 0.5f * u * (1.0f + erf_as(u * 0.70710678118654752f, gauss));
}
__device__ inline float gelu_grad_f(float u) {
  float gauss;
  const float cdf = 0.5f * (1.0f + erf_as(u * 0.70710678118654752f, gauss));
  return fmaf(u * 0.39894228040143268f, gauss, cdf);
}

template <int V> struct IC { static constexpr int value = V; };   // compile-time flag for generic lambdas
// f(IC<0>{}), ..., f(IC<N-1>{}): a loop whose index is a compile-time constant in the body
template <class F, int... I> __device__ __forceinline__ void sfor_impl(F&& f, std::integer_sequence<int, I...>) { (f(IC<I>{}), ...); }
template <int N, class F> __device__ __forceinline__ void sfor(F&& f) { sfor_impl(f, std::make_integer_sequence<int, N>{}); }

// LDS chunk swizzle: 16 consecutive rows reading the same logical 16-byte chunk hit 16 different
// (row parity, chunk position) pairs, i.e. all 64 banks once; 8 consecutive rows hit 8 positions.
__device__ inline int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// Logical tile id of this workgroup: XCD x owns the contiguous range [start(x), start(x+1)).
__device__ inline int xcd_remap(int pid, int nblocks) {
  const int base = nblocks / NXCD, rem = nblocks % NXCD;
  const int x = pid % NXCD, local = pid / NXCD;
  return x * base + min(x, rem) + local;
}

// Eight consecutive columns of output row m, accumulated in fp32: the statistics of a folded LayerNorm, bias,
// positional embedding (with the row remap of the patch embedding), GELU with its stored pre-activation or
// GELU', the residual, and the store (16 bytes of bf16, or 32 bytes of fp32).
__device__ __forceinline__ void finish8(const GemmDesc& g, float (&v)[8], int m, int col, const float (&bias)[8],
                                        const float (&cs)[8], const float2* st) {
  if (st) {
    const float2 ms = *st;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = ms.y * fmaf(-ms.x, cs[j], v[j]);
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) v[j] += bias[j];
  int64_t row = m;
  if (g.remap_np > 0) {
    row = (int64_t)m + m / g.remap_np + 1;
    const float* pr = g.pos + (int64_t)(m % g.remap_np + 1) * g.N + col;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] += pr[j];
  }
  const int64_t off = row * g.ldc + col;
  if (g.act == ACT_GELU) {
    if (g.aux) {
      bf16x8 u;
#pragma unroll
      for (int j = 0; j < 8; ++j) u[j] = (bf16)v[j];
      *(bf16x8*)((bf16*)g.aux + off) = u;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = gelu_f(v[j]);
  } else if (g.act == ACT_GELU_BWD) {
    const bf16x8 u = *(const bf16x8*)((const bf16*)g.aux + off);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] *= gelu_grad_f((float)u[j]);
  }
  if (g.out_f32) {
    float* c = (float*)g.C + off;
    *(float4*)c = make_float4(v[0], v[1], v[2], v[3]);
    *(float4*)(c + 4) = make_float4(v[4], v[5], v[6], v[7]);
  } else {
    if (g.res) {
      const bf16x8 rr = *(const bf16x8*)((const bf16*)g.res + off);
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] += (float)rr[j];
    }
    bf16x8 o;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[j] = (bf16)v[j];
    *(bf16x8*)((bf16*)g.C + off) = o;
  }
}

// Epilogue of one wave tile.  The fp32 accumulators (element r of a 32x32 tile sits at row
// 8*(r/4) + 4*(lane/32) + r%4, column lane%32) go through a per-wave LDS patch, 32 rows at a time,
// and come back row-major so that each lane owns 8 consecutive columns of one row: bias, GELU,
// GELU', positional embedding and residual are applied on 8-wide vectors and C is written with
// 16-byte stores (32 bytes for fp32 output).
template <int MI, int NI>
__device__ __forceinline__ void epilogue(const GemmDesc& g, f32x16 (&acc)[MI][NI], int row0, int col0, int lane,
                                float* patch, const float2* rowstat = nullptr) {
  constexpr int TN = NI * 32, LDP = TN + 4;     // +4 floats: rows start in different banks
  constexpr int CPR = TN / 8;                   // 8-column chunks per row
  constexpr int RPI = 64 / CPR;                 // rows handled per pass of the wave
  const int lc = lane & 31, lh = lane >> 5;
  const int my_chunk = lane % CPR, my_row = lane / CPR;
  const int col = col0 + my_chunk * 8;
  const bool col_ok = col < g.N;                // N is a multiple of 8 on this path
  float bias[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) bias[j] = (g.bias && col_ok) ? g.bias[col + j] : 0.f;
  // folded LayerNorm: rowstat holds (mean, 1/std) of the wave tile's rows of A, cs the column sums of W'
  float cs[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) cs[j] = (rowstat && col_ok) ? g.ln_colsum[col + j] : 0.f;
  // (row blocks and passes are loops, the accumulators of block mi picked by a switch: written out, this code was
  // most of the kernel, and a launch that follows another kernel fetches its code anew)
#pragma nounroll
  for (int mi = 0; mi < MI; ++mi) {
    sfor<MI>([&](auto I) __attribute__((always_inline)) {
      constexpr int i = decltype(I)::value;
      if (mi != i) return;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          patch[(8 * (r >> 2) + 4 * lh + (r & 3)) * LDP + ni * 32 + lc] = acc[i][ni][r];
    });
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma nounroll
    for (int pass = 0; pass < 32 / RPI; ++pass) {
      const int lr = pass * RPI + my_row;
      const int m = row0 + mi * 32 + lr;
      if (m >= g.M || !col_ok) continue;
      float v[8];
      const float4 p0 = *(const float4*)(patch + lr * LDP + my_chunk * 8);
      const float4 p1 = *(const float4*)(patch + lr * LDP + my_chunk * 8 + 4);
      v[0] = p0.x; v[1] = p0.y; v[2] = p0.z; v[3] = p0.w; v[4] = p1.x; v[5] = p1.y; v[6] = p1.z; v[7] = p1.w;
      finish8(g, v, m, col, bias, cs, rowstat ? rowstat + mi * 32 + lr : nullptr);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// A weight-gradient launch folded into an input-gradient launch (both read the same dy and neither reads
// what the other writes): workgroups past nt_tiles do the work of workgroup (i % gx, i / gx) of the
// gx x gy weight-gradient grid.
struct TnArgs {
  GemmDesc g;
  float *partial, *bpartial;
  int kt_per, tn_rows;
  TnReduce red;
  int gx, gy;
  int nt_tiles;
};
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void tn_body(GemmDesc g, float* partial, float* bpartial, int kt_per, int tn_rows,
                                        const TnReduce& red, int bx, int by, int gx, int gy);

// ------------------------------------------------------------------------------------------ NT
// LDS tile: rows of 8 chunks (16 B each), chunk kc of row r stored at position kc ^ swz(r).
// Software pipeline of one k-tile (4 MFMA steps of k = 16):
//   step 0,1: MFMAs on fragment set s while the fragments of the next step load into set s^1
//   step 2  : as above; the registers holding k-tile kt+1 go to the other LDS buffer and the global
//             loads of k-tile kt+1+PF are issued into the registers just freed
//   barrier ; step 3: MFMAs of the last fragments while the first fragments of k-tile kt+1 load.
// PF register stages hold the k-tiles kt+1 .. kt+PF on their way from global memory (k-tile j in stage
// j % PF): with PF = 1 a load has one k-tile of matrix work to land, which a small tile that is alone on
// its CU finishes long before an L2 or HBM access returns; such tiles run with PF = 3.
// Rows beyond M (or N) are clamped to the last valid row: they only feed accumulators that are
// never stored.  KTAIL zero-fills chunks beyond K (K % 64 != 0).
// (A folded 8-wave kernel whose tiles leave room for two workgroups per CU is held to the 128 registers that
// two workgroups need: the row sums would otherwise push the 192 x 128 shape to 132 and halve its occupancy.)
template <int BM, int BN, int WM, int WN, bool KTAIL, int PF = 1, bool FUSE = false, bool LNF = false>
__global__ __launch_bounds__(WM * WN * 64, (LNF && PF == 1 && WM * WN == 8 && (BM + BN) * 256 <= 80 * 1024) ? 4 : 1)
void gemm_nt_kernel(GemmDesc g, TnArgs tn) {
  static_assert(!LNF || (!FUSE && !KTAIL), "the folded LayerNorm reads whole rows of A in whole k-tiles");
  constexpr int NT = WM * WN * 64;
  if (FUSE && (int)blockIdx.x >= tn.nt_tiles) {          // uniform over the workgroup
    static_assert(!FUSE || NT == 512, "the weight-gradient body runs with 8 waves");
    const int i = blockIdx.x - tn.nt_tiles;
    tn_body<128, 128, 4, 2>(tn.g, tn.partial, tn.bpartial, tn.kt_per, tn.tn_rows, tn.red, i % tn.gx, i / tn.gx, tn.gx, tn.gy);
    return;
  }
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int ACH = (BM * 8 + NT - 1) / NT, BCH = (BN * 8 + NT - 1) / NT;   // 16-byte chunks per thread per tile
  constexpr bool AEVEN = (BM * 8) % NT == 0, BEVEN = (BN * 8) % NT == 0;      // else the last chunk is partial
  static_assert(MI >= 1 && NI >= 1 && TM % 32 == 0 && TN % 32 == 0, "wave tiles are made of 32x32 MFMA tiles");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* As = (u32x4*)smem;                    // [2][BM*8]
  u32x4* Bs = As + 2 * BM * 8;                 // [2][BN*8]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int ntn = (g.N + BN - 1) / BN;
  const int tile = xcd_remap(blockIdx.x, FUSE ? tn.nt_tiles : (int)gridDim.x);
  int m0 = (tile / ntn) * BM;
  const int n0 = (tile % ntn) * BN;
  if (g.grp_off) {
    // grouped form: the tile index counts row tiles group after group (a group's last tile may be
    // partial); workgroups past the last group have nothing to do
    int mt = tile / ntn, e = 0, found = 0;
    for (; e < g.groups; ++e) {
      const int r0 = g.grp_off[e], r1 = g.grp_off[e + 1];
      const int nt_e = (r1 - r0 + BM - 1) / BM;
      if (mt < nt_e) {
        m0 = r0 + mt * BM;
        g.M = r1;                                   // rows of this tile stop at the end of its group
        found = 1;
        break;
      }
      mt -= nt_e;
    }
    if (!found) return;
    g.B = (const bf16*)g.B + (int64_t)e * g.b_gs;
    if (g.bias) g.bias += (int64_t)e * g.bias_gs;
  }
  const bf16* __restrict__ A = (const bf16*)g.A;
  const bf16* __restrict__ Bt = (const bf16*)g.B;

  // per-thread chunk coordinates are the same for every k-tile
  const bf16* pa[ACH];
  const bf16* pb[BCH];
  int sa[ACH], sb[BCH];
  const int kc8 = (tid & 7) * 8;               // NT is a multiple of 8: every chunk of a thread has the same kc
  // (threads past the end of an uneven tile repeat its last row: same data, same LDS slot)
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int row = AEVEN ? (tid + NT * i) >> 3 : min((tid + NT * i) >> 3, BM - 1);
    pa[i] = A + (int64_t)min(m0 + row, g.M - 1) * g.a_rs + kc8;
    sa[i] = row * 8 + ((tid & 7) ^ swz(row));
  }
#pragma unroll
  for (int i = 0; i < BCH; ++i) {
    const int row = BEVEN ? (tid + NT * i) >> 3 : min((tid + NT * i) >> 3, BN - 1);
    pb[i] = Bt + (int64_t)min(n0 + row, g.N - 1) * g.b_cs + kc8;
    sb[i] = row * 8 + ((tid & 7) ^ swz(row));
  }
  u32x4 ra[PF][ACH], rb[PF][BCH];        // the next PF k-tiles wait here while the current one is multiplied
  auto fetch = [&](auto ST, int k0) __attribute__((always_inline)) {
    constexpr int st = decltype(ST)::value;
    if (KTAIL) {
      const bool oob = k0 + kc8 >= g.K;
      const int kk = oob ? 0 : k0;
#pragma unroll
      for (int i = 0; i < ACH; ++i) {
        ra[st][i] = *(const u32x4*)(pa[i] + kk - (oob ? kc8 : 0));
        if (oob) ra[st][i] = u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int i = 0; i < BCH; ++i) {
        rb[st][i] = *(const u32x4*)(pb[i] + kk - (oob ? kc8 : 0));
        if (oob) rb[st][i] = u32x4{0u, 0u, 0u, 0u};
      }
    } else {
#pragma unroll
      for (int i = 0; i < ACH; ++i) ra[st][i] = *(const u32x4*)(pa[i] + k0);
#pragma unroll
      for (int i = 0; i < BCH; ++i) rb[st][i] = *(const u32x4*)(pb[i] + k0);
    }
  };
  // Folded LayerNorm (LNF): the workgroup sees every element of its rows of A on the way to LDS, so it
  // takes their mean and variance itself: each thread adds up its chunks (always the same 8 of the 64
  // columns of a k-tile, k-tiles in ascending order; two bf16 per dot instruction), and the 8 threads of a
  // row are combined after the last k-tile.  The order does not depend on the tile shape.
  float rsum[LNF ? ACH : 1], rsq[LNF ? ACH : 1];
#pragma unroll
  for (int i = 0; i < (LNF ? ACH : 1); ++i) rsum[i] = rsq[i] = 0.f;
  auto stash = [&](auto ST, int buf) __attribute__((always_inline)) {
    constexpr int st = decltype(ST)::value;
#pragma unroll
    for (int i = 0; i < ACH; ++i) As[buf * BM * 8 + sa[i]] = ra[st][i];
#pragma unroll
    for (int i = 0; i < BCH; ++i) Bs[buf * BN * 8 + sb[i]] = rb[st][i];
    if constexpr (LNF) {
      const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
#pragma unroll
      for (int i = 0; i < ACH; ++i)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          // (the empty asm pins the word in a register of its own: without it the compiler folds the
          // extract-and-cast of all four words of a chunk onto word 0)
          unsigned word = ra[st][i][w];
          asm("" : "+v"(word));
          const bf16x2 pr = __builtin_bit_cast(bf16x2, word);
          rsum[i] = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, rsum[i], false);
          rsq[i] = __builtin_amdgcn_fdot2_f32_bf16(pr, pr, rsq[i], false);
        }
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  const int lr = lane & 31, lh = lane >> 5;
  int offa[MI], offb[NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) offa[mi] = (wm * TM + mi * 32 + lr) * 8;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) offb[ni] = (wn * TN + ni * 32 + lr) * 8;
  const int sw = swz(lr);

  bf16x8 fa[2][MI], fb[2][NI];
  auto load_frags = [&](int set, const u32x4* Ab, const u32x4* Bb, int ks) __attribute__((always_inline)) {
    const int kc = (ks * 2 + lh) ^ sw;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) fa[set][mi] = *(const bf16x8*)(Ab + offa[mi] + kc);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) fb[set][ni] = *(const bf16x8*)(Bb + offb[ni] + kc);
  };
  auto mma = [&](int set) __attribute__((always_inline)) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][mi], fb[set][ni], acc[mi][ni], 0, 0, 0);
  };

  const int nk = (g.K + BK - 1) / BK;
  // prologue: k-tile 0 into LDS buffer 0, k-tiles 1 .. PF in flight in the register stages
  fetch(IC<0>{}, 0);
  stash(IC<0>{}, 0);
  auto pro = [&](auto J) __attribute__((always_inline)) {
    constexpr int j = decltype(J)::value;
    if (j <= PF && j < nk) fetch(IC<j % PF>{}, j * BK);
  };
  pro(IC<1>{}); pro(IC<2>{}); pro(IC<3>{}); pro(IC<4>{});
  static_assert(PF >= 1 && PF <= 4, "");
  __syncthreads();
  load_frags(0, As, Bs, 0);
  // One k-tile.  ST: the register stage of k-tile kt + 1.  do_stash: k-tile kt + 1 exists (stage -> other
  // LDS buffer, and its first fragments are loaded after the barrier); do_fetch: k-tile kt + 1 + PF exists.
  // The steady-state loop has both set and no branches, so that the compiler can interleave the whole body.
  auto ktile = [&](auto ST, auto STEADY, bool do_stash, bool do_fetch, int kt) __attribute__((always_inline)) {
    constexpr bool steady = decltype(STEADY)::value != 0;      // both flags known to be set: no branches
    const int buf = kt & 1;
    const u32x4* Ab = As + buf * BM * 8;
    const u32x4* Bb = Bs + buf * BN * 8;
    load_frags(1, Ab, Bb, 1);
    mma(0);
    load_frags(0, Ab, Bb, 2);
    mma(1);
    load_frags(1, Ab, Bb, 3);
    if (steady || do_stash) stash(ST, buf ^ 1);
    if (steady || do_fetch) fetch(ST, (kt + 1 + PF) * BK);
    mma(0);
    __syncthreads();
    if (steady || do_stash) load_frags(0, As + (buf ^ 1) * BM * 8, Bs + (buf ^ 1) * BN * 8, 0);
    mma(1);
  };
  // k-tile kt + j of a run that starts at a multiple of PF has k-tile kt + j + 1 in stage (j + 1) % PF
  auto steady_one = [&](auto J, int kt) __attribute__((always_inline)) {
    constexpr int j = decltype(J)::value;
    if (j < PF) ktile(IC<(j + 1) % PF>{}, IC<1>{}, true, true, kt + j);
  };
  auto tail_one = [&](auto J, int kt) __attribute__((always_inline)) {
    constexpr int j = decltype(J)::value;
    if (j < 2 * PF && kt + j < nk) ktile(IC<(j + 1) % PF>{}, IC<0>{}, kt + j + 1 < nk, kt + j + 1 + PF < nk, kt + j);
  };
  int kt = 0;
  for (; kt + 2 * PF < nk; kt += PF) {      // every k-tile of the group stashes and fetches
    steady_one(IC<0>{}, kt); steady_one(IC<1>{}, kt); steady_one(IC<2>{}, kt); steady_one(IC<3>{}, kt);
  }
  // at most 2 PF k-tiles are left
  tail_one(IC<0>{}, kt); tail_one(IC<1>{}, kt); tail_one(IC<2>{}, kt); tail_one(IC<3>{}, kt);
  tail_one(IC<4>{}, kt); tail_one(IC<5>{}, kt); tail_one(IC<6>{}, kt); tail_one(IC<7>{}, kt);
  __syncthreads();
  // the tile buffers are free now: reuse them as per-wave epilogue patches
  float* patch = (float*)smem + wave * (32 * (TN + 4));
  // folded LayerNorm: (mean, 1/std) of the tile's rows go behind the epilogue patches (inside the tile
  // buffers, which are free by now, whenever those are the larger of the two)
  constexpr size_t LDS_PATCH = (size_t)WM * WN * 32 * (TN + 4) * sizeof(float);
  float2* rowstat = (float2*)(smem + LDS_PATCH);
  if constexpr (LNF) {
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
      float sm = rsum[i], sq = rsq[i];
      sm += __shfl_xor(sm, 1); sq += __shfl_xor(sq, 1);
      sm += __shfl_xor(sm, 2); sq += __shfl_xor(sq, 2);
      sm += __shfl_xor(sm, 4); sq += __shfl_xor(sq, 4);
      const float mean = sm / (float)g.K;
      const float var = fmaxf(sq / (float)g.K - mean * mean, 0.f);
      const int row = AEVEN ? (tid + NT * i) >> 3 : min((tid + NT * i) >> 3, BM - 1);
      if ((tid & 7) == 0) rowstat[row] = make_float2(mean, rsqrtf(var + g.ln_eps));
    }
    __syncthreads();
  }
  epilogue<MI, NI>(g, acc, m0 + wm * TM, n0 + wn * TN, lane, patch, LNF ? rowstat + wm * TM : nullptr);
}

template <int BM, int BN, int WM, int WN, int PF = 1>
void launch_nt(const GemmDesc& g, hipStream_t s) {
  static bool attr_set = false;
  constexpr size_t lds_tiles = (size_t)2 * (BM + BN) * BK * sizeof(bf16);
  constexpr size_t lds_patch = (size_t)WM * WN * 32 * (BN / WN + 4) * sizeof(float);   // epilogue patches
  constexpr size_t lds = lds_tiles > lds_patch ? lds_tiles : lds_patch;
  constexpr size_t lds_stat = lds_patch + BM * sizeof(float2);           // (mean, 1/std) of the tile's rows behind the patches
  constexpr size_t lds_lnf = lds > lds_stat ? lds : lds_stat;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)gemm_nt_kernel<BM, BN, WM, WN, false, PF>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)hipFuncSetAttribute((const void*)gemm_nt_kernel<BM, BN, WM, WN, true, PF>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)hipFuncSetAttribute((const void*)gemm_nt_kernel<BM, BN, WM, WN, false, PF, false, true>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_lnf);
    attr_set = true;
  }
  // grouped: every group may end in one partial row tile
  const int tiles = ((g.M + BM - 1) / BM + (g.grp_off ? g.groups : 0)) * ((g.N + BN - 1) / BN);
  if (g.ln_colsum) gemm_nt_kernel<BM, BN, WM, WN, false, PF, false, true><<<tiles, WM * WN * 64, lds_lnf, s>>>(g, TnArgs());
  else if (g.K % BK == 0) gemm_nt_kernel<BM, BN, WM, WN, false, PF><<<tiles, WM * WN * 64, lds, s>>>(g, TnArgs());
  else gemm_nt_kernel<BM, BN, WM, WN, true, PF><<<tiles, WM * WN * 64, lds, s>>>(g, TnArgs());
}

// ------------------------------------------------------------------------------------------ NT, operands straight into LDS
// The same product for K a multiple of 64, built around three facts measured on gfx950: LDS takes writes from
// registers at only 64 - 72 bytes per clock, a wavefront that is alone on its SIMD has nobody to hide its waits,
// and under matrix load the clock is set by power.  So (1) the operand tiles go from global memory straight into
// LDS with global_load_lds_dwordx4 (lane l of a wavefront writes 16 bytes at M0 + 16 l: one instruction fills 8 tile
// rows of 8 chunks, and the chunk swizzle of the LDS tile is applied to the global address a lane reads), which
// costs no registers and no LDS-write instructions; (2) NST stages of (BM + BN) x 64 and ONE barrier per k-tile:
// at the barrier every wavefront has finished reading k-tile kt and its own part of k-tile kt + 1 has landed
// (s_waitcnt vmcnt counts such a load when its data is in LDS), so behind the barrier k-tile kt + NST can go into
// the stage of k-tile kt; (3) the order of the k-loop is written out, every MFMA followed by at most one fragment
// read or a few loads, and pinned with scheduling barriers (the compiler's own order bunches the reads in front
// of the MFMAs and waits for them).  Wave tiles are at least 64 x 64 (128 x 64 in the 256 x 256 shape): per MFMA
// a wavefront reads 0.75 - 1 KB of fragments instead of the 1.5 KB of a 64 x 32 wave tile.
// The MFMA operands are swapped (weight rows first), so an accumulator holds the TRANSPOSED 32 x 32 output tile:
// a lane owns one output row and four runs of four consecutive columns.  That lets the epilogue round to bf16
// before the tile goes through LDS whenever nothing has to be added in fp32 afterwards (8-byte LDS writes of four
// bf16 instead of sixteen 4-byte writes per tile), and use 16-byte LDS writes otherwise.
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xF | (0x3 << 14) | (0x7 << 4)); }
#define BSR_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)
#define BSR_GLOBAL_PTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define BSR_LDS_VOID(p) ((void __attribute__((address_space(3)))*)(p))

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// Epilogue of one wave tile whose accumulators hold transposed output tiles: element r of acc[mi][ni] is output
// row mi*32 + lane%32, column ni*32 + 8*(r/4) + 4*(lane/32) + r%4.  32 rows at a time go through a per-wave LDS
// patch and come back with a lane owning 8 consecutive columns of a row (16-byte global stores).
// The code is kept short on purpose: a launch that follows another kernel fetches its code anew, and a version of
// this epilogue with every row block and pass written out (13 700 of the kernel's 14 400 instructions) cost a
// launch about 3 us.  So the row blocks are a loop (the accumulators of block mi are picked by a switch, which
// is all that has to be written out per block) and so are the passes: the finishing code exists once.
template <int MI, int NI>
__device__ __forceinline__ void epilogue_t(const GemmDesc& g, f32x16 (&acc)[MI][NI], int row0, int col0, int lane,
                                           unsigned char* patch) {
  constexpr int TN = NI * 32;
  constexpr int CPR = TN / 8, RPP = 64 / CPR;       // 8-column chunks per row, rows per pass of the wave
  constexpr int NPASS = (32 + RPP - 1) / RPP;       // (with 12 chunks per row 60 lanes work and the last pass is partial)
  const int lm = lane & 31, lh = lane >> 5;
  const int my_chunk = lane % CPR, my_row = lane / CPR;
  const int col = col0 + my_chunk * 8;
  const bool col_ok = col < g.N && my_row < RPP;    // N is a multiple of 8 on this path
  // nothing but the bias to add: round first, move half the bytes
  const bool direct = !g.out_f32 && !g.res && g.remap_np == 0 && g.act == ACT_NONE;
  if (direct) {
    constexpr int LDB = TN * 2 + 16;                // bytes per patch row
    bf16* dst = (bf16*)g.C;
#pragma nounroll
    for (int mi = 0; mi < MI; ++mi) {
      f32x4 bq[NI][4];                              // bias of the columns this lane holds (read per row block: the
#pragma unroll                                      // accumulators leave no registers to keep it in)
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int c = col0 + ni * 32 + 8 * rg + 4 * lh;
          bq[ni][rg] = (g.bias && c < g.N) ? *(const f32x4*)(g.bias + c) : f32x4{0.f, 0.f, 0.f, 0.f};
        }
      sfor<MI>([&](auto I) __attribute__((always_inline)) {
        constexpr int i = decltype(I)::value;
        if (mi != i) return;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int rg = 0; rg < 4; ++rg) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)(acc[i][ni][4 * rg + e] + bq[ni][rg][e]);
            *(bf16x4*)(patch + lm * LDB + (ni * 32 + 8 * rg + 4 * lh) * 2) = o;
          }
      });
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma nounroll
      for (int p = 0; p < NPASS; ++p) {
        const int lr = p * RPP + my_row;
        const int m = row0 + mi * 32 + lr;
        if (lr >= 32 || m >= g.M || !col_ok) continue;
        *(bf16x8*)(dst + (int64_t)m * g.ldc + col) = *(const bf16x8*)(patch + lr * LDB + my_chunk * 16);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    return;
  }
  constexpr int LDF = TN * 4 + 16;
  float bias[8], cs[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { bias[j] = (g.bias && col_ok) ? g.bias[col + j] : 0.f; cs[j] = 0.f; }
#pragma nounroll
  for (int mi = 0; mi < MI; ++mi) {
    sfor<MI>([&](auto I) __attribute__((always_inline)) {
      constexpr int i = decltype(I)::value;
      if (mi != i) return;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg)
          *(f32x4*)(patch + lm * LDF + (ni * 32 + 8 * rg + 4 * lh) * 4) =
              f32x4{acc[i][ni][4 * rg], acc[i][ni][4 * rg + 1], acc[i][ni][4 * rg + 2], acc[i][ni][4 * rg + 3]};
    });
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma nounroll
    for (int p = 0; p < NPASS; ++p) {
      const int lr = p * RPP + my_row;
      const int m = row0 + mi * 32 + lr;
      if (lr >= 32 || m >= g.M || !col_ok) continue;
      const f32x4 p0 = *(const f32x4*)(patch + lr * LDF + my_chunk * 32);
      const f32x4 p1 = *(const f32x4*)(patch + lr * LDF + my_chunk * 32 + 16);
      float v[8] = {p0[0], p0[1], p0[2], p0[3], p1[0], p1[1], p1[2], p1[3]};
      finish8(g, v, m, col, bias, cs, nullptr);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// (a shape whose stages take at most half of the 160 KB is held to the registers that let two workgroups share a CU)
template <int BM, int BN, int WM, int WN, int NST>
__global__ __launch_bounds__(WM * WN * 64, (NST * (BM + BN) * 128 <= 80 * 1024 && WM * WN <= 4) ? 2 : 1)
void gemm_ntd_kernel(GemmDesc g) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32, NMF = MI * NI, NFR = MI + NI;
  constexpr int RPI = NT / 8;                       // tile rows one load instruction of the workgroup fills
  constexpr int AL = BM / RPI, BL = BN / RPI;       // load instructions per thread and k-tile
  constexpr int LPT = AL + BL;
  constexpr int STAGE = (BM + BN) * 128;            // bytes of a stage: rows of 8 chunks of 16 bytes, A rows first
  static_assert(BM % RPI == 0 && BN % RPI == 0 && RPI % 16 == 0, "a load instruction covers whole groups of 16 rows");
  static_assert(NST >= 2 && NST <= 4 && (NST - 1) * LPT <= 60, "vmcnt has 6 bits");
  static_assert(NMF >= NFR && NMF <= 16 && MI >= 1 && NI >= 1, "");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int ntn = (g.N + BN - 1) / BN;
  const int tile = xcd_remap(blockIdx.x, (int)gridDim.x);
  const int m0 = (tile / ntn) * BM, n0 = (tile % ntn) * BN;
  const bf16* __restrict__ A = (const bf16*)g.A;
  const bf16* __restrict__ Bt = (const bf16*)g.B;

  // loader: thread t of load instruction i brings chunk kc of tile row i*RPI + t/8 to LDS slot (row, t%8); rows
  // past M (or N) repeat the last valid row: they only feed accumulators that are never stored
  const int lrow = tid >> 3;
  const int kc = (tid & 7) ^ swz(lrow);
  unsigned off[LPT];
#pragma unroll
  for (int i = 0; i < AL; ++i) off[i] = (unsigned)min(m0 + i * RPI + lrow, g.M - 1) * (unsigned)g.a_rs + kc * 8;
#pragma unroll
  for (int i = 0; i < BL; ++i) off[AL + i] = (unsigned)min(n0 + i * RPI + lrow, g.N - 1) * (unsigned)g.b_cs + kc * 8;
  auto issue1 = [&](auto I, int kt, int st) __attribute__((always_inline)) {
    constexpr int i = decltype(I)::value;
    const bf16* src = (i < AL ? A : Bt) + (size_t)kt * 64;
    unsigned char* dst = smem + st * STAGE + wave * 1024 + (i < AL ? i * RPI * 128 : BM * 128 + (i - AL) * RPI * 128);
    __builtin_amdgcn_global_load_lds(BSR_GLOBAL_PTR(src + off[i]), BSR_LDS_VOID(dst), 16, 0, 0);
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  // fragments: read order A0, B0 .. B(NI-1), A1 .. A(MI-1), so that the first MFMAs of a k-step can start early
  const int lr = lane & 31, lh = lane >> 5, sw = swz(lr);
  int offr[NFR];
  bf16x8 fr[2][NFR];
#pragma unroll
  for (int j = 0; j < NFR; ++j) {
    const bool isA = j == 0 || j > NI;
    const int idx = j == 0 ? 0 : (j <= NI ? j - 1 : j - NI);
    offr[j] = isA ? (wm * TM + idx * 32 + lr) * 128 : BM * 128 + (wn * TN + idx * 32 + lr) * 128;
  }
  auto rd1 = [&](auto SET, auto J, int st, int ks) __attribute__((always_inline)) {
    constexpr int set = decltype(SET)::value, j = decltype(J)::value;
    fr[set][j] = *(const bf16x8*)(smem + st * STAGE + (((ks * 2 + lh) ^ sw) << 4) + offr[j]);
  };
  auto mf1 = [&](auto SET, auto J) __attribute__((always_inline)) {
    constexpr int set = decltype(SET)::value, j = decltype(J)::value, mi = j / NI, ni = j % NI;
    constexpr int ja = mi == 0 ? 0 : NI + mi, jb = 1 + ni;
    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[set][jb], fr[set][ja], acc[mi][ni], 0, 0, 0);
  };
  // one k-step: MFMAs on fragment set SET; the fragments of (stage st, k-step ks) go into the other set
  auto kstep = [&](auto SET, int st, int ks) __attribute__((always_inline)) {
    constexpr int set = decltype(SET)::value;
    sfor<NMF>([&](auto J) __attribute__((always_inline)) {
      constexpr int j = decltype(J)::value;
      mf1(IC<set>{}, J);
      if constexpr (j < NFR) rd1(IC<set ^ 1>{}, J, st, ks);
      BSR_SCHED_FENCE();
    });
  };
  // The last k-step of k-tile kt (fragments in set 1) with the barrier.  VMW >= 0: loads that may stay in flight
  // at the barrier (steady state, k-tile kt + NST is issued behind it); VMW < 0: tail, nothing is issued and the
  // count follows from rem, the number of k-tiles after this one (after the last one barrier and reads are idle).
  auto klast = [&](auto VMW, int kt, int st, int stn, int rem) __attribute__((always_inline)) {
    constexpr int vmw = decltype(VMW)::value;
    constexpr int PRE = NMF >= 16 ? 4 : (NMF >= 8 ? 2 : 1);       // MFMAs in front of the barrier
    constexpr int POST = NMF - PRE;
    constexpr int RPP = (NFR + POST - 1) / POST, LPP = (LPT + POST - 1) / POST;
    sfor<PRE>([&](auto J) __attribute__((always_inline)) { mf1(IC<1>{}, J); BSR_SCHED_FENCE(); });
    wait_lgkmcnt0();
    if constexpr (vmw >= 0) wait_vmcnt<vmw>();
    else if (rem >= 3) wait_vmcnt<2 * LPT>();
    else if (rem == 2) wait_vmcnt<LPT>();
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    BSR_SCHED_FENCE();
    sfor<POST>([&](auto P) __attribute__((always_inline)) {
      constexpr int p = decltype(P)::value;
      mf1(IC<1>{}, IC<PRE + p>{});
      sfor<RPP>([&](auto R) __attribute__((always_inline)) {
        constexpr int r = p * RPP + decltype(R)::value;
        if constexpr (r < NFR) rd1(IC<0>{}, IC<r>{}, stn, 0);
      });
      if constexpr (vmw >= 0)
        sfor<LPP>([&](auto L) __attribute__((always_inline)) {
          constexpr int l = p * LPP + decltype(L)::value;
          if constexpr (l < LPT) issue1(IC<l>{}, kt + NST, st);
        });
      BSR_SCHED_FENCE();
    });
  };

  const int nk = g.K / BK;
  // prologue: every stage filled (k-tiles 0 .. NST-1), k-tile 0 landed
#pragma unroll
  for (int j = 0; j < NST; ++j)
    if (j < nk) sfor<LPT>([&](auto I) __attribute__((always_inline)) { issue1(I, j, j); });
  {
    const int fl = min(nk, NST) - 1;            // k-tiles that may stay in flight
    if (fl >= 3) wait_vmcnt<3 * LPT>(); else if (fl == 2) wait_vmcnt<2 * LPT>(); else if (fl == 1) wait_vmcnt<LPT>(); else wait_vmcnt<0>();
  }
  __builtin_amdgcn_s_barrier();
  sfor<NFR>([&](auto J) __attribute__((always_inline)) { rd1(IC<0>{}, J, 0, 0); });
  int st = 0, kt = 0;
  for (; kt + NST < nk; ++kt) {          // steady state
    const int stn = (st + 1 == NST) ? 0 : st + 1;
    kstep(IC<0>{}, st, 1);
    kstep(IC<1>{}, st, 2);
    kstep(IC<0>{}, st, 3);
    klast(IC<(NST - 2) * LPT>{}, kt, st, stn, 0);
    st = stn;
  }
  for (; kt < nk; ++kt) {                // the last NST k-tiles: nothing left to issue
    const int stn = (st + 1 == NST) ? 0 : st + 1;
    kstep(IC<0>{}, st, 1);
    kstep(IC<1>{}, st, 2);
    kstep(IC<0>{}, st, 3);
    klast(IC<-1>{}, kt, st, stn, nk - 1 - kt);
    st = stn;
  }
  // every wavefront is past the last barrier, i.e. has read its last fragments: the stages are free
  epilogue_t<MI, NI>(g, acc, m0 + wm * TM, n0 + wn * TN, lane, smem + wave * (32 * (TN * 4 + 16)));
}

template <int BM, int BN, int WM, int WN, int NST>
void launch_ntd(const GemmDesc& g, hipStream_t s) {
  static bool attr_set = false;
  constexpr size_t lds_tiles = (size_t)NST * (BM + BN) * 128;
  constexpr size_t lds_patch = (size_t)WM * WN * 32 * ((BN / WN) * 4 + 16);
  static_assert(lds_patch <= lds_tiles, "the epilogue patches live in the stage buffers");
  auto kern = gemm_ntd_kernel<BM, BN, WM, WN, NST>;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_tiles);
    attr_set = true;
  }
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  kern<<<tiles, WM * WN * 64, lds_tiles, s>>>(g);
}
// what the direct-to-LDS kernels take: whole k-tiles, one weight matrix, no folded LayerNorm
bool is_ntd(const GemmDesc& g) { return g.K % BK == 0 && !g.grp_off && !g.ln_colsum; }

// ------------------------------------------------------------------------------------------ TN
// Weight gradient dW[Mo,No] = sum_t X[t,Mo]^T dY[t,No] (Eq. 4): both operands have the contraction
// index t (tokens) as their row index, so an MFMA fragment (8 consecutive t for one column) is
// strided in memory.  The tiles are staged in LDS as they lie in memory - 64 token rows of 16-byte
// chunks, plain 16-byte writes - and the fragments are read with the LDS transpose read
// (ds_read_b64_tr_b16): within every 16 lanes, lane 4e+q passes the address of 4 columns of token
// row e, and lane j receives column j of the four rows, i.e. 4 consecutive tokens of one column.
// A fragment is two such reads (token rows r..r+3 and r+4..r+7).  One half-wave reads 4 rows x 64
// bytes; the 64-byte segments of a row are permuted by segment ^ (row & 3) so that those four land
// in four different bank groups (a row of 128 columns spans all 64 banks exactly once).
// Split-K: workgroup z handles k-tiles [z*kt_per, (z+1)*kt_per) and writes its own fp32 partial;
// a second kernel adds the partials in a fixed order (bit-reproducible, no atomics).
// Bias gradient: the workgroups of the first row of tiles also multiply every dY fragment by an
// all-ones A fragment, which leaves the column sums of dY (db = 1^T dY) in one more accumulator per
// 32 columns; they travel through the same partial / reduce path as dW.
#define BSR_LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))

// four elements of a split-K sum (or, past the matrix, up to four of the column sums): partials added in
// ascending split order
__device__ inline void splitk_reduce_item(const TnReduce& r, int64_t item) {
  const int64_t i = item * 4;
  if (i >= r.n) {
    for (int64_t j = i - r.n; j < min(i - r.n + 4, (int64_t)r.nb); ++j) {
      float s = r.bpartial[j];
      for (int z = 1; z < r.splits; ++z) s += r.bpartial[(int64_t)z * r.nb + j];
      r.bout[j] = s;
    }
    return;
  }
  float4 s = *(const float4*)(r.partial + i);
  for (int z = 1; z < r.splits; ++z) {
    const float4 v = *(const float4*)(r.partial + (int64_t)z * r.n + i);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  *(float4*)(r.out + i) = s;
}
__device__ inline int64_t splitk_reduce_items(const TnReduce& r) { return r.n / 4 + (r.nb + 3) / 4; }
inline int64_t splitk_reduce_items_host(const TnReduce& r) { return r.n / 4 + (r.nb + 3) / 4; }

// Grid rows [0, tn_rows) multiply; rows past them (if any) add up the partials of the previous weight
// gradient (red), a bandwidth-bound job that overlaps with this launch's matrix work.
// The work of workgroup (bx, by) of a gx x gy grid (the kernel below passes its own block index; the fused
// input-gradient + weight-gradient launch passes the coordinates of its extra workgroups).
template <int BM, int BN, int WM, int WN>
__device__ __forceinline__ void tn_body(GemmDesc g, float* partial, float* bpartial, int kt_per, int tn_rows,
                                        const TnReduce& red, int bx, int by, int gx, int gy) {
  constexpr int NT = WM * WN * 64;
  if (by >= tn_rows) {
    const int64_t nthreads = (int64_t)(gy - tn_rows) * gx * NT;
    const int64_t first = ((int64_t)(by - tn_rows) * gx + bx) * NT + threadIdx.x;
    const int64_t items = splitk_reduce_items(red);
    for (int64_t it = first; it < items; it += nthreads) splitk_reduce_item(red, it);
    return;
  }
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int ACPR = BM / 8, BCPR = BN / 8;                  // 16-byte chunks per token row
  constexpr int ACH = BK * ACPR / NT, BCH = BK * BCPR / NT;    // chunks per thread per k-tile
  static_assert(BM % 128 == 0 && BN % 128 == 0, "the segment permutation needs a multiple of 4 segments per row");
  static_assert(ACH >= 1 && BCH >= 1 && (BK * ACPR) % NT == 0 && (BK * BCPR) % NT == 0 && MI >= 1 && NI >= 1, "");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* As = smem;                            // [2][64 token rows][BM columns] bf16
  unsigned char* Bs = smem + 2 * BK * BM * 2;          // [2][64 token rows][BN columns] bf16
  constexpr int ABUF = BK * BM * 2, BBUF = BK * BN * 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int ntn = (g.N + BN - 1) / BN;
  const int ntiles = gx;
  const int tile = xcd_remap(bx, ntiles);
  // an XCD's contiguous range of tiles runs along the side with fewer tiles first, so that it spans that side
  // and its L2 fetches the longer operand's token rows once instead of once per XCD
  const int ntm = (g.M + BM - 1) / BM;
  const bool mfast = ntm < ntn;
  const int m0 = (mfast ? tile % ntm : tile / ntn) * BM, n0 = (mfast ? tile / ntm : tile % ntn) * BN;
  if (g.grp_off) {
    // grouped form: by is the group; the contraction runs over its token rows only
    const int e = by, r0 = g.grp_off[e], r1 = g.grp_off[e + 1];
    g.A = (const bf16*)g.A + (int64_t)r0 * g.a_cs;
    g.B = (const bf16*)g.B + (int64_t)r0 * g.b_rs;
    g.K = r1 - r0;
    g.C = (float*)g.C + (int64_t)e * g.c_gs;
    if (g.bsum) g.bsum += (int64_t)e * g.bsum_gs;
    partial = nullptr;
    bpartial = nullptr;
    kt_per = (g.K + BK - 1) / BK;
  }
  const int nk_all = (g.K + BK - 1) / BK;
  const int kt0 = g.grp_off ? 0 : by * kt_per, kt1 = min(kt0 + kt_per, nk_all);
  const bf16* __restrict__ X = (const bf16*)g.A;     // [K tokens, Mo], row stride a_cs
  const bf16* __restrict__ Y = (const bf16*)g.B;     // [K tokens, No], row stride b_rs

  // chunk c of a tile: token row c / chunks-per-row, chunk position c % chunks-per-row
  int ar[ACH], br[BCH], sa[ACH], sb[BCH];
  const bf16* pa[ACH];
  const bf16* pb[BCH];
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int c = tid + NT * i, r = c / ACPR, q = c % ACPR;
    ar[i] = r;
    pa[i] = X + min(m0 + q * 8, g.M - 8);              // columns past Mo repeat valid ones: never stored
    sa[i] = r * (BM * 2) + ((((q >> 2) ^ (r & 3)) << 2) + (q & 3)) * 16;
  }
#pragma unroll
  for (int i = 0; i < BCH; ++i) {
    const int c = tid + NT * i, r = c / BCPR, q = c % BCPR;
    br[i] = r;
    pb[i] = Y + min(n0 + q * 8, g.N - 8);
    sb[i] = r * (BN * 2) + ((((q >> 2) ^ (r & 3)) << 2) + (q & 3)) * 16;
  }
  u32x4 ra[ACH], rb[BCH];
  auto fetch = [&](int kt) {                           // token rows past K are zero
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
      const int t = kt * BK + ar[i];
      ra[i] = *(const u32x4*)(pa[i] + (int64_t)min(t, g.K - 1) * g.a_cs);
      if (t >= g.K) ra[i] = u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < BCH; ++i) {
      const int t = kt * BK + br[i];
      rb[i] = *(const u32x4*)(pb[i] + (int64_t)min(t, g.K - 1) * g.b_rs);
      if (t >= g.K) rb[i] = u32x4{0u, 0u, 0u, 0u};
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < ACH; ++i) *(u32x4*)(As + buf * ABUF + sa[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < BCH; ++i) *(u32x4*)(Bs + buf * BBUF + sb[i]) = rb[i];
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

  // transpose-read coordinates of this lane: j = lane % 16 inside its block of 16 lanes, the block
  // covers columns cb*16 .. +16 of the 32-column fragment for k-group kg (tokens kg*8 .. +8 of a k-step)
  const int lr = lane & 31, lh = lane >> 5;
  const int j = lane & 15, cb = (lane >> 4) & 1, kg = lh;
  const int rj = j >> 2;                               // token row inside a group of four (= row & 3)
  int oa[MI], ob[NI];                                  // byte offset inside a token row, segment-permuted
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int off = (wm * TM + mi * 32 + cb * 16 + (j & 3) * 4) * 2, q = off >> 4;
    oa[mi] = ((((q >> 2) ^ rj) << 2) + (q & 3)) * 16 + (off & 15);
  }
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    const int off = (wn * TN + ni * 32 + cb * 16 + (j & 3) * 4) * 2, q = off >> 4;
    ob[ni] = ((((q >> 2) ^ rj) << 2) + (q & 3)) * 16 + (off & 15);
  }

  const bool do_bsum = g.bsum && m0 == 0 && wm == 0;     // uniform over the wavefront
  f32x16 accb[NI];
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (bf16)1.0f;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int r = 0; r < 16; ++r) accb[ni][r] = 0.f;

  typedef short s16x4 __attribute__((ext_vector_type(4)));
  union Frag { bf16x8 v; s16x4 h[2]; };
  Frag fa[2][MI], fb[2][NI];
  auto load_frags = [&](int set, const unsigned char* Ab, const unsigned char* Bb, int ks) {
    const int row = ks * 16 + kg * 8 + rj;             // and row + 4: both have (row & 3) == rj
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const unsigned char* a = Ab + row * (BM * 2) + oa[mi];
      fa[set][mi].h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(BSR_LDS_PTR(s16x4, a));
      fa[set][mi].h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(BSR_LDS_PTR(s16x4, a + 4 * BM * 2));
    }
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const unsigned char* bp = Bb + row * (BN * 2) + ob[ni];
      fb[set][ni].h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(BSR_LDS_PTR(s16x4, bp));
      fb[set][ni].h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(BSR_LDS_PTR(s16x4, bp + 4 * BN * 2));
    }
  };
  auto mma = [&](int set) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][mi].v, fb[set][ni].v, acc[mi][ni], 0, 0, 0);
    if (do_bsum) {
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        accb[ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, fb[set][ni].v, accb[ni], 0, 0, 0);
    }
  };

  const int nk = kt1 - kt0;
  if (nk > 0) {
    fetch(kt0);
    stash(0);
    if (nk > 1) fetch(kt0 + 1);
    __syncthreads();
    load_frags(0, As, Bs, 0);
    for (int kt = 0; kt < nk; ++kt) {
      const int buf = kt & 1;
      const unsigned char* Ab = As + buf * ABUF;
      const unsigned char* Bb = Bs + buf * BBUF;
      load_frags(1, Ab, Bb, 1);
      mma(0);
      load_frags(0, Ab, Bb, 2);
      mma(1);
      load_frags(1, Ab, Bb, 3);
      if (kt + 1 < nk) stash(buf ^ 1);
      if (kt + 2 < nk) fetch(kt0 + kt + 2);
      mma(0);
      __syncthreads();
      if (kt + 1 < nk) load_frags(0, As + (buf ^ 1) * ABUF, Bs + (buf ^ 1) * BBUF, 0);
      mma(1);
    }
    __syncthreads();
  }
  GemmDesc o = g;
  if (partial) {                                   // split-K: plain fp32 partial, no epilogue terms
    o.C = partial + (int64_t)by * g.M * g.N;
    o.ldc = g.N; o.bias = nullptr; o.act = ACT_NONE; o.res = nullptr; o.remap_np = 0; o.out_f32 = true;
  }
  float* patch = (float*)smem + wave * (32 * (TN + 4));
  epilogue<MI, NI>(o, acc, m0 + wm * TM, n0 + wn * TN, lane, patch);
  if (do_bsum && lh == 0) {                        // every row of accb holds the column sums
    float* dst = bpartial ? bpartial + (int64_t)by * g.N : g.bsum;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      const int col = n0 + wn * TN + ni * 32 + lr;
      if (col < g.N) dst[col] = accb[ni][0];
    }
  }
}

template <int BM, int BN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void gemm_tn_kernel(GemmDesc g, float* partial, float* bpartial, int kt_per,
                                                              int tn_rows, TnReduce red) {
  tn_body<BM, BN, WM, WN>(g, partial, bpartial, kt_per, tn_rows, red, blockIdx.x, blockIdx.y, gridDim.x, gridDim.y);
}

// the same reduction as a launch of its own
__global__ void splitk_reduce_kernel(TnReduce r) {
  const int64_t it = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (it < splitk_reduce_items(r)) splitk_reduce_item(r, it);
}

void launch_reduce(const TnReduce& r, hipStream_t s) {
  splitk_reduce_kernel<<<(unsigned)((splitk_reduce_items_host(r) + 255) / 256), 256, 0, s>>>(r);
}

bool is_tn(const GemmDesc& g) {
  return !g.in_f32 && g.out_f32 && g.a_rs == 1 && g.b_cs == 1 && g.M % 8 == 0 && g.N % 8 == 0 && g.M >= 8 &&
         g.N >= 8 && g.a_cs % 8 == 0 && g.b_rs % 8 == 0 && g.ldc % 8 == 0 && g.K > 0 && !g.res && g.act == ACT_NONE &&
         g.remap_np == 0 && (((uintptr_t)g.A | (uintptr_t)g.B | (uintptr_t)g.C) & 15) == 0;
}

constexpr int TN_BM = 128, TN_BN = 128, TN_WM = 4, TN_WN = 2, TN_THREADS = TN_WM * TN_WN * 64;
constexpr size_t TN_LDS_TILES = (size_t)2 * (TN_BM + TN_BN) * BK * sizeof(bf16);
constexpr size_t TN_LDS_PATCH = (size_t)TN_WM * TN_WN * 32 * (TN_BN / TN_WN + 4) * sizeof(float);   // epilogue patches
constexpr size_t TN_LDS = TN_LDS_TILES > TN_LDS_PATCH ? TN_LDS_TILES : TN_LDS_PATCH;

// Everything a weight-gradient launch needs beyond the kernel itself: the split, the workspace half, the
// reduction of the previous launch that rides along (taken from the chain) and the one this launch leaves.
struct TnPlan {
  GemmDesc g;
  float *partial = nullptr, *bpartial = nullptr;
  int kt_per = 0, tn_rows = 1, grid_x = 0, grid_y = 1;
  TnReduce prev;                 // added up by the extra grid rows of this launch
  TnReduce mine;                 // what this launch leaves to add up (mine.splits == 0: nothing)
};

TnPlan plan_tn(const GemmDesc& g, float* ws, size_t ws_floats, TnChain* chain) {
  TnPlan p;
  p.g = g;
  const int tiles = ((g.M + TN_BM - 1) / TN_BM) * ((g.N + TN_BN - 1) / TN_BN);
  p.grid_x = tiles;
  if (chain) {       // this launch takes one half of the workspace, the pending reduction reads the other
    ws_floats /= 2;
    ws_floats &= ~(size_t)3;
    if (ws) ws += (size_t)chain->slot * ws_floats;
  }
  const int nk = (g.K + BK - 1) / BK;
  // enough splits for about 1.5 workgroups per CU, each with at least 4 k-tiles (measured with the launch
  // sharing the chip with an input-gradient product: at 35 - 49 k-tiles of tokens, 384 workgroups beat 512
  // and 320 by 1 % of the step); two per CU once the token dimension is long (at 138 - 194 k-tiles 512 beat
  // 384 by 3 % and 256 by 12 %)
  int splits = 1;
  const size_t mn = (size_t)g.M * g.N;
  const size_t per_split = mn + (g.bsum ? (size_t)g.N : 0);   // partial dW, then partial column sums
  if (ws && mn % 4 == 0) {
    const int target = nk >= 96 ? 512 : 384;
    splits = std::max(1, std::min({target / tiles, nk / 4, (int)(ws_floats / per_split), 16}));
  }
  p.kt_per = (nk + splits - 1) / splits;
  splits = (nk + p.kt_per - 1) / p.kt_per;
  p.tn_rows = splits;
  // the previous weight gradient's reduction rides along: about four items per thread
  int red_rows = 0;
  if (chain && chain->pending.splits > 0) {
    p.prev = chain->pending;
    chain->pending = TnReduce();
    const int64_t per_row = (int64_t)tiles * TN_THREADS * 4;
    red_rows = (int)std::min<int64_t>(8, std::max<int64_t>(1, (splitk_reduce_items_host(p.prev) + per_row - 1) / per_row));
  }
  p.grid_y = splits + red_rows;
  if (splits > 1) {
    p.partial = ws;
    p.bpartial = g.bsum ? ws + (size_t)splits * mn : nullptr;
    p.mine.partial = ws; p.mine.n = (int64_t)mn; p.mine.splits = splits; p.mine.out = (float*)g.C;
    p.mine.bpartial = p.bpartial; p.mine.nb = g.bsum ? g.N : 0; p.mine.bout = g.bsum;
    if (chain) {
      chain->pending = p.mine;
      chain->slot ^= 1;
    }
  }
  return p;
}

void launch_tn(const GemmDesc& g, float* ws, size_t ws_floats, hipStream_t s, TnChain* chain) {
  static bool attr_set = false;
  auto kern = gemm_tn_kernel<TN_BM, TN_BN, TN_WM, TN_WN>;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)TN_LDS);
    attr_set = true;
  }
  if (g.grp_off) {   // one grid row per group, no split: tiles x groups already fills the machine
    gemm_tn_flush(chain, s);
    const int tiles = ((g.M + TN_BM - 1) / TN_BM) * ((g.N + TN_BN - 1) / TN_BN);
    kern<<<dim3(tiles, g.groups), TN_THREADS, TN_LDS, s>>>(g, nullptr, nullptr, 0, g.groups, TnReduce());
    return;
  }
  const TnPlan p = plan_tn(g, ws, ws_floats, chain);
  kern<<<dim3(p.grid_x, p.grid_y), TN_THREADS, TN_LDS, s>>>(p.g, p.partial, p.bpartial, p.kt_per, p.tn_rows, p.prev);
  if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s);
}

// One launch for an input gradient (NT, tile BM x BN) and the weight gradient of the same layer.
template <int BM, int BN, int WM, int WN, int PF>
void launch_nt_fused(const GemmDesc& g, const TnPlan& p, hipStream_t s) {
  static_assert(WM * WN * 64 == TN_THREADS, "");
  static bool attr_set = false;
  constexpr size_t lds_tiles = (size_t)2 * (BM + BN) * BK * sizeof(bf16);
  constexpr size_t lds_patch = (size_t)WM * WN * 32 * (BN / WN + 4) * sizeof(float);
  constexpr size_t lds_nt = lds_tiles > lds_patch ? lds_tiles : lds_patch;
  constexpr size_t lds = lds_nt > TN_LDS ? lds_nt : TN_LDS;
  auto kern = gemm_nt_kernel<BM, BN, WM, WN, false, PF, true>;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_set = true;
  }
  TnArgs t;
  t.g = p.g; t.partial = p.partial; t.bpartial = p.bpartial; t.kt_per = p.kt_per; t.tn_rows = p.tn_rows;
  t.red = p.prev; t.gx = p.grid_x; t.gy = p.grid_y;
  t.nt_tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  kern<<<t.nt_tiles + p.grid_x * p.grid_y, TN_THREADS, lds, s>>>(g, t);
}

bool is_nt(const GemmDesc& g) {
  return !g.in_f32 && g.a_cs == 1 && g.b_rs == 1 && g.K % 8 == 0 && g.a_rs % 8 == 0 && g.b_cs % 8 == 0 &&
         g.N % 8 == 0 && g.ldc % 8 == 0 && (((uintptr_t)g.A | (uintptr_t)g.B | (uintptr_t)g.C) & 15) == 0 &&
         (((uintptr_t)g.aux | (uintptr_t)g.res) & 15) == 0 && g.M > 0 && g.N > 0 && g.K > 0;
}

}  // namespace

// two halves (a launch writes one while the previous launch's partials are added up from the other), each
// with room for 8 partial copies of the largest weight gradient of a block ([D,3D] or [D,F]) and of its
// bias gradient (16 for the smaller matrices, which split further)
size_t gemm_splitk_ws_floats(int dim, int mlp_hidden) {
  return 2 * ((size_t)8 * std::max((size_t)3 * dim * dim, (size_t)dim * mlp_hidden) +
              (size_t)16 * std::max(3 * dim, mlp_hidden));
}

bool gemm_mfma_supported(const GemmDesc& g) { return is_nt(g) || is_tn(g); }

// Tile choice.  What bounds these kernels on a CU is operand delivery, not the matrix cores: LDS
// takes writes at about 64 bytes per clock, so a k-tile of a BM x BN block tile costs 2 (BM + BN)
// clocks of LDS writes (plus the fragment reads) against BM * BN / 32 clocks of MFMA work.  Only
// 256 x 256 tiles keep that ratio well below one, but at M = 2144 .. 6304 rows they leave most CUs
// without a tile, so each launch takes the shape that a two-parameter model predicts to be fastest:
//   time = ceil(tiles / 256 CUs) * (fixed + per_ktile * K / 64)
// with (fixed, per_ktile) in microseconds fitted per tile shape to the durations of the step's own
// GEMMs (N and K in {768, 2304, 3072}, epilogues included) with every shape forced in turn.  The
// model's picks cost 2.5 % more than the per-launch best of those runs (its residual is 3 - 5 us per
// launch), which is why a context can instead time every shape on its own launches and keep the
// fastest (bsr_autotune).  The large tiles pay a long fixed part because their single workgroup per
// CU cannot hide its prologue and epilogue.  Every shape accumulates an output element over k in the
// same order, so the choice never changes a result.
struct NtShape { int id, bm, bn; float fixed_us, per_ktile_us; };
static const NtShape kNtShapes[] = {
    {256128, 256, 128, 9.77f, 0.714f},  {128128, 128, 128, 2.78f, 0.577f}, {192128, 192, 128, 4.17f, 0.734f},
    {160256, 160, 256, 11.85f, 0.975f}, {256256, 256, 256, 17.70f, 1.300f},
    {128064, 128, 64, 1.39f, 0.351f},   {96128, 96, 128, 2.38f, 0.507f},
    // offered to the measured choice only (no fitted constants: fixed_us < 0 keeps them out of the model)
    {64128, 64, 128, -1.f, 0.f},        {128256, 128, 256, -1.f, 0.f},     {192256, 192, 256, -1.f, 0.f},
    {256064, 256, 64, -1.f, 0.f},       {96256, 96, 256, -1.f, 0.f},
    // with deeper register prefetch (id = PF * 1000000 + shape)
    {3128064, 128, 64, -1.f, 0.f},      {3064128, 64, 128, -1.f, 0.f},     {2192128, 192, 128, -1.f, 0.f},
    {2256128, 256, 128, -1.f, 0.f},     {2128128, 128, 128, -1.f, 0.f},
    // operands straight into LDS (id = 7000000 + shape; K a multiple of 64, one weight matrix, no folded LayerNorm:
    // a launch outside that takes the model's shape instead)
    {7256256, 256, 256, -1.f, 0.f},     {7320256, 320, 256, -1.f, 0.f},    {7192256, 192, 256, -1.f, 0.f},
    {7256192, 256, 192, -1.f, 0.f},     {7256128, 256, 128, -1.f, 0.f},    {7128256, 128, 256, -1.f, 0.f},
    {7192128, 192, 128, -1.f, 0.f},     {7128128, 128, 128, -1.f, 0.f},
};
// stages of the direct-to-LDS shapes (0: not one of them)
static int ntd_stages(int id) {
  switch (id) {
    case 7256256: case 7320256: case 7192256: case 7256192: case 7192128: case 7128128: return 2;
    case 7256128: case 7128256: return 3;
    default: return 0;
  }
}

int gemm_nt_model_tile(int M, int N, int K) {
  int pick = 0;
  float best = 0.f;
  for (const NtShape& t : kNtShapes) {
    if (t.fixed_us < 0.f) continue;
    const int64_t tiles = (int64_t)((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn);
    const float us = (float)((tiles + 255) / 256) * (t.fixed_us + t.per_ktile_us * (float)((K + BK - 1) / BK));
    if (!pick || us < best) { pick = t.id; best = us; }
  }
  return pick;
}
size_t gemm_nt_tile_lds_bytes(int id) {
  const int bm = id % 1000000 / 1000, bn = id % 1000, nst = ntd_stages(id);
  return (size_t)(nst ? nst : 2) * (bm + bn) * BK * sizeof(bf16);
}
int gemm_nt_tile_count() { return (int)(sizeof(kNtShapes) / sizeof(kNtShapes[0])); }
int gemm_nt_tile_id(int i) { return kNtShapes[i].id; }
bool gemm_nt_tile_is_free(const GemmDesc& g) { return is_nt(g) && !g.grp_off; }

void gemm_tn_flush(TnChain* chain, hipStream_t s) {
  if (!chain || chain->pending.splits <= 0) return;
  launch_reduce(chain->pending, s);
  chain->pending = TnReduce();
}

void gemm_mfma(const GemmDesc& g, float* splitk_ws, size_t splitk_ws_floats, hipStream_t s, int tile, TnChain* chain) {
  if (is_tn(g)) {
    launch_tn(g, splitk_ws, splitk_ws_floats, s, chain);
    return;
  }
  // groups are a few hundred rows and each ends in a partial row tile: 128-row tiles, 64-row ones where a group
  // averages under four of those (the last tile of a 268-row group is 9 % full at 128 rows, 19 % at 64)
  int pick = g.grp_off ? (g.M < 512 * g.groups ? 64128 : 128128) : tile;
  if (!pick || (ntd_stages(pick) && !is_ntd(g))) pick = gemm_nt_model_tile(g.M, g.N, g.K);
  switch (pick) {
    case 7256256: launch_ntd<256, 256, 2, 4, 2>(g, s); break;
    case 7320256: launch_ntd<320, 256, 2, 4, 2>(g, s); break;
    case 7192256: launch_ntd<192, 256, 2, 4, 2>(g, s); break;
    case 7256192: launch_ntd<256, 192, 4, 2, 2>(g, s); break;
    case 7256128: launch_ntd<256, 128, 4, 2, 3>(g, s); break;
    case 7128256: launch_ntd<128, 256, 2, 4, 3>(g, s); break;
    case 7192128: launch_ntd<192, 128, 2, 2, 2>(g, s); break;
    case 7128128: launch_ntd<128, 128, 2, 2, 2>(g, s); break;
    case 256256: launch_nt<256, 256, 2, 4>(g, s); break;
    case 256128: launch_nt<256, 128, 4, 4>(g, s); break;
    case 192128: launch_nt<192, 128, 2, 4>(g, s); break;
    case 160256: launch_nt<160, 256, 1, 8>(g, s); break;
    case 128064: launch_nt<128, 64, 4, 2>(g, s); break;
    case 96128: launch_nt<96, 128, 1, 4>(g, s); break;
    case 64128: launch_nt<64, 128, 2, 4>(g, s); break;
    case 128256: launch_nt<128, 256, 2, 4>(g, s); break;
    case 192256: launch_nt<192, 256, 2, 4>(g, s); break;
    case 256064: launch_nt<256, 64, 4, 2>(g, s); break;
    case 96256: launch_nt<96, 256, 1, 8>(g, s); break;
    case 3128064: launch_nt<128, 64, 4, 2, 3>(g, s); break;
    case 3064128: launch_nt<64, 128, 2, 4, 3>(g, s); break;
    case 2192128: launch_nt<192, 128, 2, 4, 2>(g, s); break;
    case 2256128: launch_nt<256, 128, 4, 4, 2>(g, s); break;
    case 2128128: launch_nt<128, 128, 4, 2, 2>(g, s); break;
    default: launch_nt<128, 128, 4, 2>(g, s); break;
  }
}

// The input gradient (NT) and the weight gradient (TN) of one layer.  When the tile shape chosen for the
// NT part runs with 8 waves they go out as one launch (the weight-gradient workgroups fill the machine
// behind the input-gradient tiles), otherwise as two.
void gemm_mfma_pair(const GemmDesc& nt, const GemmDesc& tn, float* splitk_ws, size_t splitk_ws_floats, hipStream_t s,
                    int tile, TnChain* chain) {
  int pick = tile;
  if (!pick) pick = gemm_nt_model_tile(nt.M, nt.N, nt.K);
  const bool can = is_nt(nt) && is_tn(tn) && !nt.grp_off && !tn.grp_off && nt.K % BK == 0;
  if (can) {
    switch (pick) {
      case 128064: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<128, 64, 4, 2, 1>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      case 64128: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<64, 128, 2, 4, 1>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      case 192128: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<192, 128, 2, 4, 1>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      case 128128: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<128, 128, 4, 2, 1>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      case 3128064: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<128, 64, 4, 2, 3>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      case 3064128: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<64, 128, 2, 4, 3>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      case 2192128: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<192, 128, 2, 4, 2>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      case 2128128: { const TnPlan p = plan_tn(tn, splitk_ws, splitk_ws_floats, chain); launch_nt_fused<128, 128, 4, 2, 2>(nt, p, s); if (!chain && p.mine.splits > 0) launch_reduce(p.mine, s); return; }
      default: break;
    }
  }
  gemm_mfma(nt, splitk_ws, splitk_ws_floats, s, pick, chain);
  gemm_mfma(tn, splitk_ws, splitk_ws_floats, s, 0, chain);
}

}  // namespace bsr
