// High-precision lane for the CLS rows of the bf16 path (gfx950).
//
// The slide loss reaches the encoder through one row per tile: the CLS row of the last block (Method: the
// feature matrix is what the aggregator sees).  The aggregator's gate gradients depend on the features only
// through differences between tiles, which are several times smaller than the features themselves, so the
// rounding of that one row is what decides their accuracy: with every CLS row carried in bf16 like the other
// 196 rows of its tile the features are 1e-2 off and the gate gradients 4e-2; with the CLS row's residual
// stream, LayerNorm output, MLP activation and branch sums kept in fp32 they are 1e-3 and 6e-3, while the
// other rows stay on the bf16 kernels.  The lane is n rows out of n * T, so it costs next to nothing.
//
// Per block the lane repeats the row-wise work of the CLS rows (projection + residual, LayerNorm, MLP +
// residual) on an fp32 copy of the CLS stream.  The attention output of the CLS query comes from the main
// path (bf16); after each residual sum the lane writes its value, rounded once, over the CLS row of the main
// path's stream, so the main path's queries, keys, values and saved activations of that row follow the lane.
//   lane_gemm_k : C[n,N] = A[n,K] W[N,K]^T + bias, then + residual or GELU.  W are the bf16 weights of the
//                 step.  An fp32 A is split into two bf16 terms (a = hi + lo up to 2^-17 |a|) and multiplied
//                 in two MFMAs, so the product keeps fp32-grade operands on the bf16 matrix cores; a bf16 A
//                 (rows of the attention output) is exact as it is.  fp32 accumulation, fp32 result.
//   lane_ln_k   : LayerNorm of fp32 rows, fp32 result.
#include "slide_internal.h"

namespace sl {

namespace {

constexpr int LBM = 64, LBN = 64, LBK = 32, LLD = LBK + 8;   // tile, K step, LDS row stride (bf16 elements)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

struct LaneGemm {
  const void* A; long long lda;     // fp32 or bf16 [n][K]
  const bf16* W; long long ldw;     // [N][K]
  long long n; int N, K;
  const float* bias;                // [N]
  const float* resid; long long ldr;  // MODE 0
  float* out; long long ldc;
  bf16* copy; long long ldcopy;     // optional bf16 copy of the result rows (MODE 0), may be null
};

__device__ __forceinline__ unsigned bf16_bits(float v) { return (unsigned)__builtin_bit_cast(unsigned short, (bf16)v); }

// MODE 0: out = resid + A W^T + bias (and the optional rounded copy); MODE 1: out = gelu(A W^T + bias)
template <int MODE, bool A_BF16>
__global__ void __launch_bounds__(256) lane_gemm_k(LaneGemm g) {
  __shared__ __attribute__((aligned(16))) bf16 Ah[2][LBM * LLD];
  __shared__ __attribute__((aligned(16))) bf16 Al[2][A_BF16 ? 8 : LBM * LLD];
  __shared__ __attribute__((aligned(16))) bf16 Ws[2][LBN * LLD];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const long long m0 = (long long)blockIdx.x * LBM;
  const int n0 = blockIdx.y * LBN;
  const int nk = g.K / LBK;
  // loaders: W and a bf16 A: 64 rows x 4 chunks of 8 elements, one chunk per thread; an fp32 A: 64 rows x 8 chunks of
  // 4 elements, two per thread.  Rows past the end are redirected to the last row (valid memory, never stored).
  const int wr = tid >> 2, wc = (tid & 3) * 8;
  const bf16* wp = g.W + (long long)(n0 + wr) * g.ldw + wc;
  long long ar16 = m0 + wr; if (ar16 > g.n - 1) ar16 = g.n - 1;
  const bf16* ap16 = (const bf16*)g.A + ar16 * g.lda + wc;
  const int fr = tid >> 3, fc = (tid & 7) * 4;
  long long ar0 = m0 + fr, ar1 = m0 + fr + 32;
  if (ar0 > g.n - 1) ar0 = g.n - 1;
  if (ar1 > g.n - 1) ar1 = g.n - 1;
  const float* ap0 = (const float*)g.A + ar0 * g.lda + fc;
  const float* ap1 = (const float*)g.A + ar1 * g.lda + fc;

  u32x4 rw, ra16;
  float4 ra0, ra1;
  auto fetch = [&](int k0) {
    rw = *reinterpret_cast<const u32x4*>(wp + k0);
    if (A_BF16) ra16 = *reinterpret_cast<const u32x4*>(ap16 + k0);
    else { ra0 = *reinterpret_cast<const float4*>(ap0 + k0); ra1 = *reinterpret_cast<const float4*>(ap1 + k0); }
  };
  auto split_store = [&](int st, int row, float4 v) {
    float x[4] = {v.x, v.y, v.z, v.w};
    unsigned h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      bf16 hi = (bf16)x[i];
      h[i] = (unsigned)__builtin_bit_cast(unsigned short, hi);
      l[i] = bf16_bits(x[i] - (float)hi);
    }
    u32x2 ph = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)}, pl = {l[0] | (l[1] << 16), l[2] | (l[3] << 16)};
    *reinterpret_cast<u32x2*>(&Ah[st][row * LLD + fc]) = ph;
    *reinterpret_cast<u32x2*>(&Al[st][row * LLD + fc]) = pl;
  };
  auto stash = [&](int st) {
    *reinterpret_cast<u32x4*>(&Ws[st][wr * LLD + wc]) = rw;
    if (A_BF16) *reinterpret_cast<u32x4*>(&Ah[st][wr * LLD + wc]) = ra16;
    else { split_store(st, fr, ra0); split_store(st, fr + 32, ra1); }
  };

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  fetch(0);
  stash(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) fetch((kt + 1) * LBK);
#pragma unroll
    for (int ks = 0; ks < LBK / 16; ++ks) {
      bf16x8 fb = *reinterpret_cast<const bf16x8*>(&Ws[cur][(wn * 32 + frow) * LLD + fk + ks * 16]);
      bf16x8 fa = *reinterpret_cast<const bf16x8*>(&Ah[cur][(wm * 32 + frow) * LLD + fk + ks * 16]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc, 0, 0, 0);
      if (!A_BF16) {
        bf16x8 fl = *reinterpret_cast<const bf16x8*>(&Al[cur][(wm * 32 + frow) * LLD + fk + ks * 16]);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fl, fb, acc, 0, 0, 0);
      }
    }
    if (kt + 1 < nk) stash(cur ^ 1);   // the other stage: its readers finished before the last barrier
    __syncthreads();
  }
  // accumulator element r of lane l: row (r / 4) * 8 + (l / 32) * 4 + r % 4, column l % 32 of the wave's block
  const int col = n0 + wn * 32 + (lane & 31);
  const float b = g.bias[col];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    long long m = m0 + wm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
    if (m < g.n) {
      float v = acc[r] + b;
      if (MODE == 0) {
        v += g.resid[m * g.ldr + col];
        if (g.copy) g.copy[m * g.ldcopy + col] = (bf16)v;
      } else {
        v = gelu_f(v);
      }
      g.out[m * g.ldc + col] = v;
    }
  }
}

// LayerNorm of fp32 rows (D <= 1024): one wavefront per row, statistics in two passes over registers.
__global__ void __launch_bounds__(256) lane_ln_k(const float* __restrict__ x, long long xs, const float* __restrict__ gam,
                                                 const float* __restrict__ bet, float* __restrict__ out, long long os,
                                                 long long rows, int D, float eps) {
  const int lane = threadIdx.x & 63;
  const long long r = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  float v[16];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int d = lane + 64 * i;
    v[i] = d < D ? x[r * xs + d] : 0.f;
    s += v[i];
  }
  const float mu = wave_sum(s) / (float)D;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int d = lane + 64 * i;
    float c = d < D ? v[i] - mu : 0.f;
    q += c * c;
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)D + eps);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    int d = lane + 64 * i;
    if (d < D) out[r * os + d] = (v[i] - mu) * rstd * gam[d] + bet[d];
  }
}

// the CLS stream before the first block: cls + pos[0], the same row for every tile
__global__ void __launch_bounds__(256) lane_init_k(const float* __restrict__ cls, const float* __restrict__ pos,
                                                   float* __restrict__ xc, long long total, int D) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < total) { int d = (int)(i % D); xc[i] = cls[d] + pos[d]; }
}

}  // namespace

bool cls_lane_ok(int D, int F) { return D % 64 == 0 && F % 64 == 0 && D <= 1024; }

hipError_t launch_lane_init(const float* cls, const float* pos, float* xc, long long n, int D, hipStream_t s) {
  long long total = n * D;
  hipLaunchKernelGGL(lane_init_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, cls, pos, xc, total, D);
  return hipGetLastError();
}

hipError_t launch_lane_ln(const float* x, long long xs, const float* gam, const float* bet, float* out, long long os,
                          long long rows, int D, float eps, hipStream_t s) {
  hipLaunchKernelGGL(lane_ln_k, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x, xs, gam, bet, out, os, rows, D, eps);
  return hipGetLastError();
}

hipError_t launch_lane_gemm(bool gelu, bool a_bf16, const void* A, long long lda, const void* W, long long ldw, long long n,
                            int N, int K, const float* bias, const float* resid, long long ldr, float* out, long long ldc,
                            void* copy, long long ldcopy, hipStream_t s) {
  if (N % LBN || K % LBK || n <= 0) return hipErrorInvalidValue;
  LaneGemm g{A, lda, (const bf16*)W, ldw, n, N, K, bias, resid, ldr, out, ldc, (bf16*)copy, ldcopy};
  dim3 grid((unsigned)((n + LBM - 1) / LBM), (unsigned)(N / LBN));
  if (gelu) {
    if (a_bf16) return hipErrorInvalidValue;
    hipLaunchKernelGGL((lane_gemm_k<1, false>), grid, dim3(256), 0, s, g);
  } else if (a_bf16) {
    hipLaunchKernelGGL((lane_gemm_k<0, true>), grid, dim3(256), 0, s, g);
  } else {
    hipLaunchKernelGGL((lane_gemm_k<0, false>), grid, dim3(256), 0, s, g);
  }
  return hipGetLastError();
}

}  // namespace sl
