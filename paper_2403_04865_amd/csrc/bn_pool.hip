// Row-wise kernels of the ResNet tile encoder (gfx950): batch normalisation with the statistics of all rows of the
// call, its backward, max and average pooling.  Tensors are bf16 [rows][C], C a power of two between 64 and 2048;
// every thread moves 16-byte pieces (8 channels).  All of them are bound by memory traffic.
//
// Reductions over the rows (statistics, gain / shift gradients) are two-stage and deterministic: a fixed number of
// workgroups each sums a contiguous range of rows in fp32 (8 channels per thread, rows strided over the threads, then
// one pass through LDS), and one wavefront per channel adds the workgroups' partial sums in double, in a fixed order.
#include "resnet_internal.h"

namespace sl {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void unpack8(const u32x4& t, float (&v)[8]) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    v[2 * w] = __uint_as_float(t[w] << 16);
    v[2 * w + 1] = __uint_as_float(t[w] & 0xffff0000u);
  }
}
__device__ __forceinline__ u32x4 ld16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ void st8(bf16* p, const float (&v)[8]) {
  bf16x8 t;
#pragma unroll
  for (int e = 0; e < 8; ++e) t[e] = (bf16)v[e];
  *reinterpret_cast<bf16x8*>(p) = t;
}

// 8 consecutive floats of a 16-byte aligned per-channel array
__device__ __forceinline__ void ld8f(const float* p, float (&v)[8]) {
  const float4 lo = *reinterpret_cast<const float4*>(p), hi = *reinterpret_cast<const float4*>(p + 4);
  v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w;
  v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
}

constexpr int BN_MAX_BLOCKS = 4096;

// Two per-channel sums over the rows of one workgroup's range.  F(row pointer offset, channel base, out a[8], out b[8])
// yields the two summands of 8 channels of one row.
template <typename F>
__device__ __forceinline__ void two_sums(long long M, int C, float* part, F f) {
  __shared__ float red[2][256 * 8];
  const int tcols = C >> 3, rpp = 256 / tcols;          // threads per row, rows per pass
  const int tc = threadIdx.x % tcols, tr = threadIdx.x / tcols;
  const long long per = (M + gridDim.x - 1) / gridDim.x;
  const long long lo = (long long)blockIdx.x * per, hi = lo + per < M ? lo + per : M;
  float s[8], q[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) s[e] = q[e] = 0.f;
  for (long long m = lo + tr; m < hi; m += rpp) {
    float a[8], b[8];
    f(m * C + tc * 8, tc * 8, a, b);
#pragma unroll
    for (int e = 0; e < 8; ++e) { s[e] += a[e]; q[e] += b[e]; }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { red[0][threadIdx.x * 8 + e] = s[e]; red[1][threadIdx.x * 8 + e] = q[e]; }
  __syncthreads();
  // thread (tr, tc) -> flat index (tr * tcols + tc) * 8 + e = tr * C + channel
  for (int ch = threadIdx.x; ch < C; ch += 256) {
    float a = 0.f, b = 0.f;
    for (int r = 0; r < rpp; ++r) { a += red[0][r * C + ch]; b += red[1][r * C + ch]; }
    part[((long long)blockIdx.x * 2 + 0) * C + ch] = a;
    part[((long long)blockIdx.x * 2 + 1) * C + ch] = b;
  }
}

// The workgroups' partial sums of one channel, added in double by one wavefront: lane l takes partials l, l + 64, ...
// in order, then the lanes are combined in a fixed butterfly (the same bits on every run).
__device__ __forceinline__ void channel_sums(const float* __restrict__ part, int blocks, int C, int ch, double& s, double& q) {
  const int lane = threadIdx.x & 63;
  s = 0.0; q = 0.0;
  for (int b = lane; b < blocks; b += 64) {
    s += (double)part[((long long)b * 2) * C + ch];
    q += (double)part[((long long)b * 2 + 1) * C + ch];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { s += __shfl_xor(s, o, 64); q += __shfl_xor(q, o, 64); }
}

__global__ void __launch_bounds__(256) bn_stats_final_k(const float* __restrict__ part, int blocks, long long M, int C,
                                                         const float* __restrict__ gamma, const float* __restrict__ beta,
                                                         float eps, float* __restrict__ stats) {
  const int ch = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (ch >= C) return;
  double s, q;
  channel_sums(part, blocks, C, ch, s, q);
  if (threadIdx.x & 63) return;
  const double mean = s / (double)M;
  double var = q / (double)M - mean * mean;
  if (var < 0.0) var = 0.0;
  const double rstd = 1.0 / sqrt(var + (double)eps);
  const double a = (double)gamma[ch] * rstd;
  stats[ch] = (float)mean;
  stats[C + ch] = (float)rstd;
  stats[2 * C + ch] = (float)a;
  stats[3 * C + ch] = (float)((double)beta[ch] - mean * a);
}

// tile_part[tiles][2 C] -> part[workgroups][2 C]: every workgroup adds a contiguous range of tiles, column by column
__global__ void __launch_bounds__(256) bn_tiles_part_k(const float* __restrict__ tp, int tiles, int C2, float* __restrict__ part) {
  const int per = (tiles + gridDim.x - 1) / gridDim.x;
  const int lo = blockIdx.x * per, hi = lo + per < tiles ? lo + per : tiles;
  for (int col = threadIdx.x; col < C2; col += 256) {
    float a = 0.f;
    for (int t = lo; t < hi; ++t) a += tp[(long long)t * C2 + col];
    part[(long long)blockIdx.x * C2 + col] = a;
  }
}

// A thread of the two streaming kernels below takes SPT pieces 256 pieces apart: C / 8 divides 256, so they are the
// same 8 channels of different rows and the per-channel coefficients are fetched once for all of them (fetched per
// piece they are four to ten 16-byte loads against two or three of data); every load instruction of a wavefront still
// covers 1 KB of consecutive addresses, and a thread has SPT rows in flight.
// (measured on the ResNet18 step: forward 0.56 -> 0.45 ms per launch with 2, backward 0.64 -> 0.55 ms with 4)
constexpr int SPT_APPLY = 2, SPT_BWD = 4;

template <int SPT>
__global__ void __launch_bounds__(256) bn_apply_k(const bf16* __restrict__ x, long long chunks, int C,
                                                   const float* __restrict__ stats, const bf16* __restrict__ resid,
                                                   const float* __restrict__ rstats, int relu, bf16* __restrict__ y,
                                                   unsigned char* __restrict__ bits) {
  const long long i0 = (long long)blockIdx.x * (256 * SPT) + threadIdx.x;
  const int c0 = (int)(threadIdx.x & ((C >> 3) - 1)) * 8;   // 256 * SPT * blockIdx.x is a multiple of C / 8
  u32x4 xv[SPT], rv[SPT];
#pragma unroll
  for (int j = 0; j < SPT; ++j) {
    const long long i = i0 + j * 256;
    if (i < chunks) {
      xv[j] = ld16(x + i * 8);
      if (resid) rv[j] = ld16(resid + i * 8);
    }
  }
  float a[8], b[8], ra[8], rb[8];
  ld8f(stats + 2 * C + c0, a);
  ld8f(stats + 3 * C + c0, b);
  if (resid) {   // (without a projection the values are not used; no branch per element around the loads)
    const float* rs = rstats ? rstats : stats;
    ld8f(rs + 2 * C + c0, ra);
    ld8f(rs + 3 * C + c0, rb);
  }
#pragma unroll
  for (int j = 0; j < SPT; ++j) {
    const long long i = i0 + j * 256;
    if (i >= chunks) break;
    float v[8];
    unpack8(xv[j], v);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = a[e] * v[e] + b[e];
    if (resid) {
      float r[8];
      unpack8(rv[j], r);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += rstats ? ra[e] * r[e] + rb[e] : r[e];
    }
    if (relu) {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
    }
    bf16x8 t;
    unsigned m = 0;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      t[e] = (bf16)v[e];
      m |= ((float)t[e] > 0.f ? 1u : 0u) << e;   // of the value as stored
    }
    __builtin_nontemporal_store(t, reinterpret_cast<bf16x8*>(y + i * 8));   // streamed: the reader is a later kernel
    if (bits) bits[i] = (unsigned char)m;
  }
}

__global__ void __launch_bounds__(256) bn_bwd_part_k(const bf16* __restrict__ dy, const unsigned char* __restrict__ mask,
                                                      const bf16* __restrict__ x, long long M, int C,
                                                      const float* __restrict__ stats, float* __restrict__ part) {
  two_sums(M, C, part, [&](long long off, int c0, float (&a)[8], float (&b)[8]) {
    float xv[8];
    unpack8(ld16(dy + off), a);
    unpack8(ld16(x + off), xv);
    if (mask) {
      const unsigned m = mask[off >> 3];
#pragma unroll
      for (int e = 0; e < 8; ++e) a[e] = (m >> e) & 1u ? a[e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) b[e] = a[e] * ((xv[e] - stats[c0 + e]) * stats[C + c0 + e]);
  });
}

// coef[0][c] = dbeta / M, coef[1][c] = dgamma / M; parameter gradients written or added to
__global__ void __launch_bounds__(256) bn_bwd_final_k(const float* __restrict__ part, int blocks, long long M, int C,
                                                       float* __restrict__ coef, float* __restrict__ dgamma,
                                                       float* __restrict__ dbeta, int accumulate) {
  const int ch = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (ch >= C) return;
  double s, q;
  channel_sums(part, blocks, C, ch, s, q);
  if (threadIdx.x & 63) return;
  coef[ch] = (float)(s / (double)M);
  coef[C + ch] = (float)(q / (double)M);
  dbeta[ch] = accumulate ? dbeta[ch] + (float)s : (float)s;
  dgamma[ch] = accumulate ? dgamma[ch] + (float)q : (float)q;
}

template <int SPT>
__global__ void __launch_bounds__(256) bn_bwd_apply_k(const bf16* __restrict__ dy, const unsigned char* __restrict__ mask,
                                                       const bf16* __restrict__ x, long long chunks, int C,
                                                       const float* __restrict__ stats, const float* __restrict__ coef,
                                                       bf16* __restrict__ dx) {
  const long long i0 = (long long)blockIdx.x * (256 * SPT) + threadIdx.x;
  const int c0 = (int)(threadIdx.x & ((C >> 3) - 1)) * 8;
  u32x4 dv[SPT], xv[SPT];
  unsigned mv[SPT];
#pragma unroll
  for (int j = 0; j < SPT; ++j) {
    const long long i = i0 + j * 256;
    if (i < chunks) {
      dv[j] = ld16(dy + i * 8);
      xv[j] = ld16(x + i * 8);
      mv[j] = mask ? mask[i] : 0xffu;
    }
  }
  float mean[8], rstd[8], ga[8], k0[8], k1[8];
  ld8f(stats + c0, mean);
  ld8f(stats + C + c0, rstd);
  ld8f(stats + 2 * C + c0, ga);
  ld8f(coef + c0, k0);
  ld8f(coef + C + c0, k1);
#pragma unroll
  for (int j = 0; j < SPT; ++j) {
    const long long i = i0 + j * 256;
    if (i >= chunks) break;
    float d[8], xf[8];
    unpack8(dv[j], d);
    unpack8(xv[j], xf);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      d[e] = (mv[j] >> e) & 1u ? d[e] : 0.f;
      const float xh = (xf[e] - mean[e]) * rstd[e];
      d[e] = ga[e] * (d[e] - k0[e] - xh * k1[e]);
    }
    st8(dx + i * 8, d);
  }
}

// ---- pooling ---------------------------------------------------------------------------------------------------
// forward: the maximum and, per output element, which of the nine taps it came from (the first in (kh, kw) order of
// equal maxima), one byte each
__global__ void __launch_bounds__(256) maxpool_fwd_k(const bf16* __restrict__ x, bf16* __restrict__ y,
                                                      unsigned char* __restrict__ arg, long long chunks, int H, int W, int C) {
  const int tcols = C >> 3, OH = H / 2, OW = W / 2;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= chunks) return;
  const int tc = (int)(i % tcols);
  long long pos = i / tcols;
  const int ox = (int)(pos % OW); pos /= OW;
  const int oy = (int)(pos % OH);
  const long long n = pos / OH;
  float best[8];
  unsigned at[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { best[e] = -INFINITY; at[e] = 0; }
  for (int kh = 0; kh < 3; ++kh)
    for (int kw = 0; kw < 3; ++kw) {
      const int iy = 2 * oy + kh - 1, ix = 2 * ox + kw - 1;
      if ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) {
        float v[8];
        unpack8(ld16(x + (((n * H + iy) * W + ix) * C + tc * 8)), v);
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (v[e] > best[e]) { best[e] = v[e]; at[e] = (unsigned)(kh * 3 + kw); }
      }
    }
  st8(y + i * 8, best);
  uint2 packed;
  packed.x = at[0] | (at[1] << 8) | (at[2] << 16) | (at[3] << 24);
  packed.y = at[4] | (at[5] << 8) | (at[6] << 16) | (at[7] << 24);
  *reinterpret_cast<uint2*>(arg + i * 8) = packed;
}

// backward: a thread owns a 2 x 2 block of input positions (2 qy + {0, 1}, 2 qx + {0, 1}) of 8 channels.  The windows
// that cover it are (qy, qx), (qy, qx + 1), (qy + 1, qx), (qy + 1, qx + 1): each is fetched once (gradient and
// winning taps) and handed to the positions it covers; a position adds its windows in (oy, ox) order.  No lane
// diverges on the parity of its position, and every store instruction of a wavefront writes whole rows of channels.
__global__ void __launch_bounds__(256) maxpool_bwd_k(const unsigned char* __restrict__ arg, const bf16* __restrict__ dy,
                                                      bf16* __restrict__ dx, long long quads, int H, int W, int C) {
  const int tcols = C >> 3, OH = H / 2, OW = W / 2;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= quads) return;
  const int tc = (int)(i % tcols);
  long long pos = i / tcols;
  const int qx = (int)(pos % OW); pos /= OW;
  const int qy = (int)(pos % OH);
  const long long n = pos / OH;
  const bool hx = qx + 1 < OW, hy = qy + 1 < OH;
  // window (qy + a, qx + b): gradient d[a][b], taps t[a][b]; absent windows contribute nothing (tap 255 matches none)
  float d[2][2][8];
  uint2 t[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const bool have = (a == 0 || hy) && (b == 0 || hx);
      const long long o = (((n * OH + qy + (have ? a : 0)) * OW + qx + (have ? b : 0)) * C + tc * 8);
      const uint2 tt = *reinterpret_cast<const uint2*>(arg + o);
      unpack8(ld16(dy + o), d[a][b]);
      t[a][b] = have ? tt : uint2{0xffffffffu, 0xffffffffu};
    }
  auto take = [&](float (&g)[8], int a, int b, unsigned tap) __attribute__((always_inline)) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const unsigned at = ((e < 4 ? t[a][b].x : t[a][b].y) >> (8 * (e & 3))) & 0xffu;
      g[e] += at == tap ? d[a][b][e] : 0.f;
    }
  };
  // tap of window (oy, ox) at input (iy, ix): (iy - 2 oy + 1) * 3 + (ix - 2 ox + 1)
  float g00[8], g01[8], g10[8], g11[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) g00[e] = g01[e] = g10[e] = g11[e] = 0.f;
  take(g00, 0, 0, 4);
  take(g01, 0, 0, 5); take(g01, 0, 1, 3);
  take(g10, 0, 0, 7); take(g10, 1, 0, 1);
  take(g11, 0, 0, 8); take(g11, 0, 1, 6); take(g11, 1, 0, 2); take(g11, 1, 1, 0);
  bf16* o0 = dx + (((n * H + 2 * qy) * W + 2 * qx) * C + tc * 8);
  bf16* o1 = o0 + (long long)W * C;
  st8(o0, g00);
  st8(o0 + C, g01);
  st8(o1, g10);
  st8(o1 + C, g11);
}

// one workgroup per tile; thread t sums channels t, t + 256, ... over the positions (neighbouring threads read
// neighbouring channels)
__global__ void __launch_bounds__(256) avgpool_fwd_k(const bf16* __restrict__ x, float* __restrict__ feats, int HW, int C) {
  const long long n = blockIdx.x;
  for (int ch = threadIdx.x; ch < C; ch += 256) {
    float a = 0.f;
    for (int p = 0; p < HW; ++p) a += (float)x[(n * HW + p) * C + ch];
    feats[n * C + ch] = a / (float)HW;
  }
}

__global__ void __launch_bounds__(256) avgpool_bwd_k(const float* __restrict__ df, bf16* __restrict__ dx, long long chunks,
                                                      int HW, int C) {
  const int tcols = C >> 3;
  const float inv = 1.0f / (float)HW;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < chunks; i += (long long)gridDim.x * 256) {
    const int c0 = (int)(i % tcols) * 8;
    const long long n = i / tcols / HW;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = df[n * C + c0 + e] * inv;
    st8(dx + i * 8, v);
  }
}

bool chan_ok(int C) { return C >= 64 && C <= 2048 && (C & (C - 1)) == 0; }
bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }
// one 16-byte piece per thread where the grid allows it (measured: 4.1 -> 4.5 TB/s against 16384 workgroups that loop)
unsigned stream_grid(long long chunks) {
  long long b = (chunks + 255) / 256;
  return (unsigned)(b < 1 ? 1 : (b > 4194304 ? 4194304 : b));
}

}  // namespace

int bn_blocks(long long M, int C) {
  (void)C;
  long long b = M / 128;
  return (int)(b < 1 ? 1 : (b > BN_MAX_BLOCKS ? BN_MAX_BLOCKS : b));
}

hipError_t launch_bn_stats_tiles(const float* tile_part, int tiles, long long M, int C, const float* gamma, const float* beta,
                                 float eps, float* part, float* stats, hipStream_t s) {
  if (!tile_part || tiles <= 0 || !gamma || !beta || !part || !stats || M <= 0 || !chan_ok(C)) return hipErrorInvalidValue;
  int blocks = (tiles + 15) / 16;
  if (blocks > BN_MAX_BLOCKS) blocks = BN_MAX_BLOCKS;
  hipLaunchKernelGGL(bn_tiles_part_k, dim3(blocks), dim3(256), 0, s, tile_part, tiles, 2 * C, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bn_stats_final_k, dim3((C + 3) / 4), dim3(256), 0, s, part, blocks, M, C, gamma, beta, eps, stats);
  return hipGetLastError();
}

hipError_t launch_bn_apply(const bf16* x, long long M, int C, const float* stats, const bf16* resid, const float* rstats,
                           int relu, bf16* y, unsigned char* bits, hipStream_t s) {
  if (!x || !stats || !y || M <= 0 || !chan_ok(C) || !al16(x) || !al16(y) || !al16(resid) || !al16(stats) || !al16(rstats))
    return hipErrorInvalidValue;
  const long long chunks = M * (C >> 3);
  constexpr int SPT = SPT_APPLY;
  if ((chunks + 256 * SPT - 1) / (256 * SPT) >= (1LL << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bn_apply_k<SPT>, dim3((unsigned)((chunks + 256 * SPT - 1) / (256 * SPT))), dim3(256), 0, s, x, chunks, C, stats,
                     resid, rstats, relu, y, bits);
  return hipGetLastError();
}

hipError_t launch_bn_bwd(const bf16* dy, const unsigned char* mask, const bf16* x, long long M, int C, const float* stats,
                         float* part, float* coef, float* dgamma, float* dbeta, int accumulate, bf16* dx, hipStream_t s) {
  if (!dy || !x || !stats || !part || !coef || !dgamma || !dbeta || !dx || M <= 0 || !chan_ok(C) || !al16(dy) ||
      !al16(x) || !al16(dx) || !al16(stats) || !al16(coef))
    return hipErrorInvalidValue;
  const int blocks = bn_blocks(M, C);
  hipLaunchKernelGGL(bn_bwd_part_k, dim3(blocks), dim3(256), 0, s, dy, mask, x, M, C, stats, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bn_bwd_final_k, dim3((C + 3) / 4), dim3(256), 0, s, part, blocks, M, C, coef, dgamma, dbeta, accumulate);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long long chunks = M * (C >> 3);
  constexpr int SPT = SPT_BWD;
  if ((chunks + 256 * SPT - 1) / (256 * SPT) >= (1LL << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(bn_bwd_apply_k<SPT>, dim3((unsigned)((chunks + 256 * SPT - 1) / (256 * SPT))), dim3(256), 0, s, dy, mask, x,
                     chunks, C, stats, coef, dx);
  return hipGetLastError();
}

hipError_t launch_maxpool_fwd(const bf16* x, bf16* y, unsigned char* arg, long long n, int H, int W, int C, hipStream_t s) {
  if (!x || !y || !arg || ((uintptr_t)arg & 7) || n <= 0 || H <= 0 || W <= 0 || H % 2 || W % 2 || !chan_ok(C) || !al16(x) || !al16(y)) return hipErrorInvalidValue;
  const long long chunks = n * (H / 2) * (W / 2) * (C >> 3);
  if ((chunks + 255) / 256 >= (1LL << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(maxpool_fwd_k, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, s, x, y, arg, chunks, H, W, C);
  return hipGetLastError();
}

hipError_t launch_maxpool_bwd(const unsigned char* arg, const bf16* dy, bf16* dx, long long n, int H, int W, int C,
                              hipStream_t s) {
  if (!arg || !dy || !dx || n <= 0 || H <= 0 || W <= 0 || H % 2 || W % 2 || !chan_ok(C) || ((uintptr_t)arg & 7) || !al16(dy) ||
      !al16(dx))
    return hipErrorInvalidValue;
  const long long quads = n * (H / 2) * (W / 2) * (C >> 3);
  if ((quads + 255) / 256 >= (1LL << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(maxpool_bwd_k, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, s, arg, dy, dx, quads, H, W, C);
  return hipGetLastError();
}

hipError_t launch_avgpool_fwd(const bf16* x, float* feats, long long n, int HW, int C, hipStream_t s) {
  if (!x || !feats || n <= 0 || n >= (1LL << 31) || HW <= 0 || !chan_ok(C)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(avgpool_fwd_k, dim3((unsigned)n), dim3(256), 0, s, x, feats, HW, C);
  return hipGetLastError();
}

hipError_t launch_avgpool_bwd(const float* dfeats, bf16* dx, long long n, int HW, int C, hipStream_t s) {
  if (!dfeats || !dx || n <= 0 || HW <= 0 || !chan_ok(C) || !al16(dx)) return hipErrorInvalidValue;
  const long long chunks = n * HW * (C >> 3);
  hipLaunchKernelGGL(avgpool_bwd_k, dim3(stream_grid(chunks)), dim3(256), 0, s, dfeats, dx, chunks, HW, C);
  return hipGetLastError();
}

}  // namespace sl
