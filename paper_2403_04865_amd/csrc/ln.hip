// LayerNorm forward / backward, statistics in fp32.  No per-row statistics are stored: the backward takes the two
// row reductions again from the saved layer input.  Three generations of kernels, picked by the launchers at the
// end of the file: ln_*_row16_k (bf16 path, D = 384 / 768: 16 or 32 lanes per row, 16-byte accesses, several rows
// per wavefront; the ones the large workloads run), ln_*_fast_k (paired elements, any D up to 1024) and ln_*_k (one
// wavefront per row, any element types; the fp32 path).  The backward can also write the normalised rows
// x_hat * gamma + beta next to dx (the operand of the weight gradient behind the LayerNorm) where the forward's own
// copy was not kept.
#include "slide_internal.h"

namespace sl {

constexpr int LN_MAXV = 16;  // D <= 64 * LN_MAXV

template <typename RS, typename T>
__global__ void __launch_bounds__(256) ln_fwd_k(const RS* __restrict__ x, long long xs, const float* __restrict__ gam,
                                                const float* __restrict__ bet, T* __restrict__ out, long long os,
                                                long long rows, int D, float eps) {
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  long long r = (long long)blockIdx.x * 4 + w;
  if (r >= rows) return;
  const RS* xr = x + r * xs;
  float v[LN_MAXV];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXV; ++i) {
    int c = lane + 64 * i;
    v[i] = c < D ? to_f(xr[c]) : 0.f;
    sum += v[i];
  }
  float mean = wave_sum(sum) / D;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < LN_MAXV; ++i) {
    int c = lane + 64 * i;
    float d = c < D ? v[i] - mean : 0.f;
    sq += d * d;
  }
  float rstd = 1.0f / sqrtf(wave_sum(sq) / D + eps);
  T* o = out + r * os;
#pragma unroll
  for (int i = 0; i < LN_MAXV; ++i) {
    int c = lane + 64 * i;
    if (c < D) o[c] = from_f<T>((v[i] - mean) * rstd * gam[c] + bet[c]);
  }
}


// ---- fast path: D == 128 * NP, each lane owns NP column pairs {2*(lane + 64*i), +1} -----------
template <typename E> struct Pair;
template <> struct Pair<float> { typedef float2 type; };
template <> struct Pair<bf16> { typedef unsigned int type; };

__device__ __forceinline__ float2 ld2(const float* p) { return *reinterpret_cast<const float2*>(p); }
__device__ __forceinline__ float2 ld2(const bf16* p) {
  unsigned int u = *reinterpret_cast<const unsigned int*>(p);
  return make_float2(__uint_as_float(u << 16), __uint_as_float(u & 0xffff0000u));
}
__device__ __forceinline__ void st2(float* p, float a, float b) { *reinterpret_cast<float2*>(p) = make_float2(a, b); }
__device__ __forceinline__ void st2(bf16* p, float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v = {(bf16)a, (bf16)b};
  *reinterpret_cast<bf16x2*>(p) = v;
}

template <typename RS, typename T, int NP>
__global__ void __launch_bounds__(256) ln_fwd_fast_k(const RS* __restrict__ x, long long xs,
                                                     const float* __restrict__ gam, const float* __restrict__ bet,
                                                     T* __restrict__ out, long long os, long long rows, float eps) {
  constexpr int D = 128 * NP;
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  long long r = (long long)blockIdx.x * 4 + w;
  if (r >= rows) return;
  const RS* xr = x + r * xs;
  float2 v[NP];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    v[i] = ld2(xr + 2 * (lane + 64 * i));
    sum += v[i].x + v[i].y;
  }
  float mean = wave_sum(sum) * (1.0f / D);
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    v[i].x -= mean;
    v[i].y -= mean;
    sq += v[i].x * v[i].x + v[i].y * v[i].y;
  }
  float rstd = 1.0f / sqrtf(wave_sum(sq) * (1.0f / D) + eps);
  T* o = out + r * os;
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    int c = 2 * (lane + 64 * i);
    float2 g = ld2(gam + c), b = ld2(bet + c);
    st2(o + c, v[i].x * rstd * g.x + b.x, v[i].y * rstd * g.y + b.y);
  }
}

template <typename RS, typename TDY, typename T, bool SAME, int NP>
__global__ void __launch_bounds__(256) ln_bwd_fast_k(const RS* __restrict__ x, long long xs,
                                                     const TDY* __restrict__ dy, long long dys,
                                                     const float* __restrict__ gam, const RS* __restrict__ dres,
                                                     RS* __restrict__ dxo, T* __restrict__ dxo_t, long long os,
                                                     long long rows, float eps, float* __restrict__ part) {
  constexpr int D = 128 * NP;
  __shared__ float red[4 * 2 * D];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float2 dg[NP], db[NP], g[NP];
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    dg[i] = make_float2(0.f, 0.f);
    db[i] = make_float2(0.f, 0.f);
    g[i] = ld2(gam + 2 * (lane + 64 * i));
  }
  for (long long r = (long long)blockIdx.x * 4 + w; r < rows; r += (long long)gridDim.x * 4) {
    const RS* xr = x + r * xs;
    const TDY* dyr = dy + r * dys;
    float2 v[NP], d[NP], rs_[NP];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      int c = 2 * (lane + 64 * i);
      v[i] = ld2(xr + c);
      d[i] = ld2(dyr + c);
      if (dres) rs_[i] = ld2(dres + r * os + c);
      sum += v[i].x + v[i].y;
    }
    float mean = wave_sum(sum) * (1.0f / D);
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      v[i].x -= mean;
      v[i].y -= mean;
      sq += v[i].x * v[i].x + v[i].y * v[i].y;
    }
    float rstd = 1.0f / sqrtf(wave_sum(sq) * (1.0f / D) + eps);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      v[i].x *= rstd;
      v[i].y *= rstd;
      dg[i].x += d[i].x * v[i].x;
      dg[i].y += d[i].y * v[i].y;
      db[i].x += d[i].x;
      db[i].y += d[i].y;
      d[i].x *= g[i].x;
      d[i].y *= g[i].y;
      s1 += d[i].x + d[i].y;
      s2 += d[i].x * v[i].x + d[i].y * v[i].y;
    }
    s1 = wave_sum(s1) * (1.0f / D);
    s2 = wave_sum(s2) * (1.0f / D);
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      int c = 2 * (lane + 64 * i);
      float a = rstd * (d[i].x - s1 - v[i].x * s2);
      float b = rstd * (d[i].y - s1 - v[i].y * s2);
      if (dres) { a += rs_[i].x; b += rs_[i].y; }
      st2(dxo + r * os + c, a, b);
      if (!SAME) st2(dxo_t + r * os + c, a, b);
    }
  }
#pragma unroll
  for (int i = 0; i < NP; ++i) {
    int c = 2 * (lane + 64 * i);
    red[(w * 2 + 0) * D + c] = dg[i].x;
    red[(w * 2 + 0) * D + c + 1] = dg[i].y;
    red[(w * 2 + 1) * D + c] = db[i].x;
    red[(w * 2 + 1) * D + c + 1] = db[i].y;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * D; i += 256) {
    float a = (red[0 * 2 * D + i] + red[1 * 2 * D + i]) + (red[2 * 2 * D + i] + red[3 * 2 * D + i]);
    part[(size_t)blockIdx.x * 2 * D + i] = a;
  }
}

template <typename RS, typename T>
bool ln_fwd_fast(const void* x, long long xs, const float* gam, const float* bet, void* out, long long os,
                 long long rows, int D, float eps, hipStream_t s) {
  if ((xs & 1) || (os & 1)) return false;
  dim3 grid((unsigned)((rows + 3) / 4));
#define GO(NP) hipLaunchKernelGGL((ln_fwd_fast_k<RS, T, NP>), grid, dim3(256), 0, s, (const RS*)x, xs, gam, bet, (T*)out, os, rows, eps)
  if (D == 384) { GO(3); return true; }
  if (D == 768) { GO(6); return true; }
  if (D == 128) { GO(1); return true; }
#undef GO
  return false;
}

template <typename RS, typename TDY, typename T, bool SAME>
bool ln_bwd_fast(dim3 grid, const void* x, long long xs, const void* dy, long long dys, const float* gam,
                 const void* dres, void* dxo, void* dxo_t, long long os, long long rows, int D, float eps, float* part,
                 hipStream_t s) {
  if ((xs & 1) || (os & 1) || (dys & 1)) return false;
#define GO(NP) hipLaunchKernelGGL((ln_bwd_fast_k<RS, TDY, T, SAME, NP>), grid, dim3(256), 0, s, (const RS*)x, xs, (const TDY*)dy, dys, gam, (const RS*)dres, (RS*)dxo, (T*)dxo_t, os, rows, eps, part)
  if (D == 384) { GO(3); return true; }
  if (D == 768) { GO(6); return true; }
  if (D == 128) { GO(1); return true; }
#undef GO
  return false;
}


// ---- bf16 rows, 16 lanes per row: D == 128 * NP, every lane owns NP chunks of 8 columns (16-byte accesses), a
// wavefront works on four rows at a time.  LayerNorm is pure streaming: what matters is how many bytes a
// wavefront keeps in flight, and one row of 2 * D bytes per wavefront (4-byte accesses) left HBM mostly idle.
typedef unsigned int lnu4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void ln_ld8(const bf16* p, float (&v)[8]) {
  lnu4 t = __builtin_nontemporal_load(reinterpret_cast<const lnu4*>(p));   // streamed: read once
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    v[2 * w] = __uint_as_float(t[w] << 16);
    v[2 * w + 1] = __uint_as_float(t[w] & 0xffff0000u);
  }
}
__device__ __forceinline__ void ln_unpack8(const lnu4& t, float (&v)[8]) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    v[2 * w] = __uint_as_float(t[w] << 16);
    v[2 * w + 1] = __uint_as_float(t[w] & 0xffff0000u);
  }
}
__device__ __forceinline__ void ln_st8(bf16* p, const float (&v)[8]) {
  typedef float lnf2 __attribute__((ext_vector_type(2)));
  typedef __bf16 lnb2 __attribute__((ext_vector_type(2)));
  lnu4 r;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    lnf2 f = {v[2 * w], v[2 * w + 1]};
    lnb2 h = __builtin_convertvector(f, lnb2);
    r[w] = __builtin_bit_cast(unsigned, h);
  }
  __builtin_nontemporal_store(r, reinterpret_cast<lnu4*>(p));   // streamed: the reader is a later kernel
}
template <int LPR>
__device__ __forceinline__ float sum_row(float v) {   // over the LPR lanes of a row group
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float sum16(float v) {   // over the 16 lanes of a row group
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// A group of 16 lanes takes ln_fwd_rpg(NP) rows (4 rows apart): their loads are all in flight together and gain and
// shift are fetched once for them (two rows at 384 columns: 0.40 -> 0.37 ms per launch, four no better; at 768
// columns the gain and shift alone are 96 registers, one row).
constexpr int ln_fwd_rpg(int np) { return np <= 3 ? 2 : 1; }
template <int NP>
__global__ void __launch_bounds__(256) ln_fwd_row16_k(const bf16* __restrict__ x, long long xs,
                                                      const float* __restrict__ gam, const float* __restrict__ bet,
                                                      bf16* __restrict__ out, long long os, long long rows, float eps) {
  constexpr int D = 128 * NP, RPG = ln_fwd_rpg(NP);
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6, l16 = lane & 15, grp = lane >> 4;
  const long long r0 = ((long long)blockIdx.x * 4 + w) * (4 * RPG) + grp;
  lnu4 raw[RPG][NP];
#pragma unroll
  for (int j = 0; j < RPG; ++j) {
    const long long r = r0 + 4 * j;
    const bf16* xr = x + (r < rows ? r : rows - 1) * xs;
#pragma unroll
    for (int k = 0; k < NP; ++k) raw[j][k] = __builtin_nontemporal_load(reinterpret_cast<const lnu4*>(xr + (l16 + 16 * k) * 8));
  }
  float gg[NP][8], bb[NP][8];
#pragma unroll
  for (int k = 0; k < NP; ++k) {
    int c = (l16 + 16 * k) * 8;
    float4 g0 = *reinterpret_cast<const float4*>(gam + c), g1 = *reinterpret_cast<const float4*>(gam + c + 4);
    float4 b0 = *reinterpret_cast<const float4*>(bet + c), b1 = *reinterpret_cast<const float4*>(bet + c + 4);
    gg[k][0] = g0.x; gg[k][1] = g0.y; gg[k][2] = g0.z; gg[k][3] = g0.w; gg[k][4] = g1.x; gg[k][5] = g1.y; gg[k][6] = g1.z; gg[k][7] = g1.w;
    bb[k][0] = b0.x; bb[k][1] = b0.y; bb[k][2] = b0.z; bb[k][3] = b0.w; bb[k][4] = b1.x; bb[k][5] = b1.y; bb[k][6] = b1.z; bb[k][7] = b1.w;
  }
#pragma unroll
  for (int j = 0; j < RPG; ++j) {
    const long long r = r0 + 4 * j;
    float v[NP][8];
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
      ln_unpack8(raw[j][k], v[k]);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += v[k][e];
    }
    float mean = sum16(sum) * (1.0f / D);
    float sq = 0.f;
#pragma unroll
    for (int k = 0; k < NP; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[k][e] -= mean;
        sq += v[k][e] * v[k][e];
      }
    float rstd = 1.0f / sqrtf(sum16(sq) * (1.0f / D) + eps);
    if (r < rows) {
      bf16* o = out + r * os;
#pragma unroll
      for (int k = 0; k < NP; ++k) {
        float y[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = v[k][e] * rstd * gg[k][e] + bb[k][e];
        ln_st8(o + (l16 + 16 * k) * 8, y);
      }
    }
  }
}

// dx = (dres ? dres : 0) + rstd * (dxh - mean(dxh) - xh * mean(dxh * xh)), dxh = dy * gamma;
// dgamma / dbeta partials of the workgroup -> part[block][0][D], part[block][1][D]
// LPR lanes per row (16 or 32), NP chunks of 8 columns per lane: D = 8 * LPR * NP.  (768 columns on 16 lanes would
// need 240 registers for the per-lane arrays and leave one wavefront per SIMD: 35 % of the HBM rate instead of 70 %.)
template <int NP, int LPR>
__global__ void __launch_bounds__(256) ln_bwd_row16_k(const bf16* __restrict__ x, long long xs,
                                                      const bf16* __restrict__ dy, long long dys,
                                                      const float* __restrict__ gam, const bf16* __restrict__ dres,
                                                      bf16* __restrict__ dxo, long long os, long long rows, float eps,
                                                      float* __restrict__ part, const float* __restrict__ bet,
                                                      bf16* __restrict__ uo, long long us, int dres_period) {
  // dres_period != 0: dres has a term only for rows r with r % dres_period == 0 (the other rows of it are not read)
  // uo != nullptr: the normalised rows xh * gamma + beta (the forward output, which the weight gradient of the
  // following linear map needs and the forward did not keep) are written on the way, [rows][us]
  constexpr int D = 8 * LPR * NP, RPW = 64 / LPR;   // rows per wavefront
  __shared__ float red[4 * 2 * D];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6, l16 = lane & (LPR - 1), grp = lane / LPR;
  float dg[NP][8], db[NP][8], g[NP][8];
#pragma unroll
  for (int k = 0; k < NP; ++k) {
    int c = (l16 + LPR * k) * 8;
    float4 g0 = *reinterpret_cast<const float4*>(gam + c), g1 = *reinterpret_cast<const float4*>(gam + c + 4);
    g[k][0] = g0.x; g[k][1] = g0.y; g[k][2] = g0.z; g[k][3] = g0.w; g[k][4] = g1.x; g[k][5] = g1.y; g[k][6] = g1.z; g[k][7] = g1.w;
#pragma unroll
    for (int e = 0; e < 8; ++e) { dg[k][e] = 0.f; db[k][e] = 0.f; }
  }
  long long nsets = (rows + RPW - 1) / RPW;   // sets of RPW rows; a wavefront takes every (gridDim * 4)-th set
  // the rows of the wavefront's next set are requested before the current set is worked on
  lnu4 nx[NP], nd[NP];
  auto fetch = [&](long long set) __attribute__((always_inline)) {
    long long r = set * RPW + grp;
    long long rc = r < rows ? r : rows - 1;
    const bf16* xr = x + rc * xs;
    const bf16* dyr = dy + rc * dys;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
      int c = (l16 + LPR * k) * 8;
      nx[k] = __builtin_nontemporal_load(reinterpret_cast<const lnu4*>(xr + c));
      nd[k] = __builtin_nontemporal_load(reinterpret_cast<const lnu4*>(dyr + c));
    }
  };
  const long long set0 = (long long)blockIdx.x * 4 + w, sstep = (long long)gridDim.x * 4;
  if (set0 < nsets) fetch(set0);
  for (long long set = set0; set < nsets; set += sstep) {
    long long r = set * RPW + grp;
    bool ok = r < rows;
    float okf = ok ? 1.f : 0.f;
    float v[NP][8], d[NP][8];
    float sum = 0.f;
#pragma unroll
    for (int k = 0; k < NP; ++k) {
      ln_unpack8(nx[k], v[k]);
      ln_unpack8(nd[k], d[k]);
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += v[k][e];
    }
    if (set + sstep < nsets) fetch(set + sstep);
    float mean = sum_row<LPR>(sum) * (1.0f / D);
    float sq = 0.f;
#pragma unroll
    for (int k = 0; k < NP; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[k][e] -= mean;
        sq += v[k][e] * v[k][e];
      }
    float rstd = 1.0f / sqrtf(sum_row<LPR>(sq) * (1.0f / D) + eps);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int k = 0; k < NP; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[k][e] *= rstd;
        float dd = d[k][e] * okf;     // rows past the end contribute nothing
        dg[k][e] += dd * v[k][e];
        db[k][e] += dd;
        d[k][e] *= g[k][e];
        s1 += d[k][e];
        s2 += d[k][e] * v[k][e];
      }
    s1 = sum_row<LPR>(s1) * (1.0f / D);
    s2 = sum_row<LPR>(s2) * (1.0f / D);
    if (uo && ok) {
#pragma unroll
      for (int k = 0; k < NP; ++k) {
        int c = (l16 + LPR * k) * 8;
        float4 b0 = *reinterpret_cast<const float4*>(bet + c), b1 = *reinterpret_cast<const float4*>(bet + c + 4);
        float bb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w}, o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = v[k][e] * g[k][e] + bb[e];
        ln_st8(uo + r * us + c, o);
      }
    }
    if (ok) {
#pragma unroll
      for (int k = 0; k < NP; ++k) {
        int c = (l16 + LPR * k) * 8;
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = rstd * (d[k][e] - s1 - v[k][e] * s2);
        if (dres && (dres_period == 0 || (unsigned)r % (unsigned)dres_period == 0)) {
          float t[8];
          ln_ld8(dres + r * os + c, t);
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] += t[e];
        }
        ln_st8(dxo + r * os + c, o);
      }
    }
  }
  // the row groups of a wavefront, then the four wavefronts
#pragma unroll
  for (int k = 0; k < NP; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
      for (int o = LPR; o < 64; o <<= 1) {
        dg[k][e] += __shfl_xor(dg[k][e], o, 64);
        db[k][e] += __shfl_xor(db[k][e], o, 64);
      }
    }
  if (grp == 0) {
#pragma unroll
    for (int k = 0; k < NP; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        int c = (l16 + LPR * k) * 8 + e;
        red[(w * 2 + 0) * D + c] = dg[k][e];
        red[(w * 2 + 1) * D + c] = db[k][e];
      }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * D; i += 256) {
    float a = (red[0 * 2 * D + i] + red[1 * 2 * D + i]) + (red[2 * 2 * D + i] + red[3 * 2 * D + i]);
    part[(size_t)blockIdx.x * 2 * D + i] = a;
  }
}

static bool ln_row16_ok(const void* a, const void* b, const void* c, long long s1, long long s2, long long s3, int D) {
  auto al = [](const void* p) { return ((uintptr_t)p & 15) == 0; };
  return sizeof(rs_bf16path_t) == 2 && (D == 384 || D == 768) && al(a) && al(b) && al(c) && s1 % 8 == 0 && s2 % 8 == 0 &&
         s3 % 8 == 0;
}

hipError_t launch_ln_fwd(int dt, const void* x, long long x_stride, const float* gam, const float* bet, void* out,
                         long long out_stride, long long rows, int D, float eps, bool out_f32, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (dt == DT_BF16 && !out_f32 && ln_row16_ok(x, out, gam, x_stride, out_stride, 0, D) && ((uintptr_t)bet & 15) == 0) {
    const int rpw = 16 * ln_fwd_rpg(D / 128);   // rows per workgroup
    dim3 g16((unsigned)((rows + rpw - 1) / rpw));
    if (D == 384) hipLaunchKernelGGL(ln_fwd_row16_k<3>, g16, dim3(256), 0, s, (const bf16*)x, x_stride, gam, bet, (bf16*)out, out_stride, rows, eps);
    else hipLaunchKernelGGL(ln_fwd_row16_k<6>, g16, dim3(256), 0, s, (const bf16*)x, x_stride, gam, bet, (bf16*)out, out_stride, rows, eps);
    return hipGetLastError();
  }
  dim3 grid((unsigned)((rows + 3) / 4));
  bool fast;
  if (dt != DT_F32 && out_f32) fast = ln_fwd_fast<rs_bf16path_t, float>(x, x_stride, gam, bet, out, out_stride, rows, D, eps, s);
  else if (dt == DT_F32) fast = ln_fwd_fast<float, float>(x, x_stride, gam, bet, out, out_stride, rows, D, eps, s);
  else fast = ln_fwd_fast<rs_bf16path_t, bf16>(x, x_stride, gam, bet, out, out_stride, rows, D, eps, s);
  if (fast) return hipGetLastError();
  if (dt != DT_F32 && out_f32)
    hipLaunchKernelGGL((ln_fwd_k<rs_bf16path_t, float>), grid, dim3(256), 0, s, (const rs_bf16path_t*)x, x_stride, gam,
                       bet, (float*)out, out_stride, rows, D, eps);
  else if (dt == DT_F32)
    hipLaunchKernelGGL((ln_fwd_k<float, float>), grid, dim3(256), 0, s, (const float*)x, x_stride, gam, bet, (float*)out,
                       out_stride, rows, D, eps);
  else
    hipLaunchKernelGGL((ln_fwd_k<rs_bf16path_t, bf16>), grid, dim3(256), 0, s, (const rs_bf16path_t*)x, x_stride, gam,
                       bet, (bf16*)out, out_stride, rows, D, eps);
  return hipGetLastError();
}

// dx = rstd * (dxh - mean(dxh) - xh * mean(dxh * xh)),  dxh = dy * gamma
// dgamma = sum_rows dy * xh, dbeta = sum_rows dy  -> part[block][0][D], part[block][1][D]
template <typename RS, typename TDY, typename T, bool SAME>
__global__ void __launch_bounds__(256) ln_bwd_k(const RS* __restrict__ x, long long xs, const TDY* __restrict__ dy,
                                                long long dys, const float* __restrict__ gam,
                                                const RS* __restrict__ dres, RS* __restrict__ dxo,
                                                T* __restrict__ dxo_t, long long os, long long rows, int D, float eps,
                                                float* __restrict__ part) {
  extern __shared__ float red[];  // [4][2][D]
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float dg[LN_MAXV], db[LN_MAXV], g[LN_MAXV];
#pragma unroll
  for (int i = 0; i < LN_MAXV; ++i) {
    int c = lane + 64 * i;
    dg[i] = 0.f;
    db[i] = 0.f;
    g[i] = c < D ? gam[c] : 0.f;
  }
  for (long long r = (long long)blockIdx.x * 4 + w; r < rows; r += (long long)gridDim.x * 4) {
    const RS* xr = x + r * xs;
    const TDY* dyr = dy + r * dys;
    float v[LN_MAXV], d[LN_MAXV];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      int c = lane + 64 * i;
      v[i] = c < D ? to_f(xr[c]) : 0.f;
      d[i] = c < D ? to_f(dyr[c]) : 0.f;
      sum += v[i];
    }
    float mean = wave_sum(sum) / D;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      int c = lane + 64 * i;
      v[i] = c < D ? v[i] - mean : 0.f;
      sq += v[i] * v[i];
    }
    float rstd = 1.0f / sqrtf(wave_sum(sq) / D + eps);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      v[i] *= rstd;  // xh
      dg[i] += d[i] * v[i];
      db[i] += d[i];
      d[i] *= g[i];  // dxh
      s1 += d[i];
      s2 += d[i] * v[i];
    }
    s1 = wave_sum(s1) / D;
    s2 = wave_sum(s2) / D;
#pragma unroll
    for (int i = 0; i < LN_MAXV; ++i) {
      int c = lane + 64 * i;
      if (c < D) {
        float o = rstd * (d[i] - s1 - v[i] * s2);
        if (dres) o += to_f(dres[r * os + c]);
        dxo[r * os + c] = from_f<RS>(o);
        if (!SAME) dxo_t[r * os + c] = from_f<T>(o);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < LN_MAXV; ++i) {
    int c = lane + 64 * i;
    if (c < D) {
      red[(w * 2 + 0) * D + c] = dg[i];
      red[(w * 2 + 1) * D + c] = db[i];
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 2 * D; i += 256) {
    float a = (red[0 * 2 * D + i] + red[1 * 2 * D + i]) + (red[2 * 2 * D + i] + red[3 * 2 * D + i]);
    part[(size_t)blockIdx.x * 2 * D + i] = a;
  }
}

int ln_bwd_slabs(long long rows) {
  long long s = (rows + 3) / 4;
  if (s > 512) s = 512;
  if (s < 1) s = 1;
  return (int)s;
}

// the backward kernel that can also write the normalised rows is the 16-lanes-per-row one
bool ln_bwd_emits_u(int dt, const void* x, long long x_stride, const void* dy, long long dy_stride, const float* gam,
                    const void* dres, const void* dx_out, long long o_stride, int D, bool dy_f32, const float* bet,
                    const void* u_out, long long u_stride) {
  return dt == DT_BF16 && !dy_f32 && ln_row16_ok(x, dy, dx_out, x_stride, dy_stride, o_stride, D) &&
         ((uintptr_t)gam & 15) == 0 && ((uintptr_t)dres & 15) == 0 && ((uintptr_t)bet & 15) == 0 &&
         ((uintptr_t)u_out & 15) == 0 && u_stride % 8 == 0;
}

// a residual-gradient term on every dres_period-th row only: the kernel with 16 (32) lanes per row takes it
bool ln_bwd_periodic_ok(int dt, const void* x, long long x_stride, const void* dy, long long dy_stride, const float* gam,
                        const void* dres, const void* dx_out, long long o_stride, int D, bool dy_f32) {
  return dt == DT_BF16 && !dy_f32 && ln_row16_ok(x, dy, dx_out, x_stride, dy_stride, o_stride, D) &&
         ((uintptr_t)gam & 15) == 0 && ((uintptr_t)dres & 15) == 0;
}

hipError_t launch_ln_bwd(int dt, const void* x, long long x_stride, const void* dy, long long dy_stride,
                         const float* gam, const void* dres, void* dx_out, void* dx_out_t, long long o_stride,
                         long long rows, int D, float eps, float* part, bool dy_f32, hipStream_t s, const float* bet,
                         void* u_out, long long u_stride, int dres_period) {
  if (rows <= 0) return hipSuccess;
  if (dres_period && !ln_bwd_periodic_ok(dt, x, x_stride, dy, dy_stride, gam, dres, dx_out, o_stride, D, dy_f32))
    return hipErrorInvalidValue;
  if (u_out && !ln_bwd_emits_u(dt, x, x_stride, dy, dy_stride, gam, dres, dx_out, o_stride, D, dy_f32, bet, u_out, u_stride))
    return hipErrorInvalidValue;
  dim3 grid(ln_bwd_slabs(rows));
  size_t lds = (size_t)4 * 2 * D * sizeof(float);
  if (dt == DT_BF16 && !dy_f32 && ln_row16_ok(x, dy, dx_out, x_stride, dy_stride, o_stride, D) &&
      ((uintptr_t)gam & 15) == 0 && ((uintptr_t)dres & 15) == 0) {
    if (D == 384) hipLaunchKernelGGL((ln_bwd_row16_k<3, 16>), grid, dim3(256), 0, s, (const bf16*)x, x_stride, (const bf16*)dy, dy_stride, gam, (const bf16*)dres, (bf16*)dx_out, o_stride, rows, eps, part, bet, (bf16*)u_out, u_stride, dres_period);
    else hipLaunchKernelGGL((ln_bwd_row16_k<3, 32>), grid, dim3(256), 0, s, (const bf16*)x, x_stride, (const bf16*)dy, dy_stride, gam, (const bf16*)dres, (bf16*)dx_out, o_stride, rows, eps, part, bet, (bf16*)u_out, u_stride, dres_period);
    return hipGetLastError();
  }
  {
    constexpr bool same = sizeof(rs_bf16path_t) == sizeof(bf16);
    bool fast;
    if (dt == DT_F32)
      fast = ln_bwd_fast<float, float, float, true>(grid, x, x_stride, dy, dy_stride, gam, dres, dx_out, nullptr,
                                                    o_stride, rows, D, eps, part, s);
    else if (dy_f32)
      fast = ln_bwd_fast<rs_bf16path_t, float, bf16, same>(grid, x, x_stride, dy, dy_stride, gam, dres, dx_out,
                                                           dx_out_t, o_stride, rows, D, eps, part, s);
    else
      fast = ln_bwd_fast<rs_bf16path_t, bf16, bf16, same>(grid, x, x_stride, dy, dy_stride, gam, dres, dx_out,
                                                          dx_out_t, o_stride, rows, D, eps, part, s);
    if (fast) return hipGetLastError();
  }
  if (dt == DT_F32) {
    hipLaunchKernelGGL((ln_bwd_k<float, float, float, true>), grid, dim3(256), lds, s, (const float*)x, x_stride,
                       (const float*)dy, dy_stride, gam, (const float*)dres, (float*)dx_out, (float*)nullptr, o_stride,
                       rows, D, eps, part);
  } else {
    constexpr bool same = sizeof(rs_bf16path_t) == sizeof(bf16);
    if (dy_f32)
      hipLaunchKernelGGL((ln_bwd_k<rs_bf16path_t, float, bf16, same>), grid, dim3(256), lds, s,
                         (const rs_bf16path_t*)x, x_stride, (const float*)dy, dy_stride, gam,
                         (const rs_bf16path_t*)dres, (rs_bf16path_t*)dx_out, (bf16*)dx_out_t, o_stride, rows, D, eps,
                         part);
    else
      hipLaunchKernelGGL((ln_bwd_k<rs_bf16path_t, bf16, bf16, same>), grid, dim3(256), lds, s,
                         (const rs_bf16path_t*)x, x_stride, (const bf16*)dy, dy_stride, gam,
                         (const rs_bf16path_t*)dres, (rs_bf16path_t*)dx_out, (bf16*)dx_out_t, o_stride, rows, D, eps,
                         part);
  }
  return hipGetLastError();
}

}  // namespace sl
