// LayerNorm forward / backward: one 64-lane wavefront per token row, statistics in fp32.
// Rows are re-normalised from the saved layer input wherever the normalised value is needed
// again (weight-gradient operand, backward), so no per-row statistics are stored.
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

hipError_t launch_ln_fwd(int dt, const void* x, long long x_stride, const float* gam, const float* bet, void* out,
                         long long out_stride, long long rows, int D, float eps, bool out_f32, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  dim3 grid((unsigned)((rows + 3) / 4));
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
  if (s > 1024) s = 1024;
  if (s < 1) s = 1;
  return (int)s;
}

hipError_t launch_ln_bwd(int dt, const void* x, long long x_stride, const void* dy, long long dy_stride,
                         const float* gam, const void* dres, void* dx_out, void* dx_out_t, long long o_stride,
                         long long rows, int D, float eps, float* part, bool dy_f32, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  dim3 grid(ln_bwd_slabs(rows));
  size_t lds = (size_t)4 * 2 * D * sizeof(float);
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
