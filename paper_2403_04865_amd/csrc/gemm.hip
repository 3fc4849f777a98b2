// Plain FMA GEMMs (fp32 path, and the fall-back of the bf16 path) + dispatch to the MFMA kernels.
#include "gemm_epi.h"

namespace sl {

hipError_t launch_gemm_nt_mfma(const GemmNT& g, hipStream_t s);  // gemm_mfma.hip
hipError_t launch_gemm_tn_mfma(const GemmTN& g, hipStream_t s);
bool gemm_nt_mfma_ok(const GemmNT& g);
bool gemm_tn_mfma_ok(const GemmTN& g);

// C[m][n] = sum_k A[amap(m)][k] * B[n][k]; 64x64 tile, 4x4 per thread, BK = 16
template <typename T, typename RS>
__global__ void __launch_bounds__(256) gemm_nt_fma_k(GemmNT g) {
  __shared__ float As[16][68];
  __shared__ float Bs[16][68];
  const T* A = (const T*)g.A;
  const T* B = (const T*)g.B;
  int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  long long m0 = (long long)blockIdx.x * 64;
  int n0 = blockIdx.y * 64;
  int lr = tid >> 2, lk = (tid & 3) * 4;  // loader: row lr, k lk..lk+3
  long long am = m0 + lr;
  long long arow = am < g.M ? g.amap(am) : -1;
  int bn = n0 + lr;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < g.K; k0 += 16) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int k = k0 + lk + j;
      As[lk + j][lr] = (arow >= 0 && k < g.K) ? to_f(A[arow * g.lda + k]) : 0.f;
      Bs[lk + j][lr] = (bn < g.N && k < g.K) ? to_f(B[(long long)bn * g.ldb + k]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = As[k][ty * 4 + i];
        b[i] = Bs[k][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    long long m = m0 + ty * 4 + i;
    if (m >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n < g.N) epi_store<T, RS>(g, m, n, acc[i][j]);
    }
  }
}

// part[s][i][j] = sum_{m in slab s} A[amap(m)][i] * B[bmap(m)][j]
template <typename T>
__global__ void __launch_bounds__(256) gemm_tn_fma_k(GemmTN g) {
  __shared__ float As[16][68];
  __shared__ float Bs[16][68];
  const T* A = (const T*)g.A;
  const T* B = (const T*)g.B;
  int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  int i0 = blockIdx.x * 64, j0 = blockIdx.y * 64, s = blockIdx.z;
  long long per = (g.M + g.slabs - 1) / g.slabs;
  long long lo = (long long)s * per, hi = lo + per < g.M ? lo + per : g.M;
  int lm = tid >> 4, lc = (tid & 15) * 4;  // loader: row lm of the 16-row step, cols lc..lc+3
  float acc[4][4] = {};
  for (long long mb = lo; mb < hi; mb += 16) {
    long long m = mb + lm;
    bool ok = m < hi;
    long long ar = ok ? g.amap(m) : 0, br = ok ? g.bmap(m) : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      As[lm][lc + j] = (ok && i0 + lc + j < g.N1) ? to_f(A[ar * g.lda + i0 + lc + j]) : 0.f;
      Bs[lm][lc + j] = (ok && j0 + lc + j < g.N2) ? to_f(B[br * g.ldb + j0 + lc + j]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = As[k][ty * 4 + i];
        b[i] = Bs[k][tx * 4 + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
  float* P = g.part + (size_t)s * g.N1 * g.N2;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int r = i0 + ty * 4 + i;
    if (r >= g.N1) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int c = j0 + tx * 4 + j;
      if (c < g.N2) P[(size_t)r * g.N2 + c] = acc[i][j];
    }
  }
}

int gemm_tn_pick_slabs(long long M, int N1, int N2, int max_slabs) {
  // enough workgroups to cover the chip several times, slabs of at least 256 rows
  long long tiles = (long long)((N1 + 127) / 128) * ((N2 + 127) / 128);
  long long want = (2048 + tiles - 1) / tiles;
  long long by_rows = (M + 255) / 256;
  long long s = want < by_rows ? want : by_rows;
  if (s > max_slabs) s = max_slabs;
  if (s < 1) s = 1;
  return (int)s;
}

bool gemm_tn_fuses_colsum(int dt, const GemmTN& g, bool use_mfma) {
  return dt == DT_BF16 && use_mfma && gemm_tn_mfma_ok(g);
}

hipError_t launch_gemm_nt(int dt, const GemmNT& g, bool use_mfma, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  // the periodic-table epilogue exists in the large-M kernel only (callers ask gemm_nt_big_ok first)
  if (g.epi == EPI_ROWTAB && !(dt == DT_BF16 && use_mfma && gemm_nt_mfma_ok(g) && gemm_nt_big_ok(g))) return hipErrorInvalidValue;
  if (dt == DT_BF16 && use_mfma && gemm_nt_mfma_ok(g)) return launch_gemm_nt_mfma(g, s);
  dim3 grid((unsigned)((g.M + 63) / 64), (g.N + 63) / 64);
  if (dt == DT_F32)
    hipLaunchKernelGGL((gemm_nt_fma_k<float, float>), grid, dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL((gemm_nt_fma_k<bf16, rs_bf16path_t>), grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

hipError_t launch_gemm_tn(int dt, const GemmTN& g, bool use_mfma, hipStream_t s) {
  if (g.N1 <= 0 || g.N2 <= 0 || g.slabs <= 0) return hipSuccess;
  if (dt == DT_BF16 && use_mfma && g.big) return launch_gemm_tn_big(g, s);
  if (dt == DT_BF16 && use_mfma && gemm_tn_mfma_ok(g)) return launch_gemm_tn_mfma(g, s);
  dim3 grid((g.N1 + 63) / 64, (g.N2 + 63) / 64, g.slabs);
  if (dt == DT_F32)
    hipLaunchKernelGGL(gemm_tn_fma_k<float>, grid, dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_tn_fma_k<bf16>, grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace sl
