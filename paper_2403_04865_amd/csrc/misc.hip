// Element-wise, layout and reduction kernels of the slide step (gfx950).
#include "slide_internal.h"

namespace sl {

// ---------------------------------------------------------------------------------------
// fp32 master weight [R,C] -> T copy [R,C] (optional) and T transpose [C,R] (optional)
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) cast_transpose_k(const float* __restrict__ src, int R, int C,
                                                        T* __restrict__ dstW, T* __restrict__ dstWT) {
  __shared__ float tile[32][33];
  int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    int r = r0 + i, c = c0 + tx;
    float v = (r < R && c < C) ? src[(size_t)r * C + c] : 0.f;
    tile[i][tx] = v;
    if (dstW && r < R && c < C) dstW[(size_t)r * C + c] = from_f<T>(v);
  }
  __syncthreads();
  if (dstWT) {
    for (int i = ty; i < 32; i += 8) {
      int c = c0 + i, r = r0 + tx;
      if (r < R && c < C) dstWT[(size_t)c * R + r] = from_f<T>(tile[tx][i]);
    }
  }
}

hipError_t launch_cast_transpose(int dt, const float* src, int R, int C, void* dstW, void* dstWT, hipStream_t s) {
  dim3 grid((C + 31) / 32, (R + 31) / 32);
  if (dt == DT_F32)
    hipLaunchKernelGGL(cast_transpose_k<float>, grid, dim3(256), 0, s, src, R, C, (float*)dstW, (float*)dstWT);
  else
    hipLaunchKernelGGL(cast_transpose_k<bf16>, grid, dim3(256), 0, s, src, R, C, (bf16*)dstW, (bf16*)dstWT);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// pixels [n,3,S,S] <-> patches [n*g*g, 3*P*P]   (patch order (gy,gx), flatten order (c,py,px))
// ---------------------------------------------------------------------------------------
// Patch matrix: tile n owns rows n * (g * g + lead) .. of 3 P P columns: `lead` rows of zeros (the slots of the tokens
// that are no patches, so that the matrix lines up row by row with the token matrix), then its g * g patches.
template <typename T>
__global__ void __launch_bounds__(256) patchify_k(const T* __restrict__ pix, T* __restrict__ pat, long long total,
                                                  int S, int P, int lead) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  int g = S / P, Kp = 3 * P * P;
  int col = (int)(i % Kp);
  long long row = i / Kp;
  int px = col % P, py = (col / P) % P, c = col / (P * P);
  int gx = (int)(row % g), gy = (int)((row / g) % g);
  long long n = row / (g * g);
  long long base = n * (g * g + lead);
  pat[(base + lead + row % (g * g)) * Kp + col] = pix[((n * 3 + c) * S + gy * P + py) * S + gx * P + px];
  if (row % (g * g) == 0)
    for (int l = 0; l < lead; ++l) pat[(base + l) * Kp + col] = from_f<T>(0.f);
}

// bf16, P % 8 == 0, S % 8 == 0: one workgroup per band of patches (tile n, patch row gy).  The band's 3 x P image
// rows are read with 16-byte accesses along the rows into LDS and written as whole patch rows, again 16 bytes
// per lane and contiguous (the element-wise kernel above moves 2 bytes per lane).
__global__ void __launch_bounds__(256) patchify_band_k(const bf16* __restrict__ pix, bf16* __restrict__ pat, int S, int P,
                                                       int lead) {
  extern __shared__ uint4 band[];   // [3 * P][S / 8] chunks of 8 pixels
  const int g = S / P, SC = S / 8, PC = P / 8, rows = 3 * P;
  const long long n = blockIdx.x / g;
  const int gy = blockIdx.x % g;
  for (int i = threadIdx.x; i < rows * SC; i += 256) {
    int r = i / SC, xc = i % SC, c = r / P, py = r % P;
    band[i] = *reinterpret_cast<const uint4*>(pix + ((n * 3 + c) * S + gy * P + py) * (long long)S + xc * 8);
  }
  __syncthreads();
  const int KC = rows * PC;          // chunks per patch row of the output
  bf16* out = pat + ((n * (g * g + lead) + lead) + gy * g) * (long long)(3 * P * P);
  if (gy == 0)   // the tile's leading rows of zeros
    for (int i = threadIdx.x; i < lead * KC; i += 256)
      *reinterpret_cast<uint4*>(pat + n * (g * g + lead) * (long long)(3 * P * P) + (long long)i * 8) = make_uint4(0, 0, 0, 0);
  for (int i = threadIdx.x; i < g * KC; i += 256) {
    int gx = i / KC, k = i % KC, r = k / PC, pc = k % PC;   // r = c * P + py
    *reinterpret_cast<uint4*>(out + (long long)i * 8) = band[r * SC + gx * PC + pc];
  }
}

template <typename T>
__global__ void __launch_bounds__(256) unpatchify_k(const T* __restrict__ dpat, T* __restrict__ dpix, long long total,
                                                    int S, int P) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;  // index into dpix
  if (i >= total) return;
  int g = S / P, Kp = 3 * P * P;
  int x = (int)(i % S), y = (int)((i / S) % S), c = (int)((i / ((long long)S * S)) % 3);
  long long n = i / (3LL * S * S);
  long long row = (n * g + y / P) * g + x / P;
  int col = c * P * P + (y % P) * P + (x % P);
  dpix[i] = dpat[row * Kp + col];
}

hipError_t launch_patchify(int dt, const void* pixels, void* patches, long long n, int S, int P, hipStream_t s, int lead) {
  long long total = n * 3LL * S * S;
  unsigned grid = (unsigned)((total + 255) / 256);
  if (dt == DT_F32)
    hipLaunchKernelGGL(patchify_k<float>, dim3(grid), dim3(256), 0, s, (const float*)pixels, (float*)patches, total, S, P, lead);
  else if (P % 8 == 0 && S % P == 0 && n * (S / P) < (1LL << 31) && (size_t)3 * P * S * 2 <= 65536)
    hipLaunchKernelGGL(patchify_band_k, dim3((unsigned)(n * (S / P))), dim3(256), (size_t)3 * P * S * 2, s,
                       (const bf16*)pixels, (bf16*)patches, S, P, lead);
  else
    hipLaunchKernelGGL(patchify_k<bf16>, dim3(grid), dim3(256), 0, s, (const bf16*)pixels, (bf16*)patches, total, S, P, lead);
  return hipGetLastError();
}

hipError_t launch_unpatchify(int dt, const void* dpatches, void* dpix, long long n, int S, int P, hipStream_t s) {
  long long total = n * 3LL * S * S;
  unsigned grid = (unsigned)((total + 255) / 256);
  if (dt == DT_F32)
    hipLaunchKernelGGL(unpatchify_k<float>, dim3(grid), dim3(256), 0, s, (const float*)dpatches, (float*)dpix, total, S, P);
  else
    hipLaunchKernelGGL(unpatchify_k<bf16>, dim3(grid), dim3(256), 0, s, (const bf16*)dpatches, (bf16*)dpix, total, S, P);
  return hipGetLastError();
}

// x[n, 0, :] = cls + pos[0]
template <typename RS>
__global__ void __launch_bounds__(256) cls_rows_k(RS* __restrict__ x, const float* __restrict__ cls,
                                                  const float* __restrict__ pos, long long n, int T, int D) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n * D) return;
  int d = (int)(i % D);
  long long t = i / D;
  x[t * T * D + d] = from_f<RS>(cls[d] + pos[d]);
}

hipError_t launch_cls_rows(int dt, void* x, const float* cls, const float* pos, long long n, int T, int D, hipStream_t s) {
  unsigned grid = (unsigned)((n * D + 255) / 256);
  if (dt == DT_F32)
    hipLaunchKernelGGL(cls_rows_k<float>, dim3(grid), dim3(256), 0, s, (float*)x, cls, pos, n, T, D);
  else
    hipLaunchKernelGGL(cls_rows_k<rs_bf16path_t>, dim3(grid), dim3(256), 0, s, (rs_bf16path_t*)x, cls, pos, n, T, D);
  return hipGetLastError();
}

// The rows the patch embedding adds to its product, one per token position, as the residual-stream type:
// tab[0] = cls + pos[0] (the patch matrix has a row of zeros there), tab[t] = bias + pos[t] for the patch tokens.
__global__ void __launch_bounds__(256) pos_table_k(rs_bf16path_t* __restrict__ tab, const float* __restrict__ cls,
                                                   const float* __restrict__ pos, const float* __restrict__ bias, int T, int D) {
  int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= T * D) return;
  int d = i % D;
  tab[i] = from_f<rs_bf16path_t>(pos[i] + (i < D ? cls[d] : bias[d]));
}

hipError_t launch_pos_table(void* tab, const float* cls, const float* pos, const float* bias, int T, int D, hipStream_t s) {
  hipLaunchKernelGGL(pos_table_k, dim3((unsigned)((T * D + 255) / 256)), dim3(256), 0, s, (rs_bf16path_t*)tab, cls, pos, bias, T, D);
  return hipGetLastError();
}

// zero fill in 16-byte words (bytes must be a multiple of 16; all arena regions are)
__global__ void __launch_bounds__(256) fill_zero_k(uint4* __restrict__ p, size_t words) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  size_t stride = (size_t)gridDim.x * 256;
  for (; i < words; i += stride) p[i] = make_uint4(0, 0, 0, 0);
}

// plain copy, 16 bytes per lane, grid-stride: the known-size kernel that hardware traffic counters are scaled with
__global__ void __launch_bounds__(256) calib_copy_k(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t words) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, step = (size_t)gridDim.x * 256;
  for (; i < words; i += step) dst[i] = src[i];
}

hipError_t launch_calib_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  size_t words = bytes / 16;
  if (!words) return hipSuccess;
  size_t blocks = (words + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(calib_copy_k, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, words);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  size_t words = bytes / 16;
  if (words == 0) return hipSuccess;
  size_t blocks = (words + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(fill_zero_k, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)p, words);
  return hipGetLastError();
}

template <typename T>
__global__ void __launch_bounds__(256) gelu_k(const T* __restrict__ m, T* __restrict__ a, long long count) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  long long stride = (long long)gridDim.x * 256;
  for (; i < count; i += stride) a[i] = from_f<T>(gelu_f(to_f(m[i])));
}

hipError_t launch_gelu(int dt, const void* m, void* a, long long count, hipStream_t s) {
  long long blocks = (count + 255) / 256;
  if (blocks > 262144) blocks = 262144;
  if (blocks == 0) return hipSuccess;
  if (dt == DT_F32)
    hipLaunchKernelGGL(gelu_k<float>, dim3((unsigned)blocks), dim3(256), 0, s, (const float*)m, (float*)a, count);
  else
    hipLaunchKernelGGL(gelu_k<bf16>, dim3((unsigned)blocks), dim3(256), 0, s, (const bf16*)m, (bf16*)a, count);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// column sums, two-stage and deterministic: part[s][c] = sum over rows of slab s
// ---------------------------------------------------------------------------------------
template <typename E>
__global__ void __launch_bounds__(256) colsum_k(const E* __restrict__ A, long long lda, RowMap map, long long M, int N,
                                                float* __restrict__ part, int slabs) {
  __shared__ float red[4][64];
  int cl = threadIdx.x & 63, q = threadIdx.x >> 6;
  int c = blockIdx.x * 64 + cl;
  int s = blockIdx.y;
  long long per = (M + slabs - 1) / slabs;
  long long lo = (long long)s * per, hi = lo + per < M ? lo + per : M;
  float acc = 0.f;
  if (c < N)
    for (long long r = lo + q; r < hi; r += 4) acc += to_f(A[map(r) * lda + c]);
  red[q][cl] = acc;
  __syncthreads();
  if (q == 0 && c < N) part[(size_t)s * N + c] = (red[0][cl] + red[1][cl]) + (red[2][cl] + red[3][cl]);
}

// The same sums for bf16 rows read 16 bytes per lane (a lane owns 8 neighbouring columns), four rows of a quarter in
// flight: the element-wise kernel above moves 2 bytes per lane and load, which is a third of the memory rate on the
// position gradient (a [tiles] x [T * D] matrix, 1.2 GB on the 8192-tile slide).  Identity row map, N and lda
// multiples of 8, 16-byte aligned rows.  Fixed order of additions (four chains per element, combined pairwise).
__global__ void __launch_bounds__(256) colsum8_k(const bf16* __restrict__ A, long long lda, long long M, int N,
                                                 float* __restrict__ part, int slabs) {
  __shared__ float red[4][64][9];
  typedef unsigned int cu4 __attribute__((ext_vector_type(4)));
  const int cl = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int c = (blockIdx.x * 64 + cl) * 8;
  const int s = blockIdx.y;
  const long long per = (M + slabs - 1) / slabs;
  const long long lo = (long long)s * per, hi = lo + per < M ? lo + per : M;
  float acc[4][8];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[u][e] = 0.f;
  if (c < N) {
    long long r = lo + q;
    for (; r + 12 < hi; r += 16) {
      cu4 t[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) t[u] = __builtin_nontemporal_load(reinterpret_cast<const cu4*>(A + (r + 4 * u) * lda + c));
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          acc[u][2 * w] += __uint_as_float(t[u][w] << 16);
          acc[u][2 * w + 1] += __uint_as_float(t[u][w] & 0xffff0000u);
        }
    }
    for (; r < hi; r += 4) {
      cu4 t = *reinterpret_cast<const cu4*>(A + r * lda + c);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        acc[0][2 * w] += __uint_as_float(t[w] << 16);
        acc[0][2 * w + 1] += __uint_as_float(t[w] & 0xffff0000u);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[q][cl][e] = (acc[0][e] + acc[1][e]) + (acc[2][e] + acc[3][e]);
  __syncthreads();
  if (q == 0 && c < N) {
#pragma unroll
    for (int e = 0; e < 8; ++e) part[(size_t)s * N + c + e] = (red[0][cl][e] + red[1][cl][e]) + (red[2][cl][e] + red[3][cl][e]);
  }
}

int colsum_slabs(long long M) {
  long long s = (M + 511) / 512;
  if (s < 1) s = 1;
  if (s > 128) s = 128;
  return (int)s;
}

// 64 outputs per workgroup; the slabs are dealt to 4 quarter-groups whose sums are then added
// in a fixed order, so the result does not depend on scheduling.
__global__ void __launch_bounds__(256) reduce_partials_k(const float* __restrict__ part, int slabs, long long stride,
                                                         long long len, float* __restrict__ out, int accumulate) {
  __shared__ float red[4][64];
  int cl = threadIdx.x & 63, q = threadIdx.x >> 6;
  long long i = (long long)blockIdx.x * 64 + cl;
  float acc = 0.f;
  if (i < len)
    for (int s = q; s < slabs; s += 4) acc += part[(size_t)s * stride + i];
  red[q][cl] = acc;
  __syncthreads();
  if (q == 0 && i < len) {
    float v = (red[0][cl] + red[1][cl]) + (red[2][cl] + red[3][cl]);
    out[i] = accumulate ? out[i] + v : v;
  }
}

// The same sums in the same order, four neighbouring outputs per thread (16-byte accesses): 256 outputs per workgroup.
__global__ void __launch_bounds__(256) reduce_partials4_k(const float* __restrict__ part, int slabs, long long stride,
                                                          long long len, float* __restrict__ out, int accumulate) {
  __shared__ float4 red[4][64];
  int cl = threadIdx.x & 63, q = threadIdx.x >> 6;
  long long i = ((long long)blockIdx.x * 64 + cl) * 4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (i < len)
    for (int s = q; s < slabs; s += 4) {
      float4 v = *reinterpret_cast<const float4*>(part + (size_t)s * stride + i);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
  red[q][cl] = acc;
  __syncthreads();
  if (q == 0 && i < len) {
    float4 a = red[0][cl], b = red[1][cl], c = red[2][cl], d = red[3][cl];
    float4 v = make_float4((a.x + b.x) + (c.x + d.x), (a.y + b.y) + (c.y + d.y), (a.z + b.z) + (c.z + d.z),
                           (a.w + b.w) + (c.w + d.w));
    float4* o = reinterpret_cast<float4*>(out + i);
    if (accumulate) { float4 w = *o; v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w; }
    *o = v;
  }
}

// Short results (bias, gain and shift gradients: a few hundred outputs, up to a thousand slabs): 16 outputs per
// workgroup and the slabs dealt to 16 groups of lanes, so that a launch has four times the workgroups and a quarter of
// the loads per thread of the kernel above; the 16 group sums are added as a fixed binary tree.
__global__ void __launch_bounds__(256) reduce_partials16_k(const float* __restrict__ part, int slabs, long long stride,
                                                           long long len, float* __restrict__ out, int accumulate) {
  __shared__ float red[16][17];
  const int cl = threadIdx.x & 15, q = threadIdx.x >> 4;
  const long long i = (long long)blockIdx.x * 16 + cl;
  float a0 = 0.f, a1 = 0.f;
  if (i < len) {
    int s = q;
    for (; s + 16 < slabs; s += 32) {
      a0 += part[(size_t)s * stride + i];
      a1 += part[(size_t)(s + 16) * stride + i];
    }
    if (s < slabs) a0 += part[(size_t)s * stride + i];
  }
  red[q][cl] = a0 + a1;
  __syncthreads();
  if (q == 0 && i < len) {
    float t[16];
#pragma unroll
    for (int g = 0; g < 16; ++g) t[g] = red[g][cl];
#pragma unroll
    for (int w = 8; w > 0; w >>= 1)
#pragma unroll
      for (int g = 0; g < w; ++g) t[g] += t[g + w];
    out[i] = accumulate ? out[i] + t[0] : t[0];
  }
}

hipError_t launch_reduce_partials(const float* part, int slabs, long long stride, long long len, float* out,
                                  int accumulate, hipStream_t s) {
  if (len <= 0) return hipSuccess;
  if (len < 4096 && slabs >= 64) {
    hipLaunchKernelGGL(reduce_partials16_k, dim3((unsigned)((len + 15) / 16)), dim3(256), 0, s, part, slabs, stride, len, out,
                       accumulate);
    return hipGetLastError();
  }
  if (len >= 4096 && len % 4 == 0 && stride % 4 == 0 && ((uintptr_t)part & 15) == 0 && ((uintptr_t)out & 15) == 0) {
    hipLaunchKernelGGL(reduce_partials4_k, dim3((unsigned)((len / 4 + 63) / 64)), dim3(256), 0, s, part, slabs, stride,
                       len, out, accumulate);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(reduce_partials_k, dim3((unsigned)((len + 63) / 64)), dim3(256), 0, s, part, slabs, stride, len,
                     out, accumulate);
  return hipGetLastError();
}

hipError_t launch_colsum_part(int elem, const void* A, long long lda, RowMap map, long long M, int N, float* part,
                              int slabs, hipStream_t s) {
  if (elem != DT_F32 && map.g2 == 0 && N % 8 == 0 && lda % 8 == 0 && ((size_t)A & 15) == 0 && M >= 64) {
    hipLaunchKernelGGL(colsum8_k, dim3((N / 8 + 63) / 64, slabs), dim3(256), 0, s, (const bf16*)A, lda, M, N, part, slabs);
    return hipGetLastError();
  }
  dim3 grid((N + 63) / 64, slabs);
  if (elem == DT_F32)
    hipLaunchKernelGGL(colsum_k<float>, grid, dim3(256), 0, s, (const float*)A, lda, map, M, N, part, slabs);
  else
    hipLaunchKernelGGL(colsum_k<bf16>, grid, dim3(256), 0, s, (const bf16*)A, lda, map, M, N, part, slabs);
  return hipGetLastError();
}

}  // namespace sl
