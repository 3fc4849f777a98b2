// AdamW update of the fp32 master parameters (paper, Experiments: the optimiser of both training set-ups; Adam with
// decoupled weight decay as in the work cited there):
//   m = b1 m + (1 - b1) g,  v = b2 v + (1 - b2) g^2,  theta -= lr (m c1 / (sqrt(v c2) + eps) + wd theta)
// with the bias corrections c1 = 1 / (1 - b1^t), c2 = 1 / (1 - b2^t) formed on the host in double.  One streaming pass:
// 16 bytes read and 12 bytes written per parameter, 16-byte accesses; nothing to fuse it with (the gradients are
// complete only after the last kernel of the backward).
#include "slide_internal.h"

#include <cmath>

namespace sl {

namespace {

struct AdamW {
  float lr, b1, b2, eps, wd, c1, c2;
};

__device__ __forceinline__ void adamw_one(float& p, float g, float& m, float& v, const AdamW& a) {
  m = fmaf(a.b1, m, (1.0f - a.b1) * g);
  v = fmaf(a.b2, v, (1.0f - a.b2) * g * g);
  float upd = (m * a.c1) / (sqrtf(v * a.c2) + a.eps) + a.wd * p;
  p = fmaf(-a.lr, upd, p);
}

__global__ void __launch_bounds__(256) adamw_vec_k(float4* __restrict__ p, const float4* __restrict__ g,
                                                   float4* __restrict__ m, float4* __restrict__ v, size_t n4, AdamW a) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 P = p[i], G = g[i], M = m[i], V = v[i];
  adamw_one(P.x, G.x, M.x, V.x, a);
  adamw_one(P.y, G.y, M.y, V.y, a);
  adamw_one(P.z, G.z, M.z, V.z, a);
  adamw_one(P.w, G.w, M.w, V.w, a);
  p[i] = P; m[i] = M; v[i] = V;
}

__global__ void __launch_bounds__(256) adamw_scalar_k(float* __restrict__ p, const float* __restrict__ g,
                                                      float* __restrict__ m, float* __restrict__ v, size_t n, AdamW a) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float P = p[i], M = m[i], V = v[i];
  adamw_one(P, g[i], M, V, a);
  p[i] = P; m[i] = M; v[i] = V;
}

}  // namespace

hipError_t launch_adamw(float* p, const float* g, float* m, float* v, size_t n, long long step, float lr, float b1,
                        float b2, float eps, float wd, hipStream_t s) {
  AdamW a;
  a.lr = lr; a.b1 = b1; a.b2 = b2; a.eps = eps; a.wd = wd;
  a.c1 = (float)(1.0 / (1.0 - std::pow((double)b1, (double)step)));
  a.c2 = (float)(1.0 / (1.0 - std::pow((double)b2, (double)step)));
  const bool al = (((uintptr_t)p | (uintptr_t)g | (uintptr_t)m | (uintptr_t)v) & 15) == 0;
  size_t n4 = al ? n / 4 : 0, done = n4 * 4;
  if (n4) {
    hipLaunchKernelGGL(adamw_vec_k, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, (float4*)p, (const float4*)g,
                       (float4*)m, (float4*)v, n4, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (done < n) {
    size_t r = n - done;
    hipLaunchKernelGGL(adamw_scalar_k, dim3((unsigned)((r + 255) / 256)), dim3(256), 0, s, p + done, g + done, m + done,
                       v + done, r, a);
    return hipGetLastError();
  }
  return hipSuccess;
}

}  // namespace sl
