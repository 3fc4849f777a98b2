// Softmax attention inside one tile, plain-ALU version (fp32 path and fall-back).
// One workgroup per (tile, head); K and V (or Q and dO) of that head live in LDS as fp32.
//
// qkv is the token matrix [n*T, 3D]: columns [0,D) queries, [D,2D) keys, [2D,3D) values,
// head h owning columns h*dh .. h*dh+dh-1 of each third.
#include "slide_internal.h"

namespace sl {

hipError_t launch_attn_fwd_mfma(const void* qkv, void* O, float* lse, long long n, int T, int H, int dh, int cls_only,
                                hipStream_t s);
hipError_t launch_attn_bwd_mfma(const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv, float* delta_ws,
                                long long n, int T, int H, int dh, int cls_only, hipStream_t s);
bool attn_mfma_ok(int T, int dh);

template <typename T, int DH>
__global__ void __launch_bounds__(256) attn_fwd_k(const T* __restrict__ qkv, T* __restrict__ O,
                                                  float* __restrict__ lse, int Tn, int H) {
  extern __shared__ float lds[];
  float* Ks = lds;             // [Tn][DH]
  float* Vs = lds + Tn * DH;   // [Tn][DH]
  int h = blockIdx.x % H;
  long long tile = blockIdx.x / H;
  int D = H * DH;
  const T* base = qkv + tile * Tn * 3LL * D;
  for (int i = threadIdx.x; i < Tn * DH; i += 256) {
    int j = i / DH, e = i % DH;
    Ks[i] = to_f(base[(long long)j * 3 * D + D + h * DH + e]);
    Vs[i] = to_f(base[(long long)j * 3 * D + 2 * D + h * DH + e]);
  }
  __syncthreads();
  float scale = 1.0f / sqrtf((float)DH);
  for (int i = threadIdx.x; i < Tn; i += 256) {
    float q[DH], o[DH];
#pragma unroll
    for (int e = 0; e < DH; ++e) {
      q[e] = to_f(base[(long long)i * 3 * D + h * DH + e]) * scale;
      o[e] = 0.f;
    }
    float mx = -INFINITY;
    for (int j = 0; j < Tn; ++j) {
      float sc = 0.f;
#pragma unroll
      for (int e = 0; e < DH; ++e) sc += q[e] * Ks[j * DH + e];
      mx = fmaxf(mx, sc);
    }
    float l = 0.f;
    for (int j = 0; j < Tn; ++j) {
      float sc = 0.f;
#pragma unroll
      for (int e = 0; e < DH; ++e) sc += q[e] * Ks[j * DH + e];
      float p = __expf(sc - mx);
      l += p;
#pragma unroll
      for (int e = 0; e < DH; ++e) o[e] += p * Vs[j * DH + e];
    }
    float inv = 1.0f / l;
    T* orow = O + (tile * Tn + i) * D + h * DH;
#pragma unroll
    for (int e = 0; e < DH; ++e) orow[e] = from_f<T>(o[e] * inv);
    lse[(tile * H + h) * Tn + i] = mx + logf(l);
  }
}

// dV = P^T dO, dP = dO V^T, dS = P * (dP - delta), delta_i = dO_i . O_i,
// dQ = dS K / sqrt(dh), dK = dS^T Q / sqrt(dh);  P recomputed from the saved row log-sum-exp.
template <typename T, int DH>
__global__ void __launch_bounds__(256) attn_bwd_k(const T* __restrict__ qkv, const T* __restrict__ O,
                                                  const float* __restrict__ lse, const T* __restrict__ dO,
                                                  T* __restrict__ dqkv, int Tn, int H) {
  extern __shared__ float lds[];
  float* As = lds;             // phase A: K, phase B: Q (pre-scaled)
  float* Bs = lds + Tn * DH;   // phase A: V, phase B: dO
  float* dl = lds + 2 * Tn * DH;  // [Tn] delta
  float* ls = dl + Tn;            // [Tn] lse
  int h = blockIdx.x % H;
  long long tile = blockIdx.x / H;
  int D = H * DH;
  const T* base = qkv + tile * Tn * 3LL * D;
  T* dbase = dqkv + tile * Tn * 3LL * D;
  float scale = 1.0f / sqrtf((float)DH);
  for (int i = threadIdx.x; i < Tn * DH; i += 256) {
    int j = i / DH, e = i % DH;
    As[i] = to_f(base[(long long)j * 3 * D + D + h * DH + e]);
    Bs[i] = to_f(base[(long long)j * 3 * D + 2 * D + h * DH + e]);
  }
  for (int i = threadIdx.x; i < Tn; i += 256) ls[i] = lse[(tile * H + h) * Tn + i];
  __syncthreads();
  // phase A: one query row per thread -> delta_i, dQ_i
  for (int i = threadIdx.x; i < Tn; i += 256) {
    float q[DH], go[DH], dq[DH];
    float delta = 0.f;
    const T* orow = O + (tile * Tn + i) * D + h * DH;
    const T* gor = dO + (tile * Tn + i) * D + h * DH;
#pragma unroll
    for (int e = 0; e < DH; ++e) {
      q[e] = to_f(base[(long long)i * 3 * D + h * DH + e]) * scale;
      go[e] = to_f(gor[e]);
      delta += go[e] * to_f(orow[e]);
      dq[e] = 0.f;
    }
    dl[i] = delta;
    float li = ls[i];
    for (int j = 0; j < Tn; ++j) {
      float sc = 0.f, dp = 0.f;
#pragma unroll
      for (int e = 0; e < DH; ++e) {
        sc += q[e] * As[j * DH + e];
        dp += go[e] * Bs[j * DH + e];
      }
      float ds = __expf(sc - li) * (dp - delta);
#pragma unroll
      for (int e = 0; e < DH; ++e) dq[e] += ds * As[j * DH + e];
    }
#pragma unroll
    for (int e = 0; e < DH; ++e) dbase[(long long)i * 3 * D + h * DH + e] = from_f<T>(dq[e] * scale);
  }
  __syncthreads();
  // phase B: one key row per thread -> dK_j, dV_j
  for (int i = threadIdx.x; i < Tn * DH; i += 256) {
    int j = i / DH, e = i % DH;
    As[i] = to_f(base[(long long)j * 3 * D + h * DH + e]) * scale;
    Bs[i] = to_f(dO[(tile * Tn + j) * D + h * DH + e]);
  }
  __syncthreads();
  for (int j = threadIdx.x; j < Tn; j += 256) {
    float k[DH], v[DH], dk[DH], dv[DH];
#pragma unroll
    for (int e = 0; e < DH; ++e) {
      k[e] = to_f(base[(long long)j * 3 * D + D + h * DH + e]);
      v[e] = to_f(base[(long long)j * 3 * D + 2 * D + h * DH + e]);
      dk[e] = 0.f;
      dv[e] = 0.f;
    }
    for (int i = 0; i < Tn; ++i) {
      float sc = 0.f, dp = 0.f;
#pragma unroll
      for (int e = 0; e < DH; ++e) {
        sc += As[i * DH + e] * k[e];
        dp += Bs[i * DH + e] * v[e];
      }
      float p = __expf(sc - ls[i]);
      float ds = p * (dp - dl[i]);
#pragma unroll
      for (int e = 0; e < DH; ++e) {
        dk[e] += ds * As[i * DH + e];  // As holds q * scale
        dv[e] += p * Bs[i * DH + e];
      }
    }
#pragma unroll
    for (int e = 0; e < DH; ++e) {
      dbase[(long long)j * 3 * D + D + h * DH + e] = from_f<T>(dk[e]);
      dbase[(long long)j * 3 * D + 2 * D + h * DH + e] = from_f<T>(dv[e]);
    }
  }
}

size_t attn_lds_bytes(int Tn, int dh) { return ((size_t)2 * Tn * dh + 2 * Tn) * sizeof(float); }

template <typename K>
static hipError_t set_lds(K kernel, size_t bytes) {
  if (bytes <= 65536) return hipSuccess;
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

bool attn_cls_only_ok(int dt, int T, int dh, bool use_mfma) { return dt == DT_BF16 && use_mfma && attn_mfma_ok(T, dh); }

hipError_t launch_attn_fwd(int dt, const void* qkv, void* O, float* lse, long long n, int T, int H, int dh,
                           bool use_mfma, hipStream_t s, bool cls_only) {
  if (n <= 0) return hipSuccess;
  if (dt == DT_BF16 && use_mfma && attn_mfma_ok(T, dh)) return launch_attn_fwd_mfma(qkv, O, lse, n, T, H, dh, cls_only, s);
  if (cls_only) return hipErrorInvalidValue;
  size_t lds = attn_lds_bytes(T, dh);
  dim3 grid((unsigned)(n * H));
  hipError_t e = hipSuccess;
#define GO(TT, DHH)                                                                                            \
  do {                                                                                                         \
    e = set_lds(attn_fwd_k<TT, DHH>, lds);                                                                     \
    if (e != hipSuccess) return e;                                                                             \
    hipLaunchKernelGGL((attn_fwd_k<TT, DHH>), grid, dim3(256), lds, s, (const TT*)qkv, (TT*)O, lse, T, H);     \
  } while (0)
  if (dt == DT_F32) { if (dh == 64) GO(float, 64); else if (dh == 32) GO(float, 32); else if (dh == 8) GO(float, 8); else return hipErrorInvalidValue; }
  else { if (dh == 64) GO(bf16, 64); else if (dh == 32) GO(bf16, 32); else if (dh == 8) GO(bf16, 8); else return hipErrorInvalidValue; }
#undef GO
  return hipGetLastError();
}

hipError_t launch_attn_bwd(int dt, const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv,
                           long long n, int T, int H, int dh, bool use_mfma, hipStream_t s, bool cls_only, float* delta_ws) {
  if (n <= 0) return hipSuccess;
  if (dt == DT_BF16 && use_mfma && attn_mfma_ok(T, dh)) {
    if (!delta_ws) return hipErrorInvalidValue;
    return launch_attn_bwd_mfma(qkv, O, lse, dO, dqkv, delta_ws, n, T, H, dh, cls_only, s);
  }
  if (cls_only) return hipErrorInvalidValue;
  size_t lds = attn_lds_bytes(T, dh);
  dim3 grid((unsigned)(n * H));
  hipError_t e = hipSuccess;
#define GO(TT, DHH)                                                                                            \
  do {                                                                                                         \
    e = set_lds(attn_bwd_k<TT, DHH>, lds);                                                                     \
    if (e != hipSuccess) return e;                                                                             \
    hipLaunchKernelGGL((attn_bwd_k<TT, DHH>), grid, dim3(256), lds, s, (const TT*)qkv, (const TT*)O, lse,      \
                       (const TT*)dO, (TT*)dqkv, T, H);                                                        \
  } while (0)
  if (dt == DT_F32) { if (dh == 64) GO(float, 64); else if (dh == 32) GO(float, 32); else if (dh == 8) GO(float, 8); else return hipErrorInvalidValue; }
  else { if (dh == 64) GO(bf16, 64); else if (dh == 32) GO(bf16, 32); else if (dh == 8) GO(bf16, 8); else return hipErrorInvalidValue; }
#undef GO
  return hipGetLastError();
}

}  // namespace sl
