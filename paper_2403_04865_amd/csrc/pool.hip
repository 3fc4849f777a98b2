// Gated-attention MIL pooling over the tile features of a slide, forward and backward.
//   t_n = tanh(V h_n + b_V), s_n = sigmoid(U h_n + b_U), a_n = w . (t_n * s_n),
//   alpha = softmax_n(a), z = sum_n alpha_n h_n, y = W_c z + b_c, loss = BCE / CE(y, label).
// The softmax over tiles is a two-level online reduction: every workgroup keeps a running
// (max, sum, weighted feature sum) over its row groups, one workgroup combines them.
#include "slide_internal.h"

namespace sl {

constexpr int PR_WIDE = 16;   // rows per group
constexpr int PR_NARROW = 8;  // ... where 16 rows of features do not fit the LDS (feature width 2048)

// Gate activations of PR feature rows held in LDS (hs [PR][D] fp32):
// tl[r][j] = tanh(V_j.h_r + bV_j), sg[r][j] = sigmoid(U_j.h_r + bU_j).  One wave per gate unit j.
template <int PR>
__device__ __forceinline__ void gate_rows(const float* hs, int D, int Mh, const float* __restrict__ VW,
                                          const float* __restrict__ Vb, const float* __restrict__ UW,
                                          const float* __restrict__ Ub, float* tl, float* sg) {
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int j = w; j < Mh; j += 4) {
    float av[PR], au[PR];
#pragma unroll
    for (int r = 0; r < PR; ++r) { av[r] = 0.f; au[r] = 0.f; }
    for (int d = lane; d < D; d += 64) {
      float v = VW[(size_t)j * D + d], u = UW[(size_t)j * D + d];
#pragma unroll
      for (int r = 0; r < PR; ++r) {
        float h = hs[r * D + d];
        av[r] += v * h;
        au[r] += u * h;
      }
    }
#pragma unroll
    for (int r = 0; r < PR; ++r) {
      av[r] = wave_sum(av[r]);
      au[r] = wave_sum(au[r]);
    }
    if (lane == 0) {
      float bv = Vb[j], bu = Ub[j];
#pragma unroll
      for (int r = 0; r < PR; ++r) {
        tl[r * Mh + j] = tanhf(av[r] + bv);
        sg[r * Mh + j] = 1.0f / (1.0f + __expf(-(au[r] + bu)));
      }
    }
  }
}

template <int PR>
__device__ __forceinline__ void load_rows(const float* __restrict__ H, long long n0, long long N, int D, float* hs) {
  for (int i = threadIdx.x; i < PR * D; i += 256) {
    long long n = n0 + i / D;
    hs[i] = n < N ? H[n * D + i % D] : 0.f;
  }
}

// forward, stage 1: attention logits a[n] and per-workgroup partials part[b] = {max, sum, zsum[D]}
template <int PR>
__global__ void __launch_bounds__(256) pool_gate_part_k(PoolArgs p) {
  extern __shared__ float lds[];
  int D = p.D, Mh = p.Mh;
  float* hs = lds;                // [PR][D]
  float* tl = hs + PR * D;        // [PR][Mh]
  float* sg = tl + PR * Mh;       // [PR][Mh]
  float* ar = sg + PR * Mh;       // [PR] logits of the group
  float* er = ar + PR;            // [PR] exp weights
  double* zb = (double*)(er + PR);  // [D] running weighted sum (fp64: z feeds a cancelling difference later)
  __shared__ float run_m, resc;
  __shared__ double run_l;
  const float* H = p.H;
  for (int d = threadIdx.x; d < D; d += 256) zb[d] = 0.0;
  if (threadIdx.x == 0) { run_m = -INFINITY; run_l = 0.0; }
  long long groups = (p.N + PR - 1) / PR;
  for (long long gi = blockIdx.x; gi < groups; gi += gridDim.x) {
    long long n0 = gi * PR;
    __syncthreads();
    load_rows<PR>(H, n0, p.N, D, hs);
    __syncthreads();
    gate_rows<PR>(hs, D, Mh, p.VW, p.Vb, p.UW, p.Ub, tl, sg);
    __syncthreads();
    if (threadIdx.x < PR) {
      int r = threadIdx.x;
      float a = 0.f;
      for (int j = 0; j < Mh; ++j) a += p.w[j] * tl[r * Mh + j] * sg[r * Mh + j];
      bool ok = n0 + r < p.N;
      ar[r] = ok ? a : -INFINITY;
      if (ok) p.a[n0 + r] = a;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      float m = run_m;
      for (int r = 0; r < PR; ++r) m = fmaxf(m, ar[r]);
      float sc = __expf(run_m - m);  // exp(-inf) = 0 on the first group
      double l = run_l * (double)sc;
      for (int r = 0; r < PR; ++r) {
        float e = __expf(ar[r] - m);
        er[r] = e;
        l += (double)e;
      }
      run_m = m; run_l = l; resc = sc;
    }
    __syncthreads();
    for (int d = threadIdx.x; d < D; d += 256) {
      double z = zb[d] * (double)resc;
#pragma unroll
      for (int r = 0; r < PR; ++r) z += (double)er[r] * (double)hs[r * D + d];
      zb[d] = z;
    }
  }
  __syncthreads();
  double* out = p.part + (size_t)blockIdx.x * (2 + D);
  if (threadIdx.x == 0) { out[0] = (double)run_m; out[1] = run_l; }
  for (int d = threadIdx.x; d < D; d += 256) out[2 + d] = zb[d];
}

// Softmax statistics over the partials of stage 1: running max m and normaliser Z of the whole slide; wts[b] (if
// given) is the weight exp(m_b - m) of partial b.  Called by all 256 threads of a workgroup.
__device__ void pool_partial_stats(const PoolArgs& p, float* sm, double* smd, float* wts, float& m_out, double& Z_out) {
  const int D = p.D, B = p.blocks;
  float m = -INFINITY;
  for (int b = threadIdx.x; b < B; b += 256) m = fmaxf(m, (float)p.part[(size_t)b * (2 + D)]);
  sm[threadIdx.x] = m;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) sm[threadIdx.x] = fmaxf(sm[threadIdx.x], sm[threadIdx.x + o]);
    __syncthreads();
  }
  m = sm[0];
  double l = 0.0;
  for (int b = threadIdx.x; b < B; b += 256) {
    const double* q = p.part + (size_t)b * (2 + D);
    float wt = __expf((float)q[0] - m);
    if (wts) wts[b] = wt;
    l += q[1] * (double)wt;
  }
  smd[threadIdx.x] = l;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) smd[threadIdx.x] += smd[threadIdx.x + o];
    __syncthreads();
  }
  m_out = m;
  Z_out = smd[0];
}

// forward, stage 2a: z = sum_b wts[b] z_b / Z.  One workgroup per 16 columns, 16 slices of the partials per column:
// a single compute unit fetching all partials (written by every other unit a moment ago) is bound by its own
// handful of outstanding misses, so the sum is spread over D / 16 units with every load of a thread in flight at once.
__global__ void __launch_bounds__(256) pool_combine_z_k(PoolArgs p) {
  __shared__ float sm[256];
  __shared__ double smd[256];
  __shared__ float wts[1024];   // at most 1024 workgroups in stage 1
  __shared__ double red[16][17];
  const int D = p.D, B = p.blocks;
  float* z = p.scal + 4 + 2 * p.C;
  float* zlo = z + 2 * D;
  float m;
  double Z;
  pool_partial_stats(p, sm, smd, wts, m, Z);
  const int c = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int d = blockIdx.x * 16 + c, dc = d < D ? d : D - 1;
  double acc = 0.0;
#pragma unroll 8
  for (int b = sl; b < B; b += 16) acc += p.part[(size_t)b * (2 + D) + 2 + dc] * (double)wts[b];
  red[sl][c] = acc;
  __syncthreads();
  if (threadIdx.x < 16 && d < D) {
    double t = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i][c];
    t /= Z;
    float hi = (float)t;
    z[d] = hi;
    zlo[d] = (float)(t - (double)hi);   // z = z[d] + zlo[d] to fp64 accuracy
  }
}

// forward, stage 2b (one workgroup): m, Z, logits, loss, dy, dz, z.dz
__global__ void __launch_bounds__(256) pool_combine_k(PoolArgs p) {
  __shared__ float sm[256];
  __shared__ double smd[256];
  int D = p.D, C = p.C;
  float* scal = p.scal;
  float* y = scal + 4;
  float* dy = y + C;
  float* z = dy + C;
  float* dz = z + D;
  float m;
  double Z;
  pool_partial_stats(p, sm, smd, nullptr, m, Z);
  __syncthreads();
  // logits: one wave per class round-robin
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (int c = w; c < C; c += 4) {
    float acc = 0.f;
    for (int d = lane; d < D; d += 64) acc += p.cW[(size_t)c * D + d] * z[d];
    acc = wave_sum(acc);
    if (lane == 0) y[c] = acc + p.cb[c];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float loss;
    if (C == 1) {
      float v = y[0];
      loss = fmaxf(v, 0.f) - v * (float)p.label + log1pf(__expf(-fabsf(v)));
      dy[0] = 1.0f / (1.0f + __expf(-v)) - (float)p.label;
    } else {
      float mx = y[0];
      for (int c = 1; c < C; ++c) mx = fmaxf(mx, y[c]);
      float se = 0.f;
      for (int c = 0; c < C; ++c) se += __expf(y[c] - mx);
      float lse = mx + logf(se);
      loss = lse - y[p.label];
      for (int c = 0; c < C; ++c) dy[c] = __expf(y[c] - lse) - (c == p.label ? 1.f : 0.f);
    }
    scal[0] = m; scal[1] = (float)Z; scal[2] = loss;
    if (p.loss) p.loss[0] = loss;
    if (p.logits) for (int c = 0; c < C; ++c) p.logits[c] = y[c];
  }
  __syncthreads();
  float part = 0.f;
  for (int d = threadIdx.x; d < D; d += 256) {
    float acc = 0.f;
    for (int c = 0; c < C; ++c) acc += p.cW[(size_t)c * D + d] * dy[c];
    dz[d] = acc;
    part += acc * z[d];
  }
  sm[threadIdx.x] = part;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) sm[threadIdx.x] += sm[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) scal[3] = sm[0];
}

__global__ void __launch_bounds__(256) pool_alpha_k(const float* __restrict__ a, const float* __restrict__ scal,
                                                    float* __restrict__ alpha, long long N) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < N) alpha[i] = __expf(a[i] - scal[0]) / scal[1];
}

// backward rows: G and the per-row gate gradients Dp [N, 3*Mh] (fp32: their column sums cancel
// almost completely because sum_n da_n = 0, so they are not rounded to the storage type):
//   [0,Mh)   dpV = da * w * s * (1 - t^2)     (gradient at V's pre-activation)
//   [Mh,2Mh) dpU = da * w * t * s * (1 - s)   (gradient at U's pre-activation)
//   [2Mh,3Mh) da * t * s                      (summed over rows this is dw)
template <int PR>
__global__ void __launch_bounds__(256) pool_bwd_rows_k(PoolArgs p, float* __restrict__ Dp) {
  extern __shared__ float lds[];
  int D = p.D, Mh = p.Mh, C = p.C;
  float* hs = lds;                // [PR][D]
  float* tl = hs + PR * D;        // [PR][Mh] -> reused as dpV
  float* sg = tl + PR * Mh;       // [PR][Mh] -> reused as dpU
  float* al = sg + PR * Mh;       // [PR] alpha
  float* da = al + PR;            // [PR]
  const float* H = p.H;
  float* G = p.G;
  const float* scal = p.scal;
  const float* zv = scal + 4 + 2 * C;
  const float* dz = zv + D;
  const float* zlo = dz + D;
  float m = scal[0], Z = scal[1];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  long long groups = (p.N + PR - 1) / PR;
  for (long long gi = blockIdx.x; gi < groups; gi += gridDim.x) {
    long long n0 = gi * PR;
    __syncthreads();
    load_rows<PR>(H, n0, p.N, D, hs);
    __syncthreads();
    gate_rows<PR>(hs, D, Mh, p.VW, p.Vb, p.UW, p.Ub, tl, sg);
    for (int r = w; r < PR; r += 4) {  // softmax backward: da_n = alpha_n (h_n - z) . dz
      float acc = 0.f;
      for (int d = lane; d < D; d += 64) acc += ((hs[r * D + d] - zv[d]) - zlo[d]) * dz[d];
      acc = wave_sum(acc);
      if (lane == 0) {
        bool ok = n0 + r < p.N;
        float a = ok ? __expf(p.a[n0 + r] - m) / Z : 0.f;
        al[r] = a;
        da[r] = a * acc;
      }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < PR * Mh; i += 256) {
      int r = i / Mh, j = i % Mh;
      float t = tl[i], s = sg[i], g = da[r], wj = p.w[j];
      float dv = g * wj * s * (1.f - t * t);
      float du = g * wj * t * s * (1.f - s);
      tl[i] = dv;
      sg[i] = du;
      if (n0 + r < p.N) {
        float* row = Dp + (n0 + r) * 3LL * Mh;
        row[j] = dv;
        row[Mh + j] = du;
        row[2 * Mh + j] = g * t * s;
      }
    }
    __syncthreads();
    for (int d = threadIdx.x; d < D; d += 256) {
      float acc[PR];
      float dzd = dz[d];
#pragma unroll
      for (int r = 0; r < PR; ++r) acc[r] = al[r] * dzd;
      for (int j = 0; j < Mh; ++j) {
        float v = p.VW[(size_t)j * D + d], u = p.UW[(size_t)j * D + d];
#pragma unroll
        for (int r = 0; r < PR; ++r) acc[r] += tl[r * Mh + j] * v + sg[r * Mh + j] * u;
      }
#pragma unroll
      for (int r = 0; r < PR; ++r)
        if (n0 + r < p.N) G[(n0 + r) * D + d] = acc[r];
    }
  }
}

// head.W grad = dy z^T, head.b grad = dy
__global__ void __launch_bounds__(256) pool_head_grads_k(PoolArgs p) {
  int D = p.D, C = p.C;
  const float* dy = p.scal + 4 + C;
  const float* z = dy + C;
  float* gW = p.grads + p.ocW;
  float* gb = p.grads + p.ocb;
  for (int i = threadIdx.x + blockIdx.x * 256; i < C * D; i += 256 * gridDim.x) {
    float v = dy[i / D] * z[i % D];
    gW[i] = p.accumulate ? gW[i] + v : v;
  }
  if (blockIdx.x == 0 && threadIdx.x < C) {
    float v = dy[threadIdx.x];
    gb[threadIdx.x] = p.accumulate ? gb[threadIdx.x] + v : v;
  }
}

int pool_blocks(long long N) {
  long long g = (N + PR_WIDE - 1) / PR_WIDE;
  if (g > 1024) g = 1024;
  if (g < 1) g = 1;
  return (int)g;
}

static size_t pool_lds(int PR, int D, int Mh) { return ((size_t)PR * D + 2 * PR * Mh + 2 * PR + 2 * D) * sizeof(float); }
// rows per group: 16 where that fits the 160 KB of LDS, else 8
static int pool_pr(int D, int Mh) { return pool_lds(PR_WIDE, D, Mh) <= 160 * 1024 ? PR_WIDE : PR_NARROW; }

template <typename K>
static hipError_t set_lds(K kernel, size_t bytes) {
  if (bytes <= 65536) return hipSuccess;
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

hipError_t launch_pool_fwd(const PoolArgs& p0, hipStream_t s) {
  PoolArgs p = p0;
  const int pr = pool_pr(p.D, p.Mh);
  size_t lds = pool_lds(pr, p.D, p.Mh);
  hipError_t e;
  if (p.use_mfma && pool_mfma_ok(p)) {
    // persistent grid: one workgroup per compute unit (it owns almost all of the unit's LDS)
    static int cus = 0;
    if (!cus) {
      int dev = 0;
      hipDeviceProp_t prop;
      if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
      if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
      cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
    }
    int rb = pool_mfma_rows(p);
    long long groups = (p.N + rb - 1) / rb;
    p.blocks = (int)(groups < cus ? groups : cus);
    if (p.blocks > 1024) p.blocks = 1024;
    if ((e = launch_pool_gate_part_mfma(p, s)) != hipSuccess) return e;
  } else {
    if (pr == PR_WIDE) {
      if ((e = set_lds(pool_gate_part_k<PR_WIDE>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL(pool_gate_part_k<PR_WIDE>, dim3(p.blocks), dim3(256), lds, s, p);
    } else {
      if ((e = set_lds(pool_gate_part_k<PR_NARROW>, lds)) != hipSuccess) return e;
      hipLaunchKernelGGL(pool_gate_part_k<PR_NARROW>, dim3(p.blocks), dim3(256), lds, s, p);
    }
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (p.blocks > 1024) return hipErrorInvalidValue;
  hipLaunchKernelGGL(pool_combine_z_k, dim3((unsigned)((p.D + 15) / 16)), dim3(256), 0, s, p);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(pool_combine_k, dim3(1), dim3(256), 0, s, p);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (p.alpha) {
    hipLaunchKernelGGL(pool_alpha_k, dim3((unsigned)((p.N + 255) / 256)), dim3(256), 0, s, p.a, p.scal, p.alpha, p.N);
    e = hipGetLastError();
  }
  return e;
}

hipError_t launch_pool_bwd_rows(const PoolArgs& p, float* Dp, hipStream_t s) {
  const int pr = pool_pr(p.D, p.Mh);
  size_t lds = pool_lds(pr, p.D, p.Mh);
  hipError_t e;
  if (pr == PR_WIDE) {
    if ((e = set_lds(pool_bwd_rows_k<PR_WIDE>, lds)) != hipSuccess) return e;
    hipLaunchKernelGGL(pool_bwd_rows_k<PR_WIDE>, dim3(p.blocks), dim3(256), lds, s, p, Dp);
  } else {
    if ((e = set_lds(pool_bwd_rows_k<PR_NARROW>, lds)) != hipSuccess) return e;
    hipLaunchKernelGGL(pool_bwd_rows_k<PR_NARROW>, dim3(p.blocks), dim3(256), lds, s, p, Dp);
  }
  if ((e = hipGetLastError()) != hipSuccess) return e;
  return launch_pool_head_grads(p, s);
}

hipError_t launch_pool_head_grads(const PoolArgs& p, hipStream_t s) {
  hipLaunchKernelGGL(pool_head_grads_k, dim3(4), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace sl
