// Gated-attention MIL pooling, backward over the feature rows on the matrix cores (gfx950, bf16 path, the shape
// whose gate weights fit the register file: D = 384, M_h = 128; M_h = 256 runs as two such halves of the gate units).
//
// Per feature row h_n (attention logit a_n saved by the forward; m, Z, z, dz from the combine kernel):
//   alpha_n = exp(a_n - m) / Z,   da_n = alpha_n * dz . (h_n - z)
//   t = tanh(V h_n + b_V), s = sigmoid(U h_n + b_U)
//   dpV = da_n w s (1 - t^2),  dpU = da_n w t s (1 - s),  dw += da_n t s,  db_V += dpV,  db_U += dpU
//   G_n = alpha_n dz + [dpV dpU] [V;U]          dV += dpV (x) h_n,  dU += dpU (x) h_n
// Three contractions with three different contracted indices, and [V;U] (192 KB as bf16) fills the register file in
// one orientation only, so the work is two passes over the rows plus the ordinary weight-gradient GEMM:
//   pass 1: gate GEMM (weights as MFMA operands in registers, as in the forward), the row dot products from the fp32
//           registers, the elementwise gradients; writes [dpV dpU] and the features as bf16 and sums dw (db_V and
//           db_U are column sums of the written array, taken by the weight-gradient GEMM).
//   pass 2: G = alpha dz + [dpV dpU] [V;U] with the transposed weights in registers; rows are the M index so that a
//           lane owns a column of G and every store instruction writes whole 128-byte lines.
//   dV, dU: large-M TN GEMM of the two bf16 arrays written by pass 1.
#include "slide_internal.h"

namespace sl {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

template <int V>
struct IC { static constexpr int value = V; };
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(IC<I>{});
    static_for<I + 1, N>(f);
  }
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// out[d][u] (bf16, [D][2 Mh]) = u < Mh ? V[u][d] : U[u - Mh][d]
__global__ void __launch_bounds__(256) pool_cast_vut_k(const float* __restrict__ V, const float* __restrict__ U,
                                                       bf16* __restrict__ out, int Mh, int D) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)D * 2 * Mh) return;
  int d = (int)(i / (2 * Mh)), u = (int)(i % (2 * Mh));
  out[i] = (bf16)(u < Mh ? V[(size_t)u * D + d] : U[(size_t)(u - Mh) * D + d]);
}

// out (bf16, [2 Mh][D]) = [V; U]
__global__ void __launch_bounds__(256) pool_cast_vu2_k(const float* __restrict__ V, const float* __restrict__ U,
                                                       bf16* __restrict__ out, long long n) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) { out[i] = (bf16)V[i]; out[n + i] = (bf16)U[i]; }
}

// Pass 1.  Same skeleton as the forward kernel with register-resident weights: persistent workgroups of 4
// wavefronts over blocks of 32 rows, a wavefront owns 32 gate units, a thread owns 4 rows x 12 columns of every block
// in fp32 registers (two sets), LDS holds the bf16 image of the block for the MFMA fragments.
//   Dp  [N][2 Mh] bf16: dpV | dpU     Hb16 [N][D] bf16: the features
//   csp [gridDim.x][Mh] fp32: this workgroup's sum of da t s (dw)
template <int D, int MH>
__global__ void __launch_bounds__(256) pool_bwd_gate_k(PoolArgs p, const bf16* __restrict__ VU, bf16* __restrict__ Dp,
                                                       bf16* __restrict__ Hb16, float* __restrict__ csp) {
  constexpr int RB = 32, LDB = D + 8, KS = D / 16, CJ = D / 128, NR = 4 * CJ, KU = 2 * MH, LDP = KU + 8;
  static_assert(MH == 128 && D % 128 == 0, "shape");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Hb = reinterpret_cast<bf16*>(smem);                            // [2][RB][LDB]
  bf16* Dps = Hb + 2 * RB * LDB;                                       // [RB][LDP]
  float* gb = reinterpret_cast<float*>(Dps + RB * LDP);                // scaled bV[MH], scaled bU[MH], w[MH]
  float* dotr = gb + 3 * MH;                                           // [RB] dz . (h_n - z)
  float* zds = dotr + RB;                                              // z[D], dz[D]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, h2 = lane >> 5;
  const int rgrp = tid >> 5, cl = tid & 31;   // loads: rows 4 rgrp .. + 3 of a block, column groups cl + 32 j
  const float* H = p.H;
  const long long groups = (p.N + RB - 1) / RB;
  constexpr float C1 = -2.0f * 1.44269504088896f, C2 = -1.44269504088896f;   // exp(-2x) and exp(-x) as exp2
  const float m = p.scal[0], Zinv = 1.0f / p.scal[1];

  for (int j = tid; j < MH; j += 256) { gb[j] = C1 * p.Vb[j]; gb[MH + j] = C2 * p.Ub[j]; gb[2 * MH + j] = p.w[j]; }
  bf16x8 wv[KS], wu[KS];
  {
    const bf16* wr = VU + (size_t)(32 * wave + li) * D + h2 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 a = *reinterpret_cast<const u32x4*>(wr + ks * 16);
      u32x4 b = *reinterpret_cast<const u32x4*>(wr + (size_t)MH * D + ks * 16);
      asm volatile("" : "+a"(a), "+a"(b));   // accumulation half of the register file, read by the MFMA directly
      wv[ks] = __builtin_bit_cast(bf16x8, a);
      wu[ks] = __builtin_bit_cast(bf16x8, b);
    }
  }
  // z = zv + zlo to fp64 accuracy; the zlo part of the dot product is a constant of the thread's 12 columns
  float kz = 0.f;
  {
    const float* zv = p.scal + 4 + 2 * p.C;
    const float* dz = zv + D;
    const float* zlo = dz + D;
    for (int d = tid; d < D; d += 256) { zds[d] = zv[d]; zds[D + d] = dz[d]; }
#pragma unroll
    for (int j = 0; j < CJ; ++j)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int col = (cl + 32 * j) * 4 + c;
        kz = fmaf(zlo[col], dz[col], kz);
      }
  }
  float4 ra[NR], rb[NR];
  auto issue_h = [&](float4 (&r)[NR], long long g) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      long long row = g * RB + 4 * rgrp + k;   // past the end: the last row again (its alpha is set to zero)
      row = row < p.N ? row : p.N - 1;
      const float* hr = H + row * D + cl * 4;
#pragma unroll
      for (int j = 0; j < CJ; ++j) r[k * CJ + j] = *reinterpret_cast<const float4*>(hr + j * 128);
    }
  };
  // one of the NR loads of block g (i = k * CJ + j); spread over the MFMA loop: issued as one burst they hold the
  // wavefronts in the issue for the ~770 clocks the address unit needs for a block's 48 KB
  const float* hrp = H;   // row base of the loads in progress
  auto issue_one = [&](float4 (&r)[NR], long long g, auto ic) __attribute__((always_inline)) {
    constexpr int i = decltype(ic)::value, k = i / CJ, j = i % CJ;
    if constexpr (j == 0) {
      long long row = g * RB + 4 * rgrp + k;
      row = row < p.N ? row : p.N - 1;
      hrp = H + row * D + cl * 4;
    }
    r[i] = *reinterpret_cast<const float4*>(hrp + j * 128);
  };
  // bf16 image of block g: to LDS for the MFMA, and to the bf16 feature copy the weight-gradient GEMM reads
  auto stash_h = [&](const float4 (&r)[NR], int buf, long long g) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const long long row = g * RB + 4 * rgrp + k;
#pragma unroll
      for (int j = 0; j < CJ; ++j) {
        float4 v = r[k * CJ + j];
        uint2 w2;
        w2.x = pack_bf16(v.x, v.y);
        w2.y = pack_bf16(v.z, v.w);
        *reinterpret_cast<uint2*>(Hb + (buf * RB + 4 * rgrp + k) * LDB + (cl + 32 * j) * 4) = w2;
        if (row < p.N) *reinterpret_cast<uint2*>(Hb16 + row * D + (cl + 32 * j) * 4) = w2;
      }
    }
  };
  float sW[16];   // sum over this lane's rows of da t s, per gate unit of the accumulator layout
#pragma unroll
  for (int i = 0; i < 16; ++i) sW[i] = 0.f;
  auto block = [&](float4 (&cur)[NR], float4 (&nxt)[NR], int buf, long long gi) __attribute__((always_inline)) {
    const long long n0 = gi * RB;
    const bool ok = n0 + li < p.N;
    const float a_n = p.a[ok ? n0 + li : p.N - 1];
    // dz . (h - z) of this thread's 4 rows over its 12 columns, then over the 32 threads that share the rows
    {
      float pd[4] = {-kz, -kz, -kz, -kz};
#pragma unroll
      for (int j = 0; j < CJ; ++j) {
        const float4 zc = *reinterpret_cast<const float4*>(zds + (cl + 32 * j) * 4);
        const float4 dc = *reinterpret_cast<const float4*>(zds + D + (cl + 32 * j) * 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float4 v = cur[k * CJ + j];
          float s = pd[k];
          s = fmaf(v.x - zc.x, dc.x, s);
          s = fmaf(v.y - zc.y, dc.y, s);
          s = fmaf(v.z - zc.z, dc.z, s);
          s = fmaf(v.w - zc.w, dc.w, s);
          pd[k] = s;
        }
      }
#pragma unroll
      for (int o = 1; o < 32; o <<= 1)
#pragma unroll
        for (int k = 0; k < 4; ++k) pd[k] += __shfl_xor(pd[k], o, 64);
      if (cl < 4) dotr[4 * rgrp + cl] = cl == 0 ? pd[0] : cl == 1 ? pd[1] : cl == 2 ? pd[2] : pd[3];
    }
    f32x16 av, au;
#pragma unroll
    for (int r = 0; r < 16; ++r) { av[r] = 0.f; au[r] = 0.f; }
    const bf16* hrow = Hb + (buf * RB + li) * LDB + h2 * 8;
    constexpr int PF = 4;
    u32x4 hf[PF];
#pragma unroll
    for (int ks = 0; ks < PF; ++ks) hf[ks] = *reinterpret_cast<const u32x4*>(hrow + ks * 16);
    static_for<0, KS>([&](auto kc) __attribute__((always_inline)) {
      constexpr int ks = decltype(kc)::value;
      bf16x8 f = __builtin_bit_cast(bf16x8, hf[ks % PF]);
      if constexpr (ks + PF < KS) hf[ks % PF] = *reinterpret_cast<const u32x4*>(hrow + (ks + PF) * 16);
      if constexpr (ks % 2 == 0 && ks / 2 < NR) issue_one(nxt, gi + (long long)gridDim.x, IC<ks / 2>{});
      av = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[ks], f, av, 0, 0, 0);
      au = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wu[ks], f, au, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
    __syncthreads();   // (A) the row dot products are there; the previous block's gradient image has been copied out
    {
      // lane = feature row li; accumulator register r = gate unit (r / 4) * 8 + h2 * 4 + r % 4 of the wave's 32
      const float alpha = ok ? __expf(a_n - m) * Zinv : 0.f;
      const float da = alpha * dotr[li];
      bf16* prow = Dps + li * LDP + 32 * wave + h2 * 4;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int j = 32 * wave + q * 8 + h2 * 4;
        float4 bv = *reinterpret_cast<const float4*>(gb + j);
        float4 bu = *reinterpret_cast<const float4*>(gb + MH + j);
        float4 wj = *reinterpret_cast<const float4*>(gb + 2 * MH + j);
        float bvv[4] = {bv.x, bv.y, bv.z, bv.w}, buu[4] = {bu.x, bu.y, bu.z, bu.w}, ww[4] = {wj.x, wj.y, wj.z, wj.w};
        float dv[4], du[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // t = tanh(xv) = (1 - e1) / (1 + e1), s = sigmoid(xu) = 1 / (1 + e2), e1 = exp(-2 xv), e2 = exp(-xu)
          float e1 = __builtin_amdgcn_exp2f(fminf(fmaf(av[4 * q + e], C1, bvv[e]), 57.f));
          float e2 = __builtin_amdgcn_exp2f(fminf(fmaf(au[4 * q + e], C2, buu[e]), 57.f));
          float t = (1.0f - e1) * __builtin_amdgcn_rcpf(1.0f + e1);
          float s = __builtin_amdgcn_rcpf(1.0f + e2);
          float ts = t * s, gw = da * ww[e];
          dv[e] = gw * s * fmaf(-t, t, 1.0f);
          du[e] = gw * ts * (1.0f - s);
          sW[4 * q + e] = fmaf(da, ts, sW[4 * q + e]);
        }
        uint2 pv, pu;
        pv.x = pack_bf16(dv[0], dv[1]); pv.y = pack_bf16(dv[2], dv[3]);
        pu.x = pack_bf16(du[0], du[1]); pu.y = pack_bf16(du[2], du[3]);
        *reinterpret_cast<uint2*>(prow + q * 8) = pv;
        *reinterpret_cast<uint2*>(prow + MH + q * 8) = pu;
      }
    }
    stash_h(nxt, buf ^ 1, gi + (long long)gridDim.x);  // the next block (loaded during the previous one)
    __syncthreads();   // (B) the gradient image and the next bf16 image are visible; dotr is free again
    // gradient image -> Dp: 32 threads write one row of 512 bytes
#pragma unroll
    for (int i = 0; i < RB * KU / 8 / 256; ++i) {
      int ch = tid + 256 * i, row = ch / (KU / 8), c16 = ch % (KU / 8);
      if (n0 + row < p.N)
        *reinterpret_cast<u32x4*>(Dp + (n0 + row) * KU + c16 * 8) =
            *reinterpret_cast<const u32x4*>(Dps + row * LDP + c16 * 8);
    }
  };

  long long gi = blockIdx.x;
  const long long st = gridDim.x;
  issue_h(ra, gi);
  stash_h(ra, 0, gi);
  __syncthreads();
  while (true) {
    if (gi >= groups) break;
    block(ra, rb, 0, gi);
    gi += st;
    if (gi >= groups) break;
    block(rb, ra, 1, gi);
    gi += st;
  }
  // dw: sum over the rows (the 32 lanes of a half hold the same gate units)
#pragma unroll
  for (int o = 1; o < 32; o <<= 1)
#pragma unroll
    for (int i = 0; i < 16; ++i) sW[i] += __shfl_xor(sW[i], o, 64);
  if (li == 0) {
    float* out = csp + (size_t)blockIdx.x * MH + 32 * wave + h2 * 4;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) out[q * 8 + e] = sW[4 * q + e];
  }
}

// Pass 2.  G[n][d] = alpha_n dz[d] + sum_u Dp[n][u] VUT[d][u]; with ADD the first term is what G already holds (the
// second half of the gate units when M_h = 256 is taken as two halves).  A wavefront holds the transposed weights of its
// D / 4 columns (3 tiles of 32 x 256: 192 registers); the block's gradient rows go through LDS (double buffered, the
// next block in flight in registers).  Rows are the M index: accumulator register r of a lane is row
// (r / 4) * 8 + h2 * 4 + r % 4, the lane is the column, so a store instruction writes two 128-byte lines.
template <int D, int MH, bool ADD>
__global__ void __launch_bounds__(256) pool_bwd_g_k(PoolArgs p, const bf16* __restrict__ VUT,
                                                    const bf16* __restrict__ Dp) {
  constexpr int RB = 32, KU = 2 * MH, KS = KU / 16, LDP = KU + 8, NT = D / 128, CH = RB * KU / 8 / 256, LDG = 2 * MH;
  static_assert(MH == 128 && D % 128 == 0, "shape");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Dps = reinterpret_cast<bf16*>(smem);                           // [2][RB][LDP]
  float* als = reinterpret_cast<float*>(Dps + 2 * RB * LDP);           // [2][RB] alpha
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, h2 = lane >> 5;
  const long long groups = (p.N + RB - 1) / RB;
  const float m = p.scal[0], Zinv = 1.0f / p.scal[1];
  const int dcol = (D / 4) * wave + li;   // + 32 t
  bf16x8 wt[NT][KS];
  float dzr[NT];
  {
    const float* dz = p.scal + 4 + 2 * p.C + D;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      dzr[t] = dz[dcol + 32 * t];
      const bf16* wr = VUT + (size_t)(dcol + 32 * t) * KU + h2 * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4 a = *reinterpret_cast<const u32x4*>(wr + ks * 16);
        asm volatile("" : "+a"(a));   // accumulation half of the register file, read by the MFMA directly
        wt[t][ks] = __builtin_bit_cast(bf16x8, a);
      }
    }
  }
  u32x4 rp[CH];
  float ra = 0.f;
  auto issue_one = [&](long long g, auto ic) __attribute__((always_inline)) {
    constexpr int i = decltype(ic)::value;
    if constexpr (i < CH) {
      int ch = tid + 256 * i, row = ch / (KU / 8), c16 = ch % (KU / 8);
      long long gr = g * RB + row;   // past the end: the last row again (never stored)
      gr = gr < p.N ? gr : p.N - 1;
      rp[i] = *reinterpret_cast<const u32x4*>(Dp + gr * LDG + c16 * 8);
    } else if (tid < RB) {
      long long gr = g * RB + tid;
      ra = p.a[gr < p.N ? gr : p.N - 1];
    }
  };
  auto issue = [&](long long g) __attribute__((always_inline)) {
    static_for<0, CH + 1>([&](auto ic) __attribute__((always_inline)) { issue_one(g, ic); });
  };
  auto stash = [&](int buf, long long g) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      int ch = tid + 256 * i, row = ch / (KU / 8), c16 = ch % (KU / 8);
      *reinterpret_cast<u32x4*>(Dps + (buf * RB + row) * LDP + c16 * 8) = rp[i];
    }
    if (tid < RB) als[buf * RB + tid] = g * RB + tid < p.N ? __expf(ra - m) * Zinv : 0.f;
  };

  long long gi = blockIdx.x;
  const long long st = gridDim.x;
  issue(gi);
  stash(0, gi);
  __syncthreads();
  for (int buf = 0; gi < groups; gi += st, buf ^= 1) {
    const long long n0 = gi * RB;
    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    const bf16* prow = Dps + (buf * RB + li) * LDP + h2 * 8;
    constexpr int PF = 4;
    u32x4 pf[PF];
#pragma unroll
    for (int ks = 0; ks < PF; ++ks) pf[ks] = *reinterpret_cast<const u32x4*>(prow + ks * 16);
    static_for<0, KS>([&](auto kc) __attribute__((always_inline)) {
      constexpr int ks = decltype(kc)::value;
      bf16x8 f = __builtin_bit_cast(bf16x8, pf[ks % PF]);
      if constexpr (ks + PF < KS) pf[ks % PF] = *reinterpret_cast<const u32x4*>(prow + (ks + PF) * 16);
      // the next block's loads, spread over the loop
      if constexpr (ks % 2 == 0 && ks / 2 < CH + 1) issue_one(gi + st, IC<ks / 2>{});
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, wt[t][ks], acc[t], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
    float al[16];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      float4 v = *reinterpret_cast<const float4*>(als + buf * RB + q * 8 + h2 * 4);
      al[4 * q + 0] = v.x; al[4 * q + 1] = v.y; al[4 * q + 2] = v.z; al[4 * q + 3] = v.w;
    }
    float* gout = p.G + n0 * D + dcol;
    if (n0 + RB <= p.N) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float* o = gout + (size_t)((r / 4) * 8 + h2 * 4 + r % 4) * D + 32 * t;
          *o = ADD ? *o + acc[t][r] : fmaf(al[r], dzr[t], acc[t][r]);
        }
    } else {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int row = (r / 4) * 8 + h2 * 4 + r % 4;
          float* o = gout + (size_t)row * D + 32 * t;
          if (n0 + row < p.N) *o = ADD ? *o + acc[t][r] : fmaf(al[r], dzr[t], acc[t][r]);
        }
    }
    stash(buf ^ 1, gi + st);     // the next block (loaded during this one)
    __syncthreads();             // the next gradient image and its alpha are visible
  }
}

}  // namespace

bool pool_bwd_mfma_ok(const PoolArgs& p) {
  return p.use_mfma && pool_mfma_ok(p) && p.D == 384 && (p.Mh == 128 || p.Mh == 256);
}

int pool_bwd_mfma_blocks(const PoolArgs& p) {
  static int cus = 0;
  if (!cus) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 1;
    cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
  }
  long long groups = (p.N + 31) / 32;
  long long b = groups < cus ? groups : cus;
  return (int)(b > 1024 ? 1024 : b);
}

// Dp: [N][2 Mh] bf16, Hb16: [N][D] bf16, csp: [pool_bwd_mfma_blocks][Mh] fp32 partial sums of dw.  p.vub has room for two
// bf16 copies of [V;U] (plain and transposed).
// M_h = 256 does not fit the register file (2 M_h D bf16 = 384 KB) and is taken as two halves of 128 gate units, which
// are independent given the softmax gradient of the row: each half is the M_h = 128 problem on its rows of V, U, b_V, b_U
// and w; the second half adds its part of G to the first's.  Then Dp is [2][N][256] (half h: dpV | dpU of its units),
// csp [2][blocks][128], and the feature copy is written twice.
hipError_t launch_pool_bwd_mfma(const PoolArgs& p0, void* Dp, void* Hb16, float* csp, hipStream_t s) {
  constexpr int D = 384, MH = 128;
  if (!pool_bwd_mfma_ok(p0)) return hipErrorInvalidValue;
  const int blocks = pool_bwd_mfma_blocks(p0);
  const int halves = p0.Mh / MH;
  hipError_t e;
  for (int h = 0; h < halves; ++h) {
    PoolArgs p = p0;
    p.Mh = MH;
    p.VW = p0.VW + (size_t)h * MH * D; p.UW = p0.UW + (size_t)h * MH * D;
    p.Vb = p0.Vb + h * MH; p.Ub = p0.Ub + h * MH; p.w = p0.w + h * MH;
    bf16* vu = (bf16*)p0.vub + (size_t)h * 2 * (2 * MH * D);
    bf16* vut = vu + (size_t)2 * MH * D;
    bf16* dp = (bf16*)Dp + (size_t)h * p0.N * 2 * MH;
    const long long n = (long long)MH * D;
    hipLaunchKernelGGL(pool_cast_vu2_k, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p.VW, p.UW, vu, n);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    hipLaunchKernelGGL(pool_cast_vut_k, dim3((unsigned)((2 * MH * D + 255) / 256)), dim3(256), 0, s, p.VW, p.UW, vut, MH, D);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    {
      auto kern = pool_bwd_gate_k<D, MH>;
      size_t lds = (size_t)2 * 32 * (D + 8) * 2 + (size_t)32 * (2 * MH + 8) * 2 + (size_t)3 * MH * 4 + 32 * 4 + 2 * D * 4;
      if ((e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) != hipSuccess)
        return e;
      hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, s, p, (const bf16*)vu, dp, (bf16*)Hb16,
                         csp + (size_t)h * blocks * MH);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    {
      size_t lds = (size_t)2 * 32 * (2 * MH + 8) * 2 + (size_t)2 * 32 * 4;
      auto k0 = pool_bwd_g_k<D, MH, false>;
      auto k1 = pool_bwd_g_k<D, MH, true>;
      auto kern = h == 0 ? k0 : k1;
      if ((e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) != hipSuccess)
        return e;
      hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, s, p, (const bf16*)vut, (const bf16*)dp);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

}  // namespace sl
