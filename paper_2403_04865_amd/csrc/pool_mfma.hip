// Gated-attention MIL pooling, forward stage 1 on the matrix cores (gfx950, bf16 path).
//
// a_n = w . (tanh(V h_n + b_V) * sigmoid(U h_n + b_U)) needs 4 * M_h * D flop per feature row of D * 4 bytes:
// 128 flop/byte at M_h = 128, far more than the vector ALUs deliver at HBM speed, so the two projections are one
// bf16 MFMA GEMM [rows] x [V;U]^T with fp32 accumulation.  Everything else stays fp32 / fp64 on the
// unrounded features: the softmax over tiles is a two-level online reduction (every workgroup keeps a running
// max, sum and weighted feature sum over its row blocks; one workgroup combines them afterwards).
// Two kernels:
//   * pool_gate_part_reg_k (D = 384, M_h = 128; M_h = 256 as two passes over halves of the gate units above
//     32768 rows): the main one.  One persistent workgroup (4 wavefronts) per compute unit; the bf16 copy of
//     [V;U] is 192 kB, which is what the accumulation half of a compute unit's register file holds, so every
//     wavefront keeps the fragments of its 32 gate units in registers for the whole kernel and the only traffic is
//     the feature rows, each read from HBM exactly once into fp32 registers (a bf16 image in LDS feeds the MFMAs;
//     the weighted feature sum is taken from the unrounded registers).  The gate arithmetic of block i - 1 is
//     issued between the MFMAs of block i.
//   * pool_gate_part_mfma_k (the other built shapes: M_h = 256 below 32768 rows, D = 768): rows in LDS as fp32,
//     [V;U] streams from L2 through a double-buffered LDS ring, BK columns per step.
//   Operands are passed swapped (weights first): a lane then owns one feature row and 16 gate units per
//   accumulator, so the sum over gate units is in-lane plus one exchange between the lane halves.
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

__device__ __forceinline__ bf16x8 cvt8(float4 a, float4 b) {
  f32x2 p0 = {a.x, a.y}, p1 = {a.z, a.w}, p2 = {b.x, b.y}, p3 = {b.z, b.w};
  bf16x2 h0 = __builtin_convertvector(p0, bf16x2), h1 = __builtin_convertvector(p1, bf16x2);
  bf16x2 h2 = __builtin_convertvector(p2, bf16x2), h3 = __builtin_convertvector(p3, bf16x2);
  bf16x8 r = {h0[0], h0[1], h1[0], h1[1], h2[0], h2[1], h3[0], h3[1]};
  return r;
}

// [V;U] fp32 -> bf16, rows 0..Mh-1 = V, Mh..2Mh-1 = U
__global__ void __launch_bounds__(256) pool_cast_vu_k(const float* __restrict__ V, const float* __restrict__ U,
                                                      bf16* __restrict__ out, long long n) {
  long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) { out[i] = (bf16)V[i]; out[n + i] = (bf16)U[i]; }
}

template <int RB, int MH, int BK>
struct PoolCfg {
  static constexpr int RG = RB / 32;          // row groups of 32 (wavefronts along the rows)
  static constexpr int JG = 4 / RG;           // wavefronts along the gate units
  static constexpr int JW = MH / JG;          // gate units per wavefront
  static constexpr int NBK = JW / 32;         // 32 x 32 accumulators per wavefront for V (and as many for U)
  static constexpr int LDW = BK + 8;          // LDS row stride of the weight ring (bf16)
  static constexpr int WCH = 2 * MH * (BK / 8) / 256;  // 16-byte weight chunks per thread and step
  static_assert(JW % 32 == 0 && WCH >= 1, "shape");
  static size_t lds_bytes(int D) {
    return (size_t)RB * (D + 4) * 4 + (size_t)2 * 2 * MH * LDW * 2 + (size_t)D * 8 + (size_t)3 * MH * 4 +
           (size_t)JG * RB * 4 + (size_t)RB * 4 + 64;
  }
};

template <int RB, int MH, int BK, int HCH>   // HCH: float4 chunks of the row block per thread (RB * D / 1024)
__global__ void __launch_bounds__(256) pool_gate_part_mfma_k(PoolArgs p, const bf16* __restrict__ VU) {
  using C = PoolCfg<RB, MH, BK>;
  constexpr int LDW = C::LDW, NBK = C::NBK, JW = C::JW;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int D = p.D, LDH = D + 4;
  float* Hs = reinterpret_cast<float*>(smem);                          // [RB][LDH]
  bf16* Ws = reinterpret_cast<bf16*>(Hs + RB * LDH);                   // [2][2 MH][LDW]
  double* zb = reinterpret_cast<double*>(Ws + 2 * 2 * MH * LDW);       // [D]
  float* gb = reinterpret_cast<float*>(zb + D);                        // bV[MH], bU[MH], w[MH]
  float* apart = gb + 3 * MH;                                          // [JG][RB]
  float* er = apart + C::JG * RB;                                      // [RB]
  float* misc = er + RB;                                               // run_m, resc; run_l as double behind
  double* run_l = reinterpret_cast<double*>(misc + 2);

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rg = wave % C::RG, jg = wave / C::RG;
  const int li = lane & 31, h2 = lane >> 5;
  const int nk = D / BK;
  const float* H = p.H;
  const long long total = p.N * (long long)D;   // feature elements

  for (int d = tid; d < D; d += 256) zb[d] = 0.0;
  for (int j = tid; j < MH; j += 256) { gb[j] = p.Vb[j]; gb[MH + j] = p.Ub[j]; gb[2 * MH + j] = p.w[j]; }
  if (tid == 0) { misc[0] = -INFINITY; misc[1] = 0.f; *run_l = 0.0; }

  const long long groups = (p.N + RB - 1) / RB;
  // weight ring loader: chunk c = tid + i * 256 -> row c / (BK / 8), 16-byte column c % (BK / 8)
  u32x4 rw[C::WCH];
  auto issue_w = [&](int kt) {
#pragma unroll
    for (int i = 0; i < C::WCH; ++i) {
      int c = tid + i * 256;
      int row = c / (BK / 8), kc = c % (BK / 8);
      rw[i] = *reinterpret_cast<const u32x4*>(VU + (size_t)row * D + kt * BK + kc * 8);
    }
  };
  auto stash_w = [&](int buf) {
#pragma unroll
    for (int i = 0; i < C::WCH; ++i) {
      int c = tid + i * 256;
      int row = c / (BK / 8), kc = c % (BK / 8);
      *reinterpret_cast<u32x4*>(Ws + ((size_t)buf * 2 * MH + row) * LDW + kc * 8) = rw[i];
    }
  };
  // feature block loader: the block is one contiguous span of RB * D floats
  float4 rh[HCH];
  auto issue_h = [&](long long g) {
    long long e0 = g * RB * (long long)D;
#pragma unroll
    for (int i = 0; i < HCH; ++i) {
      long long e = e0 + (long long)(tid + i * 256) * 4;
      rh[i] = e < total ? *reinterpret_cast<const float4*>(H + e) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto stash_h = [&]() {
    int q4 = D / 4;
#pragma unroll
    for (int i = 0; i < HCH; ++i) {
      int c = tid + i * 256;
      int row = c / q4, col = (c - row * q4) * 4;
      *reinterpret_cast<float4*>(Hs + row * LDH + col) = rh[i];
    }
  };

  long long gi = blockIdx.x;
  if (gi < groups) issue_h(gi);
  issue_w(0);
  __syncthreads();
  for (; gi < groups; gi += gridDim.x) {
    const long long n0 = gi * RB;
    stash_h();
    long long gnext = gi + gridDim.x;
    if (gnext < groups) issue_h(gnext);   // in flight during the whole block

    f32x16 acc[2 * NBK];
#pragma unroll
    for (int b = 0; b < 2 * NBK; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[b][r] = 0.f;

    for (int kt = 0; kt < nk; ++kt) {
      int buf = kt & 1;
      stash_w(buf);
      issue_w(kt + 1 < nk ? kt + 1 : 0);
      __syncthreads();   // ring stage (and, at kt == 0, the feature block) visible; the other stage is free
      const float* hrow = Hs + (rg * 32 + li) * LDH + kt * BK + h2 * 8;
      const bf16* wbase = Ws + (size_t)buf * 2 * MH * LDW + h2 * 8;
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        float4 a = *reinterpret_cast<const float4*>(hrow + ks * 16);
        float4 b4 = *reinterpret_cast<const float4*>(hrow + ks * 16 + 4);
        bf16x8 hf = cvt8(a, b4);
#pragma unroll
        for (int b = 0; b < 2 * NBK; ++b) {
          int row = (b < NBK ? 0 : MH) + jg * JW + (b % NBK) * 32 + li;
          bf16x8 wf = *reinterpret_cast<const bf16x8*>(wbase + row * LDW + ks * 16);
          acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, hf, acc[b], 0, 0, 0);
        }
      }
    }
    // gate: lane = feature row rg * 32 + li; accumulator register r = gate unit (r / 4) * 8 + h2 * 4 + r % 4 of its block
    float part = 0.f;
#pragma unroll
    for (int b = 0; b < NBK; ++b)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        int j = jg * JW + b * 32 + q * 8 + h2 * 4;
        float4 bv = *reinterpret_cast<const float4*>(gb + j);
        float4 bu = *reinterpret_cast<const float4*>(gb + MH + j);
        float4 wj = *reinterpret_cast<const float4*>(gb + 2 * MH + j);
        float bvv[4] = {bv.x, bv.y, bv.z, bv.w}, buu[4] = {bu.x, bu.y, bu.z, bu.w}, ww[4] = {wj.x, wj.y, wj.z, wj.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float xv = acc[b][4 * q + e] + bvv[e], xu = acc[NBK + b][4 * q + e] + buu[e];
          // tanh(xv) * sigmoid(xu) = (1 - e1) / ((1 + e1) (1 + e2)), e1 = exp(-2 xv), e2 = exp(-xu)
          float e1 = __expf(fminf(-2.0f * xv, 40.f)), e2 = __expf(fminf(-xu, 40.f));
          part += ww[e] * ((1.0f - e1) * __builtin_amdgcn_rcpf((1.0f + e1) * (1.0f + e2)));
        }
      }
    part += __shfl_xor(part, 32, 64);
    if (h2 == 0) apart[jg * RB + rg * 32 + li] = part;
    __syncthreads();
    if (tid < 64) {   // wavefront 0: logits of the block, online softmax state
      float a = 0.f;
      if (tid < RB) {
#pragma unroll
        for (int j = 0; j < C::JG; ++j) a += apart[j * RB + tid];
      }
      bool ok = tid < RB && n0 + tid < p.N;
      if (ok) p.a[n0 + tid] = a;
      a = ok ? a : -INFINITY;
      float m_old = misc[0];
      float m = fmaxf(m_old, wave_max(a));   // finite: the block has at least one row
      float e = __expf(a - m);
      if (tid < RB) er[tid] = e;
      float es = wave_sum(e);
      if (tid == 0) {
        float sc = __expf(m_old - m);   // exp(-inf) = 0 on the first block
        misc[0] = m; misc[1] = sc;
        *run_l = *run_l * (double)sc + (double)es;
      }
    }
    __syncthreads();
    {
      float sc = misc[1];
      for (int d = tid; d < D; d += 256) {
        double z = zb[d] * (double)sc;
#pragma unroll 8
        for (int r = 0; r < RB; ++r) z += (double)er[r] * (double)Hs[r * LDH + d];
        zb[d] = z;
      }
    }
    __syncthreads();   // the feature block and er are free again
  }
  double* out = p.part + (size_t)blockIdx.x * (2 + D);
  if (tid == 0) { out[0] = (double)misc[0]; out[1] = *run_l; }
  for (int d = tid; d < D; d += 256) out[2 + d] = zb[d];
}

// Variant for the shape whose [V;U] fits the register file (D = 384, M_h = 128: 2 M_h * D bf16 = 192 KB, 192
// registers per lane): each wavefront holds the MFMA fragments of its 32 gate units for the whole kernel, so the only
// traffic per block of 32 feature rows is the block itself (the kernel above re-reads the weights from L2 for every
// block, twice the bytes of the features).
//   * A thread owns 4 rows x 12 columns of every block (fixed columns), in fp32 registers.  LDS holds only the bf16
//     image of a block (double buffered) for the MFMA fragments; the weighted feature sum is taken from the fp32
//     registers: per lane in fp32 (4 rows per block, a few thousand terms at most), over row groups and workgroups
//     in fp64 (z feeds a cancelling difference in the backward).
//   * The gate of block i - 1 runs under the MFMAs of block i inside each wavefront (the matrix pipe and the vector
//     ALU are separate, and with one wavefront per SIMD nothing else overlaps them).  The pre-activations of two
//     blocks are alive (two accumulator sets), and the softmax terms, hence the weighted sum, of a block come one
//     iteration after its MFMAs: three fp32 row sets rotate (block i - 1 waiting for its weights, block i whose bf16
//     image is being multiplied, block i + 1 in flight).  The set that the weighted sum frees takes the first loads
//     of block i + 2 at once.  The roles repeat every 6 iterations (2 images x 3 row sets), which are written out.
//   * Every wavefront computes the block's softmax terms itself from the four partial logits (no serial section).
//   * Two barriers per block: partial logits visible; next bf16 image visible.
constexpr int POOL_REG_NL = 4;   // weight slices read from LDS (the rest stay in registers)
template <int D, int MH>
__global__ void __launch_bounds__(256) pool_gate_part_reg_k(PoolArgs p, const bf16* __restrict__ VU) {
  constexpr int RB = 32, LDB = D + 8, KS = D / 16, CJ = D / 128, NR = 4 * CJ, EARLY = CJ;
  constexpr int NL = POOL_REG_NL, KR = KS - NL;   // the last NL slices of the weights are read from LDS
  static_assert(MH == 128 && D % 128 == 0 && KS % 3 == 0 && KS / 3 * 2 == 16 && NR - EARLY <= KS && EARLY % CJ == 0, "shape");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Hb = reinterpret_cast<bf16*>(smem);                            // [2][RB][LDB]
  u32x4* Wl = reinterpret_cast<u32x4*>(Hb + 2 * RB * LDB);             // [4 waves][NL][2][64 lanes] weight fragments
  float* gb = reinterpret_cast<float*>(Wl + 4 * NL * 2 * 64);          // scaled bV[MH], scaled bU[MH], w[MH]
  float* apart = gb + 3 * MH;                                          // [4][RB]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, h2 = lane >> 5;
  const int rgrp = tid >> 5, cl = tid & 31;   // loads: rows 4 rgrp .. + 3 of a block, column groups cl + 32 j
  const float* H = p.H;
  const long long groups = (p.N + RB - 1) / RB;
  constexpr float C1 = -2.0f * 1.44269504088896f, C2 = -1.44269504088896f;   // exp(-2x) and exp(-x) as exp2

  for (int j = tid; j < MH; j += 256) { gb[j] = C1 * p.Vb[j]; gb[MH + j] = C2 * p.Ub[j]; gb[2 * MH + j] = p.w[j]; }
  // this wavefront's gate units 32 wave .. + 31 of V and of U: slices 0 .. KR - 1 of their weights stay in the
  // accumulation half of the register file (the MFMA reads them there), the last NL go to LDS in fragment order
  // (each lane reads back what it wrote): with all of them in registers the two accumulator sets fill that half
  // to the last register and the allocator spills
  bf16x8 wv[KR], wu[KR];
  u32x4* wl = Wl + (size_t)wave * NL * 2 * 64 + lane;
  {
    const bf16* wr = VU + (size_t)(32 * wave + li) * D + h2 * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      u32x4 a = *reinterpret_cast<const u32x4*>(wr + ks * 16);
      u32x4 b = *reinterpret_cast<const u32x4*>(wr + (size_t)MH * D + ks * 16);
      if (ks < KR) {
        asm volatile("" : "+a"(a), "+a"(b));
        wv[ks] = __builtin_bit_cast(bf16x8, a);
        wu[ks] = __builtin_bit_cast(bf16x8, b);
      } else {
        wl[((ks - KR) * 2 + 0) * 64] = a;
        wl[((ks - KR) * 2 + 1) * 64] = b;
      }
    }
  }
  float4 rs[3][NR];
  f32x16 acc[2][2];
  // The blocks of a workgroup are loaded strictly one after the other (load 0 .. NR - 1 of a block, then the next
  // block), so one running row index serves every load site; 32-bit (N < 2^31 - 2^24 is checked on the host).
  const unsigned lastrow = (unsigned)(p.N - 1), lstep = gridDim.x * RB;
  unsigned lrow = blockIdx.x * RB + 4 * rgrp;   // first of this thread's 4 rows of the block being loaded
  const float* hrp = H;                         // row base of the loads in progress
  // load i = k * CJ + j; rows past the end re-read the last row (their softmax term is set to zero)
  auto issue_one = [&](float4 (&r)[NR], auto ic) __attribute__((always_inline)) {
    constexpr int i = decltype(ic)::value, k = i / CJ, j = i % CJ;
    if constexpr (j == 0) {
      unsigned row = lrow + k;
      row = row < lastrow ? row : lastrow;
      hrp = H + (size_t)row * D + cl * 4;
    }
    r[i] = *reinterpret_cast<const float4*>(hrp + j * 128);
    if constexpr (i == NR - 1) lrow += lstep;
  };
  auto stash_one = [&](const float4 (&r)[NR], int buf, auto ic) __attribute__((always_inline)) {
    constexpr int i = decltype(ic)::value, k = i / CJ, j = i % CJ;
    float4 v = r[i];
    f32x2 p0 = {v.x, v.y}, p1 = {v.z, v.w};
    bf16x2 h0 = __builtin_convertvector(p0, bf16x2), h1 = __builtin_convertvector(p1, bf16x2);
    uint2 w2;
    w2.x = __builtin_bit_cast(unsigned, h0);
    w2.y = __builtin_bit_cast(unsigned, h1);
    *reinterpret_cast<uint2*>(Hb + (buf * RB + 4 * rgrp + k) * LDB + (cl + 32 * j) * 4) = w2;
  };
  auto stash_h = [&](const float4 (&r)[NR], int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int j = 0; j < CJ; ++j) {
        float4 v = r[k * CJ + j];
        f32x2 p0 = {v.x, v.y}, p1 = {v.z, v.w};
        bf16x2 h0 = __builtin_convertvector(p0, bf16x2), h1 = __builtin_convertvector(p1, bf16x2);
        uint2 w2;
        w2.x = __builtin_bit_cast(unsigned, h0);
        w2.y = __builtin_bit_cast(unsigned, h1);
        *reinterpret_cast<uint2*>(Hb + (buf * RB + 4 * rgrp + k) * LDB + (cl + 32 * j) * 4) = w2;
      }
  };
  // fp32 partial sums: a lane adds 4 rows per block, a few thousand terms at most (N < 2^31, 256 workgroups x 8 row
  // groups), before the fp64 reduction over row groups and workgroups
  float z[4 * CJ];
#pragma unroll
  for (int i = 0; i < 4 * CJ; ++i) z[i] = 0.f;
  float wabs = 0.f;
  for (int j = lane; j < MH; j += 64) wabs += fabsf(p.w[j]) + (p.w_other ? fabsf(p.w_other[j]) : 0.f);
  wabs = wave_sum(wabs);
  const bool fixed = wabs <= 40.f;   // a bound of every logit serves as the softmax shift
  float run_m = fixed ? wabs : -INFINITY;
  double lsum = 0.0;
  const int st = gridDim.x;
  const int nblk = (int)((groups - blockIdx.x + st - 1) / st);   // blocks of this workgroup (>= 1)

  // iteration `it` (role phase ph = it mod 6): MFMAs of block it (on the last image again when it == nblk: unused),
  // gate, softmax terms and weighted sum of block it - 1, loads of block it + 1 (and the first of block it + 2)
  auto iter = [&](auto phc, int it) __attribute__((always_inline)) {
    constexpr int ph = decltype(phc)::value, buf = ph & 1, ls = (ph + 1) % 3, zs = (ph + 2) % 3;
    f32x16 (&ac)[2] = acc[ph & 1];
    const f32x16 (&ap)[2] = acc[(ph & 1) ^ 1];
#pragma unroll
    for (int r = 0; r < 16; ++r) { ac[0][r] = 0.f; ac[1][r] = 0.f; }
    const bf16* hrow = Hb + (buf * RB + li) * LDB + h2 * 8;
    constexpr int PF = 3;
    u32x4 hf[PF];
#pragma unroll
    for (int ks = 0; ks < PF; ++ks) hf[ks] = *reinterpret_cast<const u32x4*>(hrow + ks * 16);
    float part = 0.f, part2 = 0.f;
    u32x4 lw[2][2];
    const float* gbl = gb + 32 * wave + h2 * 4;   // scaled biases and w of this lane's gate units
    float2 bv2 = *reinterpret_cast<const float2*>(gbl), bu2, w2;
    float ge1[2], ge2[2], gnum[2];
    // Gate of the previous block, two elements (accumulator registers 2t, 2t + 1) at a time in three stages, one per
    // slice, a new pair every second slice (slices 2t, 2t + 1, 2t + 2): the vector ALU always has independent chains
    // and a slice's share stays under the 64 clocks of its two MFMAs.  Accumulator register r of a lane = gate unit
    // (r / 4) * 8 + h2 * 4 + r % 4 of the wavefront's 32, row li.  The finished accumulators are read where they are,
    // in the accumulation half of the register file (left to itself the allocator moves them to 32 ordinary registers
    // first, which the three row sets need).
    // tanh(xv) * sigmoid(xu) = (1 - e1) / ((1 + e1) (1 + e2)), e1 = exp(-2 xv), e2 = exp(-xu)
    auto gate0 = [&](auto tc) __attribute__((always_inline)) {
      constexpr int t = decltype(tc)::value, r0 = 2 * t, off = (r0 / 4) * 8 + r0 % 4;
      bu2 = *reinterpret_cast<const float2*>(gbl + MH + off);
      w2 = *reinterpret_cast<const float2*>(gbl + 2 * MH + off);
      float xa, xb;
      asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(xa) : "a"(ap[0][r0]));
      asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(xb) : "a"(ap[0][r0 + 1]));
      ge1[0] = __builtin_amdgcn_exp2f(fminf(fmaf(xa, C1, bv2.x), 57.f));
      ge1[1] = __builtin_amdgcn_exp2f(fminf(fmaf(xb, C1, bv2.y), 57.f));
    };
    auto gate1 = [&](auto tc) __attribute__((always_inline)) {
      constexpr int t = decltype(tc)::value, r0 = 2 * t;
      float xa, xb;
      asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(xa) : "a"(ap[1][r0]));
      asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(xb) : "a"(ap[1][r0 + 1]));
      ge2[0] = __builtin_amdgcn_exp2f(fmaf(xa, C2, bu2.x));   // inf is fine: 1 / inf = 0, e1 is finite
      ge2[1] = __builtin_amdgcn_exp2f(fmaf(xb, C2, bu2.y));
      gnum[0] = fmaf(-w2.x, ge1[0], w2.x);
      gnum[1] = fmaf(-w2.y, ge1[1], w2.y);
      ge1[0] = fmaf(ge1[0] + 1.0f, ge2[0], ge1[0] + 1.0f);   // (1 + e1) (1 + e2)
      ge1[1] = fmaf(ge1[1] + 1.0f, ge2[1], ge1[1] + 1.0f);
      if constexpr (t + 1 < 8) {   // the next pair's first constants
        constexpr int r1 = r0 + 2, off1 = (r1 / 4) * 8 + r1 % 4;
        bv2 = *reinterpret_cast<const float2*>(gbl + off1);
      }
    };
    float gden[2];
    auto gate2 = [&]() __attribute__((always_inline)) {
      part = fmaf(gnum[0], __builtin_amdgcn_rcpf(gden[0]), part);
      part2 = fmaf(gnum[1], __builtin_amdgcn_rcpf(gden[1]), part2);
    };
    // After the last gate stage (slice GA): the partial logits are exchanged, and the softmax terms, the weighted sum
    // of block it - 1, the first loads of block it + 2 and the bf16 image of block it + 1 run under the remaining
    // slices' MFMAs.
    constexpr int GA = 16, SP = (KS - 1 - GA - CJ);   // SP slices share the NR registers of the image
    static_assert(GA + CJ + 1 < KS && NR % SP == 0, "tail schedule");
    const long long n0 = ((long long)blockIdx.x + (long long)(it - 1) * st) * RB;   // first row of block it - 1
    float a_out = 0.f, sc = 1.0f, ek[4] = {0.f, 0.f, 0.f, 0.f};
    float a_prev = 0.f;   // the other half's partial logit of this lane's row (two-pass use)
    if (p.a_in != nullptr && it >= 1) a_prev = p.a_in[n0 + li < p.N ? n0 + li : p.N - 1];   // uniform
    static_for<0, KS>([&](auto kc) __attribute__((always_inline)) {
      constexpr int ks = decltype(kc)::value;
      bf16x8 f = __builtin_bit_cast(bf16x8, hf[ks % PF]);
      if constexpr (ks + PF < KS) hf[ks % PF] = *reinterpret_cast<const u32x4*>(hrow + (ks + PF) * 16);
      // one load per slice: issued as one burst they hold the wavefronts in the issue for the ~770 clocks the address
      // unit needs for a block's 48 KB
      if constexpr (ks + EARLY < NR) issue_one(rs[ls], IC<ks + EARLY>{});
      if constexpr (ks < KR) {
        ac[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv[ks], f, ac[0], 0, 0, 0);
        ac[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wu[ks], f, ac[1], 0, 0, 0);
      } else {
        ac[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, lw[(ks - KR) % 2][0]), f, ac[0], 0, 0, 0);
        ac[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, lw[(ks - KR) % 2][1]), f, ac[1], 0, 0, 0);
      }
      if constexpr (ks + 2 >= KR && ks + 2 < KS) {   // weight fragments from LDS, two slices ahead
        lw[(ks + 2 - KR) % 2][0] = wl[((ks + 2 - KR) * 2 + 0) * 64];
        lw[(ks + 2 - KR) % 2][1] = wl[((ks + 2 - KR) * 2 + 1) * 64];
      }
      if constexpr (ks % 2 == 0 && ks >= 2 && ks <= GA) gate2();                      // pair (ks - 2) / 2
      if constexpr (ks % 2 == 0 && ks / 2 < 8) gate0(IC<ks / 2>{});
      if constexpr (ks % 2 == 1 && ks / 2 < 8) { gate1(IC<ks / 2>{}); gden[0] = ge1[0]; gden[1] = ge1[1]; }
      if constexpr (ks == GA) {
        part += part2;
        part += __shfl_xor(part, 32, 64);
        if (h2 == 0) apart[wave * RB + li] = part;
        __syncthreads();   // (A) the four partial logits of every row of block it - 1 are there
        if (it >= 1) {     // uniform
          float a = apart[li] + apart[RB + li] + apart[2 * RB + li] + apart[3 * RB + li] + a_prev;
          const bool ok = n0 + li < p.N;
          a_out = a;
          float e;
          if (p.partial) {   // uniform: only the partial logits are wanted
            e = 0.f;
          } else if (fixed) {   // uniform
            e = ok ? __expf(a - run_m) : 0.f;
          } else {
            a = ok ? a : -INFINITY;
            float m = fmaxf(run_m, wave_max(a));   // finite: the block has at least one row
            e = __expf(a - m);                     // lanes li and li + 32: row li
            sc = __expf(run_m - m);                // exp(-inf) = 0 on the first block
            run_m = m;
            lsum *= (double)sc;
          }
          lsum += (double)e;   // summed over the rows once, at the end
#pragma unroll
          for (int k = 0; k < 4; ++k) ek[k] = __shfl(e, 4 * (rgrp & 7) + k, 64);
        }
      }
      if constexpr (ks > GA && ks <= GA + CJ) {   // weighted sum, one group of 4 columns per slice (all zero when it = 0)
        constexpr int j = ks - GA - 1;
        float4 s = make_float4(z[4 * j] * sc, z[4 * j + 1] * sc, z[4 * j + 2] * sc, z[4 * j + 3] * sc);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float4 v = rs[zs][k * CJ + j];
          s.x = fmaf(ek[k], v.x, s.x); s.y = fmaf(ek[k], v.y, s.y);
          s.z = fmaf(ek[k], v.z, s.z); s.w = fmaf(ek[k], v.w, s.w);
        }
        z[4 * j] = s.x; z[4 * j + 1] = s.y; z[4 * j + 2] = s.z; z[4 * j + 3] = s.w;
      }
      if constexpr (ks == GA + CJ) {
        // the freed set takes the first loads of block it + 2 (the next iteration continues with load EARLY); they
        // must not move above the weighted sum, which still reads the registers they land in
        asm volatile("" ::: "memory");
        static_for<0, EARLY>([&](auto ic) __attribute__((always_inline)) { issue_one(rs[zs], ic); });
      }
      if constexpr (ks > GA + CJ) {   // bf16 image of block it + 1 (replaces that of block it - 1), NR / SP registers per slice
        constexpr int q = ks - GA - CJ - 1;
        static_for<q * (NR / SP), (q + 1) * (NR / SP)>([&](auto ic) __attribute__((always_inline)) { stash_one(rs[ls], buf ^ 1, ic); });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    // both accumulator sets stay in the accumulation half of the register file (left to itself the allocator moves
    // the finished one to 32 ordinary registers, which the three row sets need)
    asm volatile("" : "+a"(ac[0]), "+a"(ac[1]));
    if (it >= 1 && wave == 0 && h2 == 0 && n0 + li < p.N) p.a[n0 + li] = a_out;   // kept for the backward
    __syncthreads();   // (B) the next bf16 image is visible; apart is free again
  };

  // prologue: block 0 of this workgroup, and the first loads of block 1
  static_for<0, NR>([&](auto ic) __attribute__((always_inline)) { issue_one(rs[0], ic); });
  static_for<0, EARLY>([&](auto ic) __attribute__((always_inline)) { issue_one(rs[1], ic); });
  stash_h(rs[0], 0);
  // iteration 0 has no previous block: its gate reads zeros and its weighted sum adds zero times zero
#pragma unroll
  for (int i = 0; i < NR; ++i) rs[2][i] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc[1][0][r] = 0.f; acc[1][1][r] = 0.f; }
  __syncthreads();
  for (int it = 0;;) {
    iter(IC<0>{}, it); if (++it > nblk) break;
    iter(IC<1>{}, it); if (++it > nblk) break;
    iter(IC<2>{}, it); if (++it > nblk) break;
    iter(IC<3>{}, it); if (++it > nblk) break;
    iter(IC<4>{}, it); if (++it > nblk) break;
    iter(IC<5>{}, it); if (++it > nblk) break;
  }
  // column sums over the 8 row groups (the bf16 images are dead: every wavefront is past the last barrier (B))
  double* zred = reinterpret_cast<double*>(smem);   // [8][D]
  static_assert(8 * D * 8 <= 2 * RB * LDB * 2, "reduction buffer");
#pragma unroll
  for (int j = 0; j < CJ; ++j)
#pragma unroll
    for (int c = 0; c < 4; ++c) zred[rgrp * D + (cl + 32 * j) * 4 + c] = (double)z[4 * j + c];
  __syncthreads();
  double* out = p.part + (size_t)blockIdx.x * (2 + D);
  // lanes li and li + 32 hold the same rows: sum over one half
  for (int o = 1; o < 32; o <<= 1) lsum += __shfl_xor(lsum, o, 64);
  if (tid == 0) { out[0] = (double)run_m; out[1] = lsum; }
  for (int d = tid; d < D; d += 256) {
    double t = 0.0;
#pragma unroll
    for (int g = 0; g < 8; ++g) t += zred[g * D + d];
    out[2 + d] = t;
  }
}

template <int D, int MH>
hipError_t go_reg(const PoolArgs& p, hipStream_t s) {
  auto kern = pool_gate_part_reg_k<D, MH>;
  size_t lds = (size_t)2 * 32 * (D + 8) * 2 + (size_t)4 * POOL_REG_NL * 2 * 64 * 16 + (size_t)3 * MH * 4 + 4 * 32 * 4;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  long long n = (long long)MH * p.D;
  hipLaunchKernelGGL(pool_cast_vu_k, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p.VW, p.UW, (bf16*)p.vub, n);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(256), lds, s, p, (const bf16*)p.vub);
  return hipGetLastError();
}

// M_h = 256 as two passes of the M_h = 128 kernel over the rows (the features are read twice, against the weights
// streaming from L2 for every block of rows in the one-pass kernel): pass 1 leaves the partial logits of gate units
// 0..127 in a_tmp, pass 2 adds those of units 128..255 and does the softmax partials.
hipError_t go_reg_halves(const PoolArgs& p0, hipStream_t s) {
  constexpr int MH = 128;
  if (!p0.a_tmp) return hipErrorInvalidValue;
  PoolArgs p = p0;
  p.Mh = MH; p.partial = 1; p.a_in = nullptr; p.w_other = nullptr; p.a = p0.a_tmp;
  hipError_t e = go_reg<384, MH>(p, s);
  if (e != hipSuccess) return e;
  p = p0;
  p.Mh = MH; p.partial = 0; p.a_in = p0.a_tmp; p.w_other = p0.w;
  p.VW = p0.VW + (size_t)MH * p0.D; p.UW = p0.UW + (size_t)MH * p0.D;
  p.Vb = p0.Vb + MH; p.Ub = p0.Ub + MH; p.w = p0.w + MH;
  return go_reg<384, MH>(p, s);
}

template <int RB, int MH, int BK, int HCH>
hipError_t go(const PoolArgs& p, hipStream_t s) {
  using C = PoolCfg<RB, MH, BK>;
  auto kern = pool_gate_part_mfma_k<RB, MH, BK, HCH>;
  size_t lds = C::lds_bytes(p.D);
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  long long n = (long long)p.Mh * p.D;
  hipLaunchKernelGGL(pool_cast_vu_k, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p.VW, p.UW, (bf16*)p.vub, n);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(p.blocks), dim3(256), lds, s, p, (const bf16*)p.vub);
  return hipGetLastError();
}

}  // namespace

// shapes built: (D, M_h) in {384, 768} x {128, 256}
bool pool_mfma_ok(const PoolArgs& p) {
  return p.vub && p.N >= 512 && p.N < (1LL << 31) - (1 << 24) && (p.D == 384 || p.D == 768) && (p.Mh == 128 || p.Mh == 256) &&
         ((uintptr_t)p.H & 15) == 0 && ((uintptr_t)p.vub & 15) == 0;
}

// above this many rows M_h = 256 goes through the register-resident kernel in two passes (below it the launches cost
// more than the weights streaming from L2)
static bool pool_two_pass(const PoolArgs& p) { return p.D == 384 && p.Mh == 256 && p.N >= 32768 && p.a_tmp != nullptr; }

int pool_mfma_rows(const PoolArgs& p) { return (p.D == 384 && p.Mh == 256 && !pool_two_pass(p)) ? 64 : 32; }

hipError_t launch_pool_gate_part_mfma(const PoolArgs& p, hipStream_t s) {
  if (p.D == 384 && p.Mh == 128) return go_reg<384, 128>(p, s);
  if (pool_two_pass(p)) return go_reg_halves(p, s);
  if (p.D == 384 && p.Mh == 256) return go<64, 256, 16, 24>(p, s);
  if (p.D == 768 && p.Mh == 128) return go<32, 128, 32, 24>(p, s);
  if (p.D == 768 && p.Mh == 256) return go<32, 256, 16, 24>(p, s);
  return hipErrorInvalidValue;
}

}  // namespace sl
