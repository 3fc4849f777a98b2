// bf16 MFMA softmax attention inside one tile for gfx950 (v_mfma_f32_32x32x16_bf16).
//
// One workgroup per (tile, head), one wavefront per block of 32 queries (seven at 197 tokens; the key-owned
// backward keeps four); all keys/values of the head (queries and output gradients in the key-owned pass) sit in LDS.
// Scores are produced TRANSPOSED (keys x queries): a 32x32 accumulator block then holds one
// query per lane column and the keys down the registers, so the softmax over keys is a
// reduction inside each lane plus one exchange between the two lane halves, and the
// probabilities are already in the lane layout the next MFMA wants as its B operand.
// Operands whose contraction index is the row index of a row-major matrix (V in P.V, K in
// dS.K, Q and dO in the key-owned backward) stay row-major in LDS and are fetched with LDS
// transpose reads (ds_read_b64_tr_b16); no transposed copy is kept.
//
// Backward is two deterministic passes, both recomputing P from the saved row log-sum-exp:
//   pass Q (query blocks owned by a wave): dQ = scale * dS K
//   pass K (key blocks owned by a wave):   dV = P^T dO,  dK = scale * dS^T Q
// with dS = P * (dP - delta), dP = dO V^T, delta_i = dO_i . O_i.  No atomics.
#include "slide_internal.h"

#include <type_traits>

namespace sl {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ u32x4 ldg16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// pack 8 floats into the bf16x8 B operand
__device__ __forceinline__ bf16x8 pack8(const float* p) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (bf16)p[i];
  return o;
}

// A operand whose contraction index runs along the ROWS of a row-major LDS matrix X[row][col] (row stride ld):
// lane l gets column c0 + l % 32 and the rows j0 + 4*h2 + {0..3}, j0 + 8 + 4*h2 + {0..3} (h2 = l / 32), the order
// of accumulator registers 8t..8t+7.  Two LDS transpose reads (ds_read_b64_tr_b16): within a group of 16
// lanes, lane s addresses 4 consecutive columns of row s / 4 and receives, for column s of the group's 16, the
// four rows.  No transposed copy of X is kept.
typedef short s16x4 __attribute__((ext_vector_type(4)));
// The lane-dependent part of the address is taken out: lp = X + tr_lane_off(ld, lane) is formed once,
// off = j0 * ld + c0 is a compile-time or wave-uniform element offset (LDS instructions carry it as an immediate).
__device__ __forceinline__ int tr_lane_off(int ld, int lane) {
  int g = lane >> 4, s = lane & 15;
  return (4 * (g >> 1) + (s >> 2)) * ld + 16 * (g & 1) + (s & 3) * 4;
}
__device__ __forceinline__ bf16x8 frag_tr_at(const bf16* lp, int ld, int off) {
  const bf16* p = lp + off;
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 8 * ld));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// Copies rows [0,T) x DH of two row-major global matrices (row strides gs0, gs1) into LDS row-major [TP][DH+8], by a
// workgroup of NTHR threads, all global loads issued before the first LDS store (a copy loop with a run-time trip
// count waits for every load before it stores, which puts one memory latency per iteration in front of the
// kernel's work, as long as the work itself).
// Rows past T0 / T1 are filled with zeros.
template <int DH, int TP, int NTHR, bool FENCE, typename MID>
__device__ __forceinline__ void load_rm2(const bf16* __restrict__ g0, long long gs0, int T0, bf16* dst0,
                                         const bf16* __restrict__ g1, long long gs1, int T1, bf16* dst1, MID mid) {
  constexpr int CH = DH / 8, TOTAL = TP * CH, ITER = (TOTAL + NTHR - 1) / NTHR;
  u32x4 va[ITER], vb[ITER];
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    int c = threadIdx.x + i * NTHR;
    int row = c / CH, kc = c % CH;
    int r0 = row < T0 ? row : T0 - 1, r1 = row < T1 ? row : T1 - 1;
    va[i] = ldg16(g0 + r0 * gs0 + kc * 8);
    vb[i] = ldg16(g1 + r1 * gs1 + kc * 8);
  }
  // everything requested so far (also by the caller, before this call) is in flight before anything is waited for:
  // `mid` is the caller's arithmetic on its own, older loads
  if (FENCE) __builtin_amdgcn_sched_barrier(0);
  mid();
#pragma unroll
  for (int i = 0; i < ITER; ++i) {
    int c = threadIdx.x + i * NTHR;
    int row = c / CH, kc = c % CH;
    if (TOTAL % NTHR == 0 || c < TOTAL) {
      u32x4 z = {0, 0, 0, 0};
      *reinterpret_cast<u32x4*>(dst0 + row * (DH + 8) + kc * 8) = row < T0 ? va[i] : z;
      *reinterpret_cast<u32x4*>(dst1 + row * (DH + 8) + kc * 8) = row < T1 ? vb[i] : z;
    }
  }
}

constexpr float LOG2E = 1.4426950408889634f;

// Workgroup size: one wavefront per block of 32 queries (keys) where a head has seven of them: no
// wavefront then carries two blocks while another carries one.
template <int NB> constexpr int attn_threads() { return NB >= 7 ? NB * 64 : 256; }

// --------------------------------------------------------------------------------------------
// forward
// --------------------------------------------------------------------------------------------
template <int DH, int NB>
__global__ void __launch_bounds__(attn_threads<NB>(), 2) attn_fwd_mfma_k(const bf16* __restrict__ qkv, bf16* __restrict__ O,
                                                       float* __restrict__ lse, int T, int H, long long ntiles, int cls_only) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int TP = NB * 32, LDR = DH + 8, KS = DH / 16, DB = DH / 32;
  bf16* Ks = reinterpret_cast<bf16*>(smem);  // [TP][LDR]
  bf16* Vs = Ks + TP * LDR;                  // [TP][LDR]
  // workgroup ids are dealt round-robin to the 8 XCDs: the heads of one tile go to one XCD, next to each other
  // in time, so the neighbouring 128-byte head slices of its token rows meet in one L2
  int h = (blockIdx.x / 8) % H;
  long long tile = (long long)(blockIdx.x / 8 / H) * 8 + blockIdx.x % 8;
  if (tile >= ntiles) return;
  int D = H * DH;
  long long gs = 3LL * D;
  const bf16* base = qkv + tile * T * gs + h * DH;
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int li = lane & 31, h2 = lane >> 5;
  // the wavefront's query fragments are requested before the K/V copy so that they arrive with it (asked for after
  // the barrier they would cost a memory latency of their own)
  bf16x8 fq[KS];
  {
    int q0 = wave * 32 + li;
    q0 = q0 < T ? q0 : T - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fq[ks] = as_bf16x8(ldg16(base + q0 * gs + ks * 16 + h2 * 8));
  }
  load_rm2<DH, TP, attn_threads<NB>(), false>(base + D, gs, T, Ks, base + 2 * D, gs, T, Vs, [] {});
  __syncthreads();
  float sl2 = LOG2E / sqrtf((float)DH);
  // lane-dependent parts of the LDS addresses, formed once; the key-block loop only advances them
  const bf16* const krow0 = Ks + li * LDR + h2 * 8;
  const bf16* const vtr0 = Vs + tr_lane_off(LDR, lane);
  const int nqb = cls_only ? 1 : NB;   // cls_only: only query 0 is needed (its block of 32 is computed)
  const int nlast = T - (NB - 1) * 32;   // real keys in the last block (1 .. 32)
  for (int qb = wave; qb < nqb; qb += attn_threads<NB>() / 64) {
    int q = qb * 32 + li;
    int qc = q < T ? q : T - 1;
    if (qb != wave) {   // uniform; later query blocks of a wavefront (workgroups with fewer wavefronts than blocks)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) fq[ks] = as_bf16x8(ldg16(base + qc * gs + ks * 16 + h2 * 8));
    }
    // keys are taken one block of 32 at a time with a running maximum and sum (the whole row of
    // scores never sits in registers); o is rescaled when the maximum moves
    f32x16 o[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[d][r] = 0.f;
    float mx = -INFINITY, l = 0.f;
    const bf16* krow = krow0;
    const bf16* vtr = vtr0;
    // one block of 32 keys; LASTB: the head's last block, the only one that holds padded keys (its own copy of the
    // loop body, so that the other blocks carry no mask arithmetic)
    auto key_block = [&](auto lastb) __attribute__((always_inline)) {
      constexpr bool LASTB = decltype(lastb)::value;
      f32x16 sc;
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 a = *reinterpret_cast<const bf16x8*>(krow + ks * 16);
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, fq[ks], sc, 0, 0, 0);
      }
      // In the last block only the first nlast keys exist.  Accumulator registers 4g .. 4g + 3 hold keys 8g .. 8g + 7
      // of the block: a group of registers past the last real key takes no part in the maximum, gets no exponential
      // (its probabilities are zero) and, where the block's upper 16 keys are all padding, no second P V slice.
      float bm = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (LASTB) {
          if ((r >> 2) * 8 < nlast) {   // uniform
            int key = (r >> 2) * 8 + h2 * 4 + (r & 3);
            if (key >= nlast) sc[r] = -INFINITY;
            bm = fmaxf(bm, sc[r]);
          }
        } else {
          bm = fmaxf(bm, sc[r]);
        }
      }
      bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
      float mn = fmaxf(mx, bm);                                  // finite: every block has a real key
      float resc = __builtin_amdgcn_exp2f((mx - mn) * sl2);       // 0 at the first block
      float ms = mn * sl2;
      float ls = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (!LASTB || (r >> 2) * 8 < nlast) {   // uniform
          float pe = __builtin_amdgcn_exp2f(sc[r] * sl2 - ms);
          sc[r] = pe;
          ls += pe;
        } else {
          sc[r] = 0.f;
        }
      }
      l = l * resc + ls;
      mx = mn;
      if (__builtin_amdgcn_ballot_w64(resc != 1.0f) != 0) {   // uniform: after the first blocks the maximum rarely moves
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[d][r] *= resc;
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (LASTB && t == 1 && nlast <= 16) continue;   // uniform: all of these probabilities are zero
        float pv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) pv[i] = sc[8 * t + i];
        bf16x8 pb = pack8(pv);
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          bf16x8 a = frag_tr_at(vtr, LDR, 16 * t * LDR + d * 32);
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o[d], 0, 0, 0);
        }
      }
    };
#pragma unroll 1
    for (int kb = 0; kb < NB - 1; ++kb, krow += 32 * LDR, vtr += 32 * LDR) key_block(std::false_type{});
    key_block(std::true_type{});
    l += __shfl_xor(l, 32, 64);
    if (q < T) {
      float inv = 1.0f / l;
      bf16* orow = O + (tile * T + q) * D + h * DH;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16x4 v;
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = (bf16)(o[d][g4 * 4 + i] * inv);
          *reinterpret_cast<bf16x4*>(orow + d * 32 + g4 * 8 + h2 * 4) = v;
        }
      if (h2 == 0) lse[(tile * H + h) * T + q] = mx * (sl2 / LOG2E) + logf(l);
    }
  }
}

// --------------------------------------------------------------------------------------------
// backward, pass Q: dQ
// --------------------------------------------------------------------------------------------
template <int DH, int NB>
__global__ void __launch_bounds__(attn_threads<NB>(), 2) attn_bwd_q_mfma_k(const bf16* __restrict__ qkv, const bf16* __restrict__ O,
                                                         const float* __restrict__ lse, const bf16* __restrict__ dO,
                                                         bf16* __restrict__ dqkv, float* __restrict__ delta_ws, int T, int H,
                                                         long long ntiles, int cls_only) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int TP = NB * 32, LDR = DH + 8, KS = DH / 16, DB = DH / 32;
  bf16* Ks = reinterpret_cast<bf16*>(smem);  // [TP][LDR]
  bf16* Vs = Ks + TP * LDR;                  // [TP][LDR]
  // workgroup ids are dealt round-robin to the 8 XCDs: the heads of one tile go to one XCD, next to each other
  // in time, so the neighbouring 128-byte head slices of its token rows meet in one L2
  int h = (blockIdx.x / 8) % H;
  long long tile = (long long)(blockIdx.x / 8 / H) * 8 + blockIdx.x % 8;
  if (tile >= ntiles) return;
  int D = H * DH;
  long long gs = 3LL * D;
  const bf16* base = qkv + tile * T * gs + h * DH;
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int li = lane & 31, h2 = lane >> 5;
  // per query block: fragments of Q and dO, delta = dO . O, the row's log-sum-exp.  Requesting and consuming are
  // separate so that the first block's loads and the K/V copy's are all in flight before anything is waited for.
  bf16x8 fq[KS], fdo[KS], fo[KS];
  float delta, lq;
  auto issue_qblock = [&](int qb) __attribute__((always_inline)) {
    int q = qb * 32 + li;
    int qc = q < T ? q : T - 1;
    int qg = cls_only ? 0 : qc;   // cls_only: only row 0 of dO (and of O) is defined
    const bf16* orow = O + (tile * T + qg) * D + h * DH;
    const bf16* gor = dO + (tile * T + qg) * D + h * DH;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      fq[ks] = as_bf16x8(ldg16(base + qc * gs + ks * 16 + h2 * 8));
      fdo[ks] = as_bf16x8(ldg16(gor + ks * 16 + h2 * 8));
      fo[ks] = as_bf16x8(ldg16(orow + ks * 16 + h2 * 8));
    }
    lq = lse[(tile * H + h) * T + qc];
  };
  auto finish_qblock = [&](int qb) __attribute__((always_inline)) {
    int q = qb * 32 + li;
    delta = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (cls_only && q != 0) fdo[ks] = as_bf16x8(u32x4{0, 0, 0, 0});   // only query 0 carries a gradient
#pragma unroll
      for (int i = 0; i < 8; ++i) delta += (float)fdo[ks][i] * (float)fo[ks][i];
    }
    delta += __shfl_xor(delta, 32, 64);
    lq *= LOG2E;
    // kept for the key-owned pass (which would otherwise read dO and O once more to form it)
    if (h2 == 0 && q < T) delta_ws[(tile * H + h) * T + q] = delta;
  };
  const int qb0 = wave < NB ? wave : 0;
  issue_qblock(qb0);
  load_rm2<DH, TP, attn_threads<NB>(), true>(base + D, gs, T, Ks, base + 2 * D, gs, T, Vs, [&] { finish_qblock(qb0); });
  __syncthreads();
  float scale = 1.0f / sqrtf((float)DH);
  float sl2 = LOG2E * scale;
  const bf16* const krow0 = Ks + li * LDR + h2 * 8;
  const bf16* const vrow0 = Vs + li * LDR + h2 * 8;
  const bf16* const ktr0 = Ks + tr_lane_off(LDR, lane);
  const int nlast = T - (NB - 1) * 32;   // real keys in the last block (1 .. 32)
  for (int qb = wave; qb < NB; qb += attn_threads<NB>() / 64) {
    int q = qb * 32 + li;
    if (cls_only && qb > 0) {   // uniform: the output gradient is zero for these queries, and so is dQ
      if (q < T) {
        bf16* out = dqkv + (tile * T + q) * gs + h * DH;
#pragma unroll
        for (int c = 0; c < DH / 8; ++c)
          if ((c & 1) == h2) *reinterpret_cast<u32x4*>(out + c * 8) = u32x4{0, 0, 0, 0};   // the row's two lanes share it
      }
      continue;
    }
    if (qb != wave) {   // uniform; later blocks of a wavefront (fewer wavefronts than blocks)
      issue_qblock(qb);
      finish_qblock(qb);
    }
    f32x16 dq[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq[d][r] = 0.f;
    const bf16* krow = krow0;
    const bf16* vrow = vrow0;
    const bf16* ktr = ktr0;
    // one block of 32 keys; LASTB: the head's last block, the only one that holds padded keys (its own copy of the
    // loop body, so that the other blocks carry no mask arithmetic)
    auto key_block = [&](auto lastb) __attribute__((always_inline)) {
      constexpr bool LASTB = decltype(lastb)::value;
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 a = *reinterpret_cast<const bf16x8*>(krow + ks * 16);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, fq[ks], s, 0, 0, 0);
        bf16x8 v = *reinterpret_cast<const bf16x8*>(vrow + ks * 16);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(v, fdo[ks], dp, 0, 0, 0);
      }
      // (last block: register groups past the last real key are zero without being computed, and the second dS K
      // slice is skipped where the block's upper 16 keys are all padding; see the forward kernel)
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (!LASTB || (r >> 2) * 8 < nlast) {   // uniform
          float p = __builtin_amdgcn_exp2f(s[r] * sl2 - lq);
          if (LASTB) {
            int key = (r >> 2) * 8 + h2 * 4 + (r & 3);
            if (key >= nlast) p = 0.f;
          }
          ds[r] = p * (dp[r] - delta);
        } else {
          ds[r] = 0.f;
        }
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (LASTB && t == 1 && nlast <= 16) continue;   // uniform
        bf16x8 db = pack8(ds + 8 * t);
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          bf16x8 a = frag_tr_at(ktr, LDR, 16 * t * LDR + d * 32);
          dq[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, db, dq[d], 0, 0, 0);
        }
      }
    };
#pragma unroll 1
    for (int kb = 0; kb < NB - 1; ++kb, krow += 32 * LDR, vrow += 32 * LDR, ktr += 32 * LDR) key_block(std::false_type{});
    key_block(std::true_type{});
    if (q < T) {
      bf16* out = dqkv + (tile * T + q) * gs + h * DH;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16x4 v;
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = (bf16)(dq[d][g4 * 4 + i] * scale);
          *reinterpret_cast<bf16x4*>(out + d * 32 + g4 * 8 + h2 * 4) = v;
        }
    }
  }
}

// --------------------------------------------------------------------------------------------
// backward, pass K: dK, dV
// --------------------------------------------------------------------------------------------
template <int DH, int NB>
// (four wavefronts: this kernel needs more registers than seven wavefronts per workgroup, two workgroups per
// compute unit, would leave it, and measured slower with seven and one workgroup)
__global__ void __launch_bounds__(256, 2) attn_bwd_k_mfma_k(const bf16* __restrict__ qkv, const float* __restrict__ delta_ws,
                                                         const float* __restrict__ lse, const bf16* __restrict__ dO,
                                                         bf16* __restrict__ dqkv, int T, int H, long long ntiles, int cls_only) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int TP = NB * 32, LDR = DH + 8, KS = DH / 16, DB = DH / 32;
  bf16* Qs = reinterpret_cast<bf16*>(smem);   // [TP][LDR]
  bf16* Gs = Qs + TP * LDR;                   // [TP][LDR]  dO
  float* ls = reinterpret_cast<float*>(Gs + TP * LDR);  // [TP] lse * log2(e), +inf on padding rows
  float* dl = ls + TP;                                  // [TP] delta
  // workgroup ids are dealt round-robin to the 8 XCDs: the heads of one tile go to one XCD, next to each other
  // in time, so the neighbouring 128-byte head slices of its token rows meet in one L2
  int h = (blockIdx.x / 8) % H;
  long long tile = (long long)(blockIdx.x / 8 / H) * 8 + blockIdx.x % 8;
  if (tile >= ntiles) return;
  int D = H * DH;
  long long gs = 3LL * D;
  const bf16* base = qkv + tile * T * gs + h * DH;
  const bf16* gbase = dO + tile * T * (long long)D + h * DH;
  const int TG = cls_only ? 1 : T;   // rows of dO that are defined (cls_only: query 0 alone carries a gradient)
  static_assert(TP <= 256, "one row of delta / lse per thread");
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int li = lane & 31, h2 = lane >> 5;
  // Everything that comes from global memory before the main loop is requested up front, in one go, so that the
  // workgroup waits for one memory latency and not for one per step: delta and log-sum-exp of row i = thread id (no
  // branches around the loads: rows past the end read the last defined row and are overwritten below), the K/V
  // fragments of the wavefront's first key block, then the Q / dO copy.
  float d_row, l_row;   // delta_i = dO_i . O_i (left by the query-owned pass) and the log-sum-exp of row i = thread id
  {
    int i = threadIdx.x < TG ? threadIdx.x : TG - 1;
    d_row = delta_ws[(tile * H + h) * T + i];
    l_row = lse[(tile * H + h) * T + i];
  }
  bf16x8 fk[KS], fv[KS];
  auto load_kv = [&](int kb, bf16x8 (&k8)[KS], bf16x8 (&v8)[KS]) __attribute__((always_inline)) {
    int key = kb * 32 + li;
    int kc = key < T ? key : T - 1;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      k8[ks] = as_bf16x8(ldg16(base + D + kc * gs + ks * 16 + h2 * 8));
      v8[ks] = as_bf16x8(ldg16(base + 2 * D + kc * gs + ks * 16 + h2 * 8));
    }
  };
  load_kv(wave, fk, fv);
  load_rm2<DH, TP, 256, true>(base, gs, T, Qs, gbase, D, TG, Gs, [&] { l_row *= LOG2E; });
  if (threadIdx.x < TP) {
    bool def = threadIdx.x < TG;
    dl[threadIdx.x] = def ? d_row : 0.f;
    ls[threadIdx.x] = def ? l_row : INFINITY;   // +inf on padding rows: their probabilities come out as zero
  }
  __syncthreads();
  float scale = 1.0f / sqrtf((float)DH);
  float sl2 = LOG2E * scale;
  const bf16* const qrow0 = Qs + li * LDR + h2 * 8;
  const bf16* const grow0 = Gs + li * LDR + h2 * 8;
  const bf16* const qtr0 = Qs + tr_lane_off(LDR, lane);
  const bf16* const gtr0 = Gs + tr_lane_off(LDR, lane);
  const int nlast = T - (NB - 1) * 32;   // real queries in the last block (1 .. 32)
  for (int kb = wave; kb < NB; kb += 4) {
    int key = kb * 32 + li;
    // the fragments of the wavefront's next key block travel while this one is worked on
    const bool more = kb + 4 < NB;   // uniform
    bf16x8 nk[KS], nv[KS];
    if (more) load_kv(kb + 4, nk, nv);
    f32x16 dk[DB], dv[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) { dk[d][r] = 0.f; dv[d][r] = 0.f; }
    const bf16* qrow = qrow0;
    const bf16* grow = grow0;
    const bf16* qtr = qtr0;
    const bf16* gtr = gtr0;
    const float* lsq = ls + h2 * 4;
    const float* dlq = dl + h2 * 4;
    // one block of 32 queries; LASTQ: the head's last block, the only one with padding rows: accumulator registers
    // 4g .. 4g + 3 hold queries 8g .. 8g + 7 of the block, and a group past the last real query is zero without being
    // computed (no exponential); the second slice of both products is skipped where the upper 16 queries are padding
    auto q_block = [&](auto lastq) __attribute__((always_inline)) {
      constexpr bool LASTQ = decltype(lastq)::value;
      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 a = *reinterpret_cast<const bf16x8*>(qrow + ks * 16);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, fk[ks], s, 0, 0, 0);
        bf16x8 g = *reinterpret_cast<const bf16x8*>(grow + ks * 16);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(g, fv[ks], dp, 0, 0, 0);
      }
      float p[16], ds[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {   // accumulator registers 4 g4 .. 4 g4 + 3 are four consecutive queries
        if (LASTQ && g4 * 8 >= nlast) {   // uniform
#pragma unroll
          for (int e = 0; e < 4; ++e) { p[g4 * 4 + e] = 0.f; ds[g4 * 4 + e] = 0.f; }
          continue;
        }
        float4 lv = *reinterpret_cast<const float4*>(lsq + g4 * 8), dv4 = *reinterpret_cast<const float4*>(dlq + g4 * 8);
        float lr[4] = {lv.x, lv.y, lv.z, lv.w}, dr[4] = {dv4.x, dv4.y, dv4.z, dv4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          int r = g4 * 4 + e;
          p[r] = __builtin_amdgcn_exp2f(s[r] * sl2 - lr[e]);  // padding rows: lse = +inf -> 0
          ds[r] = p[r] * (dp[r] - dr[e]);
        }
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        if (LASTQ && t == 1 && nlast <= 16) continue;   // uniform
        bf16x8 pb = pack8(p + 8 * t);
        bf16x8 db = pack8(ds + 8 * t);
#pragma unroll
        for (int d = 0; d < DB; ++d) {
          bf16x8 ag = frag_tr_at(gtr, LDR, 16 * t * LDR + d * 32);
          dv[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ag, pb, dv[d], 0, 0, 0);
          bf16x8 aq = frag_tr_at(qtr, LDR, 16 * t * LDR + d * 32);
          dk[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, db, dk[d], 0, 0, 0);
        }
      }
    };
    const int nfull = cls_only ? 1 : NB - 1;
#pragma unroll 1
    for (int qb = 0; qb < nfull; ++qb, qrow += 32 * LDR, grow += 32 * LDR, qtr += 32 * LDR, gtr += 32 * LDR, lsq += 32, dlq += 32)
      q_block(std::false_type{});
    if (!cls_only) q_block(std::true_type{});
    if (key < T) {
      bf16* outk = dqkv + (tile * T + key) * gs + D + h * DH;
      bf16* outv = outk + D;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16x4 vk, vv;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            vk[i] = (bf16)(dk[d][g4 * 4 + i] * scale);
            vv[i] = (bf16)dv[d][g4 * 4 + i];
          }
          *reinterpret_cast<bf16x4*>(outk + d * 32 + g4 * 8 + h2 * 4) = vk;
          *reinterpret_cast<bf16x4*>(outv + d * 32 + g4 * 8 + h2 * 4) = vv;
        }
    }
    if (more) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) { fk[ks] = nk[ks]; fv[ks] = nv[ks]; }
    }
  }
}

template <int DH, int NB> constexpr size_t fwd_lds() { return (size_t)2 * NB * 32 * (DH + 8) * 2; }
template <int DH, int NB> constexpr size_t bq_lds() { return (size_t)2 * NB * 32 * (DH + 8) * 2; }
template <int DH, int NB> constexpr size_t bk_lds() {
  return (size_t)2 * NB * 32 * (DH + 8) * 2 + (size_t)2 * NB * 32 * 4;
}

template <typename K>
hipError_t set_lds(K kernel, size_t bytes) {
  if (bytes <= 65536) return hipSuccess;
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int DH, int NB>
hipError_t fwd_go(const void* qkv, void* O, float* lse, long long n, int T, int H, int cls_only, hipStream_t s) {
  size_t lds = fwd_lds<DH, NB>();
  hipError_t e = set_lds(attn_fwd_mfma_k<DH, NB>, lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_fwd_mfma_k<DH, NB>), dim3((unsigned)((n + 7) / 8 * 8 * H)), dim3(attn_threads<NB>()), lds, s,
                     (const bf16*)qkv, (bf16*)O, lse, T, H, n, cls_only);
  return hipGetLastError();
}

template <int DH, int NB>
hipError_t bwd_go(const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv, float* delta_ws,
                  long long n, int T, int H, int cls_only, hipStream_t s) {
  size_t lq = bq_lds<DH, NB>(), lk = bk_lds<DH, NB>();
  hipError_t e = set_lds(attn_bwd_q_mfma_k<DH, NB>, lq);
  if (e != hipSuccess) return e;
  e = set_lds(attn_bwd_k_mfma_k<DH, NB>, lk);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_q_mfma_k<DH, NB>), dim3((unsigned)((n + 7) / 8 * 8 * H)), dim3(attn_threads<NB>()), lq, s,
                     (const bf16*)qkv, (const bf16*)O, lse, (const bf16*)dO, (bf16*)dqkv, delta_ws, T, H, n, cls_only);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_k_mfma_k<DH, NB>), dim3((unsigned)((n + 7) / 8 * 8 * H)), dim3(256), lk, s,
                     (const bf16*)qkv, (const float*)delta_ws, lse, (const bf16*)dO, (bf16*)dqkv, T, H, n, cls_only);
  return hipGetLastError();
}

}  // namespace

// built shapes: head width 64 with 193..224 tokens (ViT-*/16 at 224 px), head width 32 with <= 32 tokens
bool attn_mfma_ok(int T, int dh) {
  int nb = (T + 31) / 32;
  return (dh == 64 && nb == 7) || (dh == 32 && nb == 1);
}

hipError_t launch_attn_fwd_mfma(const void* qkv, void* O, float* lse, long long n, int T, int H, int dh, int cls_only,
                                hipStream_t s) {
  if (dh == 64) return fwd_go<64, 7>(qkv, O, lse, n, T, H, cls_only, s);
  return fwd_go<32, 1>(qkv, O, lse, n, T, H, cls_only, s);
}

hipError_t launch_attn_bwd_mfma(const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv, float* delta_ws,
                                long long n, int T, int H, int dh, int cls_only, hipStream_t s) {
  if (dh == 64) return bwd_go<64, 7>(qkv, O, lse, dO, dqkv, delta_ws, n, T, H, cls_only, s);
  return bwd_go<32, 1>(qkv, O, lse, dO, dqkv, delta_ws, n, T, H, cls_only, s);
}

}  // namespace sl
