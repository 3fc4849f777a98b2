// bf16 MFMA "NT" GEMM for gfx950, large-M variant: C[M,N] = A[M,K] * B[N,K]^T (+ fused epilogue).
//
// The encoder's GEMMs have a short contraction (K = D or 4D) and a huge M (all tokens of the slide), so
// per output tile there is little MFMA work to hide the operand traffic behind.  What one compute unit can
// pull out of its L2 (measured: < 50 bytes per clock) bounds the tile from below: a 256 x 192 tile needs
// (256 + 192) * 2 bytes per 256 * 192 * 2 flop, about 37 bytes per MFMA clock.  192 divides every N that
// occurs (D, 3D, 4D for D = 384 and 768), so no column tile is partly empty.
//   * One persistent workgroup of 4 wavefronts per compute unit (one per SIMD, the whole register file
//     each); a wavefront owns 128 x 96 of the tile (4 x 3 accumulators of 32 x 32), so every fragment read
//     from LDS feeds three or four MFMAs.  Tiles that share an A row panel run at the same time on one XCD.
//   * Operands travel global -> registers -> LDS.  The A loads of K step k + 2 and the B loads of step
//     k + 1 are issued during step k and stay in flight (in registers) across steps and across tile
//     boundaries, which covers an HBM miss on the A panel; LDS holds two stages of [256 + 192][64 + 8]
//     bf16 (two separate arrays, so that writes to one are free to move past reads of the other) and
//     needs one barrier per step.  The order of MFMA, LDS and global instructions inside a step is pinned.
//   * The MFMA operands are passed swapped (B fragment first), so a lane's accumulator registers are runs
//     of four neighbouring columns of one row: the epilogue moves them through a wave-private LDS patch
//     with 16-byte writes and gets 8-column row segments back, all global traffic being 16-byte accesses
//     along rows.  The bias is the initial value of the accumulators.
//   * GELU and its derivative come from a table of the normal CDF and of d/dx (x cdf(x)) in LDS, linearly
//     interpolated at 1/64 steps (error < 2e-5, far below bf16 rounding): seven VALU instructions per
//     element instead of an erf evaluation; with K = 384 the VALU time of the epilogue is otherwise of the
//     order of the tile's MFMA time.
#include "gemm_epi.h"

#include <type_traits>
#include <utility>

namespace sl {

namespace {

constexpr int NXCD = 8;
constexpr int BM = 256, BN = 192, BK = 64, LDT = BK + 8, NTH = 256;
constexpr int WBM = 4, WBN = 3;                    // 32 x 32 accumulators per wavefront: 128 x 96, waves 2 x 2
constexpr int RSTEP = NTH / 8;                     // rows per loader pass
constexpr int CA = BM / RSTEP, CB = BN / RSTEP;    // 16-byte chunks per thread and K step
constexpr int STAGE = (BM + BN) * LDT;             // bf16 elements per LDS stage
constexpr int TAB_N = 1024;                        // table over [-8, 8) in steps of 1/64
constexpr int PS = 100;                            // patch row stride in floats (96 + 4)
static_assert((NTH / 64) * 32 * PS * 4 <= STAGE * 2, "epilogue patches alias stage 1 of the operand ring");

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 ldg16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }
// uniform base (scalar registers) + 32-bit per-lane byte offset
__device__ __forceinline__ u32x4 ldg16(const char* base, unsigned off) { return *reinterpret_cast<const u32x4*>(base + off); }

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// 8 floats -> 8 bf16 (round to nearest even), four packed conversions
__device__ __forceinline__ u32x4 pack8(const float (&v)[8]) {
  u32x4 r;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    f32x2 f = {v[2 * w], v[2 * w + 1]};
    bf16x2 h = __builtin_convertvector(f, bf16x2);
    r[w] = __builtin_bit_cast(unsigned, h);
  }
  return r;
}
__device__ __forceinline__ void unpack8(u32x4 t, float (&v)[8]) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    v[2 * w] = __uint_as_float(t[w] << 16);
    v[2 * w + 1] = __uint_as_float(t[w] & 0xffff0000u);
  }
}

// table entry k: {cdf(x_k), cdf(x_k+1) - cdf(x_k), dg(x_k), dg(x_k+1) - dg(x_k)}, x_k = -8 + k/64,
// cdf = standard normal distribution function, dg(x) = cdf(x) + x * pdf(x) = d/dx (x cdf(x))
__device__ __forceinline__ void table_pos(float x, int* k, float* f) {
  float t = fminf(fmaxf(x * 64.0f + 512.0f, 0.0f), 1023.0f);
  float fl = floorf(t);
  *k = (int)fl;
  *f = t - fl;
}
__device__ __forceinline__ float gelu_tab(const float4* tab, float x) {
  int k; float f;
  table_pos(x, &k, &f);
  float2 e = *reinterpret_cast<const float2*>(tab + k);
  return x * (e.x + f * e.y);
}
__device__ __forceinline__ void gelu_both_tab(const float4* tab, float x, float* gl, float* dg) {
  int k; float f;
  table_pos(x, &k, &f);
  float4 e = tab[k];
  *gl = x * (e.x + f * e.y);
  *dg = e.z + f * e.w;
}

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// ---- epilogue of one wavefront's 128 x 96 block -------------------------------------------------
// Accumulator element r of lane l (operands swapped) is row l % 32, column (r / 4) * 8 + (l / 32) * 4 + r % 4
// of its 32 x 32 block.  Per 32-row strip the wave writes its accumulators to a private LDS patch (12
// 16-byte writes per lane) and reads them back as 8-column row segments: 12 lanes per row, 5 rows per
// pass, 7 passes (lanes 60..63 idle, the last pass holds rows 30 and 31), so the lane -> (row, segment)
// map is the same in every pass and all offsets are immediates.  Everything that does not depend on the
// lane is wave-uniform (scalar registers); per-lane global offsets are 32-bit.
// A strip is processed in two halves (passes 0..3, 4..6); the auxiliary operand (residual row,
// pre-activation, position row) of a half is fetched while the half before it is processed.
template <int MODE, typename RS>
struct Epi {
  static constexpr bool HAS_AUX = MODE == EPI_BIAS_RESID || MODE == EPI_DGELU || MODE == EPI_PATCH;
  static constexpr bool AUX_F32 = MODE == EPI_PATCH || (MODE == EPI_BIAS_RESID && sizeof(RS) == 4);
  struct Aux {
    u32x4 lo[HAS_AUX ? 4 : 1];
    u32x4 hi[AUX_F32 ? 4 : 1];
  };
};

template <int MODE, typename RS, int DBG>
struct BigEpilogue {
  using E = Epi<MODE, RS>;
  using Aux = typename E::Aux;
  static constexpr int UNITS = 2 * WBM;
  const GemmNT& g;
  const float4* tab;
  int mw, nw;        // first row / column of the wave's block (uniform)
  int rl, sg8;       // lane's row inside a pass (>= 4096: idle lane) and first column of its 8-column segment
  int rl0;           // rl, or 0 for idle lanes (addresses stay valid)
  // Per-lane element offsets rl0 * ld + sg8 for the leading dimensions in use.  They are derived from a
  // lane id the optimiser cannot see through, once per tile: values that are invariant over the whole
  // kernel would otherwise be kept in registers across the K loop, where there are none to spare.
  unsigned vo_c, vo_c2, vo_a;
  int ldc, ldc2, lda_;   // leading dimensions of out, out2 and the auxiliary operand, opaque copies for the same reason

  __device__ __forceinline__ BigEpilogue(const GemmNT& g_, const float4* tab_, int mw_, int nw_, int lane)
      : g(g_), tab(tab_), mw(mw_), nw(nw_) {
    asm volatile("" : "+v"(lane));
    ldc = (int)g.ldc; ldc2 = (int)g.ldc2; lda_ = (int)(MODE == EPI_BIAS_RESID ? g.ldr : g.ldpre);
    asm volatile("" : "+s"(ldc), "+s"(ldc2), "+s"(lda_));
    rl0 = lane < 60 ? lane / 12 : 0;
    rl = lane < 60 ? rl0 : 4096;
    sg8 = (lane % 12) * 8;
    vo_c = (unsigned)(rl0 * ldc + sg8);
    vo_c2 = (unsigned)(rl0 * ldc2 + sg8);
    vo_a = (unsigned)(rl0 * lda_ + sg8);
  }
  // passes of half-strip unit u: [p0, p1)
  static constexpr int p0(int u) { return (u & 1) ? 4 : 0; }
  static constexpr int p1(int u) { return (u & 1) ? 7 : 4; }

  // rows of strip i that exist (uniform)
  __device__ __forceinline__ int rows_left(int i) const {
    long long r = g.M - ((long long)mw + i * 32);
    return r > 32 ? 32 : (int)r;
  }

  template <int U>
  __device__ __forceinline__ void fetch(Aux& a) const {
    if (!E::HAS_AUX) return;
    constexpr int i = U >> 1;
    int lim = rows_left(i);
#pragma unroll
    for (int p = p0(U); p < p1(U); ++p) {
      if (p * 5 >= lim) continue;             // uniform: no row of this pass exists
      int q = p - p0(U);
      bool ok = rl < lim - p * 5;             // lanes past the end read the pass's first row (never stored)
      long long rs = (long long)mw + i * 32;  // first row of the strip
      long long r0 = rs + p * 5;
      if (MODE == EPI_BIAS_RESID) {
        const RS* src = (const RS*)g.resid + (rs * lda_ + nw) + (unsigned)(p * 5 * lda_) + (ok ? vo_a : (unsigned)sg8);
        a.lo[q] = *reinterpret_cast<const u32x4*>(src);
        if (sizeof(RS) == 4) a.hi[q] = *reinterpret_cast<const u32x4*>((const float*)src + 4);
      } else if (MODE == EPI_DGELU) {
        const bf16* src = (const bf16*)g.pre + (rs * lda_ + nw) + (unsigned)(p * 5 * lda_) + (ok ? vo_a : (unsigned)sg8);
        a.lo[q] = *reinterpret_cast<const u32x4*>(src);
      } else if (MODE == EPI_PATCH) {
        unsigned m = (unsigned)r0 + (ok ? (unsigned)rl0 : 0u);
        const float* src = g.pos + (size_t)(1 + m % (unsigned)g.cmap.g2) * g.N + (nw + sg8);
        a.lo[q] = *reinterpret_cast<const u32x4*>(src);
        a.hi[q] = *reinterpret_cast<const u32x4*>(src + 4);
      }
    }
  }

  template <typename OT>
  __device__ __forceinline__ void put(OT* dst, const float (&v)[8]) const {
    if (sizeof(OT) == 4) {
      reinterpret_cast<float4*>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
      reinterpret_cast<float4*>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      *reinterpret_cast<u32x4*>(dst) = pack8(v);
    }
  }

  // one half strip: 3 or 4 passes read from the patch, combined with the auxiliary operand and stored
  template <int U>
  __device__ __forceinline__ void half(const float* pr, const Aux& a) const {
    constexpr int i = U >> 1;
    int lim = rows_left(i);
    float4 va[4], vb[4];
#pragma unroll
    for (int p = p0(U); p < p1(U); ++p) {
      const float4* src = reinterpret_cast<const float4*>(pr + p * 5 * PS);
      va[p - p0(U)] = src[0];
      vb[p - p0(U)] = src[1];
    }
#pragma unroll
    for (int p = p0(U); p < p1(U); ++p) {
      if (p * 5 >= lim) continue;   // uniform
      int q = p - p0(U);
      float v[8] = {va[q].x, va[q].y, va[q].z, va[q].w, vb[q].x, vb[q].y, vb[q].z, vb[q].w};
      float t[8];
      if (E::AUX_F32) {
#pragma unroll
        for (int w = 0; w < 4; ++w) { t[w] = __uint_as_float(a.lo[q][w]); t[4 + w] = __uint_as_float(a.hi[q][w]); }
      } else if (E::HAS_AUX) {
        unpack8(a.lo[q], t);
      }
      if (DBG & 32) {  // tuning: all epilogue arithmetic, no global stores
        float sacc = 0.f;
        if (MODE == EPI_BIAS_GELU) { for (int e = 0; e < 8; ++e) { float gl, dg; gelu_both_tab(tab, v[e], &gl, &dg); sacc += dg + gl; } }
        else if (E::HAS_AUX) { for (int e = 0; e < 8; ++e) sacc += v[e] + t[e]; }
        else { for (int e = 0; e < 8; ++e) sacc += v[e]; }
        if (sacc == 12345.678f) ((float*)g.out)[0] = sacc;
        continue;
      }
      long long rs = (long long)mw + i * 32;           // first row of the strip (uniform)
      long long r0 = rs + p * 5;                       // first row of the pass
      unsigned oc = (unsigned)(p * 5 * ldc), oc2 = (unsigned)(p * 5 * ldc2);
      if (rl < lim - p * 5) {
        if (MODE == EPI_PLAIN || MODE == EPI_BIAS) {
          put((bf16*)g.out + (rs * ldc + nw) + oc + vo_c, v);
        } else if (MODE == EPI_BIAS_RESID) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += t[e];
          put((RS*)g.out + (rs * ldc + nw) + oc + vo_c, v);
        } else if (MODE == EPI_BIAS_GELU) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float gl, dg;
            gelu_both_tab(tab, v[e], &gl, &dg);
            v[e] = gl;
            t[e] = dg;
          }
          put((bf16*)g.out + (rs * ldc + nw) + oc + vo_c, v);
          put((bf16*)g.out2 + (rs * ldc2 + nw) + oc2 + vo_c2, t);
        } else if (MODE == EPI_DGELU) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] *= t[e];
          put((bf16*)g.out + (rs * ldc + nw) + oc + vo_c, v);
        } else {  // EPI_PATCH: output rows go through the row map
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += t[e];
          put((RS*)g.out + g.cmap.map32((unsigned)r0 + (unsigned)rl0) * g.ldc + (nw + sg8), v);
        }
      }
    }
  }

  mutable long long et[2 * UNITS + 1];
  template <int U>
  __device__ __forceinline__ void unit(f32x16 (&acc)[WBM][WBN], float* pw, const float* pr, Aux& cur) const {
    if constexpr (U < UNITS) {
      constexpr int i = U >> 1;
      if (DBG & 64) et[2 * U] = clock64();
      if ((U & 1) == 0) {
#pragma unroll
        for (int j = 0; j < WBN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            *reinterpret_cast<float4*>(pw + j * 32 + q * 8) =
                make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
        // the patch is private to the wave and LDS operations of one wave execute in order: no barrier,
        // but the compiler must not move the reads above the writes of other lanes
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      }
      if (DBG & 64) et[2 * U + 1] = clock64();
      Aux nxt;
      if constexpr (U + 1 < UNITS) fetch<U + 1>(nxt);
      half<U>(pr, cur);
      if (DBG & 64) et[2 * U + 2] = clock64();
      if ((U & 1) == 1) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // reads done before the next strip's writes
      if constexpr (U + 1 < UNITS) {
        cur = nxt;
        unit<U + 1>(acc, pw, pr, cur);
      }
    }
  }
};

// DBG (tuning builds only): 2 = no epilogue, 4 = no operand loads, 8 = A panel always in L2, 32 = no stores
template <typename RS, int MODE, int DBG>
__global__ void __launch_bounds__(NTH) gemm_nt_big_k(GemmNT g, int MT, int NTL) {
  // two separate arrays: the compiler then knows that the LDS writes of the next step's operands do not alias
  // the fragment reads of the current one and is free to interleave them
  __shared__ __attribute__((aligned(16))) bf16 ring0[STAGE];
  __shared__ __attribute__((aligned(16))) bf16 ring1[STAGE];
  __shared__ float4 tab[TAB_N];
  __shared__ __attribute__((aligned(16))) float lbias_all[BN];  // zeros when there is no bias
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = tid >> 3, kc = tid & 7;       // loader: 32 rows x 8 chunks of 16 bytes per pass
  const int soff = row0 * LDT + kc * 8;
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  const int nk = g.K / BK;
  const int total = (MT + NXCD - 1) / NXCD * NXCD * NTL;
  constexpr bool has_bias = MODE != EPI_PLAIN && MODE != EPI_DGELU;

  if (MODE == EPI_BIAS_GELU) {
    // filled once per workgroup; the K-loop barriers order it before the first epilogue
    for (int k = tid; k < TAB_N; k += NTH) {
      float x0 = -8.0f + (float)k * (1.0f / 64.0f), x1 = x0 + (1.0f / 64.0f);
      float c0 = 0.5f * (1.0f + erff(x0 * 0.70710678118654752f)), c1 = 0.5f * (1.0f + erff(x1 * 0.70710678118654752f));
      float d0 = c0 + x0 * 0.39894228040143268f * expf(-0.5f * x0 * x0);
      float d1 = c1 + x1 * 0.39894228040143268f * expf(-0.5f * x1 * x1);
      tab[k] = make_float4(c0, c1 - c0, d0, d1 - d0);
    }
  }

  // tile id -> (row tile, column tile): ids are dealt round-robin to the XCDs and the column tiles of one
  // row panel get consecutive slots of one XCD (the grid size is a multiple of 8)
  auto tile_of = [&](int id, long long& m0, int& n0) {
    int xcd = id % NXCD, slot = id / NXCD;
    int mt = (slot / NTL) * NXCD + xcd;
    m0 = (long long)mt * BM;
    n0 = (slot % NTL) * BN;
    return mt < MT;
  };
  auto next_valid = [&](int id, long long& m0, int& n0) {
    while (id < total && !tile_of(id, m0, n0)) id += gridDim.x;
    return id;
  };

  // operand addresses of the tile whose loads are being issued: uniform base + 32-bit per-thread offsets
  const bf16* Ab;
  const bf16* Bb;
  unsigned aoff[CA], boff[CB];
  u32x4 ra[2][CA], rb[CB];   // A: two register slots (loads two steps ahead, it may miss to HBM); B: one (L2 hits)
  float rbias = 0.f;
  bool off_special = true;   // aoff must be (re)built
#pragma unroll
  for (int i = 0; i < CB; ++i) boff[i] = 2u * (unsigned)((row0 + i * RSTEP) * (int)g.ldb + kc * 8);  // bytes; N % 96 == 0: no clamp
  auto set_offsets_a = [&](long long m0) {
    if (DBG & 8) m0 = (m0 / BM % 8) * BM;  // tuning: every A load hits L2
    long long base_row = g.amap.map32((unsigned)m0);
    Ab = (const bf16*)g.A + base_row * g.lda;
    // per-thread offsets depend on the tile only through the row map and the clamp at the last row:
    // they are rebuilt for such tiles (and for the tile after one), otherwise kept
    bool special = g.amap.g2 != 0 || m0 + BM > g.M;
    if (special || off_special) {
#pragma unroll
      for (int i = 0; i < CA; ++i) {
        unsigned am = (unsigned)m0 + (unsigned)(row0 + i * RSTEP);  // M < 2^31
        if (am > (unsigned)g.M - 1u) am = (unsigned)g.M - 1u;  // rows past the end are loaded (valid memory) but never stored
        aoff[i] = 2u * (unsigned)((g.amap.map32(am) - base_row) * g.lda + kc * 8);  // bytes
      }
    }
    off_special = special;
  };
  auto set_offsets_b = [&](int n0) {
    Bb = (const bf16*)g.B + (long long)n0 * g.ldb;
    if (has_bias && tid < BN) rbias = g.bias[n0 + tid];  // else stays 0
  };
  auto issue_a = [&](auto slot, int k0) {
    constexpr int S = decltype(slot)::value;
    if (DBG & 4) return;
#pragma unroll
    for (int i = 0; i < CA; ++i) ra[S][i] = ldg16((const char*)(Ab + k0), aoff[i]);
  };
  auto issue_b = [&](int k0) {
    if (DBG & 4) return;
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[i] = ldg16((const char*)(Bb + k0), boff[i]);
  };
  auto stash = [&](auto slot) {
    constexpr int S = decltype(slot)::value;
    bf16* st = S ? ring1 : ring0;
#pragma unroll
    for (int i = 0; i < CA; ++i) *reinterpret_cast<u32x4*>(st + soff + i * RSTEP * LDT) = ra[S][i];
#pragma unroll
    for (int i = 0; i < CB; ++i) *reinterpret_cast<u32x4*>(st + BM * LDT + soff + i * RSTEP * LDT) = rb[i];
  };

  long long m0, m1;
  int n0, n1;
  int id = next_valid(blockIdx.x, m0, n0);
  if (id >= total) return;
  // prologue: step 0 in LDS stage 0, steps 1 and 2 in flight in register slots 1 and 0
  set_offsets_a(m0);
  set_offsets_b(n0);
  // (the order of these loads is fenced: the waits the compiler places in the K loop are the most
  // conservative over every way into it, this one included)
  issue_a(std::integral_constant<int, 0>{}, 0);
  issue_b(0);
  __builtin_amdgcn_sched_barrier(0);
  issue_a(std::integral_constant<int, 1>{}, BK);
  __builtin_amdgcn_sched_barrier(0);
  stash(std::integral_constant<int, 0>{});
  __builtin_amdgcn_sched_barrier(0);
  issue_b(BK);
  __builtin_amdgcn_sched_barrier(0);
  issue_a(std::integral_constant<int, 0>{}, 2 * BK);
  __builtin_amdgcn_sched_barrier(0);
  if (tid < BN) lbias_all[tid] = rbias;
  __syncthreads();

  int tcount = 0;
  long long tstamp[6];
  while (id < total) {
    if (DBG & 64) tstamp[0] = clock64();
    int nid = next_valid(id + gridDim.x, m1, n1);
    if (nid >= total) { m1 = m0; n1 = n0; }  // no further tile: the prefetches re-read this one and are dropped
    const long long mw = m0 + wm * (WBM * 32);
    const int nw = n0 + wn * (WBN * 32);

    // the bias (or zero) is the initial value of the accumulators
    f32x16 acc[WBM][WBN];
#pragma unroll
    for (int j = 0; j < WBN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        if (has_bias) b = *reinterpret_cast<const float4*>(lbias_all + wn * (WBN * 32) + j * 32 + q * 8 + (lane >> 5) * 4);
#pragma unroll
        for (int i = 0; i < WBM; ++i) {
          acc[i][j][4 * q] = b.x; acc[i][j][4 * q + 1] = b.y; acc[i][j][4 * q + 2] = b.z; acc[i][j][4 * q + 3] = b.w;
        }
      }

    // MFMA fragments: two buffers of one 16-wide slice each
    bf16x8 fa[2][WBM], fb[2][WBN];
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    // fragment t (0..3: A row blocks, 4..6: B column blocks) of slice KS of stage S -> buffer BF
    auto rd_one = [&](auto slot, auto slice, auto buf, auto frag) {
      constexpr int S = decltype(slot)::value, KS = decltype(slice)::value, BF = decltype(buf)::value;
      constexpr int T = decltype(frag)::value;
      const bf16* st = S ? ring1 : ring0;
      if constexpr (T < WBM) {
        const bf16* as = st + (wm * (WBM * 32) + frow) * LDT + fk + KS * 16;
        fa[BF][T] = *reinterpret_cast<const bf16x8*>(as + T * 32 * LDT);
      } else {
        const bf16* bs = st + BM * LDT + (wn * (WBN * 32) + frow) * LDT + fk + KS * 16;
        fb[BF][T - WBM] = *reinterpret_cast<const bf16x8*>(bs + (T - WBM) * 32 * LDT);
      }
    };
    // LDS write w of the next stage: 0..7 the A chunks of register slot S, 8..13 the B chunks
    auto wr_one = [&](auto slot, auto idx) {
      constexpr int S = decltype(slot)::value, W = decltype(idx)::value;
      bf16* st = S ? ring1 : ring0;
      if constexpr (W < CA) *reinterpret_cast<u32x4*>(st + soff + W * RSTEP * LDT) = ra[S][W];
      else *reinterpret_cast<u32x4*>(st + BM * LDT + soff + (W - CA) * RSTEP * LDT) = rb[W - CA];
    };
    // global load l of a step: 0..5 the B chunks (they are needed first and hit L2), 6..13 the A chunks.
    // Loads return in order: the B chunks, issued one step before their LDS writes, do not wait for younger A
    // loads that may miss to HBM.
    auto ld_one = [&](auto slot, auto idx, int ka, int kb) {
      constexpr int S = decltype(slot)::value, Lx = decltype(idx)::value;
      if (DBG & 4) return;
      if constexpr (Lx < CB) rb[Lx] = ldg16((const char*)(Bb + kb), boff[Lx]);
      else ra[S][Lx - CB] = ldg16((const char*)(Ab + ka), aoff[Lx - CB]);
    };
    auto mfma_one = [&](auto buf, auto tt) {
      constexpr int BF = decltype(buf)::value, T = decltype(tt)::value, i = T / WBN, j = T % WBN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[BF][j], fa[BF][i], acc[i][j], 0, 0, 0);
    };
    // One K step out of LDS stage S, in explicit issue order: one MFMA and at most two memory instructions per
    // piece, a scheduling fence after each piece (one wavefront per SIMD: nothing else hides the LDS and
    // global-memory instructions, so they are dealt out between the 48 MFMAs).  The step's barrier sits
    // between slices 2 and 3: by then every fragment of this stage has been read and the next stage
    // (A: register slot S^1, loaded two steps ago; B: loaded one step ago) is completely written, so the
    // fragments of the next step's slice 0 are fetched under the MFMAs of slice 3 and no wavefront starts a
    // step with an empty MFMA pipe.  The registers are re-used for A three steps and B two steps ahead
    // (element offsets ka, kb).  NEXT_FRAGS = 0 for the last step of a tile.
    auto step_part1 = [&](auto slot, int ka, int kb) {
      constexpr int S = decltype(slot)::value;
      using SN = std::integral_constant<int, S ^ 1>;
      static_for<36>([&](auto pc) {
        constexpr int P = decltype(pc)::value, KS = P / 12, T = P % 12;
        mfma_one(std::integral_constant<int, KS & 1>{}, std::integral_constant<int, T>{});
        if constexpr (T < WBM + WBN)
          rd_one(slot, std::integral_constant<int, KS + 1>{}, std::integral_constant<int, (KS + 1) & 1>{},
                 std::integral_constant<int, T>{});
        if constexpr (KS < 2 && T >= 7) wr_one(SN{}, std::integral_constant<int, KS * 5 + T - 7>{});
        if constexpr (KS == 2 && T < 4) wr_one(SN{}, std::integral_constant<int, 10 + T>{});
        if constexpr (KS == 2 && T >= 7) ld_one(SN{}, std::integral_constant<int, T - 7>{}, ka, kb);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    auto step_part2 = [&](auto slot, auto next_frags, int ka, int kb) {
      constexpr int S = decltype(slot)::value;
      using SN = std::integral_constant<int, S ^ 1>;
      static_for<12>([&](auto tc) {
        constexpr int T = decltype(tc)::value;
        mfma_one(I1{}, tc);
        if constexpr (decltype(next_frags)::value && T < WBM + WBN) rd_one(SN{}, I0{}, I0{}, tc);
        if constexpr (T < 9) ld_one(SN{}, std::integral_constant<int, 5 + T>{}, ka, kb);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    auto step = [&](auto slot, int ka, int kb) {
      step_part1(slot, ka, kb);
      __syncthreads();
      step_part2(slot, I1{}, ka, kb);
    };

    static_for<WBM + WBN>([&](auto tc) { rd_one(I0{}, I0{}, I0{}, tc); });
    for (int kt = 0; kt < nk - 4; kt += 2) {
      step(I0{}, (kt + 3) * BK, (kt + 2) * BK);
      step(I1{}, (kt + 4) * BK, (kt + 3) * BK);
    }
    step(I0{}, (nk - 1) * BK, (nk - 2) * BK);   // step nk - 4
    set_offsets_a(m1);  // this tile needs no further A loads
    step(I1{}, 0, (nk - 1) * BK);               // step nk - 3
    set_offsets_b(n1);
    step(I0{}, BK, 0);                          // step nk - 2
    if (DBG & 64) tstamp[1] = clock64();

    // last step: the next tile's first operands go to stage 0 and every load up to its third step is in flight
    // BEFORE this tile's stores are issued (loads issued behind stores would wait for the stores to drain).
    // The epilogue patches live in stage 1.
    float* patch = reinterpret_cast<float*>(ring1) + wave * 32 * PS;
    BigEpilogue<MODE, RS, DBG> epi(g, tab, (int)mw, nw, lane);
    {
      typename BigEpilogue<MODE, RS, DBG>::Aux aux;
      step_part1(I1{}, 2 * BK, BK);
      epi.template fetch<0>(aux);
      step_part2(I1{}, I0{}, 2 * BK, BK);
      if (tid < BN) lbias_all[tid] = rbias;  // next tile's bias; this tile's was consumed at its start
      if (DBG & 64) tstamp[2] = clock64();
      __syncthreads();  // every wave is done with stage 1
      if (DBG & 64) tstamp[3] = clock64();
      if (DBG & 2) {
        if (acc[0][0][0] + acc[1][2][5] + acc[2][1][3] + acc[3][0][7] + acc[0][2][9] + acc[1][1][11] == 12345.678f) ((float*)g.out)[0] = 1.f;
      } else if (nw < g.N) {
        float* pw = patch + (lane & 31) * PS + (lane >> 5) * 4;
        const float* pr = patch + epi.rl0 * PS + epi.sg8;
        epi.template unit<0>(acc, pw, pr, aux);
      }
    }
    if (DBG & 64) tstamp[4] = clock64();
    __syncthreads();  // patches are read before the next tile's second step overwrites stage 1
    if (DBG & 64) {
      tstamp[5] = clock64();
      if (blockIdx.x == 17 && lane == 0 && tcount < 32) {
        long long* dbgout = (long long*)g.out2 + (tcount * 4 + wave) * 8;
        for (int q = 0; q < 6; ++q) dbgout[q] = tstamp[q];
        if (tcount == 5 && wave == 0) {
          long long* d2 = (long long*)g.out2 + 4096;
          for (int q = 0; q < 17; ++q) d2[q] = epi.et[q];
        }
      }
      ++tcount;
    }
    id = nid; m0 = m1; n0 = n1;
  }
}

}  // namespace

// Shapes this kernel takes: a contraction that is a whole number of double steps, and enough rows
// to fill the chip with 256-row tiles.  Alignment requirements are those of gemm_nt_mfma_ok.
bool gemm_nt_big_ok(const GemmNT& g) { return g.M < (1LL << 31) && g.N % BN == 0 &&
         g.lda < (1 << 20) && g.ldb < (1 << 20) && g.ldc < (1 << 20) && g.ldc2 < (1 << 20) && g.ldr < (1 << 20) && g.ldpre < (1 << 20) && g.K % (2 * BK) == 0 && g.K >= 4 * BK && g.M >= 4096 && g.N >= 96; }

template <int MODE, int DBG>
hipError_t launch_big(const GemmNT& g, hipStream_t s) {
  static int cus = 0;
  auto kern = gemm_nt_big_k<rs_bf16path_t, MODE, DBG>;
  if (!cus) {
    hipError_t e;
    int dev = 0;
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
    cus = prop.multiProcessorCount / NXCD * NXCD;
    if (cus < NXCD) cus = NXCD;
  }
  int MT = (int)((g.M + BM - 1) / BM), NTL = (g.N + BN - 1) / BN;
  long long total = (long long)((MT + NXCD - 1) / NXCD) * NXCD * NTL;
  long long wgs = total < cus ? total : cus;
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(NTH), 0, s, g, MT, NTL);
  return hipGetLastError();
}

template <int DBG>
hipError_t launch_big_mode(const GemmNT& g, hipStream_t s) {
  switch (g.epi) {
    case EPI_PLAIN: return launch_big<EPI_PLAIN, DBG>(g, s);
    case EPI_BIAS: return launch_big<EPI_BIAS, DBG>(g, s);
    case EPI_BIAS_RESID: return launch_big<EPI_BIAS_RESID, DBG>(g, s);
    case EPI_BIAS_GELU: return launch_big<EPI_BIAS_GELU, DBG>(g, s);
    case EPI_DGELU: return launch_big<EPI_DGELU, DBG>(g, s);
    case EPI_PATCH: return launch_big<EPI_PATCH, DBG>(g, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sl

namespace sl {
hipError_t launch_gemm_nt_big(const GemmNT& g, hipStream_t s) {
#ifdef SLIDE_DEBUG_HOOKS
  switch (g.dbg) {
    case 2: return launch_big_mode<2>(g, s);
    case 4: return launch_big_mode<4>(g, s);
    case 6: return launch_big_mode<6>(g, s);
    case 10: return launch_big_mode<10>(g, s);
    case 32: return launch_big_mode<32>(g, s);
    case 36: return launch_big_mode<36>(g, s);
    case 64: return launch_big_mode<64>(g, s);
    default: break;
  }
#endif
  return launch_big_mode<0>(g, s);
}
}  // namespace sl
