// bf16 MFMA weight-gradient GEMM for gfx950, large-M variant: C[N1,N2] = sum_m A[m,N1]^T B[m,N2] (fp32 partials).
//
// Same machine balance as the activation GEMMs (what a compute unit can pull out of its L2 bounds the tile from
// below), so the same tile area: one persistent workgroup of 8 wavefronts per compute unit (two per SIMD, 256
// registers each: while one waits for LDS, memory or the barrier the other issues), a 128 x 384 output tile
// (wavefront: 64 x 96), 64 rows of m per step, operands global -> registers -> LDS with the loads of X two steps
// and of Y one step ahead, MFMA / LDS / global instructions dealt out by hand.  What differs:
//   * The contraction runs over the ROW index of both operands.  The 64-row slices go to LDS as they are
//     (row-major, 16-byte stores) and the MFMA fragments, which need 8 consecutive contraction indices per
//     lane, are read with LDS transpose reads (ds_read_b64_tr_b16: a group of 16 lanes addresses a 4-row x
//     16-column patch and every lane receives one column of it).  No transposition in registers.
//   * M (all tokens of the slide) is split into slabs; a work item is (slab, output tile) and writes its partial
//     tile once, a second kernel adds the slabs in a fixed order (no atomics: results are run-to-run identical).
//     All tiles of a slab run on ONE XCD at about the same time, so the slab's rows come from HBM once and the
//     other tiles find them in that XCD's L2 (with tiles spread over XCDs the rows were fetched several times).
//   * The tile is as wide as the narrow operand of most of the encoder's weight gradients (384 columns), so a wide
//     A (1152 or 1536 columns, four fifths of the bytes) is read by exactly one workgroup and streams from HBM once
//     whatever the workgroups' relative progress; only the narrow operand is shared through L2, and its window (a
//     few steps x 48 kB per slab) is a small part of the 4 MB.  With 256 x 192 tiles every row was shared by up to
//     twelve workgroups that each run three steps of loads ahead: the windows of the slabs in flight on an XCD
//     filled its L2, any drift between the sharers missed, and the kernel moved 1.7 x its operand bytes.
//   * A (the gradient rows, N1 columns) is always the side tiled by 128, so its column sums (the bias gradient) come
//     out of the registers of its loads; B takes the 384 side.  Both must be covered exactly (N1 % 128 == 0,
//     N2 % 384 == 0: all the encoder's and the pool's weight-gradient shapes).
#include "slide_internal.h"

#include <type_traits>

namespace sl {

namespace {

constexpr int NXCD = 8;
#ifndef TN_WAVES
#define TN_WAVES 8
#endif
constexpr int BX = 128, BY = 384, BK = 64, NW = TN_WAVES, NTH = 64 * NW;
constexpr int WVM = 2, WVN = NW / WVM;              // wavefronts along X and Y
constexpr int RSTEP = NTH / 16;                     // rows per loader pass (16 lanes per 256-byte row segment)
constexpr int XL = BK / RSTEP, YG = BY / 128, YL = BK / RSTEP;   // 16-byte loads per thread and step: X XL, Y YG x YL
// LDS row: 128 X columns, 384 Y columns, pad.  The pad makes the row stride 64 bytes modulo 256 (16 banks): a
// transpose read's group of 16 lanes touches 4 rows x 32 bytes, and the two groups that are served together sit 32
// bytes apart, so with this stride their eight 32-byte pieces fall on eight different bank ranges (with a 16-byte
// stride modulo 256 they overlapped: 58 % of the LDS cycles were bank-conflict cycles).
constexpr int LDW = BX + BY + 32;
constexpr int STAGE = BK * LDW;                     // bf16 elements per LDS stage
constexpr int WBM = BX / (32 * WVM), WBN = BY / (32 * WVN);   // 32 x 32 accumulators per wavefront
static_assert(YG * 128 == BY && WBM == 2 && 2 * XL + 2 * YG * YL <= 3 * WBM * WBN, "loader split, fragment and piece schedule");

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 ldg16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// MFMA operand from a row-major LDS slice S[k][col] (row stride LDW): lane l gets column c0 + l % 32 and the
// contraction indices k0 + 8 * (l / 32) + {0..7}
__device__ __forceinline__ bf16x8 frag_tr(const bf16* S, int c0, int k0, int lane) {
  int g = lane >> 4, q = lane & 15;
  const bf16* p = S + (k0 + 8 * (g >> 1) + (q >> 2)) * LDW + c0 + 16 * (g & 1) + (q & 3) * 4;
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * LDW));
  s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

struct TnBig {
  const bf16* X; long long ldx; int NX;   // A: side tiled by 128
  const bf16* Y; long long ldy; int NY;   // B: side tiled by 384
  long long M;
  float* part;                            // partial of slab s: part[s * NX * NY + x * NY + y]
  float* cs_part;                         // column sums of X per slab, [slabs][NX]; may be null
  int slabs, spx;                         // slabs = 8 * spx: slabs xcd * spx .. xcd * spx + spx - 1 run on XCD xcd
  int TX, TY;
};

// uniform base (scalar registers) + 32-bit per-lane byte offset
__device__ __forceinline__ u32x4 ldg16o(const char* base, unsigned off) { return *reinterpret_cast<const u32x4*>(base + off); }

__global__ void __launch_bounds__(NTH) gemm_tn_big_k(TnBig g) {
  __shared__ __attribute__((aligned(16))) bf16 ring0[STAGE];
  __shared__ __attribute__((aligned(16))) bf16 ring1[STAGE];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WVN, wn = wave % WVN;
  // loader: 16 lanes cover 256 contiguous bytes of one row; thread t takes 16-byte chunk t % 16 of rows
  // t / 16 + RSTEP i of X, and the chunks t % 16 + 16 q (q < 3) of the same rows of Y
  const int lr = tid >> 4, lc = tid & 15;
  const int xcd = blockIdx.x % NXCD, wg = blockIdx.x / NXCD, wgs = gridDim.x / NXCD;
  const int tiles = g.TX * g.TY;
  const int items = g.spx * tiles;
  long long per = (g.M + g.slabs - 1) / g.slabs;
  per = (per + 2 * BK - 1) / (2 * BK) * (2 * BK);          // whole double steps
  const unsigned ldxb = 2u * (unsigned)g.ldx, ldyb = 2u * (unsigned)g.ldy;   // row strides in bytes
  const unsigned xo = (unsigned)lr * ldxb + lc * 16, yo = (unsigned)lr * ldyb + lc * 16;

  u32x4 rx[2][XL], ry[YG * YL];
  for (int idx = wg; idx < items; idx += wgs) {            // uniform for the workgroup
    const int s = xcd * g.spx + idx / tiles;
    const int tile = idx % tiles;
    const int x0 = (tile / g.TY) * BX, y0 = (tile % g.TY) * BY;
    const long long lo = (long long)s * per;
    const long long hi = lo + per < g.M ? lo + per : g.M;
    const int span = lo < hi ? (int)(hi - lo) : 0;         // rows of this slab (0: the partial is written as zeros)
    const int nk = span / (2 * BK) * 2;                    // whole double steps: the pipelined loop, no row is masked
    const int rem = span - nk * BK;                        // < 128 rows left over (last slab only): done on their own
    // Operand addresses: a uniform base per item plus 32-bit byte offsets (a slab spans far less than 4 GB).  Loads
    // that run ahead past the slab's end are redirected to its last row by clamping the offset (valid memory; what
    // they fetch is never multiplied).
    const char* const Xb = (const char*)(g.X + lo * g.ldx + x0);
    const char* const Yb = (const char*)(g.Y + lo * g.ldy + y0);
    const unsigned xmax = (unsigned)(span - 1) * ldxb + lc * 16, ymax = (unsigned)(span - 1) * ldyb + lc * 16;
    auto ld_x = [&](int row0, int i) {   // row0: first row of the step, relative to the slab (uniform)
      unsigned off = xo + (unsigned)(row0 + RSTEP * i) * ldxb;
      return ldg16o(Xb, off < xmax ? off : xmax);
    };
    auto ld_y = [&](int row0, int q, int i) {
      unsigned off = yo + (unsigned)(row0 + RSTEP * i) * ldyb;
      return ldg16o(Yb + q * 256, off < ymax ? off : ymax);
    };
    auto issue_x = [&](auto slot, int kt) {
      constexpr int S = decltype(slot)::value;
#pragma unroll
      for (int i = 0; i < XL; ++i) rx[S][i] = ld_x(kt * BK, i);
    };
    auto issue_y = [&](int kt) {
#pragma unroll
      for (int q = 0; q < YG; ++q)
#pragma unroll
        for (int i = 0; i < YL; ++i) ry[q * YL + i] = ld_y(kt * BK, q, i);
    };
    // zero a register whose row (relative to the slab) does not exist
    auto mask = [&](u32x4& v, int row) {
      bool ok = row < span;
#pragma unroll
      for (int w = 0; w < 4; ++w) v[w] = ok ? v[w] : 0u;
    };
    const bool cs_x = g.cs_part != nullptr && y0 == 0;
    float cs[8];   // column sums of this thread's chunk of X
#pragma unroll
    for (int c = 0; c < 8; ++c) cs[c] = 0.f;
    auto add_cs_row = [&](const u32x4& v, float wt = 1.0f) {   // wt: 1, or 0 for rows that are not part of the product
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        cs[2 * w] = fmaf(__uint_as_float(v[w] << 16), wt, cs[2 * w]);
        cs[2 * w + 1] = fmaf(__uint_as_float(v[w] & 0xffff0000u), wt, cs[2 * w + 1]);
      }
    };
    const int sx_off = lr * LDW + lc * 8, sy_off = lr * LDW + BX + lc * 8;
    // registers -> LDS stage (prologue and the left-over rows; the steps below do the same piecewise).  row0: first
    // row of the stage relative to the slab, for the zeroing of rows that do not exist (MASK)
    auto stash = [&](auto slot, auto stage, auto csm, auto msk, int row0) {
      constexpr int S = decltype(slot)::value, ST = decltype(stage)::value;
      constexpr int CSM = decltype(csm)::value;
      constexpr bool MASK = decltype(msk)::value;
      bf16* st = ST ? ring1 : ring0;
#pragma unroll
      for (int i = 0; i < XL; ++i) {
        if (MASK) mask(rx[S][i], row0 + lr + RSTEP * i);
        if (CSM == 1) add_cs_row(rx[S][i]);
        *reinterpret_cast<u32x4*>(st + sx_off + RSTEP * i * LDW) = rx[S][i];
      }
#pragma unroll
      for (int q = 0; q < YG; ++q)
#pragma unroll
        for (int i = 0; i < YL; ++i) {
          if (MASK) mask(ry[q * YL + i], row0 + lr + RSTEP * i);
          *reinterpret_cast<u32x4*>(st + sy_off + q * 128 + RSTEP * i * LDW) = ry[q * YL + i];
        }
    };

    f32x16 acc[WBM][WBN];
#pragma unroll
    for (int i = 0; i < WBM; ++i)
#pragma unroll
      for (int j = 0; j < WBN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // One step, written out in issue order: everything that is not an MFMA is issued in the shadow of the MFMAs, and
    // the scheduler is kept from regrouping by a fence after each MFMA.  Step kt multiplies out of stage S = kt & 1.
    // Between the MFMAs: fragment reads of the next slice; the next step's operands (X: register slot S^1, loaded
    // two steps ago; Y: loaded one step ago) are written to stage S^1, which every wave left before the last
    // barrier; then the registers are re-used for the loads of X three steps and Y two steps ahead.  The step's
    // barrier sits between slices 2 and 3: by then this stage has been read and the next one is written, so the
    // fragments of the next step's slice 0 are fetched under the MFMAs of slice 3 and no wavefront starts a step
    // with an empty MFMA pipe.
    const int xc = wm * (WBM * 32), yc = BX + wn * (WBN * 32);
    // One set of fragments: within a slice the MFMAs run over (i, j) with i outermost, so fx[0] is free after the
    // first WBN MFMAs, fy[j] after MFMA (1, j) and fx[1] after the last; each is re-read for the next slice right
    // behind its last use.
    bf16x8 fx[WBM], fy[WBN];
    auto first_frags = [&]() {   // slice 0 of stage 0
#pragma unroll
      for (int i = 0; i < WBM; ++i) fx[i] = frag_tr(ring0, xc + i * 32, 0, lane);
#pragma unroll
      for (int j = 0; j < WBN; ++j) fy[j] = frag_tr(ring0, yc + j * 32, 0, lane);
    };
    auto step = [&](auto slot, int kt, auto csm) {
      constexpr int S = decltype(slot)::value;
      constexpr int N = S ^ 1;
      constexpr int CSM = decltype(csm)::value;   // 1: column sums of X in this item
      const bf16* st = S ? ring1 : ring0;
      bf16* sn = N ? ring1 : ring0;
      const float cs_wt = kt + 1 < nk ? 1.0f : 0.0f;   // the last step writes rows that are not multiplied
#pragma unroll
      for (int n = 0; n < 4 * WBM * WBN; ++n) {
        constexpr int PER = WBM * WBN;
        const int ks = n / PER, t = n % PER, i = t / WBN, j = t % WBN;
        if (n == 3 * PER) __syncthreads();
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[i], fy[j], acc[i][j], 0, 0, 0);
        {   // fragments of slice ks + 1, or of the next stage's slice 0
          const bf16* src = ks < 3 ? st : sn;
          const int kk = ks < 3 ? (ks + 1) * 16 : 0;
          if (t == WBN - 1) fx[0] = frag_tr(src, xc, kk, lane);
          if (t >= WBN) fy[t - WBN] = frag_tr(src, yc + (t - WBN) * 32, kk, lane);
          if (t == PER - 1) fx[1] = frag_tr(src, xc + 32, kk, lane);
          static_assert(WBM == 2, "two X fragments");
        }
        // pieces, in this order: store the X rows (and their column sums), store the Y rows, load Y (needed again
        // in the next step), load X (needed two steps later); all before the step's barrier
        if (n < XL) {
          if (CSM == 1) add_cs_row(rx[N][n], cs_wt);
          *reinterpret_cast<u32x4*>(sn + sx_off + RSTEP * n * LDW) = rx[N][n];
        } else if (n < XL + YG * YL) {
          const int r = n - XL, q = r / YL, ri = r % YL;
          *reinterpret_cast<u32x4*>(sn + sy_off + q * 128 + RSTEP * ri * LDW) = ry[r];
        } else if (n < XL + 2 * YG * YL) {
          const int r = n - XL - YG * YL, q = r / YL, ri = r % YL;
          ry[r] = ld_y((kt + 2) * BK, q, ri);
        } else if (n < 2 * XL + 2 * YG * YL) {
          const int r = n - XL - 2 * YG * YL;
          rx[N][r] = ld_x((kt + 3) * BK, r);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };

    auto run = [&](auto csm) {   // one instance per column-sum mode: the step stays free of branches
      using S0 = std::integral_constant<int, 0>;
      using S1 = std::integral_constant<int, 1>;
      if (nk > 0) {
        issue_x(S0{}, 0);
        issue_y(0);
        issue_x(S1{}, 1);
        __syncthreads();   // the item before may still be fetching its last (unused) fragments from stage 0
        stash(S0{}, S0{}, csm, std::false_type{}, 0);
        issue_x(S0{}, 2);
        issue_y(1);
        __syncthreads();
        first_frags();
        for (int kt = 0; kt < nk; kt += 2) {
          step(S0{}, kt, csm);
          step(S1{}, kt + 1, csm);
        }
      }
      if (rem > 0) {
        // the slab's last rows (fewer than a double step): both stages are filled at once, rows that do not exist as
        // zeros, then multiplied; no overlap of loads and MFMAs (once per item of the last slab)
        __syncthreads();   // every wavefront has left both stages
        issue_x(S0{}, nk);
        issue_y(nk);
        stash(S0{}, S0{}, csm, std::true_type{}, nk * BK);
        issue_x(S0{}, nk + 1);
        issue_y(nk + 1);
        stash(S0{}, S1{}, csm, std::true_type{}, (nk + 1) * BK);
        __syncthreads();
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            const bf16* st = h ? ring1 : ring0;
#pragma unroll
            for (int i = 0; i < WBM; ++i) fx[i] = frag_tr(st, xc + i * 32, ks * 16, lane);
#pragma unroll
            for (int j = 0; j < WBN; ++j) fy[j] = frag_tr(st, yc + j * 32, ks * 16, lane);
#pragma unroll
            for (int i = 0; i < WBM; ++i)
#pragma unroll
              for (int j = 0; j < WBN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[i], fy[j], acc[i][j], 0, 0, 0);
          }
        __syncthreads();   // the column-sum reduction below and the next item write LDS
      }
    };
    if (cs_x) run(std::integral_constant<int, 1>{});
    else run(std::integral_constant<int, 0>{});
    // (after the last step's barrier nothing reads stage 1 any more; stage 0 is still being read)

    // column sums: the RSTEP threads that share a 16-byte chunk -> one value per column
    if (cs_x) {
      float* red = reinterpret_cast<float*>(ring1);   // [RSTEP][BX]
      static_assert((size_t)RSTEP * BX * 4 <= (size_t)STAGE * 2, "reduction buffer fits a stage");
#pragma unroll
      for (int c = 0; c < 8; ++c) red[lr * BX + lc * 8 + c] = cs[c];
      __syncthreads();
      if (tid < BX) {
        float a = 0.f;
#pragma unroll
        for (int m = 0; m < RSTEP; ++m) a += red[m * BX + tid];
        g.cs_part[(size_t)s * g.NX + x0 + tid] = a;
      }
      __syncthreads();
    }

    // accumulator element r of lane l: x = (r / 4) * 8 + (l / 32) * 4 + r % 4, y = l % 32 of its 32 x 32 block
    float* P = g.part + (size_t)s * g.NX * g.NY;
#pragma unroll
    for (int i = 0; i < WBM; ++i)
#pragma unroll
      for (int j = 0; j < WBN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int x = x0 + wm * (WBM * 32) + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
          int y = y0 + wn * (WBN * 32) + j * 32 + (lane & 31);
          P[(size_t)x * g.NY + y] = acc[i][j][r];
        }
  }
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

// Shapes this kernel takes: identity row maps, enough rows, an output that the tiles cover exactly with A on the
// side tiled by 128 (no column is masked in the kernel), slabs short enough for 32-bit offsets.  Returns the
// number of slabs it will use (0: not taken).
int gemm_tn_big_slabs(const GemmTN& g, int max_slabs) {
  if (g.amap.g2 != 0 || g.bmap.g2 != 0 || g.M < 65536 || max_slabs < 8) return 0;
  if (g.lda % 8 || g.ldb % 8 || !aligned16(g.A) || !aligned16(g.B)) return 0;
  if ((long long)g.N1 * g.N2 >= (1LL << 31)) return 0;
  if (g.N1 % BX || g.N2 % BY) return 0;
  int tiles = (g.N1 / BX) * (g.N2 / BY);
  // per XCD: spx slabs x tiles items over 32 workgroups; more slabs while that fills the last round of workgroups
  // noticeably better (every slab costs one partial result to write and to add)
  int spx = 1;
  double best = 0.0;
  for (int c = 1; c <= 32 && 8 * c <= max_slabs; ++c) {
    int items = c * tiles, rounds = (items + 31) / 32;
    double fill = (double)items / (rounds * 32.0);
    if (fill > best + 0.04 || (c <= 3 && fill >= best)) { best = fill; spx = c; }
  }
  long long per = (g.M + 8 * spx - 1) / (8 * spx) + 8 * BK;   // loads run up to four steps past a slab's end
  long long ldmax = g.lda > g.ldb ? g.lda : g.ldb;
  if (per * ldmax * 2 >= (1LL << 32)) return 0;
  return 8 * spx;
}

hipError_t launch_gemm_tn_big(const GemmTN& g, hipStream_t s) {
  static int cus = 0;
  if (!cus) {
    hipError_t e;
    int dev = 0;
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
    cus = prop.multiProcessorCount / NXCD * NXCD;
    if (cus < NXCD) cus = NXCD;
  }
  if (g.N1 % BX || g.N2 % BY || g.slabs % NXCD) return hipErrorInvalidValue;
  TnBig t{};
  t.M = g.M; t.part = g.part; t.cs_part = g.cs_part; t.slabs = g.slabs; t.spx = g.slabs / NXCD;
  t.X = (const bf16*)g.A; t.ldx = g.lda; t.NX = g.N1; t.Y = (const bf16*)g.B; t.ldy = g.ldb; t.NY = g.N2;
  t.TX = t.NX / BX; t.TY = t.NY / BY;
  int items_per_xcd = t.spx * t.TX * t.TY;
  int per_xcd = cus / NXCD < items_per_xcd ? cus / NXCD : items_per_xcd;
  hipLaunchKernelGGL(gemm_tn_big_k, dim3((unsigned)(per_xcd * NXCD)), dim3(NTH), 0, s, t);
  return hipGetLastError();
}

}  // namespace sl
