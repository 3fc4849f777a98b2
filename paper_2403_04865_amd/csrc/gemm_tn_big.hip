// bf16 MFMA weight-gradient GEMM for gfx950, large-M variant: C[N1,N2] = sum_m A[m,N1]^T B[m,N2] (fp32 partials).
//
// Same machine balance as the activation GEMMs (what a compute unit can pull out of its L2 bounds the tile from
// below), so the same tile area: one persistent workgroup of 4 wavefronts per compute unit, a 128 x 384 output tile
// (wavefront: 64 x 192), 64 rows of m per step, operands global -> registers -> LDS with the loads of X two steps
// and of Y one step ahead, MFMA / LDS / global instructions dealt out by hand.  What differs:
//   * The contraction runs over the ROW index of both operands.  The 64-row slices go to LDS as they are
//     (row-major, 16-byte stores) and the MFMA fragments, which need 8 consecutive contraction indices per
//     lane, are read with LDS transpose reads (ds_read_b64_tr_b16: a group of 16 lanes addresses a 4-row x
//     16-column patch and every lane receives one column of it).  No transposition in registers.
//   * M (all tokens of the slide) is split into slabs; a work item is (slab, output tile) and writes its partial
//     tile once, a second kernel adds the slabs in a fixed order (no atomics: results are run-to-run identical).
//     All tiles of a slab run on ONE XCD at about the same time, so the slab's rows come from HBM once and the
//     other tiles find them in that XCD's L2 (with tiles spread over XCDs the rows were fetched several times).
//   * The tile is as wide as the narrow operand of the encoder's weight gradients (384 columns, "Y"), so the wide
//     operand ("X": 1152 or 1536 columns, four fifths of the bytes) is read by exactly one workgroup and streams
//     from HBM once whatever the workgroups' relative progress; only the narrow operand is shared through L2, and
//     its window (a few steps x 48 kB per slab) is a small part of the 4 MB.  With 256 x 192 tiles every row was
//     shared by up to twelve workgroups that each run three steps of loads ahead: the windows of the slabs in
//     flight on an XCD filled its L2, any drift between the sharers missed, and the kernel moved 1.7 x its operand
//     bytes and ran at HBM speed.
//   * Either operand can play the 128-tiled side, whichever leaves fewer empty tile columns; the output
//     strides follow.  Column sums of A (the bias gradient) are taken from the registers of the loads.
#include "slide_internal.h"

#include <type_traits>

namespace sl {

namespace {

constexpr int NXCD = 8;
constexpr int BX = 128, BY = 384, BK = 64, NTH = 256;
constexpr int XL = BX / 8 * BK / NTH, YG = BY / 128, YL = 4;   // 16-byte loads per thread and step: X 4, Y 3 x 4
// LDS row: 128 X columns, 384 Y columns, pad.  The pad makes the row stride 64 bytes modulo 256 (16 banks): a
// transpose read's group of 16 lanes touches 4 rows x 32 bytes, and the two groups that are served together sit 32
// bytes apart, so with this stride their eight 32-byte pieces fall on eight different bank ranges (with a 16-byte
// stride modulo 256 they overlapped: 58 % of the LDS cycles were bank-conflict cycles).
constexpr int LDW = BX + BY + 32;
constexpr int STAGE = BK * LDW;                     // bf16 elements per LDS stage
constexpr int WBM = 2, WBN = 6;
static_assert(XL == 4 && YG * 128 == BY && WBM == 2, "loader split, fragment schedule");

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

// a row of zeros that loads of rows past a slab's end (and of columns past the matrix) are pointed at, so that
// the loads need no branches (a branch would cut the step into several scheduling regions)
__device__ __attribute__((aligned(16))) unsigned int g_zero_row[64];

struct TnBig {
  const bf16* X; long long ldx; int NX;   // side tiled by 128
  const bf16* Y; long long ldy; int NY;   // side tiled by 384
  long long M;
  float* part; long long sx, sy;          // partial of slab s: part[s * NX * NY + x * sx + y * sy]
  float* cs_part; int cs_on_x;            // column sums of X (1) or Y (0) per slab, [slabs][N of that side]; may be null
  int slabs, spx;                         // slabs = 8 * spx: slabs xcd * spx .. xcd * spx + spx - 1 run on XCD xcd
  int TX, TY;
};

template <bool LANE_IS_X>
__global__ void __launch_bounds__(NTH) gemm_tn_big_k(TnBig g) {
  __shared__ __attribute__((aligned(16))) bf16 ring0[STAGE];
  __shared__ __attribute__((aligned(16))) bf16 ring1[STAGE];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  // loader: 16 lanes cover 256 contiguous bytes of one row; thread t takes 16-byte chunk t % 16 of rows t / 16 + 16 i
  // of X, and the chunks t % 16 + 16 g (g < 3) of the same rows of Y
  const int lr = tid >> 4, lc = tid & 15;
  const int xcd = blockIdx.x % NXCD, wg = blockIdx.x / NXCD, wgs = gridDim.x / NXCD;
  const int tiles = g.TX * g.TY;
  const int items = g.spx * tiles;
  long long per = (g.M + g.slabs - 1) / g.slabs;
  per = (per + 2 * BK - 1) / (2 * BK) * (2 * BK);          // whole double steps

  u32x4 rx[2][XL], ry[YG * YL];
  for (int idx = wg; idx < items; idx += wgs) {            // uniform for the workgroup
    const int s = xcd * g.spx + idx / tiles;
    const int tile = idx % tiles;
    const int x0 = (tile / g.TY) * BX, y0 = (tile % g.TY) * BY;
    const long long lo = (long long)s * per;
    const long long hi = lo + per < g.M ? lo + per : g.M;
    const int nk = lo < hi ? (int)((hi - lo + 2 * BK - 1) / (2 * BK)) * 2 : 0;
    // (NX % 128 == 0 and NY % 384 == 0: every column of a tile exists)
    const bf16* zero = reinterpret_cast<const bf16*>(g_zero_row);
    const bf16* xp = g.X + (x0 + lc * 8);
    const bf16* yp = g.Y + (y0 + lc * 8);
    const long long ldx = g.ldx, ldy = g.ldy;
    // rows of step kt this thread loads: lo + kt * 64 + lr + 16 i; rows past the slab's end read the zero row
    auto issue_x = [&](auto slot, int kt) {
      constexpr int S = decltype(slot)::value;
      long long m = lo + (long long)kt * BK + lr;
      const bf16* p = xp + m * ldx;
#pragma unroll
      for (int i = 0; i < XL; ++i) rx[S][i] = ldg16(m + 16 * i < hi ? p + 16 * i * ldx : zero);
    };
    auto issue_y = [&](int kt) {
      long long m = lo + (long long)kt * BK + lr;
      const bf16* p = yp + m * ldy;
#pragma unroll
      for (int q = 0; q < YG; ++q)
#pragma unroll
        for (int i = 0; i < YL; ++i) ry[q * YL + i] = ldg16(m + 16 * i < hi ? p + 16 * i * ldy + q * 128 : zero);
    };
    const bool cs_x = g.cs_part != nullptr && g.cs_on_x && y0 == 0;
    const bool cs_y = g.cs_part != nullptr && !g.cs_on_x && x0 == 0;
    float cs[YG][8];   // column sums of this thread's chunk(s): X uses cs[0]
#pragma unroll
    for (int q = 0; q < YG; ++q)
#pragma unroll
      for (int c = 0; c < 8; ++c) cs[q][c] = 0.f;
    auto add_cs_row = [&](const u32x4& v, float (&a)[8]) {
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        a[2 * w] += __uint_as_float(v[w] << 16);
        a[2 * w + 1] += __uint_as_float(v[w] & 0xffff0000u);
      }
    };
    const int sx_off = lr * LDW + lc * 8, sy_off = lr * LDW + BX + lc * 8;
    auto stash = [&](auto slot, auto csm) {   // prologue only; the steps below do the same piecewise
      constexpr int S = decltype(slot)::value;
      constexpr int CSM = decltype(csm)::value;
      bf16* st = S ? ring1 : ring0;
#pragma unroll
      for (int i = 0; i < XL; ++i) {
        if (CSM == 1) add_cs_row(rx[S][i], cs[0]);
        *reinterpret_cast<u32x4*>(st + sx_off + 16 * i * LDW) = rx[S][i];
      }
#pragma unroll
      for (int q = 0; q < YG; ++q)
#pragma unroll
        for (int i = 0; i < YL; ++i) {
          if (CSM == 2) add_cs_row(ry[q * YL + i], cs[q]);
          *reinterpret_cast<u32x4*>(st + sy_off + q * 128 + 16 * i * LDW) = ry[q * YL + i];
        }
    };

    f32x16 acc[WBM][WBN];
#pragma unroll
    for (int i = 0; i < WBM; ++i)
#pragma unroll
      for (int j = 0; j < WBN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // One step, written out in issue order (one wavefront per SIMD: everything that is not an MFMA has to be
    // issued in the shadow of the 48 MFMAs, and the scheduler is kept from regrouping by a fence after each
    // MFMA).  Step kt multiplies out of stage S = kt & 1.  Between the MFMAs: fragment reads of the next slice;
    // the next step's operands (X: register slot S^1, loaded two steps ago; Y: loaded one step ago) are
    // written to stage S^1, which every wave left before the last barrier; then the registers are re-used
    // for the loads of X three steps and Y two steps ahead.  The step's barrier sits between slices 2 and
    // 3: by then this stage has been read and the next one is written, so the fragments of the next step's
    // slice 0 are fetched under the MFMAs of slice 3 and no wavefront starts a step with an empty MFMA pipe.
    const int xc = wm * (WBM * 32), yc = BX + wn * (WBN * 32);
    // One set of fragments: within a slice the MFMAs run over (i, j) with i outermost, so fx[0] is free after the first
    // six MFMAs, fy[j] after MFMA (1, j) and fx[1] after the last; each is re-read for the next slice right behind its
    // last use, six or more MFMAs before its next one.
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
      constexpr int CSM = decltype(csm)::value;   // 0: no column sums in this item, 1: of X, 2: of Y
      const bf16* st = S ? ring1 : ring0;
      bf16* sn = N ? ring1 : ring0;
      const bf16* px = nullptr;
      const bf16* py = nullptr;
      long long mx = 0, my = 0;
#pragma unroll
      for (int n = 0; n < 4 * WBM * WBN; ++n) {
        constexpr int PER = WBM * WBN;
        const int ks = n / PER, t = n % PER, i = t / WBN, j = t % WBN;
        if (n == 3 * PER) __syncthreads();
        acc[i][j] = LANE_IS_X ? __builtin_amdgcn_mfma_f32_32x32x16_bf16(fy[j], fx[i], acc[i][j], 0, 0, 0)
                              : __builtin_amdgcn_mfma_f32_32x32x16_bf16(fx[i], fy[j], acc[i][j], 0, 0, 0);
        {   // fragments of slice ks + 1, or of the next stage's slice 0
          const bf16* src = ks < 3 ? st : sn;
          const int kk = ks < 3 ? (ks + 1) * 16 : 0;
          if (t == WBN - 1) fx[0] = frag_tr(src, xc, kk, lane);
          if (t >= WBN) fy[t - WBN] = frag_tr(src, yc + (t - WBN) * 32, kk, lane);
          if (t == PER - 1) fx[1] = frag_tr(src, xc + 32, kk, lane);
        }
        // pieces: 0..3 store X rows (and their column sums); 4..15 store Y rows (and theirs); 16..27 load Y
        // (needed again 36 pieces later); 28..31 load X (needed two steps later)
        if (n < XL) {
          if (CSM == 1) add_cs_row(rx[N][n], cs[0]);
          *reinterpret_cast<u32x4*>(sn + sx_off + 16 * n * LDW) = rx[N][n];
        } else if (n < XL + YG * YL) {
          const int r = n - XL, q = r / YL, ri = r % YL;
          if (CSM == 2) add_cs_row(ry[r], cs[q]);
          *reinterpret_cast<u32x4*>(sn + sy_off + q * 128 + 16 * ri * LDW) = ry[r];
          if (n == XL + YG * YL - 2) { my = lo + (long long)(kt + 2) * BK + lr; py = yp + my * ldy; }
          if (n == XL + YG * YL - 1) { mx = lo + (long long)(kt + 3) * BK + lr; px = xp + mx * ldx; }
        } else if (n < XL + 2 * YG * YL) {
          const int r = n - XL - YG * YL, q = r / YL, ri = r % YL;
          ry[r] = ldg16(my + 16 * ri < hi ? py + 16 * ri * ldy + q * 128 : zero);
        } else if (n < 2 * XL + 2 * YG * YL) {
          const int r = n - XL - 2 * YG * YL;
          rx[N][r] = ldg16(mx + 16 * r < hi ? px + 16 * r * ldx : zero);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };

    auto run = [&](auto csm) {   // one instance per column-sum mode: the step stays free of branches
      issue_x(std::integral_constant<int, 0>{}, 0);
      issue_y(0);
      issue_x(std::integral_constant<int, 1>{}, 1);
      __syncthreads();   // the item before may still be fetching its last (unused) fragments from stage 0
      stash(std::integral_constant<int, 0>{}, csm);
      issue_x(std::integral_constant<int, 0>{}, 2);
      issue_y(1);
      __syncthreads();
      first_frags();
      for (int kt = 0; kt < nk; kt += 2) {       // loads past the slab's end read the zero row
        step(std::integral_constant<int, 0>{}, kt, csm);
        step(std::integral_constant<int, 1>{}, kt + 1, csm);
      }
    };
    if (nk > 0) {
      if (cs_x) run(std::integral_constant<int, 1>{});
      else if (cs_y) run(std::integral_constant<int, 2>{});
      else run(std::integral_constant<int, 0>{});
    }
    // (after the last step's barrier nothing reads stage 1 any more; stage 0 is still being read)

    // column sums: the 16 threads lr = 0..15 that share a 16-byte chunk -> one value per column
    if (cs_x || cs_y) {
      float* red = reinterpret_cast<float*>(ring1);   // [16][BX] or [16][BY]
      const int ncol = cs_x ? BX : BY;
      if (cs_x) {
#pragma unroll
        for (int c = 0; c < 8; ++c) red[lr * BX + lc * 8 + c] = cs[0][c];
      } else {
#pragma unroll
        for (int q = 0; q < YG; ++q)
#pragma unroll
          for (int c = 0; c < 8; ++c) red[lr * BY + (lc + 16 * q) * 8 + c] = cs[q][c];
      }
      __syncthreads();
      const int c0 = cs_x ? x0 : y0, nn = cs_x ? g.NX : g.NY;
      for (int col = tid; col < ncol; col += NTH)
        if (c0 + col < nn) {
          float a = 0.f;
#pragma unroll
          for (int m = 0; m < 16; ++m) a += red[m * ncol + col];
          g.cs_part[(size_t)s * nn + c0 + col] = a;
        }
      __syncthreads();
    }

    float* P = g.part + (size_t)s * g.NX * g.NY;
#pragma unroll
    for (int i = 0; i < WBM; ++i)
#pragma unroll
      for (int j = 0; j < WBN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int inner = (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), outer = lane & 31;
          int x = x0 + wm * (WBM * 32) + i * 32 + (LANE_IS_X ? outer : inner);
          int y = y0 + wn * (WBN * 32) + j * 32 + (LANE_IS_X ? inner : outer);
          if (x < g.NX && y < g.NY) P[x * g.sx + y * g.sy] = acc[i][j][r];
        }
  }
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// A on the side tiled by 128 and B on the side tiled by 384, or the other way round: whichever way the tiles cover
// the output exactly, and of two such ways the one with fewer tiles along the 384 side (the operand on the 128 side
// is then shared by fewer workgroups; with one tile along the 384 side it is read by exactly one)
bool tn_fits(int nx, int ny) { return nx % BX == 0 && ny % BY == 0; }
bool tn_a_is_x(const GemmTN& g) {
  bool ax = tn_fits(g.N1, g.N2), bx = tn_fits(g.N2, g.N1);
  if (ax && bx) return g.N2 <= g.N1;
  return ax;
}

}  // namespace

// Shapes this kernel takes: identity row maps, enough rows.  Returns the number of slabs it will use (0: not taken).
int gemm_tn_big_slabs(const GemmTN& g, int max_slabs) {
  if (g.amap.g2 != 0 || g.bmap.g2 != 0 || g.M < 65536) return 0;
  if (g.lda % 8 || g.ldb % 8 || !aligned16(g.A) || !aligned16(g.B)) return 0;
  if ((long long)g.N1 * g.N2 >= (1LL << 31)) return 0;
  // the tiles must cover the output exactly, one way round or the other (no column is masked in the kernel)
  if (!tn_fits(g.N1, g.N2) && !tn_fits(g.N2, g.N1)) return 0;
  bool a_is_x = tn_a_is_x(g);
  int nx = a_is_x ? g.N1 : g.N2, ny = a_is_x ? g.N2 : g.N1;
  int tiles = ((nx + BX - 1) / BX) * ((ny + BY - 1) / BY);
  // per XCD: spx slabs x tiles items over 32 workgroups; more slabs while that fills the last round of workgroups
  // noticeably better (every slab costs one partial result to write and to add)
  int spx = 1;
  double best = 0.0;
  for (int c = 1; c <= 32 && 8 * c <= max_slabs; ++c) {
    int items = c * tiles, rounds = (items + 31) / 32;
    double fill = (double)items / (rounds * 32.0);
    if (fill > best + 0.04 || (c <= 3 && fill >= best)) { best = fill; spx = c; }
  }
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
  bool a_is_x = tn_a_is_x(g);
  TnBig t{};
  t.M = g.M; t.part = g.part; t.cs_part = g.cs_part; t.slabs = g.slabs; t.spx = g.slabs / NXCD;
  if (a_is_x) {
    t.X = (const bf16*)g.A; t.ldx = g.lda; t.NX = g.N1; t.Y = (const bf16*)g.B; t.ldy = g.ldb; t.NY = g.N2;
    t.sx = g.N2; t.sy = 1; t.cs_on_x = 1;
  } else {
    t.X = (const bf16*)g.B; t.ldx = g.ldb; t.NX = g.N2; t.Y = (const bf16*)g.A; t.ldy = g.lda; t.NY = g.N1;
    t.sx = 1; t.sy = g.N2; t.cs_on_x = 0;
  }
  t.TX = (t.NX + BX - 1) / BX; t.TY = (t.NY + BY - 1) / BY;
  int items_per_xcd = t.spx * t.TX * t.TY;
  int per_xcd = cus / NXCD < items_per_xcd ? cus / NXCD : items_per_xcd;
  dim3 grid((unsigned)(per_xcd * NXCD));
  // the lanes of a store run along the output's contiguous index: y when X = A (row-major [N1][N2]), x otherwise
  if (a_is_x) hipLaunchKernelGGL(gemm_tn_big_k<false>, grid, dim3(NTH), 0, s, t);
  else hipLaunchKernelGGL(gemm_tn_big_k<true>, grid, dim3(NTH), 0, s, t);
  return hipGetLastError();
}

}  // namespace sl
