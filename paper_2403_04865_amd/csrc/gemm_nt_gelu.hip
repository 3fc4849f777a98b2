// bf16 MFMA "NT" GEMM with fused bias + GELU for gfx950, large-M variant (the first MLP GEMM of a block):
// m = A[M,K] * B[N,K]^T + bias;  out = gelu(m) as bf16, out2 = gelu'(m) as the one-byte code of slide_internal.h.
//
// Same tile and operand pipeline as the large-M kernel of the other epilogues (gemm_nt_big.hip: 256 x 192 tiles,
// one persistent workgroup per compute unit, operands global -> registers -> LDS three K steps ahead, explicit
// instruction order), but this epilogue is the heaviest of all (two outputs and a table look-up per element for
// 6 K steps of MFMAs at K = 384), and it is organised differently:
//   * 8 wavefronts per workgroup, two per SIMD with 256 registers each: while one wavefront waits for LDS, for
//     memory or at the barrier, the other one issues.  A wavefront owns 64 x 96 of the tile (2 x 3 accumulators of
//     32 x 32); the loads of K step k + 3 are issued during step k into two register slots, across tile boundaries.
//   * The epilogue runs when the tile's last step is done, by all eight wavefronts at once: the accumulators
//     (which started from the bias) go through wavefront-private fp32 patches in the (then idle) operand stages and
//     come back as 8-column row segments, GELU and its derivative are evaluated on the UNROUNDED pre-activation and
//     rounded once, and every global store is a 16-byte (derivative codes: 8-byte) access along a row.  The first two K steps of the next tile
//     are already in flight in the registers meanwhile.  (In the 4-wavefront kernel the same work rides between
//     the MFMAs of the next tile on a bf16-rounded copy of the accumulators; measured 3.74 ms per launch on the
//     8192-tile ViT-S workload against 3.2 ms here.  For the lighter epilogues the two organisations measure the
//     same, and those with an auxiliary operand are faster there.)
//   * GELU and its derivative come from a table of the normal CDF and of d/dx (x cdf(x)) in LDS, linearly
//     interpolated at 1/32 steps (error < 1e-4, far below bf16 rounding).
#include "slide_internal.h"

#include <type_traits>

namespace sl {

namespace {

constexpr int NXCD = 8;
constexpr int BM = 256, BN = 192, BK = 64, LDT = BK + 8, NW = 8, NTH = 64 * NW;
constexpr int WVM = 4, WVN = 2;                    // wavefronts along M and N
constexpr int WBM = BM / (32 * WVM), WBN = BN / (32 * WVN);   // 32 x 32 accumulators per wavefront: 2 x 3
constexpr int RSTEP = NTH / 8;                     // rows per loader pass (8 chunks of 16 bytes per row)
constexpr int CA = BM / RSTEP, CB = BN / RSTEP;    // 16-byte chunks per thread and K step: 4 + 3
constexpr int STAGE = (BM + BN) * LDT;             // bf16 elements per LDS stage
constexpr int TAB_N = 448;                         // table over [-7, 7) in steps of 1/32
constexpr int PS = WBN * 32 + 4;                   // patch row stride (floats)
constexpr int NPASS = 7;                           // 12 lanes per row, 5 rows per pass, lanes 60..63 idle
constexpr int MIN_STEPS = 6;
static_assert(WBM == 2 && WBN == 3, "fragment schedule and epilogue lane map");
static_assert((size_t)NW * 32 * PS * 4 <= (size_t)2 * STAGE * 2, "epilogue patches fit the operand stages");
static_assert(2 * (CA + CB) <= 3 * WBM * WBN, "piece schedule");

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// uniform base (scalar registers) + 32-bit per-lane byte offset
__device__ __forceinline__ u32x4 ldg16(const char* base, unsigned off) { return *reinterpret_cast<const u32x4*>(base + off); }

__device__ __forceinline__ u32x4 pack8(const float (&v)[8]) {
  bf16x8 t;
#pragma unroll
  for (int w = 0; w < 8; ++w) t[w] = (bf16)v[w];   // round to nearest even
  return __builtin_bit_cast(u32x4, t);
}

// table entry k: {cdf(x_k), cdf(x_k+1) - cdf(x_k), c(x_k), c(x_k+1) - c(x_k)}, x_k = -7 + k/32,
// cdf = standard normal distribution function, dg(x) = cdf(x) + x * pdf(x) = d/dx (x cdf(x)) and c = dg8_code(dg),
// the derivative in the code space of its one-byte storage: *dgc comes out ready for the conversion
// (entries are four halves: 8 bytes per look-up instead of 16 keep the table's LDS traffic, which every wavefront's
// epilogue shares, and its bank conflicts at half; a half has 11 significant bits against the 8 of the results)
typedef _Float16 h16x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void gelu_both_tab(const h16x4* tab, float x, float* gl, float* dgc) {
  float t = __builtin_amdgcn_fmed3f(x * 32.0f + 224.0f, 0.0f, (float)TAB_N - 0.001f);
  int k = (int)t;                       // t >= 0: truncation is the floor
  float f = __builtin_amdgcn_fractf(t);
  h16x4 e = tab[k];
  *gl = x * ((float)e[0] + f * (float)e[1]);
  *dgc = (float)e[2] + f * (float)e[3];
}

template <int V> using IC = std::integral_constant<int, V>;

__global__ void __launch_bounds__(NTH) gemm_nt_gelu_k(GemmNT g, int MT, int NTL) {
  __shared__ __attribute__((aligned(16))) bf16 ring[2 * STAGE];
  __shared__ h16x4 tab[TAB_N];
  __shared__ __attribute__((aligned(16))) float lbias[BN];   // the tile's bias columns (zeros without a bias)
  bf16* const ring0 = ring;
  bf16* const ring1 = ring + STAGE;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WVN, wn = wave % WVN;
  const int row0 = tid >> 3, kc = tid & 7;       // loader: 64 rows x 8 chunks of 16 bytes per pass
  const int soff = row0 * LDT + kc * 8;
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  const int nk = g.K / BK;
  const int total = (MT + NXCD - 1) / NXCD * NXCD * NTL;

  {
    // filled once per workgroup; the K-loop barriers order it before its first use
    for (int k = tid; k < TAB_N; k += NTH) {
      float x0 = -7.0f + (float)k * (1.0f / 32.0f), x1 = x0 + (1.0f / 32.0f);
      float c0 = 0.5f * (1.0f + erff(x0 * 0.70710678118654752f)), c1 = 0.5f * (1.0f + erff(x1 * 0.70710678118654752f));
      float d0 = c0 + x0 * 0.39894228040143268f * expf(-0.5f * x0 * x0);
      float d1 = c1 + x1 * 0.39894228040143268f * expf(-0.5f * x1 * x1);
      tab[k] = h16x4{(_Float16)c0, (_Float16)(c1 - c0), (_Float16)dg8_code(d0), (_Float16)(dg8_code(d1) - dg8_code(d0))};
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

  // ---- operand loads: uniform base + 32-bit per-thread byte offsets --------------------------------------
  // chunk i of a thread is row0 + 64 i.  Rows past the end of A (last row tile only) are redirected to row M - 1 by
  // clamping the offset: they are loaded (valid memory) but never stored.
  const unsigned aoff0 = 2u * (unsigned)(row0 * (int)g.lda + kc * 8), boff0 = 2u * (unsigned)(row0 * (int)g.ldb + kc * 8);
  const unsigned astride = 2u * RSTEP * (unsigned)g.lda, bstride = 2u * RSTEP * (unsigned)g.ldb;  // bytes
  struct Src { const char* A; const char* B; unsigned amax; };
  auto src_of = [&](long long m0, int n0) {
    Src s;
    s.A = (const char*)((const bf16*)g.A + m0 * g.lda);
    s.B = (const char*)((const bf16*)g.B + (long long)n0 * g.ldb);
    s.amax = m0 + BM > g.M ? 2u * (unsigned)((g.M - 1 - m0) * g.lda + kc * 8) : 0xffffffffu;
    return s;
  };
  u32x4 ra[2][CA], rb[2][CB];
  auto load_a = [&](const Src& s, int i, int k0) {
    unsigned off = aoff0 + (unsigned)i * astride;
    return ldg16(s.A + 2 * k0, off < s.amax ? off : s.amax);
  };
  auto load_b = [&](const Src& s, int i, int k0) {
    return ldg16(s.B + 2 * k0 + (unsigned)i * bstride, boff0);   // N % 192 == 0: no clamp
  };
  auto issue = [&](auto slot, const Src& s, int k0) {
    constexpr int S = decltype(slot)::value;
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[S][i] = load_b(s, i, k0);
#pragma unroll
    for (int i = 0; i < CA; ++i) ra[S][i] = load_a(s, i, k0);
  };
  auto stash = [&](auto slot, auto stage) {
    constexpr int S = decltype(slot)::value, ST = decltype(stage)::value;
    bf16* st = ST ? ring1 : ring0;
#pragma unroll
    for (int i = 0; i < CA; ++i) *reinterpret_cast<u32x4*>(st + soff + i * RSTEP * LDT) = ra[S][i];
#pragma unroll
    for (int i = 0; i < CB; ++i) *reinterpret_cast<u32x4*>(st + BM * LDT + soff + i * RSTEP * LDT) = rb[S][i];
  };

  // ---- MFMA side ----------------------------------------------------------------------------------------------
  // The MFMA operands are passed swapped (B first): accumulator element r of lane l is then row l % 32, column
  // (r / 4) * 8 + (l / 32) * 4 + r % 4 of its 32 x 32 block, i.e. a lane holds runs of four neighbouring columns.
  // One set of fragments: within a slice the MFMAs run over (i, j) with i outermost, so fa[0] is free after the
  // first three MFMAs, fb[j] after MFMA (1, j) and fa[1] after the last; each is re-read for the next slice right
  // behind its last use.
  f32x16 acc[WBM][WBN];
  bf16x8 fa[WBM], fb[WBN];
  const int a_lds = (wm * (WBM * 32) + frow) * LDT + fk, b_lds = BM * LDT + (wn * (WBN * 32) + frow) * LDT + fk;
  auto rd_a = [&](const bf16* st, int i, int kk) { fa[i] = *reinterpret_cast<const bf16x8*>(st + a_lds + i * 32 * LDT + kk); };
  auto rd_b = [&](const bf16* st, int j, int kk) { fb[j] = *reinterpret_cast<const bf16x8*>(st + b_lds + j * 32 * LDT + kk); };

  // One K step out of LDS stage S, in explicit issue order: one MFMA and at most one other group of instructions
  // per piece, a scheduling fence after each piece.  The step's barrier sits between slices 2 and 3: by then every
  // fragment of this stage has been read and the next stage (register slot S^1, loaded two steps ago) is
  // completely written, so the fragments of the next step's slice 0 are fetched under the MFMAs of slice 3.  The
  // registers are re-used for the loads three steps ahead (source `nx`, element offset k3).  LAST: the tile's
  // last step; nothing is written to LDS (the epilogue takes the stages) and nothing is loaded (both slots hold
  // the first two steps of the next tile).
  auto step = [&](auto slot, auto last, const Src& nx, int k3) {
    constexpr int S = decltype(slot)::value, N = S ^ 1;
    constexpr bool LAST = decltype(last)::value;
    const bf16* st = S ? ring1 : ring0;
    bf16* sn = N ? ring1 : ring0;
#pragma unroll
    for (int n = 0; n < 4 * WBM * WBN; ++n) {
      constexpr int PER = WBM * WBN;
      const int ks = n / PER, t = n % PER, i = t / WBN, j = t % WBN;
      if (n == 3 * PER && !LAST) __syncthreads();
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
      if (!(LAST && ks == 3)) {   // fragments of slice ks + 1, or of the next stage's slice 0
        const bf16* src = ks < 3 ? st : sn;
        const int kk = ks < 3 ? (ks + 1) * 16 : 0;
        if (t == WBN - 1) rd_a(src, 0, kk);
        if (t >= WBN) rd_b(src, t - WBN, kk);
        if (t == PER - 1) rd_a(src, 1, kk);
      }
      if (!LAST) {
        // pieces, in this order: store A, store B (slot N), then load B, load A three steps ahead into the slot
        if (n < CA) {
          *reinterpret_cast<u32x4*>(sn + soff + n * RSTEP * LDT) = ra[N][n];
        } else if (n < CA + CB) {
          *reinterpret_cast<u32x4*>(sn + BM * LDT + soff + (n - CA) * RSTEP * LDT) = rb[N][n - CA];
        } else if (n < CA + 2 * CB) {
          rb[N][n - CA - CB] = load_b(nx, n - CA - CB, k3);
        } else if (n < 2 * CA + 2 * CB) {
          ra[N][n - CA - 2 * CB] = load_a(nx, n - CA - 2 * CB, k3);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- epilogue ------------------------------------------------------------------------------------------------
  // Per 32-row strip the wavefront writes its 32 x 96 accumulators to its patch (a lane holds runs of four
  // neighbouring columns: 12 x 16 bytes) and reads 8-column row segments back: 12 lanes per row, 5 rows per pass,
  // 7 passes (the last holds rows 30, 31; lanes 60..63 idle).
  const int er = lane < 60 ? lane / 12 : 0;    // row inside a pass (idle lanes: a valid address)
  const int erc = lane < 60 ? lane / 12 : 64;  // the same for comparisons: idle lanes never pass
  const int esg = lane % 12;
  float* const patch = reinterpret_cast<float*>(ring) + wave * 32 * PS;
  float* const pw = patch + (lane & 31) * PS + (lane >> 5) * 4;
  const float* const pr = patch + er * PS + esg * 8;
  const unsigned ldc_b = 2u * (unsigned)g.ldc, ldc2_b = (unsigned)g.ldc2;   // bytes: bf16 and one-byte codes
  auto epilogue = [&](long long m0, int n0) {
    const long long mw = m0 + wm * (WBM * 32);
    const int nw = n0 + wn * (WBN * 32);
#pragma unroll
    for (int i = 0; i < WBM; ++i) {
      const long long ms = mw + i * 32;                 // first row of the strip
      const long long left = g.M - ms;
      const int lim = left > 32 ? 32 : (int)left;       // rows of the strip that exist (uniform, may be <= 0)
#pragma unroll
      for (int j = 0; j < WBN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *reinterpret_cast<float4*>(pw + j * 32 + q * 8) =
              make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
#pragma unroll
      for (int p = 0; p < NPASS; ++p) {
        if (p * 5 < lim) {   // uniform
          const int prow = p * 5 + er < 32 ? p * 5 + er : 31;
          float4 x0 = *reinterpret_cast<const float4*>(pr + (prow - er) * PS), x1 = *reinterpret_cast<const float4*>(pr + (prow - er) * PS + 4);
          float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
          float t[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            float gl, dg;
            gelu_both_tab(tab, v[e], &gl, &dg);
            v[e] = gl;
            t[e] = dg;
          }
          const bool ok = p * 5 + erc < lim && p * 5 + er < 32;
          char* o = (char*)g.out + ((ms + p * 5) * (long long)ldc_b + 2 * nw);
          char* o2 = (char*)g.out2 + ((ms + p * 5) * (long long)ldc2_b + nw);
          if (ok) __builtin_nontemporal_store(pack8(v), reinterpret_cast<u32x4*>(o + (unsigned)er * ldc_b + esg * 16));
          if (ok) __builtin_nontemporal_store(u32x2{dg8_pack4_code(t[0], t[1], t[2], t[3]), dg8_pack4_code(t[4], t[5], t[6], t[7])},
                                              reinterpret_cast<u32x2*>(o2 + (unsigned)er * ldc2_b + esg * 8));
        }
      }
    }
  };

  long long m0, m1;
  int n0, n1;
  int id = next_valid(blockIdx.x, m0, n0);
  if (id >= total) return;
  using S0 = IC<0>;
  using S1 = IC<1>;
  Src cur = src_of(m0, n0);
  issue(S0{}, cur, 0);
  issue(S1{}, cur, BK);
  while (id < total) {
    int nid = next_valid(id + gridDim.x, m1, n1);
    if (nid >= total) { m1 = m0; n1 = n0; }  // no further tile: the prefetches re-read this one and are dropped
    const Src nxt = src_of(m1, n1);
    // slot 0 holds step 0 and slot 1 step 1 of this tile (loaded during the previous tile or above)
    if (tid < BN) lbias[tid] = g.bias[n0 + tid];   // (its last readers passed the barrier below a tile ago)
    __syncthreads();   // the previous tile's patches are read
    stash(S0{}, S0{});
    issue(S0{}, cur, 2 * BK);
    __syncthreads();
    // the bias is the initial value of the accumulators
#pragma unroll
    for (int j = 0; j < WBN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 b = *reinterpret_cast<const float4*>(lbias + wn * (WBN * 32) + j * 32 + q * 8 + (lane >> 5) * 4);
#pragma unroll
        for (int i = 0; i < WBM; ++i) {
          acc[i][j][4 * q] = b.x; acc[i][j][4 * q + 1] = b.y; acc[i][j][4 * q + 2] = b.z; acc[i][j][4 * q + 3] = b.w;
        }
      }
#pragma unroll
    for (int i = 0; i < WBM; ++i) rd_a(ring0, i, 0);
#pragma unroll
    for (int j = 0; j < WBN; ++j) rd_b(ring0, j, 0);
    // steps 0 .. nk - 1 (nk even, >= 6); the loads three steps ahead run into the next tile near the end
    for (int kt = 0; kt < nk - 2; kt += 2) {
      const bool w0 = kt + 3 >= nk, w1 = kt + 4 >= nk;   // uniform
      step(S0{}, std::false_type{}, w0 ? nxt : cur, (w0 ? kt + 3 - nk : kt + 3) * BK);
      step(S1{}, std::false_type{}, w1 ? nxt : cur, (w1 ? kt + 4 - nk : kt + 4) * BK);
    }
    step(S0{}, std::false_type{}, nxt, BK);   // step nk - 2: writes step nk - 1, loads step 1 of the next tile
    step(S1{}, std::true_type{}, nxt, 0);     // step nk - 1
    __syncthreads();   // every wavefront has read its last fragments: the stages become the patches
    epilogue(m0, n0);
    id = nid; m0 = m1; n0 = n1; cur = nxt;
  }
}

}  // namespace

// Shapes this kernel takes: the bias + GELU epilogue, a contraction that is a whole number of double steps and at
// least six steps, enough rows to fill the chip with 256-row tiles, 32-bit operand offsets.  Alignment requirements
// are those of gemm_nt_mfma_ok.
bool gemm_nt_gelu_ok(const GemmNT& g) {
  return g.epi == EPI_BIAS_GELU && g.amap.g2 == 0 && g.M < (1LL << 31) && g.M >= 4096 && g.N % BN == 0 &&
         g.lda < (1 << 20) && g.ldb < (1 << 20) && g.ldc < (1 << 20) && g.ldc2 < (1 << 20) && g.K % (2 * BK) == 0 &&
         g.K >= MIN_STEPS * BK;
}

hipError_t launch_gemm_nt_gelu(const GemmNT& g, hipStream_t s) {
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
  int MT = (int)((g.M + BM - 1) / BM), NTL = (g.N + BN - 1) / BN;
  long long total = (long long)((MT + NXCD - 1) / NXCD) * NXCD * NTL;
  long long wgs = total < cus ? total : cus;
  hipLaunchKernelGGL(gemm_nt_gelu_k, dim3((unsigned)wgs), dim3(NTH), 0, s, g, MT, NTL);
  return hipGetLastError();
}

}  // namespace sl
