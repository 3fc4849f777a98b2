// bf16 MFMA "NT" GEMM for gfx950, large-M variant: C[M,N] = A[M,K] * B[N,K]^T (+ fused epilogue).
//
// The encoder's GEMMs have a short contraction (K = D or 4D) and a huge M (all tokens of the slide), so
// per output tile there is little MFMA work to hide the operand traffic and the epilogue behind.  What one
// compute unit can pull out of its L2 (measured: < 50 bytes per clock) bounds the tile from below: a
// 256 x 192 tile needs (256 + 192) * 2 bytes per 256 * 192 * 2 flop, about 37 bytes per MFMA clock.  192
// divides every N that occurs (D, 3D, 4D for D = 384 and 768), so no column tile is partly empty.
//   * One persistent workgroup of 4 wavefronts per compute unit (one per SIMD, the whole register file
//     each); a wavefront owns 128 x 96 of the tile (4 x 3 accumulators of 32 x 32), so every fragment read
//     from LDS feeds three or four MFMAs.  Tiles that share an A row panel run at the same time on one XCD.
//   * Operands travel global -> registers -> LDS.  The A loads of K step k + 3 and the B loads of step
//     k + 2 are issued during step k and stay in flight (in registers) across steps and across tile
//     boundaries, which covers an HBM miss on the A panel; LDS holds two stages of [256 + 192][64 + 8]
//     bf16 (two separate arrays, so that writes to one are free to move past reads of the other) and
//     needs one barrier per step.  The order of MFMA, LDS and global instructions inside a step is explicit.
//   * The epilogue of a tile runs in the background of the next tile's K steps: with one wavefront per
//     SIMD nothing else would keep the MFMA pipe busy while results are stored.  At the end of a tile the
//     accumulators (bias included) are rounded to bf16 and parked in registers (96 instead of 192), the
//     accumulators are free again and the next tile starts at once.  During its steps 1..4 the parked
//     block goes, one 32-row strip per step, through a wave-private LDS patch (the MFMA operands are
//     passed swapped, so a lane holds runs of four neighbouring columns of one row and writes 8 bytes;
//     it reads back 16-byte row segments), is combined with the residual / the stored GELU derivative or
//     run through the GELU table, and is stored with 16-byte accesses along rows.
//     The sum with the residual and the product with the GELU derivative are formed in fp32 from the
//     bf16-rounded GEMM result and rounded once more.
//   * GELU and its derivative come from a table of the normal CDF and of d/dx (x cdf(x)) in LDS, linearly
//     interpolated at 1/32 steps (error < 1e-4, far below bf16 rounding).
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
constexpr int TAB_N = 448;                         // table over [-7, 7) in steps of 1/32
constexpr int PSB = 208;                           // patch row stride in bytes (96 bf16 + 16)
constexpr int PATCH_BYTES = 32 * PSB;              // one 32 x 96 bf16 strip per wavefront
constexpr int NPASS = 7;                           // 12 lanes per row, 5 rows per pass, lanes 60..63 idle
constexpr int MIN_STEPS = 6;                       // steps 1..4 of a tile carry the previous tile's strips

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// uniform base (scalar registers) + 32-bit per-lane byte offset
__device__ __forceinline__ u32x4 ldg16(const char* base, unsigned off) { return *reinterpret_cast<const u32x4*>(base + off); }

__device__ __forceinline__ unsigned pack2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);  // round to nearest even
  return __builtin_bit_cast(unsigned, h);
}
__device__ __forceinline__ u32x4 pack8(const float (&v)[8]) {
  u32x4 r;
#pragma unroll
  for (int w = 0; w < 4; ++w) r[w] = pack2(v[2 * w], v[2 * w + 1]);
  return r;
}
__device__ __forceinline__ void unpack8(u32x4 t, float (&v)[8]) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    v[2 * w] = __uint_as_float(t[w] << 16);
    v[2 * w + 1] = __uint_as_float(t[w] & 0xffff0000u);
  }
}

// table entry k: {cdf(x_k), cdf(x_k+1) - cdf(x_k), c(x_k), c(x_k+1) - c(x_k)}, x_k = -7 + k/32,
// cdf = standard normal distribution function, dg(x) = cdf(x) + x * pdf(x) = d/dx (x cdf(x)) and c = dg8_code(dg),
// the derivative in the code space of its one-byte storage
__device__ __forceinline__ void gelu_both_tab(const float4* tab, float x, float* gl, float* dgc) {
  float t = __builtin_amdgcn_fmed3f(x * 32.0f + 224.0f, 0.0f, (float)TAB_N - 0.001f);
  int k = (int)t;                       // t >= 0: truncation is the floor
  float f = __builtin_amdgcn_fractf(t);
  float4 e = tab[k];
  *gl = x * (e.x + f * e.y);
  *dgc = e.z + f * e.w;
}

template <class F, int... Is>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

template <int V> using IC = std::integral_constant<int, V>;

template <int MODE>
__global__ void __launch_bounds__(NTH) gemm_nt_big_k(GemmNT g, int MT, int NTL) {
  constexpr bool HAS_BIAS = MODE == EPI_BIAS || MODE == EPI_BIAS_RESID || MODE == EPI_BIAS_GELU;
  constexpr bool HAS_AUX = MODE == EPI_BIAS_RESID || MODE == EPI_DGELU || MODE == EPI_ROWTAB;
  // stores issued in one burst at the end of a step measured slower than stores spread over the step
  constexpr bool LATE_STORES = false;
  // two separate arrays: the compiler then knows that the LDS writes of the next step's operands do not alias
  // the fragment reads of the current one
  __shared__ __attribute__((aligned(16))) bf16 ring0[STAGE];
  __shared__ __attribute__((aligned(16))) bf16 ring1[STAGE];
  __shared__ __attribute__((aligned(16))) unsigned char patches[(NTH / 64) * PATCH_BYTES];
  __shared__ float4 tab[MODE == EPI_BIAS_GELU ? TAB_N : 1];
  __shared__ __attribute__((aligned(16))) float lbias_all[BN];  // zeros when there is no bias
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int row0 = tid >> 3, kc = tid & 7;       // loader: 32 rows x 8 chunks of 16 bytes per pass
  const int soff = row0 * LDT + kc * 8;
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  const int nk = g.K / BK;
  const int total = (MT + NXCD - 1) / NXCD * NXCD * NTL;

  if (MODE == EPI_BIAS_GELU) {
    // filled once per workgroup; the K-loop barriers order it before its first use
    for (int k = tid; k < TAB_N; k += NTH) {
      float x0 = -7.0f + (float)k * (1.0f / 32.0f), x1 = x0 + (1.0f / 32.0f);
      float c0 = 0.5f * (1.0f + erff(x0 * 0.70710678118654752f)), c1 = 0.5f * (1.0f + erff(x1 * 0.70710678118654752f));
      float d0 = c0 + x0 * 0.39894228040143268f * expf(-0.5f * x0 * x0);
      float d1 = c1 + x1 * 0.39894228040143268f * expf(-0.5f * x1 * x1);
      tab[k] = make_float4(c0, c1 - c0, dg8_code(d0), dg8_code(d1) - dg8_code(d0));
    }
  }

  // (every lambda below is forced inline: left to its size heuristics the compiler keeps some of them as calls,
  // and the register arrays they touch would then live in memory)
  // tile id -> (row tile, column tile): ids are dealt round-robin to the XCDs and the column tiles of one
  // row panel get consecutive slots of one XCD (the grid size is a multiple of 8)
  auto tile_of = [&](int id, long long& m0, int& n0) __attribute__((always_inline)) {
    int xcd = id % NXCD, slot = id / NXCD;
    int mt = (slot / NTL) * NXCD + xcd;
    m0 = (long long)mt * BM;
    n0 = (slot % NTL) * BN;
    return mt < MT;
  };
  auto next_valid = [&](int id, long long& m0, int& n0) __attribute__((always_inline)) {
    while (id < total && !tile_of(id, m0, n0)) id += gridDim.x;
    return id;
  };

  // ---- operand loads: uniform base + 32-bit per-thread byte offsets --------------------------------------
  const bf16* Ab;
  const bf16* Bb;
  // chunk i of a thread is row0 + 32 i: one per-thread offset plus a uniform row stride serves all chunks.
  // Rows past the end of A (last row tile only) are redirected to row M - 1 by clamping the offset: they are
  // loaded (valid memory) but never stored.
  const unsigned aoff0 = 2u * (unsigned)(row0 * (int)g.lda + kc * 8), boff0 = 2u * (unsigned)(row0 * (int)g.ldb + kc * 8);
  const unsigned astride = 2u * RSTEP * (unsigned)g.lda, bstride = 2u * RSTEP * (unsigned)g.ldb;  // bytes
  unsigned amax = 0xffffffffu;   // largest valid offset of this thread: (M - 1 - m0) rows + its chunk column
  // A: two register slots (loads three steps ahead of their MFMAs; it may miss to HBM).  B: two slots and the same
  // lead where the registers allow it (with every load an L1 hit the K loop runs a third faster: it is the time
  // the L2 takes to answer that the loop waits for), one slot and one step less in the modes that keep two
  // strips of auxiliary rows in registers.
  constexpr bool B2 = !HAS_AUX;
  u32x4 ra[2][CA], rb[2][CB];
  float rbias = 0.f;
  auto set_offsets_a = [&](long long m0) __attribute__((always_inline)) {
    Ab = (const bf16*)g.A + m0 * g.lda;
    amax = m0 + BM > g.M ? 2u * (unsigned)((g.M - 1 - m0) * g.lda + kc * 8) : 0xffffffffu;
  };
  auto set_offsets_b = [&](int n0) __attribute__((always_inline)) {
    Bb = (const bf16*)g.B + (long long)n0 * g.ldb;
    if (HAS_BIAS && tid < BN) rbias = g.bias[n0 + tid];  // else stays 0
  };
  auto load_a = [&](int i, int k0) __attribute__((always_inline)) {
    unsigned off = aoff0 + (unsigned)i * astride;
    return ldg16((const char*)(Ab + k0), off < amax ? off : amax);
  };
  auto load_b = [&](int i, int k0) __attribute__((always_inline)) {
    return ldg16((const char*)(Bb + k0) + (unsigned)i * bstride, boff0);   // N % 192 == 0: no clamp
  };
  auto issue_a = [&](auto slot, int k0) __attribute__((always_inline)) {
    constexpr int S = decltype(slot)::value;
#pragma unroll
    for (int i = 0; i < CA; ++i) ra[S][i] = load_a(i, k0);
  };
  auto issue_b = [&](auto slot, int k0) __attribute__((always_inline)) {
    constexpr int S = B2 ? decltype(slot)::value : 0;
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[S][i] = load_b(i, k0);
  };
  auto stash = [&](auto slot) __attribute__((always_inline)) {
    constexpr int S = decltype(slot)::value;
    bf16* st = S ? ring1 : ring0;
#pragma unroll
    for (int i = 0; i < CA; ++i) *reinterpret_cast<u32x4*>(st + soff + i * RSTEP * LDT) = ra[S][i];
#pragma unroll
    for (int i = 0; i < CB; ++i) *reinterpret_cast<u32x4*>(st + BM * LDT + soff + i * RSTEP * LDT) = rb[B2 ? S : 0][i];
  };

  // ---- MFMA side ----------------------------------------------------------------------------------------------
  f32x16 acc[WBM][WBN];
  bf16x8 fa[2][WBM], fb[2][WBN];   // two buffers of one 16-wide slice each
  // fragment t (0..3: A row blocks, 4..6: B column blocks) of slice KS of stage S -> buffer BF
  auto rd_one = [&](auto slot, auto slice, auto buf, auto frag) __attribute__((always_inline)) {
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
  auto wr_one = [&](auto slot, auto idx) __attribute__((always_inline)) {
    constexpr int S = decltype(slot)::value, W = decltype(idx)::value;
    bf16* st = S ? ring1 : ring0;
    if constexpr (W < CA) *reinterpret_cast<u32x4*>(st + soff + W * RSTEP * LDT) = ra[S][W];
    else *reinterpret_cast<u32x4*>(st + BM * LDT + soff + (W - CA) * RSTEP * LDT) = rb[B2 ? S : 0][W - CA];
  };
  // global load l of a step: 0..5 the B chunks (they are needed first and hit L2), 6..13 the A chunks.
  // Loads return in order: the B chunks, issued one step before their LDS writes, do not wait for younger A
  // loads that may miss to HBM.
  auto ld_one = [&](auto slot, auto idx, int ka, int kb) __attribute__((always_inline)) {
    constexpr int S = decltype(slot)::value, Lx = decltype(idx)::value;
    if constexpr (Lx < CB) rb[B2 ? S : 0][Lx] = load_b(Lx, kb);
    else ra[S][Lx - CB] = load_a(Lx - CB, ka);
  };
  auto mfma_one = [&](auto buf, auto tt) __attribute__((always_inline)) {
    constexpr int BF = decltype(buf)::value, T = decltype(tt)::value, i = T / WBN, j = T % WBN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[BF][j], fa[BF][i], acc[i][j], 0, 0, 0);
  };

  // ---- background epilogue of the previous tile ------------------------------------------------------------
  // Accumulator element r of lane l (operands swapped) is row l % 32, column (r / 4) * 8 + (l / 32) * 4 + r % 4
  // of its 32 x 32 block.  park[i - 1][j][q] holds strip i (rows i * 32 ..), column block j, elements
  // 4q .. 4q + 3 as four bf16; strip 0 goes to the LDS patch when the tile ends.  Per strip the wave
  // writes 12 x 8 bytes per lane to its patch and reads 16-byte row segments back: 12 lanes per row, 5
  // rows per pass, 7 passes (the last holds rows 30 and 31), so the lane -> (row, segment) map is the
  // same in every pass and all offsets are immediates.
  u32x2 park[WBM - 1][WBN][4];
  long long pmw = 0;   // first row / column of the parked block (uniform)
  int pnw = 0;
  typedef std::conditional_t<MODE == EPI_DGELU, u32x2, u32x4> aux_t;   // eight codes / eight bf16
  u32x4 rowdat[NPASS];
  aux_t auxv[2][NPASS];   // auxiliary row segments of two strips: one in use, one in flight
  const int er = lane < 60 ? lane / 12 : 0;    // row inside a pass (idle lanes: a valid address)
  const int erc = lane < 60 ? lane / 12 : 64;  // the same for comparisons: idle lanes never pass
  const int esg = lane % 12;
  const unsigned ldc_b = 2u * (unsigned)g.ldc, ldc2_b = (unsigned)g.ldc2;   // bytes (the derivative: one per element)
  const unsigned lda_b = MODE == EPI_DGELU ? (unsigned)g.ldpre : 2u * (unsigned)g.ldr;
  constexpr int AUXW = MODE == EPI_DGELU ? 1 : 2;   // bytes per element of the auxiliary operand
  const unsigned eo_c = (unsigned)er * ldc_b + esg * 16, eo_c2 = (unsigned)er * ldc2_b + esg * 8;
  const unsigned eo_a = (unsigned)er * lda_b + esg * (8 * AUXW);
  unsigned char* const pw = patches + wave * PATCH_BYTES + (lane & 31) * PSB + (lane >> 5) * 8;
  const unsigned char* const pr = patches + wave * PATCH_BYTES + er * PSB + esg * 16;
  const char* const aux_ptr = (const char*)(MODE == EPI_DGELU ? g.pre : g.resid);
  unsigned pmod = 0;   // EPI_ROWTAB: first row of the parked block modulo the table's row count (uniform)

  // rows of strip I of the parked block that exist (uniform, may be <= 0)
  auto strip_lim = [&](int I) __attribute__((always_inline)) {
    long long r = g.M - (pmw + I * 32);
    return r > 32 ? 32 : (int)r;
  };
  auto bg_w = [&](auto ic, auto wc) __attribute__((always_inline)) {
    constexpr int I = decltype(ic)::value, W = decltype(wc)::value, j = W / 4, q = W % 4;
    *reinterpret_cast<u32x2*>(pw + j * 64 + q * 16) = park[I - 1][j][q];
  };
  auto bg_r = [&](auto pc) __attribute__((always_inline)) {
    constexpr int p = decltype(pc)::value;
    rowdat[p] = *reinterpret_cast<const u32x4*>(pr + p * 5 * PSB);
  };
  auto bg_aux = [&](auto ic, auto pc, int lim) __attribute__((always_inline)) {
    constexpr int I = decltype(ic)::value, p = decltype(pc)::value;
    if constexpr (HAS_AUX) {
      if (p * 5 < lim) {  // uniform; lanes past the end read the pass's first row (never stored)
        if constexpr (MODE == EPI_ROWTAB) {
          // the pass's rows modulo the table's row count: the block's first row is known modulo it, a pass is at
          // most 131 rows further (fewer than a table has: one conditional subtraction each)
          const unsigned per = (unsigned)g.rperiod;
          unsigned pm = pmod;
          asm volatile("" : "+s"(pm));   // formed where it is used: 28 addresses kept from the tile's start do not fit
          unsigned r0 = pm + I * 32 + p * 5;
          r0 = r0 >= per ? r0 - per : r0;
          unsigned t = r0 + (unsigned)er;
          t = t >= per ? t - per : t;
          auxv[I & 1][p] = *reinterpret_cast<const aux_t*>(aux_ptr + 2 * pnw + (t * lda_b + esg * 16));
        } else {
          const char* base = aux_ptr + ((pmw + I * 32 + p * 5) * (long long)lda_b + AUXW * pnw);
          auxv[I & 1][p] = *reinterpret_cast<const aux_t*>(base + (p * 5 + erc < lim ? eo_a : (unsigned)(esg * (8 * AUXW))));
        }
      }
    }
  };
  // pass p of strip I: combine the row segment with the auxiliary operand (results stay in registers) ...
  u32x4 res[NPASS];
  u32x2 res2[MODE == EPI_BIAS_GELU ? NPASS : 1];
  auto bg_cmp = [&](auto ic, auto pc) __attribute__((always_inline)) {
    constexpr int I = decltype(ic)::value, p = decltype(pc)::value;
    if constexpr (MODE == EPI_PLAIN || MODE == EPI_BIAS) {
      res[p] = rowdat[p];
    } else if constexpr (MODE == EPI_BIAS_RESID || MODE == EPI_ROWTAB) {
      float v[8], t[8];
      unpack8(rowdat[p], v);
      unpack8(auxv[I & 1][p], t);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] += t[e];
      res[p] = pack8(v);
    } else if constexpr (MODE == EPI_DGELU) {
      float v[8], t0[4], t1[4];
      unpack8(rowdat[p], v);
      dg8_unpack4(auxv[I & 1][p][0], t0);
      dg8_unpack4(auxv[I & 1][p][1], t1);
#pragma unroll
      for (int e = 0; e < 4; ++e) { v[e] *= t0[e]; v[4 + e] *= t1[e]; }
      res[p] = pack8(v);
    } else {  // EPI_BIAS_GELU: out = gelu(m), out2 = the code of gelu'(m), m the bf16-rounded pre-activation
      float v[8], t[8];
      unpack8(rowdat[p], v);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float gl, dg;
        gelu_both_tab(tab, v[e], &gl, &dg);
        v[e] = gl;
        t[e] = dg;
      }
      res[p] = pack8(v);
      res2[p] = u32x2{dg8_pack4_code(t[0], t[1], t[2], t[3]), dg8_pack4_code(t[4], t[5], t[6], t[7])};
    }
  };
  // ... and its stores.  They are issued after the step's operand loads: memory operations complete in
  // order, so loads queued behind stores wait for the stores to drain, and the loads of one step are
  // needed one step later; stores at the end of a step have two steps to complete before anything waits.
  auto bg_put = [&](auto ic, auto pc, int lim) __attribute__((always_inline)) {
    constexpr int I = decltype(ic)::value, p = decltype(pc)::value;
    if (p * 5 < lim) {  // uniform
      bool ok = p * 5 + erc < lim;
      char* o = (char*)g.out + ((pmw + I * 32 + p * 5) * (long long)ldc_b + 2 * pnw);
      if (ok) __builtin_nontemporal_store(res[p], reinterpret_cast<u32x4*>(o + eo_c));
      if constexpr (MODE == EPI_BIAS_GELU) {
        char* o2 = (char*)g.out2 + ((pmw + I * 32 + p * 5) * (long long)ldc2_b + pnw);
        if (ok) __builtin_nontemporal_store(res2[p], reinterpret_cast<u32x2*>(o2 + eo_c2));
      }
    }
  };

  // One K step out of LDS stage S, in explicit issue order: one MFMA and a few other instructions per piece,
  // a scheduling fence after each piece (one wavefront per SIMD: nothing else hides the LDS and
  // global-memory instructions, so they are dealt out between the 48 MFMAs).  The step's barrier sits
  // between slices 2 and 3: by then every fragment of this stage has been read and the next stage
  // (A: register slot S^1, loaded two steps ago; B: loaded one step ago) is completely written, so the
  // fragments of the next step's slice 0 are fetched under the MFMAs of slice 3 and no wavefront starts a
  // step with an empty MFMA pipe.  The registers are re-used for A three steps and B two steps ahead
  // (element offsets ka, kb).  BG = 0: nothing else; BG < 0: only the auxiliary loads of strip 0; BG = 1 + I: strip I of the previous tile's block is
  // moved through the patch and stored.
  auto step = [&](auto slot, auto bgc, int ka, int kb) __attribute__((always_inline)) {
    constexpr int S = decltype(slot)::value, BG = decltype(bgc)::value, I = BG - 1;
    using SN = IC<S ^ 1>;
    int lim = 0;
    if constexpr (BG > 0) lim = strip_lim(I);
    static_for<36>([&](auto pc) __attribute__((always_inline)) {
      constexpr int P = decltype(pc)::value, KS = P / 12, T = P % 12;
      mfma_one(IC<KS & 1>{}, IC<T>{});
      if constexpr (T < WBM + WBN) rd_one(slot, IC<KS + 1>{}, IC<(KS + 1) & 1>{}, IC<T>{});
      if constexpr (KS < 2 && T >= 7) wr_one(SN{}, IC<KS * 5 + T - 7>{});
      if constexpr (KS == 2 && T < 4) wr_one(SN{}, IC<10 + T>{});
      if constexpr (KS == 2 && T >= 7) ld_one(SN{}, IC<T - 7>{}, ka, kb);
      if constexpr (BG < 0) {
        if constexpr (P < NPASS) bg_aux(IC<0>{}, IC<P>{}, strip_lim(0));   // strip 0 is processed in the next step
      }
      if constexpr (BG > 0) {
        if constexpr (P < NPASS && I + 1 < WBM) bg_aux(IC<I + 1>{}, IC<P>{}, strip_lim(I + 1));   // needed one step later
        if constexpr (I > 0 && P < 12) bg_w(IC<I>{}, IC<P>{});
        if constexpr (P >= 17 && (P - 17) % 4 == 0 && (P - 17) / 4 < NPASS) bg_r(IC<(P - 17) / 4>{});
        if constexpr (P >= 20 && (P - 20) % 4 == 0 && (P - 20) / 4 < NPASS) {
          bg_cmp(IC<I>{}, IC<(P - 20) / 4>{});
          if constexpr (!LATE_STORES) bg_put(IC<I>{}, IC<(P - 20) / 4>{}, lim);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    __syncthreads();
    static_for<12>([&](auto tc) __attribute__((always_inline)) {
      constexpr int T = decltype(tc)::value, P = 36 + T;
      mfma_one(IC<1>{}, tc);
      if constexpr (T < WBM + WBN) rd_one(SN{}, IC<0>{}, IC<0>{}, tc);
      if constexpr (T < 9) ld_one(SN{}, IC<5 + T>{}, ka, kb);
      if constexpr (BG > 0) {
        if constexpr (P >= 17 && (P - 17) % 4 == 0 && (P - 17) / 4 < NPASS) bg_r(IC<(P - 17) / 4>{});
        if constexpr (P >= 20 && (P - 20) % 4 == 0 && (P - 20) / 4 < NPASS) {
          bg_cmp(IC<I>{}, IC<(P - 20) / 4>{});
          if constexpr (!LATE_STORES) bg_put(IC<I>{}, IC<(P - 20) / 4>{}, lim);
        }
        if constexpr (LATE_STORES && T == 9) { bg_put(IC<I>{}, IC<0>{}, lim); bg_put(IC<I>{}, IC<1>{}, lim); }
        if constexpr (LATE_STORES && T == 10) { bg_put(IC<I>{}, IC<2>{}, lim); bg_put(IC<I>{}, IC<3>{}, lim); }
        if constexpr (LATE_STORES && T == 11) { bg_put(IC<I>{}, IC<4>{}, lim); bg_put(IC<I>{}, IC<5>{}, lim); bg_put(IC<I>{}, IC<6>{}, lim); }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
  };

  // the same strip work on its own (after the last tile)
  auto strip_alone = [&](auto ic) __attribute__((always_inline)) {
    constexpr int I = decltype(ic)::value;
    int lim = strip_lim(I);
    static_for<NPASS>([&](auto pc) __attribute__((always_inline)) { bg_aux(ic, pc, lim); });
    if constexpr (I > 0) static_for<12>([&](auto wc) __attribute__((always_inline)) { bg_w(ic, wc); });
    static_for<NPASS>([&](auto pc) __attribute__((always_inline)) { bg_r(pc); });
    static_for<NPASS>([&](auto pc) __attribute__((always_inline)) { bg_cmp(ic, pc); });
    static_for<NPASS>([&](auto pc) __attribute__((always_inline)) { bg_put(ic, pc, lim); });
  };

  long long m0, m1;
  int n0, n1;
  int id = next_valid(blockIdx.x, m0, n0);
  if (id >= total) return;
  // prologue: step 0 in LDS stage 0, steps 1 and 2 in flight in register slots 1 and 0
  // (the order of these loads is fenced: the waits the compiler places in the K loop are the most
  // conservative over every way into it, this one included)
  set_offsets_a(m0);
  set_offsets_b(n0);
  issue_a(IC<0>{}, 0);
  issue_b(IC<0>{}, 0);
  __builtin_amdgcn_sched_barrier(0);
  if constexpr (B2) issue_b(IC<1>{}, BK);
  issue_a(IC<1>{}, BK);
  __builtin_amdgcn_sched_barrier(0);
  stash(IC<0>{});
  __builtin_amdgcn_sched_barrier(0);
  issue_b(IC<0>{}, B2 ? 2 * BK : BK);
  __builtin_amdgcn_sched_barrier(0);
  issue_a(IC<0>{}, 2 * BK);
  __builtin_amdgcn_sched_barrier(0);
  if (tid < BN) lbias_all[tid] = rbias;
  __syncthreads();
  static_for<WBM + WBN>([&](auto tc) __attribute__((always_inline)) { rd_one(IC<0>{}, IC<0>{}, IC<0>{}, tc); });

  // One tile: K steps 0 .. nk - 1 (nk even, >= 6); steps 1..4 carry the strips of the block parked by the
  // tile before (BGON).  Loads run ahead into the next tile: its A offsets are in place before step nk - 3,
  // its B offsets before step nk - 2.  The last step stores the next tile's first stage and fetches its
  // first fragments like any other step, so the MFMA pipe only waits while the accumulators are parked.
  auto koff = [&](int x) __attribute__((always_inline)) { return (x >= nk ? x - nk : x) * BK; };
  auto run_tile = [&](auto bgon) __attribute__((always_inline)) {
    constexpr bool BGON = decltype(bgon)::value;
    const long long mw = m0 + wm * (WBM * 32);
    const int nw = n0 + wn * (WBN * 32);
    // the bias (or zero) is the initial value of the accumulators
#pragma unroll
    for (int j = 0; j < WBN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
        if (HAS_BIAS) b = *reinterpret_cast<const float4*>(lbias_all + wn * (WBN * 32) + j * 32 + q * 8 + (lane >> 5) * 4);
#pragma unroll
        for (int i = 0; i < WBM; ++i) {
          acc[i][j][4 * q] = b.x; acc[i][j][4 * q + 1] = b.y; acc[i][j][4 * q + 2] = b.z; acc[i][j][4 * q + 3] = b.w;
        }
      }
    auto pre = [&](int s) __attribute__((always_inline)) {
      if (s == nk - 3) set_offsets_a(m1);
      if (s == nk - (B2 ? 3 : 2)) set_offsets_b(n1);
    };
    pre(0); step(IC<0>{}, IC<(BGON && HAS_AUX) ? -1 : 0>{}, koff(3), B2 ? koff(3) : koff(2));
    pre(1); step(IC<1>{}, IC<BGON ? 1 : 0>{}, koff(4), B2 ? koff(4) : koff(3));
    pre(2); step(IC<0>{}, IC<BGON ? 2 : 0>{}, koff(5), B2 ? koff(5) : koff(4));
    pre(3); step(IC<1>{}, IC<BGON ? 3 : 0>{}, koff(6), B2 ? koff(6) : koff(5));
    pre(4); step(IC<0>{}, IC<BGON ? 4 : 0>{}, koff(7), B2 ? koff(7) : koff(6));
    for (int s = 5; s < nk - 1; s += 2) {
      pre(s); step(IC<1>{}, IC<0>{}, koff(s + 3), B2 ? koff(s + 3) : koff(s + 2));
      pre(s + 1); step(IC<0>{}, IC<0>{}, koff(s + 4), B2 ? koff(s + 4) : koff(s + 3));
    }
    if (tid < BN) lbias_all[tid] = rbias;  // next tile's bias; this tile's was consumed at its start
    step(IC<1>{}, IC<0>{}, 2 * BK, B2 ? 2 * BK : BK);
    // park the block: strip 0 in the patch, strips 1..3 in registers
#pragma unroll
    for (int i = 0; i < WBM; ++i)
#pragma unroll
      for (int j = 0; j < WBN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          u32x2 pk = {pack2(acc[i][j][4 * q], acc[i][j][4 * q + 1]), pack2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3])};
          if (i == 0) *reinterpret_cast<u32x2*>(pw + j * 64 + q * 16) = pk;
          else park[i - 1][j][q] = pk;
        }
    pmw = mw;
    pnw = nw;
    if constexpr (MODE == EPI_ROWTAB) pmod = (unsigned)mw % (unsigned)g.rperiod;   // (M < 2^31)
  };

  {
    int nid = next_valid(id + gridDim.x, m1, n1);
    if (nid >= total) { m1 = m0; n1 = n0; }  // no further tile: the prefetches re-read this one and are dropped
    run_tile(std::false_type{});
    id = nid; m0 = m1; n0 = n1;
  }
  while (id < total) {
    int nid = next_valid(id + gridDim.x, m1, n1);
    if (nid >= total) { m1 = m0; n1 = n0; }
    run_tile(std::true_type{});
    id = nid; m0 = m1; n0 = n1;
  }
  strip_alone(IC<0>{});
  strip_alone(IC<1>{});
  strip_alone(IC<2>{});
  strip_alone(IC<3>{});
}

}  // namespace

// Shapes this kernel takes: a contraction that is a whole number of double steps and at least six steps,
// enough rows to fill the chip with 256-row tiles, a bf16 residual stream.  Alignment requirements are those
// of gemm_nt_mfma_ok.  The patch-embedding epilogue (row-mapped output) stays with the small kernel.
bool gemm_nt_big_ok(const GemmNT& g) {
  bool shape = g.M < (1LL << 31) && g.N % BN == 0 && g.lda < (1 << 20) && g.ldb < (1 << 20) && g.ldc < (1 << 20) &&
               g.ldc2 < (1 << 20) && g.ldr < (1 << 20) && g.ldpre < (1 << 20) && g.K % (2 * BK) == 0 &&
               g.K >= MIN_STEPS * BK && g.M >= 4096;
  bool mode = g.epi == EPI_PLAIN || g.epi == EPI_BIAS || g.epi == EPI_BIAS_GELU || g.epi == EPI_DGELU ||
              (g.epi == EPI_BIAS_RESID && sizeof(rs_bf16path_t) == 2) ||
              (g.epi == EPI_ROWTAB && sizeof(rs_bf16path_t) == 2 && g.rperiod >= 160);
  return shape && mode && g.amap.g2 == 0;
}

template <int MODE>
hipError_t launch_big(const GemmNT& g, hipStream_t s) {
  static int cus = 0;
  auto kern = gemm_nt_big_k<MODE>;
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

hipError_t launch_gemm_nt_big(const GemmNT& g, hipStream_t s) {
  switch (g.epi) {
    case EPI_PLAIN: return launch_big<EPI_PLAIN>(g, s);
    case EPI_BIAS: return launch_big<EPI_BIAS>(g, s);
    case EPI_BIAS_RESID: return launch_big<EPI_BIAS_RESID>(g, s);
    case EPI_BIAS_GELU: return launch_big<EPI_BIAS_GELU>(g, s);
    case EPI_DGELU: return launch_big<EPI_DGELU>(g, s);
    case EPI_ROWTAB: return launch_big<EPI_ROWTAB>(g, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sl
