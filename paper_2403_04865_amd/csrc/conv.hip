// Convolutions of the ResNet tile encoder on the bf16 matrix cores of gfx950 (v_mfma_f32_32x32x16_bf16, fp32
// accumulation), as implicit GEMMs over channels-last activations: a tensor is a matrix [n * H * W][C], one row per
// position, so a tap of a convolution is a row gather and a channel slice of a tap is 128 contiguous bytes.
//
//   conv_nt_dl_k : forward and input gradient.  out[M][N] = sum_taps gather_tap(src)[M][Cs] * W_tap[N][Cs]^T.  The
//                  contraction index is (tap, channel); a K step is 64 channels of one tap, so the tap of a step is the
//                  same for the whole workgroup and only the row addresses change from step to step.  Rows that fall
//                  into the zero padding (or, for the input gradient of a strided convolution, between the taps) read
//                  zeros.  Operands go from global memory straight into LDS (see the kernel).  The MFMA takes the
//                  weights as its first operand, so a lane ends up with four consecutive output channels of one row;
//                  the tile goes through LDS once (fp32) and leaves as whole row segments, rounded once.
//   conv_wgrad_k : weight gradient.  dW[co][tap][ci] = sum_rows dout[row][co] * gather_tap(src)[row][ci]: the
//                  contraction runs over the rows, so the 32-row slices go to LDS as they are (straight from global
//                  memory, like the other kernel's operands) and the MFMA operands come from LDS transpose reads.  One workgroup owns a 64 x 64 block of (co, ci) for ALL taps (the
//                  output-gradient slice is loaded once for the nine taps) over one slab of rows; slabs are added in
//                  a fixed order by wgrad_reduce_k (no atomics: run-to-run identical), which also turns the
//                  [co][tap][ci] order of the kernels into the parameter's [co][ci][kh][kw].
#include "resnet_internal.h"
#include <type_traits>

namespace sl {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ u32x4 ldg16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }

constexpr int ROW_ABSENT = -(1 << 20);   // y of a row past the end: no tap of it is ever inside a grid

// source row of produced row (n, y, x) for tap (kh, kw), or -1
__device__ __forceinline__ long long src_row(const ConvGeom& g, int n, int y, int x, int kh, int kw) {
  int ys, xs;
  bool ok;   // bitwise combinations: no branch per condition
  if (!g.transposed) {
    ys = y * g.stride + kh - g.pad;
    xs = x * g.stride + kw - g.pad;
    ok = ((unsigned)ys < (unsigned)g.YS) & ((unsigned)xs < (unsigned)g.XS);
  } else {
    const int ty = y + g.pad - kh, tx = x + g.pad - kw;
    const int sm = g.stride - 1, sh = g.stride >> 1;   // stride is 1 or 2
    ys = ty >> sh;
    xs = tx >> sh;
    ok = ((ty | tx) >= 0) & (((ty | tx) & sm) == 0) & (ys < g.YS) & (xs < g.XS);
  }
  const long long r = ((long long)n * g.YS + ys) * g.XS + xs;
  return ok ? r : -1;
}

__device__ __forceinline__ void row_pos(long long m, long long M, const ConvGeom& g, int& n, int& y, int& x) {
  if (m < M) {
    const unsigned plane = (unsigned)(g.YO * g.XO);
    const unsigned mm = (unsigned)m;
    const unsigned q = mm / plane, rem = mm - q * plane;
    const unsigned yy = rem / (unsigned)g.XO;
    n = (int)q; y = (int)yy; x = (int)(rem - yy * (unsigned)g.XO);
  } else {
    n = 0; y = ROW_ABSENT; x = 0;
  }
}

// row m of a launch -> position (n, y, x) of the produced grid; with a parity class the rows enumerate that class only
__device__ __forceinline__ void launch_pos(long long m, long long M, const ConvGeom& g, int& n, int& y, int& x) {
  if (!g.cls) { row_pos(m, M, g, n, y, x); return; }
  if (m < M) {
    const unsigned hx = (unsigned)(g.XO >> 1), plane = (unsigned)(g.YO >> 1) * hx;
    const unsigned mm = (unsigned)m;
    const unsigned q = mm / plane, rem = mm - q * plane;
    const unsigned yy = rem / hx;
    n = (int)q; y = 2 * (int)yy + ((g.cls - 1) >> 1); x = 2 * (int)(rem - yy * hx) + ((g.cls - 1) & 1);
  } else {
    n = 0; y = ROW_ABSENT; x = 0;
  }
}

// stem geometry: element offset in the padded image of the 8 columns at contraction column k for produced row (n, y, x)
__device__ __forceinline__ long long stem_off(const ConvGeom& g, int n, int y, int x, int k) {
  int kh = k >> 5;
  kh = kh > 6 ? 6 : kh;   // the eighth kernel row has zero weights: read the seventh again
  return (((long long)n * g.YS + 2 * y + kh) * g.XS + 2 * x) * 4 + (k & 31);
}

constexpr int CBK = 64;   // channels of one tap per K step

// ---------------------------------------------------------------------------------------------------------------
// forward / input gradient
// ---------------------------------------------------------------------------------------------------------------
// The same contraction with global_load_lds_dwordx4: a wavefront instruction moves 64 x 16 bytes from 64 independent
// global addresses to 1 KB of consecutive LDS (lane l -> bytes 16 l ..), without passing through registers, so three
// K steps of operands are in flight per workgroup at no register cost and the loop waits only for the oldest.
//   * One instruction fills 8 rows x 128 bytes (8 lanes per row).  Rows are unpadded; the 16-byte pieces of a row are
//     stored permuted (piece c of row R sits in slot c ^ ((R >> 1) & 7)), which the loading lane realises by choosing
//     its global address, so that the 16-byte fragment reads of 16 consecutive rows fall on 64 different banks.
//   * A row in the zero padding reads a row of zeros in global memory instead (no branch, every lane loads).
//   * Every wavefront owns a 64 x 64 block of the tile: 256 x 64 tiles (4 x 1 wavefronts) where the output has 64
//     channels, 128 x 128 (2 x 2) otherwise.
__device__ __attribute__((aligned(128))) bf16 g_zero_row[64];

// LDS stages.  Two (64 / 80 KB per workgroup, two workgroups per compute unit, loads one step ahead) measured 22 %
// faster over the ResNet18 step than three (one workgroup per compute unit, loads two steps ahead): the second
// workgroup hides more than the deeper queue.
constexpr int CONV_STAGES = 2;

template <int N>
__device__ __forceinline__ void wait_vm() {   // until at most N vector-memory operations of this wavefront are pending
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0070 | 0x0f00);
}

// The accumulators of a tile (one 64 x 64 block per wavefront) to memory: through LDS in fp32, then whole row segments;
// what is added on the way (the output's old value, the shortcut's gradient) is added to the unrounded sums, so every
// stored element is rounded once; optionally the tile's channel sums for the batch statistics.
template <int BM, int BN>
__device__ __forceinline__ void conv_tile_out(const ConvNT& p, const f32x16 (&acc)[2][2], unsigned char* smem, long long m0,
                                              int n0, int rt, int tid, int lane, int wm, int wn) {
  __syncthreads();   // every operand read is done: the stages become the copy of the tile

  constexpr int CH = BN / 8;
  float ss[8], qq[8];   // this thread's 8 channels (the same in every iteration: 256 % CH == 0) summed over its rows
#pragma unroll
  for (int e = 0; e < 8; ++e) ss[e] = qq[e] = 0.f;
  if (!p.add && !p.extra) {   // uniform: nothing is added on the way, the tile can cross LDS as bf16 (half the LDS traffic)
    constexpr int CLDB = BN + 8;
    bf16* Cb = reinterpret_cast<bf16*>(smem);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int row = wm * 64 + i * 32 + (lane & 31);
          const int col = wn * 64 + j * 32 + q * 8 + (lane >> 5) * 4;
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)acc[i][j][q * 4 + e];
          *reinterpret_cast<bf16x4*>(&Cb[row * CLDB + col]) = v;
        }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < BM * CH / 256; ++it) {
      const int idx = tid + 256 * it;
      const int row = idx / CH, ch = idx - row * CH;
      const long long m = m0 + row;
      if (m < p.M) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(&Cb[row * CLDB + ch * 8]);
        long long orow = m;
        if (p.g.cls) {   // the produced position's row in the full grid
          int n, y, x;
          launch_pos(m, p.M, p.g, n, y, x);
          orow = ((long long)n * p.g.YO + y) * p.g.XO + x;
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {   // the statistics are those of the stored values
          const float lo = __uint_as_float(v[w] << 16), hi = __uint_as_float(v[w] & 0xffff0000u);
          ss[2 * w] += lo; qq[2 * w] += lo * lo;
          ss[2 * w + 1] += hi; qq[2 * w + 1] += hi * hi;
        }
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p.out + orow * p.N + n0 + ch * 8));
      }
    }
  } else {
  constexpr int CLDC = BN + 4;
  float* Cs = reinterpret_cast<float*>(smem);
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = wm * 64 + i * 32 + (lane & 31);
        const int col = wn * 64 + j * 32 + q * 8 + (lane >> 5) * 4;
        *reinterpret_cast<float4*>(&Cs[row * CLDC + col]) =
            make_float4(acc[i][j][q * 4], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]);
      }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < BM * CH / 256; ++it) {
    const int idx = tid + 256 * it;
    const int row = idx / CH, ch = idx - row * CH;
    const long long m = m0 + row;
    if (m < p.M) {
      const float4 lo = *reinterpret_cast<const float4*>(&Cs[row * CLDC + ch * 8]);
      const float4 hi = *reinterpret_cast<const float4*>(&Cs[row * CLDC + ch * 8 + 4]);
      float f[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      long long orow = m;
      if (p.g.cls) {   // the produced position's row in the full grid
        int n, y, x;
        launch_pos(m, p.M, p.g, n, y, x);
        orow = ((long long)n * p.g.YO + y) * p.g.XO + x;
      }
      const long long at = orow * p.N + n0 + ch * 8;
      if (p.add) {
        const u32x4 o = *reinterpret_cast<const u32x4*>(p.out + at);
#pragma unroll
        for (int w = 0; w < 4; ++w) { f[2 * w] += __uint_as_float(o[w] << 16); f[2 * w + 1] += __uint_as_float(o[w] & 0xffff0000u); }
      }
      if (p.extra) {
        const u32x4 x = *reinterpret_cast<const u32x4*>(p.extra + at);
        const unsigned k = p.mask[at >> 3];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          f[2 * w] += (k >> (2 * w)) & 1u ? __uint_as_float(x[w] << 16) : 0.f;
          f[2 * w + 1] += (k >> (2 * w + 1)) & 1u ? __uint_as_float(x[w] & 0xffff0000u) : 0.f;
        }
      }
      bf16x8 t;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        t[e] = (bf16)f[e];
        const float v = (float)t[e];   // the statistics are those of the stored values
        ss[e] += v;
        qq[e] += v * v;
      }
      __builtin_nontemporal_store(t, reinterpret_cast<bf16x8*>(p.out + at));
    }
  }
  }
  if (p.stat_part) {   // uniform
    __syncthreads();   // the tile has been read out
    float* red = reinterpret_cast<float*>(smem);   // [2][256][8]
#pragma unroll
    for (int e = 0; e < 8; ++e) { red[tid * 8 + e] = ss[e]; red[2048 + tid * 8 + e] = qq[e]; }
    __syncthreads();
    if (tid < BN) {   // channel tid of the tile: threads ch + CH j hold its pieces, added in order
      const int ch = tid >> 3, e = tid & 7;
      float a = 0.f, b = 0.f;
      for (int j = 0; j < 256 / CH; ++j) { a += red[(ch + CH * j) * 8 + e]; b += red[2048 + (ch + CH * j) * 8 + e]; }
      p.stat_part[((long long)rt * 2) * p.N + n0 + tid] = a;
      p.stat_part[((long long)rt * 2 + 1) * p.N + n0 + tid] = b;
    }
  }
}

// PW: a pointwise (1x1, stride 1) layer: produced row m reads source row m, so none of the position arithmetic below
// is needed (a tile of such a layer is one to eight K steps long, and what a wavefront spends per tile outside the
// MFMAs -- some 1000 vector instructions in the general form -- is what bounds it)
template <int BM, int BN, int NST, bool STEM, bool PW = false>
__global__ void __launch_bounds__(256) conv_nt_dl_k(ConvNT p, int row_tiles, int col_tiles) {
  constexpr int STAGE = (BM + BN) * CBK;   // bf16 elements per stage
  constexpr int WN = BN / 64, WM = 4 / WN;
  static_assert(WM * 64 == BM && (BN == 64 || BN == 128), "one 64 x 64 block per wavefront");
  constexpr int AG = BM / 32, BG = BN / 32;          // 8-row groups per wavefront and step
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* S = reinterpret_cast<bf16*>(smem);
  // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  Every XCD gets a contiguous range of
  // row tiles and walks it in order, the column tiles of a row tile one after the other: what runs on an XCD at one
  // time are neighbouring row tiles, whose gathered source rows overlap (the taps reach a row of positions up and
  // down), so those rows come from HBM once instead of once per XCD.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per_xcd = (row_tiles + 7) >> 3;
  const int rt = xcd * per_xcd + slot / col_tiles, ct = slot % col_tiles;
  if (slot / col_tiles >= per_xcd || rt >= row_tiles) return;
  const long long m0 = (long long)rt * BM;
  const int n0 = ct * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int lr = lane >> 3, ls = lane & 7;
  const int cpt = p.Cs / CBK;
  const long long ldw = (long long)p.g.KH * p.g.KW * p.Cs;
  // taps of this launch: all, or (parity class) kh = kh0 + 2 i, kw = kw0 + 2 i'
  const int tstep = p.g.cls ? 2 : 1;
  const int kh0 = p.g.cls ? ((((p.g.cls - 1) >> 1) + p.g.pad) & 1) : 0, kw0 = p.g.cls ? ((((p.g.cls - 1) & 1) + p.g.pad) & 1) : 0;
  const int nky = p.g.KH > kh0 ? (p.g.KH - kh0 + tstep - 1) / tstep : 0, nkx = p.g.KW > kw0 ? (p.g.KW - kw0 + tstep - 1) / tstep : 0;
  const int nk = nky * nkx * cpt;

  // Per row of the tile, once: the position, the address of its source row for tap offset zero and which of the
  // launch's taps exist for it.  A K step then costs a mask test and the step's uniform offset per row.
  int pn[AG], py[AG], px[AG], pc[AG];
  const bf16* rb[AG];
  unsigned rm[AG];
  const int sh = p.g.stride >> 1;
#pragma unroll
  for (int j = 0; j < AG; ++j) {
    const int R = (j * 4 + wave) * 8 + lr;
    pc[j] = (ls ^ ((R >> 1) & 7)) * 8;
    if (PW) {
      rb[j] = p.src + (m0 + R) * p.Cs + pc[j];
      rm[j] = m0 + R < p.M ? 1u : 0u;
      continue;
    }
    launch_pos(m0 + R, p.M, p.g, pn[j], py[j], px[j]);
    if (!STEM) {
      const int yb = p.g.transposed ? (py[j] + p.g.pad) >> sh : py[j] * p.g.stride - p.g.pad;
      const int xb = p.g.transposed ? (px[j] + p.g.pad) >> sh : px[j] * p.g.stride - p.g.pad;
      rb[j] = p.src + (((long long)pn[j] * p.g.YS + yb) * p.g.XS + xb) * p.Cs + pc[j];
      unsigned m = 0;
      for (int t = 0; t < nky * nkx; ++t) {
        const int ty = t / nkx;
        m |= (src_row(p.g, pn[j], py[j], px[j], kh0 + tstep * ty, kw0 + tstep * (t - ty * nkx)) >= 0 ? 1u : 0u) << t;
      }
      rm[j] = m;
    }
  }
  const bf16* wb[BG];
#pragma unroll
  for (int j = 0; j < BG; ++j) {
    const int R = (j * 4 + wave) * 8 + lr;
    wb[j] = p.W + (long long)(n0 + R) * ldw + (ls ^ ((R >> 1) & 7)) * 8;
  }
  typedef const void __attribute__((address_space(1)))* gptr_t;
  typedef void __attribute__((address_space(3)))* lptr_t;
  auto issue = [&](int kt, int st) {
    const int tap = kt / cpt, c0 = (kt - tap * cpt) * CBK;
    const int ty = tap / nkx;
    const int kh = kh0 + tstep * ty, kw = kw0 + tstep * (tap - ty * nkx);
    const long long wcol = (long long)(kh * p.g.KW + kw) * p.Cs + c0;   // column of this step in the weight rows
    // the tap's offset from a row's base address (input gradient: taps count backwards, in source steps)
    const long long soff = (p.g.transposed ? -(long long)((kh >> sh) * p.g.XS + (kw >> sh)) : (long long)(kh * p.g.XS + kw)) * p.Cs + c0;
    bf16* sa = S + st * STAGE;
#pragma unroll
    for (int j = 0; j < AG; ++j) {
      const bf16* gp;
      if (STEM) gp = py[j] != ROW_ABSENT ? p.src + stem_off(p.g, pn[j], py[j], px[j], c0 + pc[j]) : g_zero_row + pc[j];
      else gp = (rm[j] >> tap) & 1u ? rb[j] + soff : g_zero_row + pc[j];
      __builtin_amdgcn_global_load_lds((gptr_t)gp, (lptr_t)(sa + (j * 4 + wave) * 8 * CBK), 16, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < BG; ++j)
      __builtin_amdgcn_global_load_lds((gptr_t)(wb[j] + wcol), (lptr_t)(sa + BM * CBK + (j * 4 + wave) * 8 * CBK), 16, 0, 0);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frow = lane & 31, half = lane >> 5;
  // element offsets of this lane's fragment rows inside a stage and their slot permutation
  int offA[2], offB[2], swA[2], swB[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int Ra = wm * 64 + i * 32 + frow, Rb = wn * 64 + i * 32 + frow;
    offA[i] = Ra * CBK; swA[i] = (Ra >> 1) & 7;
    offB[i] = BM * CBK + Rb * CBK; swB[i] = (Rb >> 1) & 7;
  }

  if (nk > 0) issue(0, 0);   // a parity class may have no tap at all (1x1 kernels): its positions get zeros
  if (NST == 3 && nk > 1) issue(1, 1);
  int st = 0;
  for (int kt = 0; kt < nk; ++kt) {
    // this step's operands have landed (with three stages the next step's may be pending)
    if (NST == 3 && kt + 1 < nk) wait_vm<AG + BG>(); else wait_vm<0>();
    // ... for every wavefront, and the stage of step kt - 1 is free (its fragment reads were waited for before the
    // MFMAs that used them).  A bare barrier: the fence of __syncthreads would wait for every pending load.
    __builtin_amdgcn_s_barrier();
    if (NST == 3) { if (kt + 2 < nk) issue(kt + 2, st >= 1 ? st - 1 : 2); }   // (kt + 2) % 3
    else if (kt + 1 < nk) issue(kt + 1, st ^ 1);
    const bf16* sb = S + st * STAGE;
#pragma unroll
    for (int ks = 0; ks < CBK / 16; ++ks) {
      const int c = ks * 2 + half;
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8*>(sb + offA[i] + ((c ^ swA[i]) << 3));
        fb[i] = *reinterpret_cast<const bf16x8*>(sb + offB[i] + ((c ^ swB[i]) << 3));
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    st = st == NST - 1 ? 0 : st + 1;
  }
  conv_tile_out<BM, BN>(p, acc, smem, m0, n0, rt, tid, lane, wm, wn);
}

// ---------------------------------------------------------------------------------------------------------------
// forward / input gradient of 3x3 stride-1 convolutions with the tile's source rows resident in LDS
// ---------------------------------------------------------------------------------------------------------------
// For a 3x3 stride-1 pad-1 convolution (forward, or its input gradient, which is the same correlation with the taps
// mirrored) source and result live on the same grid, and in the flattened row order (n, y, x) the source row of tap
// (dy, dx) for result row m is m + dy * XO + dx wherever it exists.  The nine gathers of the general kernel fetch
// nearly the same rows nine times, and its K loop stops at a barrier every step.  Here
//   * the workgroup loads the window of source rows [m0 - XO - 1, m0 + BM + XO] once (straight into LDS, all
//     channels, pieces slot-permuted as in the general kernel); a tap is an offset into the window when the MFMA
//     fragments are read, and rows whose tap falls outside the image (a neighbouring image row or tile in the flattened
//     order) are zeroed in the fragment by a per-row tap mask;
//   * the weights do not pass through LDS at all: a second copy of the weight matrix is kept in FRAGMENT ORDER (for
//     every block of 32 output channels and 16 contraction columns the 64 lanes' 16-byte operands back to back, see
//     frag_index), so a wavefront's operand is one fully coalesced 1 KB load into registers, fetched two K steps ahead;
//   * so after the window has landed nothing in the K loop is shared between wavefronts: no barrier, every wavefront
//     runs at its own pace.
__host__ __device__ __forceinline__ long long frag_index(int row, int col, int K) {
  return ((((long long)(row >> 5) * (K >> 4) + (col >> 4)) * 64 + (row & 31) + 32 * ((col >> 3) & 1)) << 3) + (col & 7);
}

template <int BM, int BN>
__global__ void __launch_bounds__(256) conv_nt_halo_k(ConvNT p, int row_tiles, int col_tiles, int wrows) {
  constexpr int WN = BN / 64, WM = 4 / WN;
  static_assert(WM * 64 == BM && (BN == 64 || BN == 128), "one 64 x 64 block per wavefront");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* Wd = reinterpret_cast<bf16*>(smem);          // window [wrows][Cs]
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int per_xcd = (row_tiles + 7) >> 3;
  const int rt = xcd * per_xcd + slot / col_tiles, ct = slot % col_tiles;
  if (slot / col_tiles >= per_xcd || rt >= row_tiles) return;
  const long long m0 = (long long)rt * BM;
  const int n0 = ct * BN;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int cpt = p.Cs / CBK, cpr = p.Cs >> 3;       // K steps per tap, 16-byte pieces per row
  const int nk = 9 * cpt;                            // a multiple of 3
  const int halo = p.g.XO + 1;
  const int sg = p.g.transposed ? -1 : 1;
  typedef const void __attribute__((address_space(1)))* gptr_t;
  typedef void __attribute__((address_space(3)))* lptr_t;

  // the window: instruction q of this wavefront fills pieces [(q * 4 + wave) * 64, + 64) in row-major order
  const int ninst = wrows * cpr / 256;
  for (int q = 0; q < ninst; ++q) {
    const int gidx = (q * 4 + wave) * 64 + lane;
    const int j = gidx / cpr, sl = gidx - j * cpr;
    const int piece = (sl & ~7) | ((sl ^ (j >> 1)) & 7);
    const long long f = m0 - halo + j;
    const bool ok = (f >= 0) & (f < p.M) & (j < BM + 2 * halo);
    const bf16* gp = ok ? p.src + f * p.Cs + piece * 8 : g_zero_row + (piece & 7) * 8;
    __builtin_amdgcn_global_load_lds((gptr_t)gp, (lptr_t)(Wd + (long long)(q * 4 + wave) * 64 * 8), 16, 0, 0);
  }

  // weights: operand (j, ks) of K step kt is the 1 KB at slice (block of 32 channels, 16 columns) of the fragment-order copy
  const long long kslices = 9LL * p.Cs / 16;
  const bf16* wf[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) wf[j] = p.Wf + ((long long)((n0 + wn * 64 + j * 32) >> 5) * kslices * 64 + lane) * 8;
  bf16x8 breg[3][2][4];
  auto fetch_w = [&](auto sc, int kt) __attribute__((always_inline)) {
    constexpr int S = decltype(sc)::value;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        breg[S][j][ks] = *reinterpret_cast<const bf16x8*>(wf[j] + ((long long)kt * 4 + ks) * 512);
  };
  fetch_w(std::integral_constant<int, 0>{}, 0);
  fetch_w(std::integral_constant<int, 1>{}, 1);

  // this lane's two fragment rows: window row of the centre tap, and which taps exist for them
  const int frow = lane & 31, half = lane >> 5;
  int wr0[2];
  unsigned vm[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int R = wm * 64 + i * 32 + frow;
    wr0[i] = R + halo;
    int n, y, x;
    row_pos(m0 + R, p.M, p.g, n, y, x);
    unsigned m = 0;
#pragma unroll
    for (int t = 0; t < 9; ++t) m |= (src_row(p.g, n, y, x, t / 3, t % 3) >= 0 ? 1u : 0u) << t;
    vm[i] = m;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  wait_vm<0>();        // the window has landed (and the first weight operands) ...
  __syncthreads();     // ... for every wavefront.  From here on the window is only read.

  auto step = [&](auto sc, int kt) __attribute__((always_inline)) {
    constexpr int S = decltype(sc)::value;
    if (kt + 2 < nk) fetch_w(std::integral_constant<int, (S + 2) % 3>{}, kt + 2);
    const int tap = kt / cpt, cc = kt - tap * cpt;
    const int th = tap / 3;
    const int shift = sg * ((th - 1) * p.g.XO + (tap - th * 3 - 1));
    const bf16* sa[2];
    int sw[2];
    bool on[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      sa[i] = Wd + (long long)(wr0[i] + shift) * p.Cs + cc * CBK;
      sw[i] = ((wr0[i] + shift) >> 1) & 7;
      on[i] = (vm[i] >> tap) & 1u;
    }
#pragma unroll
    for (int ks = 0; ks < CBK / 16; ++ks) {
      const int c = ks * 2 + half;
      bf16x8 fa[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8*>(sa[i] + ((c ^ sw[i]) << 3));
        if (!on[i]) {
#pragma unroll
          for (int e = 0; e < 8; ++e) fa[i][e] = (bf16)0.f;
        }
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(breg[S][j][ks], fa[i], acc[i][j], 0, 0, 0);
    }
  };
  for (int kt = 0; kt < nk; kt += 3) {
    step(std::integral_constant<int, 0>{}, kt);
    step(std::integral_constant<int, 1>{}, kt + 1);
    step(std::integral_constant<int, 2>{}, kt + 2);
  }
  conv_tile_out<BM, BN>(p, acc, smem, m0, n0, rt, tid, lane, wm, wn);
}

// ---------------------------------------------------------------------------------------------------------------
// stem forward with the tile's window of the padded image resident in LDS
// ---------------------------------------------------------------------------------------------------------------
// The stem's contraction column k = kh * 32 + kw * 4 + c is 8 pixels of image row 2 y + kh from pixel 2 x on: the
// kernel rows of neighbouring positions overlap almost entirely.  Gathered per position (the general kernel) a tile of
// 256 positions pulls 128 KB of operand and 32 KB of weights through the compute unit's L1, which is what bounds it.
// Here a persistent workgroup keeps the 64 x 224 weights in LDS for its whole life (the eighth kernel row, all zero,
// is not multiplied at all), and a tile's operand is the contiguous block of image rows 2 y0 .. 2 y_last + 6 (24 KB
// for 256 positions of a 112 x 112 grid): copied straight into LDS once, fragments read from it at
// (2 (y - y0) + kh) rows + 2 x pixels.  No barrier in the K loop.  The window shares its LDS with the copy of the
// finished tile, so two workgroups fit a compute unit (with the weights in registers, 112 of them, only one did, and
// nothing covered its write-out: 3.3 ms per launch against 4.0 for the general kernel); one works while the other
// waits for its next window.
// Needs: positions per image a multiple of 256 (tiles never straddle images), 64 output channels.
constexpr int STEM_KS = 14;                       // 16-wide slices of the contraction that carry weights
constexpr int STEM_WPT = 6;                       // 16-byte pieces of the window per thread
constexpr int STEM_WIN = STEM_WPT * 256 * 16;     // window buffer: 24 KB
constexpr int STEM_OUTB = 256 * (64 + 8) * 2;     // conv_tile_out's copy of the tile (bf16 path) / its statistics
constexpr int STEM_WROW = STEM_KS * 32 + 16;      // bytes per weight row in LDS: 464 (16 rows x 16 bytes cover all banks)
constexpr int STEM_LDS = STEM_OUTB + 64 * STEM_WROW;
static_assert(STEM_WIN <= STEM_OUTB, "the window lies inside the region of the tile's copy");

__global__ void __launch_bounds__(256, 2) stem_fwd_k(ConvNT p, int tiles, int wbytes, long long img_bytes) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* const win = smem;                  // dead when the tile's copy takes its place
  unsigned char* const wsm = smem + STEM_OUTB;      // weights [64][STEM_WROW]
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int li = lane & 31, h2 = lane >> 5;
  const int XO = p.g.XO, plane = p.g.YO * p.g.XO, XS = p.g.XS, YS = p.g.YS;
  const int rowB = XS * 8;   // bytes of an image row (4 channels)
  int t = blockIdx.x;
  if (t >= tiles) return;

  for (int idx = tid; idx < 64 * STEM_KS * 2; idx += 256) {   // 16-byte pieces of the 64 x 224 weights
    const int row = idx / (STEM_KS * 2), pc = idx - row * (STEM_KS * 2);
    *reinterpret_cast<u32x4*>(wsm + row * STEM_WROW + pc * 16) = ldg16(p.W + (long long)row * 256 + pc * 8);
  }
  const unsigned char* const wl = wsm + li * STEM_WROW + h2 * 16;   // this lane's row of column block 0

  // the window of tile tt, straight into LDS (a wavefront instruction copies 1 KB): wbytes from image row 2 y0 of its
  // image on; pieces past the end of the whole image buffer (only ever the unused tail of the last tiles' windows)
  // read its last piece instead
  typedef const void __attribute__((address_space(1)))* gptr_t;
  typedef void __attribute__((address_space(3)))* lptr_t;
  auto fetch = [&](int tt) __attribute__((always_inline)) {
    const int m0 = tt * 256, n = m0 / plane, y0 = (m0 - n * plane) / XO;
    const long long woff = ((long long)(n * YS + 2 * y0) * XS) * 8;
    const char* src = reinterpret_cast<const char*>(p.src);
#pragma unroll
    for (int i = 0; i < STEM_WPT; ++i) {
      const int c = i * 4 + wave;   // 1 KB chunk of the window
      if (c * 1024 < wbytes) {      // uniform
        long long o = woff + c * 1024 + lane * 16;
        o = o > img_bytes - 16 ? img_bytes - 16 : o;
        __builtin_amdgcn_global_load_lds((gptr_t)(src + o), (lptr_t)(win + c * 1024), 16, 0, 0);
      }
    }
  };
  fetch(t);
  __syncthreads();   // (waits for the wavefront's own loads, then for the others)
  while (true) {
    const int nt = t + (int)gridDim.x;
    const bool more = nt < tiles;   // uniform
    const int m0 = t * 256, n = m0 / plane, p0 = m0 - n * plane, y0 = p0 / XO;
    int ab[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int pp = p0 + wave * 64 + i * 32 + li;
      const int y = pp / XO, x = pp - y * XO;
      ab[i] = (2 * (y - y0) * XS + 2 * x) * 8 + 16 * h2;
    }
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
#pragma unroll
    for (int s = 0; s < STEM_KS; ++s) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(win + ab[i] + (s >> 1) * rowB + (s & 1) * 32);
#pragma unroll
      for (int j = 0; j < 2; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(wl + j * 32 * STEM_WROW + s * 32);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    // (starts with a barrier: every wavefront is done with the window before the tile's copy overwrites it)
    conv_tile_out<256, 64>(p, acc, smem, (long long)m0, 0, t, tid, lane, wave, 0);
    if (!more) break;
    __syncthreads();   // the copy and the statistics have been read out
    fetch(nt);
    __syncthreads();   // (waits for the wavefront's own loads, then for the others)
    t = nt;
  }
}

// ---------------------------------------------------------------------------------------------------------------
// weight gradient
// ---------------------------------------------------------------------------------------------------------------
constexpr int WBK = 32;   // rows per step

// Operands go straight into LDS here too.  A stage holds 1 + TAPS slices of [32 rows][64 channels] (128-byte rows,
// unpadded): slice 0 the output-gradient rows, slice 1 + t the source rows of tap t.  A wavefront instruction fills 8
// rows of one slice; wavefront w always takes rows 8 w .. 8 w + 7, of every slice, so a lane resolves one row position
// per step.  The 16-byte pieces of rows 2, 3, 6, 7, ... sit in the other 64-byte half of the row (slot = piece ^ 4):
// a transpose read's two 16-lane groups that are served together touch 4 rows x 64 bytes, which then fall on four
// different quarters of the banks.
//
// MFMA operand from slice B (row-major, 64 elements per row): lane l gets column c0 + l % 32 and the contraction
// indices k0 + 8 * (l / 32) + {0..7}.  A transpose read's group of 16 lanes addresses a 4-row x 16-column patch and
// every lane receives one column of it.
__device__ __forceinline__ bf16x8 frag_tr_dl(const bf16* B, int c0, int k0, int lane) {
  const int g = lane >> 4, q = lane & 15;
  const int k = k0 + 8 * (g >> 1) + (q >> 2), col = c0 + 16 * (g & 1) + (q & 3) * 4;
  const bf16* p = B + k * 64 + ((((col >> 3) ^ (((k >> 1) & 1) << 2)) << 3) | (col & 7));
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * 64));   // row k + 4: same half
  s16x8 r = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  return __builtin_bit_cast(bf16x8, r);
}

// PW: a pointwise (1x1, stride 1) layer: the source row of output row m is row m (no position arithmetic per step)
template <int TAPS, bool STEM, bool PW = false>
__global__ void __launch_bounds__(256) conv_wgrad_k(ConvWG p) {
  constexpr int SL = 1 + TAPS, SLICE = WBK * 64, STAGE = SL * SLICE;   // bf16 elements
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* S = reinterpret_cast<bf16*>(smem);   // [2][SL][32][64]
  // Workgroup ids go round-robin to the 8 XCDs: all (c_out, c_in) blocks of one slab get ids of one XCD, one after the
  // other, so the slab's rows are fetched into that XCD's L2 once and not once per XCD that holds one of the blocks.
  const int nco = p.Co >> 6, nci = p.Cs >> 6, pairs = nco * nci;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int slab = (slot / pairs) * 8 + xcd, pair = slot % pairs;
  if (slab >= p.slabs) return;
  const int co0 = (pair % nco) * 64, ci0 = (pair / nco) * 64;
  const long long lo = (long long)slab * p.per;
  const long long hi = lo + p.per < p.M ? lo + p.per : p.M;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qa = wave >> 1, qb = wave & 1;
  const int r = wave * 8 + (lane >> 3);                          // this lane's row of every slice
  const int cl = ((lane & 7) ^ (((r >> 1) & 1) << 2)) * 8;       // the piece it fetches (its slot holds piece slot ^ ...)
  typedef const void __attribute__((address_space(1)))* gptr_t;
  typedef void __attribute__((address_space(3)))* lptr_t;

  auto issue = [&](long long mstep, int st) {   // only called with mstep < hi
    const long long m = mstep + r;
    const bool ok = m < hi;
    bf16* sa = S + st * STAGE + wave * 8 * 64;
    const bf16* gd = ok ? p.dout + m * p.Co + co0 + cl : g_zero_row + cl;
    __builtin_amdgcn_global_load_lds((gptr_t)gd, (lptr_t)sa, 16, 0, 0);
    if (PW) {
      const bf16* gp = ok ? p.src + m * p.Cs + ci0 + cl : g_zero_row + cl;
      __builtin_amdgcn_global_load_lds((gptr_t)gp, (lptr_t)(sa + SLICE), 16, 0, 0);
      return;
    }
    int n, y, x;
    row_pos(ok ? m : hi - 1, p.M, p.g, n, y, x);
    if (STEM) {   // the four 64-column groups of the stem's 256 contraction columns stand where the taps stand
#pragma unroll
      for (int t = 0; t < TAPS; ++t) {
        const bf16* gp = ok ? p.src + stem_off(p.g, n, y, x, t * 64 + cl) : g_zero_row + cl;
        __builtin_amdgcn_global_load_lds((gptr_t)gp, (lptr_t)(sa + (1 + t) * SLICE), 16, 0, 0);
      }
    } else {
      // the row's source position for tap (0, 0), once; a tap adds a uniform offset, and exists where both of its
      // coordinates fall inside the source grid
      const int ys0 = y * p.g.stride - p.g.pad, xs0 = x * p.g.stride - p.g.pad;
      const bf16* base = p.src + (((long long)n * p.g.YS + ys0) * p.g.XS + xs0) * p.Cs + ci0 + cl;
      bool oky[3], okx[3];
#pragma unroll
      for (int k = 0; k < 3; ++k) {
        oky[k] = ok & ((unsigned)(ys0 + k) < (unsigned)p.g.YS);
        okx[k] = (unsigned)(xs0 + k) < (unsigned)p.g.XS;
      }
#pragma unroll
      for (int t = 0; t < TAPS; ++t) {
        const int kh = TAPS == 1 ? 0 : t / 3, kw = TAPS == 1 ? 0 : t % 3;
        const bf16* gp = (oky[kh] & okx[kw]) ? base + (long long)(kh * p.g.XS + kw) * p.Cs : g_zero_row + cl;
        __builtin_amdgcn_global_load_lds((gptr_t)gp, (lptr_t)(sa + (1 + t) * SLICE), 16, 0, 0);
      }
    }
  };

  f32x16 acc[TAPS];
#pragma unroll
  for (int t = 0; t < TAPS; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  if (lo < hi) issue(lo, 0);
  int st = 0;
  for (long long mstep = lo; mstep < hi; mstep += WBK) {
    wait_vm<0>();                     // this step's rows have landed ...
    __builtin_amdgcn_s_barrier();     // ... for every wavefront, and the other stage is no longer read
    if (mstep + WBK < hi) issue(mstep + WBK, st ^ 1);
    const bf16* sb = S + st * STAGE;
#pragma unroll
    for (int kk = 0; kk < WBK; kk += 16) {
      const bf16x8 fa = frag_tr_dl(sb, qa * 32, kk, lane);
#pragma unroll
      for (int t = 0; t < TAPS; ++t) {
        const bf16x8 fb = frag_tr_dl(sb + (1 + t) * SLICE, qb * 32, kk, lane);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc[t], 0, 0, 0);
      }
    }
    st ^= 1;
  }
  // block rows = output channels (r / 4) * 8 + (l / 32) * 4 + r % 4, block columns = input channels l % 32.  A slab
  // without rows still writes its zeros: the reduction adds every slab.
  const long long ldk = (long long)TAPS * p.Cs;
  float* P = p.part + (long long)slab * p.Co * ldk;
#pragma unroll
  for (int t = 0; t < TAPS; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int co = co0 + qa * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
      P[(long long)co * ldk + (long long)t * p.Cs + ci0 + qb * 32 + (lane & 31)] = acc[t][e];
    }
}

// Weight gradient of the pointwise (1x1, stride 1) layers.  With 64 x 64 blocks a step of 32 rows is two MFMAs per
// wavefront between two barriers, and the Co / 64 x Cs / 64 workgroups of a slab each fetch their operands' slices
// again.  Here a workgroup owns BO x BI = 128 x 128, 256 x 64 or 64 x 256 of (c_out, c_in), a wavefront 64 x 64 of it
// (eight MFMAs per step), the source row of output row m is row m, three stages in separate LDS arrays, loads two
// steps ahead.
template <int BO, int BI>
__global__ void __launch_bounds__(256, 2) conv_wgrad_pw_k(ConvWG p) {
  constexpr int SA = BO / 64, SB = BI / 64, SL = SA + SB, SLICE = WBK * 64, STAGE = SL * SLICE;   // bf16 elements
  constexpr int WI = SB >= 4 ? 4 : SB >= 2 ? 2 : 1;   // wavefronts along c_in, the others along c_out
  static_assert(SA * SB == 4, "four 64 x 64 blocks, one per wavefront");
  __shared__ __attribute__((aligned(128))) bf16 sg0[STAGE];
  __shared__ __attribute__((aligned(128))) bf16 sg1[STAGE];
  __shared__ __attribute__((aligned(128))) bf16 sg2[STAGE];
  const int nco = p.Co / BO, nci = p.Cs / BI, pairs = nco * nci;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int slab = (slot / pairs) * 8 + xcd, pair = slot % pairs;
  if (slab >= p.slabs) return;
  const int co0 = (pair % nco) * BO, ci0 = (pair / nco) * BI;
  const long long lo = (long long)slab * p.per;
  const long long hi = lo + p.per < p.M ? lo + p.per : p.M;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave % WI, wo = wave / WI;
  const int r = wave * 8 + (lane >> 3);                          // this lane's row of every slice
  const int cl = ((lane & 7) ^ (((r >> 1) & 1) << 2)) * 8;       // the piece it fetches (its slot holds piece slot ^ ...)
  typedef const void __attribute__((address_space(1)))* gptr_t;
  typedef void __attribute__((address_space(3)))* lptr_t;

  auto issue = [&](long long mstep, auto stc) __attribute__((always_inline)) {   // only called with mstep < hi
    constexpr int ST = decltype(stc)::value;
    bf16* sa = (ST == 0 ? sg0 : ST == 1 ? sg1 : sg2) + wave * 8 * 64;
    const long long m = mstep + r;
    const bool ok = m < hi;
    const bf16* gd = ok ? p.dout + m * p.Co + co0 + cl : g_zero_row + cl;
    const bf16* gs = ok ? p.src + m * p.Cs + ci0 + cl : g_zero_row + cl;
    const int so = ok ? 64 : 0;   // the zero row has one slice
#pragma unroll
    for (int sl = 0; sl < SA; ++sl) __builtin_amdgcn_global_load_lds((gptr_t)(gd + sl * so), (lptr_t)(sa + sl * SLICE), 16, 0, 0);
#pragma unroll
    for (int sl = 0; sl < SB; ++sl) __builtin_amdgcn_global_load_lds((gptr_t)(gs + sl * so), (lptr_t)(sa + (SA + sl) * SLICE), 16, 0, 0);
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  if (lo < hi) issue(lo, std::integral_constant<int, 0>{});
  if (lo + WBK < hi) issue(lo + WBK, std::integral_constant<int, 1>{});
  auto step = [&](long long mstep, auto stc) __attribute__((always_inline)) {
    constexpr int ST = decltype(stc)::value;
    // this step's rows have landed (the next step's SL requests may be pending) ...
    if (mstep + WBK < hi) wait_vm<SL>(); else wait_vm<0>();
    __builtin_amdgcn_s_barrier();     // ... for every wavefront, and the stage of the previous step is no longer read
    if (mstep + 2 * WBK < hi) issue(mstep + 2 * WBK, std::integral_constant<int, (ST + 2) % 3>{});
    const bf16* sb = ST == 0 ? sg0 : ST == 1 ? sg1 : sg2;
#pragma unroll
    for (int kk = 0; kk < WBK; kk += 16) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int a = 0; a < 2; ++a) fa[a] = frag_tr_dl(sb + wo * SLICE, a * 32, kk, lane);
#pragma unroll
      for (int b = 0; b < 2; ++b) fb[b] = frag_tr_dl(sb + (SA + wi) * SLICE, b * 32, kk, lane);
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
    }
  };
  for (long long mstep = lo; mstep < hi; mstep += 3 * WBK) {
    step(mstep, std::integral_constant<int, 0>{});
    if (mstep + WBK < hi) step(mstep + WBK, std::integral_constant<int, 1>{});
    if (mstep + 2 * WBK < hi) step(mstep + 2 * WBK, std::integral_constant<int, 2>{});
  }
  // block rows = output channels (e / 4) * 8 + (l / 32) * 4 + e % 4, block columns = input channels l % 32.  A slab
  // without rows still writes its zeros: the reduction adds every slab.
  const long long ldk = p.Cs;
  float* P = p.part + (long long)slab * p.Co * ldk;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int co = co0 + wo * 64 + a * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        P[(long long)co * ldk + ci0 + wi * 64 + b * 32 + (lane & 31)] = acc[a][b][e];
      }
}

// Weight gradient of the 3x3 stride-1 pad-1 layers with the step's source rows fetched once.  In the flattened row
// order (n, y, x) the source row of tap (kh, kw) for output row m is m + (kh - 1) XO + (kw - 1) wherever it exists,
// so the nine slices the kernel above gathers for a step of 32 rows are three bands of consecutive rows, one per
// kh: 19 KB per step and stage instead of 40 KB, which is what that kernel is bound by (the compute unit's L1 fills
// at about 30 bytes per clock; a step is 580 clocks of MFMA).
// Where a tap leaves the image the flattened neighbour is a wrong row, and the contraction index IS the row, so such
// products must vanish element by element.  They do so by construction of the band in LDS:
//   * a band is stored in padded coordinates: after the last position of every image row comes one row of zeros, so
//     the left neighbour of x = 0 and the right neighbour of x = XO - 1 are that row.  Output row k of the step
//     (x0 + k positions after the step's first row at column x0) reads band row k + wraps(k) + kw,
//     wraps(k) = (x0 + k) / XO; the transpose read takes a row address per lane, so the uneven spacing costs nothing;
//   * a source row whose output row would need an image row above the first or below the last (kh = 0 with y = 0,
//     kh = 2 with y = YO - 1; also the neighbouring image in the flattened order) is fetched as zeros: within band
//     kh every source row serves output rows of one image row only.
// The loading lane decides per band row what to fetch (row, gap, or zeros); the K loop has no masks.  Needs XO >= 8.
// The stages being half the size, four of them fit (two workgroups per compute unit): a step's rows are requested three
// steps ahead.  With one step of lead a step cannot be shorter than a memory latency, which, not the bytes, is what
// the two-stage kernels of this file wait for (measured: the halved traffic alone changed nothing).
constexpr int WBAND = 40;   // band rows per step: 32 + 2 neighbours + at most 4 gap rows, rounded to the 8 of an instruction
constexpr int WSTAGES = 4;

__global__ void __launch_bounds__(256, 2) conv_wgrad_win_k(ConvWG p) {
  constexpr int DOUT = WBK * 64, BAND = WBAND * 64, STAGE = DOUT + 3 * BAND;   // bf16 elements
  // one array per stage: the compiler waits for every load in flight into an LDS array before it reads that array,
  // so stages that share an array cannot have loads pending while another stage is read
  __shared__ __attribute__((aligned(128))) bf16 sg0[STAGE];
  __shared__ __attribute__((aligned(128))) bf16 sg1[STAGE];
  __shared__ __attribute__((aligned(128))) bf16 sg2[STAGE];
  __shared__ __attribute__((aligned(128))) bf16 sg3[STAGE];
  static_assert(WSTAGES == 4, "four stage arrays");
  const int nco = p.Co >> 6, nci = p.Cs >> 6, pairs = nco * nci;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int slab = (slot / pairs) * 8 + xcd, pair = slot % pairs;
  if (slab >= p.slabs) return;
  const int co0 = (pair % nco) * 64, ci0 = (pair / nco) * 64;
  const long long lo = (long long)slab * p.per;
  const long long hi = lo + p.per < p.M ? lo + p.per : p.M;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int qa = wave >> 1, qb = wave & 1;
  const int XO = p.g.XO, YO = p.g.YO, P1 = XO + 1;
  const float invP1 = 1.0f / (float)P1, invXO = 1.0f / (float)XO;
  typedef const void __attribute__((address_space(1)))* gptr_t;
  typedef void __attribute__((address_space(3)))* lptr_t;

  // (y0, x0): position of row mstep
  // Load instructions of a step (1 KB each): wavefront w takes rows 8 w .. of the output gradient, band rows 8 w .. of
  // all three bands (what decides a band row -- gap, image row, source row -- is the same in the three, only the
  // image-row test and the base differ) and, w < 3, band rows 32 .. 39 of band w: five instructions (wavefront 3: four).
  const int lr = lane >> 3;
  const int rA = wave * 8 + lr, rB = 32 + lr;                       // band rows of the two row groups of this lane
  const int clA = ((lane & 7) ^ (((rA >> 1) & 1) << 2)) * 8, clB = ((lane & 7) ^ (((rB >> 1) & 1) << 2)) * 8;
  auto issue = [&](long long mstep, auto stc, int y0, int x0) __attribute__((always_inline)) {   // only called with mstep < hi
    constexpr int ST = decltype(stc)::value;
    bf16* sa = ST == 0 ? sg0 : ST == 1 ? sg1 : ST == 2 ? sg2 : sg3;
    {
      const long long m = mstep + rA;   // (rA is also this lane's output-gradient row)
      const bf16* gp = m < hi ? p.dout + m * p.Co + co0 + clA : g_zero_row + clA;
      __builtin_amdgcn_global_load_lds((gptr_t)gp, (lptr_t)(sa + wave * 8 * 64), 16, 0, 0);
    }
    // band row r of band b: padded column (one padded image row ahead so that it is not negative), image rows after
    // the step's first one (-1 only for a gap), source row relative to the row in the column of row mstep
    auto band_row = [&](int r, int cl, auto bc) __attribute__((always_inline)) {
      const int up = x0 + r - 1 + P1;
      const int wq = (int)(((float)up + 0.5f) * invP1);   // exact: up < 200, the half keeps multiples of P1 off the edge
      const int rem = up - wq * P1, w = wq - 1;
      int yo = y0 + w;
      yo = yo >= YO ? yo - YO : yo;                        // the image row of the output rows this source row serves
      const bool okx = rem != XO;
      const int rel = r - 1 - w;
      auto one = [&](int b, bf16* dst) __attribute__((always_inline)) {
        const long long f = mstep + (long long)((b - 1) * XO + rel);
        const bool ok = okx & ((unsigned)(yo + b - 1) < (unsigned)YO) & (f >= 0) & (f < p.M);
        const bf16* gp = ok ? p.src + f * p.Cs + ci0 + cl : g_zero_row + cl;
        __builtin_amdgcn_global_load_lds((gptr_t)gp, (lptr_t)dst, 16, 0, 0);
      };
      constexpr int B = decltype(bc)::value;
      if constexpr (B < 0) {
#pragma unroll
        for (int b = 0; b < 3; ++b) one(b, sa + DOUT + b * BAND + wave * 8 * 64);
      } else {
        one(wave, sa + DOUT + wave * BAND + 4 * 8 * 64);
      }
    };
    band_row(rA, clA, std::integral_constant<int, -1>{});
    if (wave < 3) band_row(rB, clB, std::integral_constant<int, 0>{});
  };

  f32x16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  // positions (wave-uniform) of the step being worked on and of the one being fetched
  int cy, cx, iy, ix;
  {
    int n;
    row_pos(lo < p.M ? lo : p.M - 1, p.M, p.g, n, cy, cx);
    iy = cy; ix = cx;
  }
  auto adv32 = [&](int& y, int& x) __attribute__((always_inline)) {
    x += WBK;
    while (x >= XO) { x -= XO; y = y + 1 == YO ? 0 : y + 1; }
  };
  // this lane's contraction rows in a transpose read: k = kk + 8 (g / 2) + s / 4 (+ 4 for the second read of a pair)
  const int g16 = lane >> 4, s16 = lane & 15;
  const int kl = 8 * (g16 >> 1) + (s16 >> 2);
  const int col = qb * 32 + 16 * (g16 & 1) + (s16 & 3) * 4, cb = col >> 3, c7 = col & 7;
  const int swz0 = (cb << 3) + c7, swz1 = ((cb ^ 4) << 3) + c7;

  // the first WSTAGES - 1 steps are requested up front; step s then requests step s + WSTAGES - 1 into the stage that
  // step s - 1 has just left
  if (lo < hi) { issue(lo, std::integral_constant<int, 0>{}, iy, ix); adv32(iy, ix); }
  if (lo + WBK < hi) { issue(lo + WBK, std::integral_constant<int, 1>{}, iy, ix); adv32(iy, ix); }
  if (lo + 2 * WBK < hi) { issue(lo + 2 * WBK, std::integral_constant<int, 2>{}, iy, ix); adv32(iy, ix); }
  auto step = [&](long long mstep, auto stc) __attribute__((always_inline)) {
    constexpr int ST = decltype(stc)::value;
    // this step's rows have landed: at most the requests of the later steps are pending (waves 0..2 issue five
    // instructions per step, wave 3 four) ...
    const long long later = (hi - mstep - 1) / WBK;   // steps after this one
    if (later >= WSTAGES - 2) { if (wave < 3) wait_vm<10>(); else wait_vm<8>(); }
    else if (later == 1) { if (wave < 3) wait_vm<5>(); else wait_vm<4>(); }
    else wait_vm<0>();
    __builtin_amdgcn_s_barrier();     // ... for every wavefront, and the stage of the previous step is no longer read
    if (mstep + (WSTAGES - 1) * WBK < hi) {
      issue(mstep + (WSTAGES - 1) * WBK, std::integral_constant<int, (ST + WSTAGES - 1) % WSTAGES>{}, iy, ix);
      adv32(iy, ix);
    }
    const bf16* sb = ST == 0 ? sg0 : ST == 1 ? sg1 : ST == 2 ? sg2 : sg3;
    // element offsets inside a band of the rows this lane addresses, per (kk, read of the pair) and kw
    int off[4][3];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int k = (a >> 1) * 16 + (a & 1) * 4 + kl;
      const int jb = k + (int)(((float)(cx + k) + 0.5f) * invXO);
#pragma unroll
      for (int kw = 0; kw < 3; ++kw) {
        const int j = jb + kw;
        off[a][kw] = j * 64 + ((j & 2) ? swz1 : swz0);   // rows 2, 3, 6, 7, ... hold their pieces in the other half
      }
    }
    adv32(cy, cx);
#pragma unroll
    for (int kk = 0; kk < WBK; kk += 16) {
      const bf16x8 fa = frag_tr_dl(sb, qa * 32, kk, lane);
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int kh = t / 3, kw = t % 3;
        const bf16* bp = sb + DOUT + kh * BAND;
        s16x4 u0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(bp + off[(kk >> 4) * 2][kw]));
        s16x4 u1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(bp + off[(kk >> 4) * 2 + 1][kw]));
        s16x8 r8 = {u0[0], u0[1], u0[2], u0[3], u1[0], u1[1], u1[2], u1[3]};
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, __builtin_bit_cast(bf16x8, r8), acc[t], 0, 0, 0);
      }
    }
  };
  for (long long mstep = lo; mstep < hi; mstep += WSTAGES * WBK) {
    step(mstep, std::integral_constant<int, 0>{});
    if (mstep + WBK < hi) step(mstep + WBK, std::integral_constant<int, 1>{});
    if (mstep + 2 * WBK < hi) step(mstep + 2 * WBK, std::integral_constant<int, 2>{});
    if (mstep + 3 * WBK < hi) step(mstep + 3 * WBK, std::integral_constant<int, 3>{});
  }
  const long long ldk = 9LL * p.Cs;
  float* P = p.part + (long long)slab * p.Co * ldk;
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int co = co0 + qa * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
      P[(long long)co * ldk + (long long)t * p.Cs + ci0 + qb * 32 + (lane & 31)] = acc[t][e];
    }
}

__global__ void __launch_bounds__(256) wgrad_reduce_k(const float* __restrict__ part, int slabs, int Co, int Cin, int taps,
                                                       int ldk, float* __restrict__ dW, int accumulate) {
  const int K = taps * Cin;
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)Co * K) return;
  const int co = (int)(i / K), col = (int)(i - (long long)co * K);
  const int tap = col / Cin, ci = col - tap * Cin;
  // eight independent running sums (slab s goes to sum s % 8), combined in a fixed order: the loads of eight slabs are
  // in flight together and the result is still the same bits on every run
  float a8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const long long st = (long long)Co * ldk;
  const float* pp = part + (long long)co * ldk + col;
  int s = 0;
  for (; s + 8 <= slabs; s += 8) {
#pragma unroll
    for (int u = 0; u < 8; ++u) a8[u] += pp[(s + u) * st];
  }
  for (; s < slabs; ++s) a8[s & 7] += pp[s * st];
  const float a = ((a8[0] + a8[1]) + (a8[2] + a8[3])) + ((a8[4] + a8[5]) + (a8[6] + a8[7]));
  const long long o = ((long long)co * Cin + ci) * taps + tap;
  dW[o] = accumulate ? dW[o] + a : a;
}

__global__ void __launch_bounds__(256) conv_cast_w_k(const float* __restrict__ W, int Co, int Cin, int taps, int ldk,
                                                      bf16* __restrict__ Wk, bf16* __restrict__ Wt, bf16* __restrict__ Wf,
                                                      bf16* __restrict__ Wtf) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long long)Co * ldk) return;
  const int co = (int)(i / ldk), col = (int)(i - (long long)co * ldk);
  float v = 0.f;
  if (col < taps * Cin) {
    const int tap = col / Cin, ci = col - tap * Cin;
    v = W[((long long)co * Cin + ci) * taps + tap];
    if (Wt) Wt[(long long)ci * taps * Co + (long long)tap * Co + co] = (bf16)v;
    if (Wf) Wf[frag_index(co, col, taps * Cin)] = (bf16)v;
    if (Wtf) Wtf[frag_index(ci, tap * Co + co, taps * Co)] = (bf16)v;
  }
  Wk[i] = (bf16)v;
}

// one thread per pixel of the padded image
__global__ void __launch_bounds__(256) stem_pad_pixels_k(const bf16* __restrict__ px, bf16* __restrict__ img, long long total,
                                                          int S) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= total) return;
  const int XS = S + 8, YS = S + 6;
  const int x = (int)(i % XS);
  const long long t = i / XS;
  const int y = (int)(t % YS);
  const long long n = t / YS;
  const int iy = y - 3, ix = x - 3;
  bf16x4 v = {(bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f};
  if ((unsigned)iy < (unsigned)S && (unsigned)ix < (unsigned)S) {
#pragma unroll
    for (int ch = 0; ch < 3; ++ch) v[ch] = px[((n * 3 + ch) * S + iy) * S + ix];
  }
  *reinterpret_cast<bf16x4*>(img + i * 4) = v;
}

__global__ void __launch_bounds__(256) stem_cast_w_k(const float* __restrict__ W, int Co, bf16* __restrict__ Wk) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= Co * 256) return;
  const int co = i >> 8, k = i & 255;
  const int kh = k >> 5, kw = (k & 31) >> 2, ch = k & 3;
  float v = 0.f;
  if (kh < 7 && kw < 7 && ch < 3) v = W[((co * 3 + ch) * 7 + kh) * 7 + kw];
  Wk[i] = (bf16)v;
}

__global__ void __launch_bounds__(256) stem_wgrad_reduce_k(const float* __restrict__ part, int slabs, int Co,
                                                            float* __restrict__ dW, int accumulate) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= Co * 147) return;
  const int co = i / 147, r = i - co * 147;
  const int ch = r / 49, kh = (r - ch * 49) / 7, kw = r - ch * 49 - kh * 7;
  const int col = kh * 32 + kw * 4 + ch;
  float a = 0.f;
  for (int s = 0; s < slabs; ++s) a += part[((long long)s * Co + co) * 256 + col];
  dW[i] = accumulate ? dW[i] + a : a;
}

bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

bool geom_ok(const ConvGeom& g) {
  if (g.stem && (g.KH != 1 || g.KW != 1 || g.transposed || g.YS != 2 * g.YO + 6 || g.XS != 2 * g.XO + 8)) return false;
  return g.YO > 0 && g.XO > 0 && g.YS > 0 && g.XS > 0 && g.KH > 0 && g.KW > 0 && (g.stride == 1 || g.stride == 2) &&
         g.pad >= 0 && g.pad < (1 << 10) && g.KH < (1 << 10) && g.KW < (1 << 10);
}

}  // namespace

int conv_nt_row_tiles(const ConvNT& p) {
  const int BMt = p.N % 128 == 0 ? 128 : 256;
  return (int)((p.M + BMt - 1) / BMt);
}

hipError_t launch_conv_nt(const ConvNT& p, hipStream_t s) {
  if (!geom_ok(p.g) || p.M <= 0 || p.M >= (1LL << 31) - 256 || p.Cs <= 0 || p.Cs % CBK || p.N <= 0 || p.N % 64 ||
      !al16(p.src) || !al16(p.W) || !al16(p.out) || !al16(p.extra) || (p.extra && !p.mask))
    return hipErrorInvalidValue;
  if (p.g.stem && p.Cs != 256) return hipErrorInvalidValue;
  if (p.stat_part && (p.add || p.extra || p.g.cls)) return hipErrorInvalidValue;   // sums of a whole, fresh output only
  if (p.g.cls && (p.g.cls < 1 || p.g.cls > 4 || !p.g.transposed || p.g.stride != 2 || p.g.YO % 2 || p.g.XO % 2))
    return hipErrorInvalidValue;
  // rows of one launch: whole tiles, or (parity class) a quarter of their positions
  const long long per_tile = p.g.cls ? (long long)(p.g.YO / 2) * (p.g.XO / 2) : (long long)p.g.YO * p.g.XO;
  if (p.M % per_tile) return hipErrorInvalidValue;
  // every source row index must fit the tensor the caller holds: n * YS * XS rows
  const long long n = p.M / per_tile;
  if (n * p.g.YS * p.g.XS >= (1LL << 31)) return hipErrorInvalidValue;
  const bool wide = p.N % 128 == 0;
  const int BMt = wide ? 128 : 256, BNt = wide ? 128 : 64;
  const int row_tiles = (int)((p.M + BMt - 1) / BMt);
  const int col_tiles = p.N / BNt;
  const unsigned grid = (unsigned)((row_tiles + 7) / 8 * 8) * (unsigned)col_tiles;   // 8 XCDs x tiles per XCD x column tiles
  // 3x3 stride-1 convolutions whose source window fits the LDS next to the weight stages: the resident-window kernel
  if (p.Wf && !p.g.stem && !p.g.cls && p.g.KH == 3 && p.g.KW == 3 && p.g.stride == 1 && p.g.pad == 1 && p.g.YS == p.g.YO &&
      p.g.XS == p.g.XO && p.Cs <= 256 && al16(p.Wf)) {
    const int cpr = p.Cs / 8, unit = 256 / cpr;   // window rows come in units of 256 pieces (one instruction per wavefront)
    const int wrows = (BMt + 2 * (p.g.XO + 1) + unit - 1) / unit * unit;
    const size_t st = (size_t)wrows * p.Cs * 2, ep = (size_t)BMt * (BNt + 4) * sizeof(float);
    const size_t lds = st > ep ? st : ep;
    if (lds <= 160 * 1024) {
      static size_t attr_w = 0, attr_n = 0;   // largest size the attribute has been raised to
      size_t& have = wide ? attr_w : attr_n;
      if (lds > have) {
        hipError_t e = wide ? hipFuncSetAttribute((const void*)conv_nt_halo_k<128, 128>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                            : hipFuncSetAttribute((const void*)conv_nt_halo_k<256, 64>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        have = lds;
      }
      if (wide) hipLaunchKernelGGL((conv_nt_halo_k<128, 128>), dim3(grid), dim3(256), lds, s, p, row_tiles, col_tiles, wrows);
      else hipLaunchKernelGGL((conv_nt_halo_k<256, 64>), dim3(grid), dim3(256), lds, s, p, row_tiles, col_tiles, wrows);
      return hipGetLastError();
    }
  }
  // the stem where its tiles never straddle images and a tile's window of image rows fits the window buffer
  if (p.g.stem && p.N == 64 && !p.add && !p.extra && !p.g.cls && per_tile % 256 == 0) {
    const int rows_out = (p.g.XO - 1 + 255) / p.g.XO + 1;            // output rows a tile of 256 positions can touch
    const long long wbytes = (long long)(2 * (rows_out - 1) + 7) * p.g.XS * 8;
    const long long img_bytes = n * p.g.YS * p.g.XS * 8;
    if (wbytes <= STEM_WIN && img_bytes >= 16) {
      static int cus = 0;
      if (!cus) {
        int dev = 0;
        hipDeviceProp_t prop;
        hipError_t e;
        if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
        if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
        cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
      }
      const int tiles = (int)(p.M / 256);
      static bool stem_attr = false;
      if (!stem_attr) {
        hipError_t e = hipFuncSetAttribute((const void*)stem_fwd_k, hipFuncAttributeMaxDynamicSharedMemorySize, STEM_LDS);
        if (e != hipSuccess) return e;
        stem_attr = true;
      }
      const int g = tiles < 2 * cus ? tiles : 2 * cus;   // two workgroups per compute unit
      hipLaunchKernelGGL(stem_fwd_k, dim3((unsigned)g), dim3(256), STEM_LDS, s, p, tiles, (int)wbytes, img_bytes);
      return hipGetLastError();
    }
  }
  static bool attr_done = false;
  constexpr int NST = CONV_STAGES;
  // the operand stages, or the fp32 copy of the tile that takes their place at the end, whichever is larger
  auto lds_of = [](size_t BM, size_t BN) {
    const size_t st = (size_t)NST * (BM + BN) * CBK * sizeof(bf16), ep = BM * (BN + 4) * sizeof(float);
    return st > ep ? st : ep;
  };
  const size_t lds_w = lds_of(128, 128), lds_n = lds_of(256, 64);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)conv_nt_dl_k<128, 128, NST, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_w);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)conv_nt_dl_k<256, 64, NST, false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_n);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)conv_nt_dl_k<128, 128, NST, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_w);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)conv_nt_dl_k<256, 64, NST, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_n);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)conv_nt_dl_k<128, 128, NST, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_w);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void*)conv_nt_dl_k<256, 64, NST, false, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_n);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  // pointwise layers (and their input gradients): produced row m reads source row m
  const bool pw = !p.g.stem && !p.g.cls && p.g.KH == 1 && p.g.KW == 1 && p.g.stride == 1 && p.g.pad == 0 && p.g.YS == p.g.YO &&
                  p.g.XS == p.g.XO;
  if (pw) {
    if (wide) hipLaunchKernelGGL((conv_nt_dl_k<128, 128, NST, false, true>), dim3(grid), dim3(256), lds_w, s, p, row_tiles, col_tiles);
    else hipLaunchKernelGGL((conv_nt_dl_k<256, 64, NST, false, true>), dim3(grid), dim3(256), lds_n, s, p, row_tiles, col_tiles);
    return hipGetLastError();
  }
  if (wide && p.g.stem) hipLaunchKernelGGL((conv_nt_dl_k<128, 128, NST, true>), dim3(grid), dim3(256), lds_w, s, p, row_tiles, col_tiles);
  else if (wide) hipLaunchKernelGGL((conv_nt_dl_k<128, 128, NST, false>), dim3(grid), dim3(256), lds_w, s, p, row_tiles, col_tiles);
  else if (p.g.stem) hipLaunchKernelGGL((conv_nt_dl_k<256, 64, NST, true>), dim3(grid), dim3(256), lds_n, s, p, row_tiles, col_tiles);
  else hipLaunchKernelGGL((conv_nt_dl_k<256, 64, NST, false>), dim3(grid), dim3(256), lds_n, s, p, row_tiles, col_tiles);
  return hipGetLastError();
}

hipError_t launch_conv_wgrad(const ConvWG& p, hipStream_t s) {
  const int taps = p.g.KH * p.g.KW;
  if (!geom_ok(p.g) || p.g.transposed || (taps != 1 && !(p.g.KH == 3 && p.g.KW == 3)) || p.M <= 0 ||
      p.M >= (1LL << 31) - WBK || p.Co <= 0 || p.Co % 64 || p.Cs <= 0 || p.Cs % 64 || p.slabs <= 0 || p.slabs > 65535 ||
      p.per <= 0 || p.per % WBK || p.per * p.slabs < p.M || !al16(p.dout) || !al16(p.src) || !p.part ||
      p.M % ((long long)p.g.YO * p.g.XO))
    return hipErrorInvalidValue;
  if (p.g.stem && (p.Cs != 64 || taps != 1)) return hipErrorInvalidValue;   // 4 column groups of 64
  const long long n = p.M / ((long long)p.g.YO * p.g.XO);
  if (n * p.g.YS * p.g.XS >= (1LL << 31)) return hipErrorInvalidValue;
  const long long nwg = (long long)((p.slabs + 7) / 8 * 8) * (p.Co / 64) * (p.Cs / 64);
  if (nwg >= (1LL << 31)) return hipErrorInvalidValue;
  dim3 grid((unsigned)nwg);
  auto lds_of = [](int taps_) { return (size_t)2 * (1 + taps_) * WBK * 64 * sizeof(bf16); };
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)conv_wgrad_k<9, false>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)lds_of(9));
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  // 3x3 stride-1 pad-1 layers on a grid at least 8 wide: the kernel that fetches a step's source rows once
  if (!p.g.stem && taps == 9 && p.g.stride == 1 && p.g.pad == 1 && p.g.YS == p.g.YO && p.g.XS == p.g.XO && p.g.XO >= 8) {
    hipLaunchKernelGGL(conv_wgrad_win_k, grid, dim3(256), 0, s, p);   // (its stages are static LDS arrays)
    return hipGetLastError();
  }
  if (p.g.stem) hipLaunchKernelGGL((conv_wgrad_k<4, true>), grid, dim3(256), lds_of(4), s, p);
  else if (taps == 1 && p.g.stride == 1 && p.g.pad == 0 && p.g.YS == p.g.YO && p.g.XS == p.g.XO) {
    const unsigned g8 = (unsigned)((p.slabs + 7) / 8 * 8);
    if (p.Co % 128 == 0 && p.Cs % 128 == 0)
      hipLaunchKernelGGL((conv_wgrad_pw_k<128, 128>), dim3(g8 * (p.Co / 128) * (p.Cs / 128)), dim3(256), 0, s, p);
    else if (p.Co % 256 == 0)
      hipLaunchKernelGGL((conv_wgrad_pw_k<256, 64>), dim3(g8 * (p.Co / 256) * (p.Cs / 64)), dim3(256), 0, s, p);
    else if (p.Cs % 256 == 0)
      hipLaunchKernelGGL((conv_wgrad_pw_k<64, 256>), dim3(g8 * (p.Co / 64) * (p.Cs / 256)), dim3(256), 0, s, p);
    else
      hipLaunchKernelGGL((conv_wgrad_k<1, false, true>), grid, dim3(256), lds_of(1), s, p);
  }
  else if (taps == 1) hipLaunchKernelGGL((conv_wgrad_k<1, false>), grid, dim3(256), lds_of(1), s, p);
  else hipLaunchKernelGGL((conv_wgrad_k<9, false>), grid, dim3(256), lds_of(9), s, p);
  return hipGetLastError();
}

hipError_t launch_wgrad_reduce(const float* part, int slabs, int Co, int Cin, int taps, int ldk, float* dW, int accumulate,
                               hipStream_t s) {
  if (!part || !dW || slabs <= 0 || Co <= 0 || Cin <= 0 || taps <= 0 || ldk < taps * Cin) return hipErrorInvalidValue;
  const long long total = (long long)Co * taps * Cin;
  hipLaunchKernelGGL(wgrad_reduce_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, part, slabs, Co, Cin, taps, ldk,
                     dW, accumulate);
  return hipGetLastError();
}

hipError_t launch_conv_cast_w(const float* W, int Co, int Cin, int taps, int ldk, bf16* Wk, bf16* Wt, bf16* Wf, bf16* Wtf,
                              hipStream_t s) {
  if (!W || !Wk || Co <= 0 || Cin <= 0 || taps <= 0 || ldk < taps * Cin) return hipErrorInvalidValue;
  if ((Wf || Wtf) && (Co % 32 || Cin % 32 || ldk != taps * Cin)) return hipErrorInvalidValue;   // whole fragments only
  const long long total = (long long)Co * ldk;
  hipLaunchKernelGGL(conv_cast_w_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, W, Co, Cin, taps, ldk, Wk, Wt, Wf, Wtf);
  return hipGetLastError();
}

hipError_t launch_stem_pad_pixels(const bf16* pixels, bf16* img, long long n, int S, hipStream_t s) {
  if (!pixels || !img || n <= 0 || S <= 0 || S % 2 || ((uintptr_t)img & 7)) return hipErrorInvalidValue;
  const long long total = n * (S + 6) * (S + 8);
  if ((total + 255) / 256 >= (1LL << 31)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stem_pad_pixels_k, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, pixels, img, total, S);
  return hipGetLastError();
}

hipError_t launch_stem_cast_w(const float* W, int Co, bf16* Wk, hipStream_t s) {
  if (!W || !Wk || Co <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stem_cast_w_k, dim3((unsigned)(Co)), dim3(256), 0, s, W, Co, Wk);
  return hipGetLastError();
}

hipError_t launch_stem_wgrad_reduce(const float* part, int slabs, int Co, float* dW, int accumulate, hipStream_t s) {
  if (!part || !dW || slabs <= 0 || Co <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(stem_wgrad_reduce_k, dim3((unsigned)((Co * 147 + 255) / 256)), dim3(256), 0, s, part, slabs, Co, dW,
                     accumulate);
  return hipGetLastError();
}

}  // namespace sl
