// bf16 MFMA "NT" GEMM for gfx950: C[M,N] = A[M,K] * B[N,K]^T (+ fused epilogue), fp32 accumulate.
//
// Every activation-side GEMM of the encoder is this kernel (forward GEMMs use W [out][in];
// input-gradient GEMMs use the pre-transposed copy W^T, so both operands are always
// K-contiguous).  K is short here (384..1536), so the output tile is made large instead: one
// workgroup of WVM x WVN wavefronts owns a (WVM*WBM*32) x (WVN*WBN*32) tile, each wavefront a
// WBM x WBN grid of 32x32 MFMA accumulators.  A large tile is what keeps the bytes moved
// global->LDS per MFMA clock under what one CU's vector memory path delivers.
//   * LDS: two stages of [BM + BN][BK + 8] bf16 (144-byte rows: conflict-free 16-byte reads);
//     global loads of K step k+1 are issued before the MFMAs of step k and parked in registers.
//   * Epilogue: each wave passes its accumulators through a private LDS patch and gets them back
//     as 8-column row segments, so bias / residual / GELU / position terms are applied with
//     16-byte loads and stores and every output row of the strip is one contiguous run
//     (partial-line stores straight from the MFMA register layout measured 25 % slower).
//   * Persistent workgroups: the grid is what fits on the chip at once and every workgroup walks
//     over tiles.  Identical tiles otherwise march in lockstep (all CUs load and multiply, then
//     all CUs store), leaving HBM idle in one phase and the MFMAs idle in the other; here a
//     tile's stores drain under the next tile's loads and MFMAs.
//   * Workgroup ids are dealt round-robin to the 8 XCDs by the hardware; the id -> tile map puts
//     the tiles that share an A row panel on the same XCD (same L2).
#include "gemm_epi.h"

namespace sl {

namespace {

constexpr int NXCD = 8;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 ldg16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }

// ---- 8-wide row segment helpers ----------------------------------------------------------------
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    float4 t = reinterpret_cast<const float4*>(p)[i];
    v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
  }
}
__device__ __forceinline__ void load8(const bf16* p, float (&v)[8]) {
  u32x4 t = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    v[2 * w] = __uint_as_float(t[w] << 16);
    v[2 * w + 1] = __uint_as_float(t[w] & 0xffff0000u);
  }
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) reinterpret_cast<float4*>(p)[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
  bf16x8 t;
#pragma unroll
  for (int w = 0; w < 8; ++w) t[w] = (bf16)v[w];
  *reinterpret_cast<bf16x8*>(p) = t;
}

// eight one-byte codes of the stored GELU derivative
__device__ __forceinline__ void load8_dg(const unsigned char* p, float (&v)[8]) {
  uint2 t = *reinterpret_cast<const uint2*>(p);
  float a[4], b[4];
  dg8_unpack4(t.x, a);
  dg8_unpack4(t.y, b);
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
}
__device__ __forceinline__ void store8_dg(unsigned char* p, const float (&v)[8]) {
  *reinterpret_cast<uint2*>(p) = make_uint2(dg8_pack4(v[0], v[1], v[2], v[3]), dg8_pack4(v[4], v[5], v[6], v[7]));
}

// Auxiliary operand of one 8-column row segment (residual / saved pre-activation / position
// row), fetched ahead of the arithmetic so that its latency overlaps the LDS round trip.
template <int MODE, typename RS>
__device__ __forceinline__ void epi_aux8(const GemmNT& g, long long m, int n, float (&t)[8]) {
  if (MODE == EPI_BIAS_RESID) load8((const RS*)g.resid + m * g.ldr + n, t);
  else if (MODE == EPI_DGELU) load8_dg((const unsigned char*)g.pre + m * g.ldpre + n, t);
  else if (MODE == EPI_PATCH) load8(g.pos + (size_t)(1 + (int)(m % g.cmap.g2)) * g.N + n, t);
}

// one row segment: columns n..n+7 of row m; `bias` and `t` (aux) were loaded by the caller
template <int MODE, typename RS>
__device__ __forceinline__ void epi_seg8(const GemmNT& g, long long m, int n, float (&v)[8], const float (&bias)[8],
                                         float (&t)[8]) {
  if (MODE != EPI_PLAIN && MODE != EPI_DGELU) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] += bias[i];
  }
  if (MODE == EPI_PLAIN || MODE == EPI_BIAS) {
    store8((bf16*)g.out + m * g.ldc + n, v);
  } else if (MODE == EPI_BIAS_RESID) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] += t[i];
    store8((RS*)g.out + m * g.ldc + n, v);
  } else if (MODE == EPI_BIAS_GELU) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float gl, dg;
      gelu_both(v[i], &gl, &dg);
      v[i] = gl;
      t[i] = dg;
    }
    store8((bf16*)g.out + m * g.ldc + n, v);
    store8_dg((unsigned char*)g.out2 + m * g.ldc2 + n, t);
  } else if (MODE == EPI_DGELU) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] *= t[i];
    store8((bf16*)g.out + m * g.ldc + n, v);
  } else {  // EPI_PATCH
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] += t[i];
    store8((RS*)g.out + g.cmap(m) * g.ldc + n, v);
  }
}

template <int WBM, int WBN, int WVM, int WVN, int BK>
struct Cfg {
  static constexpr int BM = WVM * WBM * 32, BN = WVN * WBN * 32;
  static constexpr int NT = 64 * WVM * WVN;
  static constexpr int LDT = BK + 8;
  static constexpr int CPR = BK / 8;                 // 16-byte chunks per tile row
  static constexpr int CA = BM * CPR / NT, CB = BN * CPR / NT;
  static constexpr int RSTEP = NT / CPR;             // rows between successive chunks of one thread
  static constexpr size_t LDS = (size_t)2 * (BM + BN) * LDT * sizeof(bf16);
  static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "loader split");
  static_assert(WBN == 2 || WBN == 4, "epilogue row split");
  static_assert(LDS >= (size_t)WVM * WVN * 32 * (WBN * 32 + 4) * 4, "epilogue patches fit");
};

// Epilogue: the wave's 32 x (WBN*32) strip of accumulators goes through a wave-private LDS patch
// (row stride padded to WBN*32 + 4 floats) and comes back as 8-column row segments, 4*WBN
// neighbouring lanes covering one full output row of the strip: every global load and store of
// the epilogue is a 16-byte access and each row is written as one contiguous run.
// Accumulator element r of lane l sits at row (r/4)*8 + (l/32)*4 + r%4, column l%32 of its block.
template <int MODE, typename RS, int WBM, int WBN>
__device__ __forceinline__ void nt_epilogue(const GemmNT& g, f32x16 (&acc)[WBM][WBN], long long mw, int nw, int lane,
                                            float* patch) {
  constexpr int PS = WBN * 32 + 4;      // patch row stride (floats)
  constexpr int SEG = WBN * 4;          // 8-column segments per row
  constexpr int RPP = 64 / SEG;         // rows per pass
  constexpr int NP = 32 / RPP;          // passes per strip
  int li = lane & 31, h2 = lane >> 5;
  int prow = lane / SEG, pseg = lane % SEG;
  int n = nw + pseg * 8;
  bool n_ok = n < g.N;
  float bias[8];
  if (MODE != EPI_PLAIN && MODE != EPI_DGELU && n_ok) load8(g.bias + n, bias);
#pragma unroll
  for (int i = 0; i < WBM; ++i) {
    float aux[NP][8];
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      long long m = mw + i * 32 + ps * RPP + prow;
      if (n_ok && m < g.M) epi_aux8<MODE, RS>(g, m, n, aux[ps]);
    }
#pragma unroll
    for (int j = 0; j < WBN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) patch[((r >> 2) * 8 + h2 * 4 + (r & 3)) * PS + j * 32 + li] = acc[i][j][r];
#pragma unroll
    for (int ps = 0; ps < NP; ++ps) {
      int row = ps * RPP + prow;
      float v[8];
      const float4* src = reinterpret_cast<const float4*>(patch + row * PS + pseg * 8);
      float4 a = src[0], b = src[1];
      v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
      long long m = mw + i * 32 + row;
      if (n_ok && m < g.M) epi_seg8<MODE, RS>(g, m, n, v, bias, aux[ps]);
    }
  }
}

template <typename RS, int WBM, int WBN, int WVM, int WVN, int BK>
__global__ void __launch_bounds__(64 * WVM * WVN) gemm_nt_tile_k(GemmNT g, int MT, int NTL) {
  using C = Cfg<WBM, WBN, WVM, WVN, BK>;
  constexpr int BM = C::BM, BN = C::BN, LDT = C::LDT, CA = C::CA, CB = C::CB;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* As = reinterpret_cast<bf16*>(smem);  // [2][BM][LDT]
  bf16* Bs = As + 2 * BM * LDT;              // [2][BN][LDT]
  const bf16* A = (const bf16*)g.A;
  const bf16* B = (const bf16*)g.B;
  int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int wm = wave / WVN, wn = wave % WVN;
  int row0 = tid / C::CPR, kc = tid % C::CPR;
  int soff = row0 * LDT + kc * 8;
  int frow = lane & 31, fk = (lane >> 5) * 8;
  int nk = g.K / BK;
  int total = (MT + NXCD - 1) / NXCD * NXCD * NTL;

  long long aoff[CA], boff[CB];
  u32x4 ra[CA], rb[CB];
  // tile id -> (row tile, column tile); ids are dealt round-robin to the XCDs, and the tiles of one
  // row panel get consecutive slots of one XCD.  The grid size is a multiple of 8, so a persistent
  // workgroup keeps meeting tiles of its own XCD.
  auto tile_of = [&](int id, long long& m0, int& n0) {
    int xcd = id % NXCD, slot = id / NXCD;
    int mt = (slot / NTL) * NXCD + xcd;
    m0 = (long long)mt * BM;
    n0 = (slot % NTL) * BN;
    return mt < MT;
  };
  auto fetch0 = [&](long long m0, int n0) {  // operand offsets of a tile + global loads of its first K step
#pragma unroll
    for (int i = 0; i < CA; ++i) {
      long long am = m0 + row0 + i * C::RSTEP;
      if (am > g.M - 1) am = g.M - 1;  // rows past the end are loaded (valid memory) but never stored
      aoff[i] = g.amap(am) * g.lda + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      int bn = n0 + row0 + i * C::RSTEP;
      if (bn > g.N - 1) bn = g.N - 1;
      boff[i] = (long long)bn * g.ldb + kc * 8;
    }
#pragma unroll
    for (int i = 0; i < CA; ++i) ra[i] = ldg16(A + aoff[i]);
#pragma unroll
    for (int i = 0; i < CB; ++i) rb[i] = ldg16(B + boff[i]);
  };

  bool have = false;  // ra/rb already hold the first K step of the tile about to be processed
  for (int id = blockIdx.x; id < total; id += gridDim.x) {
    long long m0;
    int n0;
    if (!tile_of(id, m0, n0)) { have = false; continue; }  // uniform for the workgroup
    if (!have) fetch0(m0, n0);
#pragma unroll
    for (int i = 0; i < CA; ++i) *reinterpret_cast<u32x4*>(As + soff + i * C::RSTEP * LDT) = ra[i];
#pragma unroll
    for (int i = 0; i < CB; ++i) *reinterpret_cast<u32x4*>(Bs + soff + i * C::RSTEP * LDT) = rb[i];
    __syncthreads();

    f32x16 acc[WBM][WBN];
#pragma unroll
    for (int i = 0; i < WBM; ++i)
#pragma unroll
      for (int j = 0; j < WBN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    for (int kt = 0; kt < nk; ++kt) {
      int cur = kt & 1;
      bool more = kt + 1 < nk;
      if (more) {
#pragma unroll
        for (int i = 0; i < CA; ++i) ra[i] = ldg16(A + aoff[i] + (kt + 1) * BK);
#pragma unroll
        for (int i = 0; i < CB; ++i) rb[i] = ldg16(B + boff[i] + (kt + 1) * BK);
      }
      const bf16* as = As + cur * BM * LDT + (wm * WBM * 32 + frow) * LDT + fk;
      const bf16* bs = Bs + cur * BN * LDT + (wn * WBN * 32 + frow) * LDT + fk;
      // fragments of k-slice ks+1 are read from LDS before the MFMAs of slice ks are issued
      bf16x8 fa[2][WBM], fb[2][WBN];
#pragma unroll
      for (int i = 0; i < WBM; ++i) fa[0][i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDT);
#pragma unroll
      for (int j = 0; j < WBN; ++j) fb[0][j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * LDT);
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        if (ks + 1 < BK / 16) {
#pragma unroll
          for (int i = 0; i < WBM; ++i)
            fa[(ks + 1) & 1][i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDT + (ks + 1) * 16);
#pragma unroll
          for (int j = 0; j < WBN; ++j)
            fb[(ks + 1) & 1][j] = *reinterpret_cast<const bf16x8*>(bs + j * 32 * LDT + (ks + 1) * 16);
        }
#pragma unroll
        for (int i = 0; i < WBM; ++i)
#pragma unroll
          for (int j = 0; j < WBN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][i], fb[ks & 1][j], acc[i][j], 0, 0, 0);
      }
      if (more) {
        int nxt = cur ^ 1;
#pragma unroll
        for (int i = 0; i < CA; ++i)
          *reinterpret_cast<u32x4*>(As + nxt * BM * LDT + soff + i * C::RSTEP * LDT) = ra[i];
#pragma unroll
        for (int i = 0; i < CB; ++i)
          *reinterpret_cast<u32x4*>(Bs + nxt * BN * LDT + soff + i * C::RSTEP * LDT) = rb[i];
      }
      __syncthreads();
    }

    // the next tile's first loads go out now: they and this tile's stores drain while the epilogue
    // arithmetic runs, and the stores keep draining under the next tile's MFMAs
    {
      long long m1;
      int n1;
      int nid = id + gridDim.x;
      have = nid < total && tile_of(nid, m1, n1);
      if (have) fetch0(m1, n1);
    }

    // operand tiles are dead past the last barrier: the patches reuse their LDS
    float* patch = reinterpret_cast<float*>(smem) + wave * 32 * (WBN * 32 + 4);
    long long mw = m0 + wm * WBM * 32;
    int nw = n0 + wn * WBN * 32;
    switch (g.epi) {
      case EPI_PLAIN: nt_epilogue<EPI_PLAIN, RS, WBM, WBN>(g, acc, mw, nw, lane, patch); break;
      case EPI_BIAS: nt_epilogue<EPI_BIAS, RS, WBM, WBN>(g, acc, mw, nw, lane, patch); break;
      case EPI_BIAS_RESID: nt_epilogue<EPI_BIAS_RESID, RS, WBM, WBN>(g, acc, mw, nw, lane, patch); break;
      case EPI_BIAS_GELU: nt_epilogue<EPI_BIAS_GELU, RS, WBM, WBN>(g, acc, mw, nw, lane, patch); break;
      case EPI_DGELU: nt_epilogue<EPI_DGELU, RS, WBM, WBN>(g, acc, mw, nw, lane, patch); break;
      default: nt_epilogue<EPI_PATCH, RS, WBM, WBN>(g, acc, mw, nw, lane, patch); break;
    }
    __syncthreads();  // patches are read before the next tile's operands overwrite them
  }
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

template <int WBM, int WBN, int WVM, int WVN, int BK>
hipError_t go(const GemmNT& g, hipStream_t s) {
  using C = Cfg<WBM, WBN, WVM, WVN, BK>;
  static int resident = 0;  // workgroups that fit on the chip at once (persistent grid size)
  auto kern = gemm_nt_tile_k<rs_bf16path_t, WBM, WBN, WVM, WVN, BK>;
  if (!resident) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
    if (e != hipSuccess) return e;
    int per_cu = 0, dev = 0;
    hipDeviceProp_t prop;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipGetDeviceProperties(&prop, dev)) != hipSuccess) return e;
    if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, C::NT, C::LDS)) != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    resident = per_cu * prop.multiProcessorCount / NXCD * NXCD;
    if (resident < NXCD) resident = NXCD;
  }
  int MT = (int)((g.M + C::BM - 1) / C::BM), NTL = (g.N + C::BN - 1) / C::BN;
  long long total = (long long)((MT + NXCD - 1) / NXCD) * NXCD * NTL;
  long long wgs = total < resident ? total : resident;
  hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(C::NT), C::LDS, s, g, MT, NTL);
  return hipGetLastError();
}

}  // namespace

bool gemm_nt_mfma_ok(const GemmNT& g) {
  bool ok = g.K % 64 == 0 && g.N % 16 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 && aligned16(g.A) && aligned16(g.B) &&
            g.M > 0 && g.ldc % 8 == 0 && aligned16(g.out) && g.N % 8 == 0;
  if (g.epi == EPI_BIAS_RESID) ok = ok && g.ldr % 8 == 0 && aligned16(g.resid);
  if (g.epi == EPI_BIAS_GELU) ok = ok && g.ldc2 % 8 == 0 && ((size_t)g.out2 & 7) == 0;   // 8-byte code segments
  if (g.epi == EPI_DGELU) ok = ok && g.ldpre % 8 == 0 && ((size_t)g.pre & 7) == 0;
  if (g.epi != EPI_PLAIN && g.epi != EPI_DGELU) ok = ok && aligned16(g.bias);
  if (g.epi == EPI_PATCH) ok = ok && aligned16(g.pos);
  return ok;
}

bool gemm_nt_big_ok(const GemmNT& g);
hipError_t launch_gemm_nt_big(const GemmNT& g, hipStream_t s);
bool gemm_nt_gelu_ok(const GemmNT& g);
hipError_t launch_gemm_nt_gelu(const GemmNT& g, hipStream_t s);

// Large problems go to the 256 x 192 persistent kernels (the bias + GELU epilogue has one of its own), the rest to the
// 128 x 128 tiles of the kernel above.
hipError_t launch_gemm_nt_mfma(const GemmNT& g, hipStream_t s) {
  if (gemm_nt_gelu_ok(g)) return launch_gemm_nt_gelu(g, s);
  if (gemm_nt_big_ok(g)) return launch_gemm_nt_big(g, s);
  return go<2, 2, 2, 2, 64>(g, s);
}

}  // namespace sl
