// bf16 MFMA weight-gradient GEMM for gfx950 (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// TN: C[N1,N2] = A[M,N1]^T * B[M,N2], contraction over the slow (row) index.  Each thread
//     transposes 8x8 bf16 blocks in registers on the way into LDS, so the LDS image is
//     [column][row-chunk] and MFMA operands are again 16-byte contiguous reads.
#include "gemm_epi.h"

namespace sl {

namespace {


typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x4 ldg16(const bf16* p) { return *reinterpret_cast<const u32x4*>(p); }

// ---------------------------------------------------------------------------------------
// TN: part[s][i][j] = sum_{m in slab s} A[amap(m)][i] * B[bmap(m)][j]
// 128x128 output tile, 64 rows of m per step.  LDS image: At[i][m-chunk], Bt[j][m-chunk].
// ---------------------------------------------------------------------------------------
constexpr int TK = 64;          // rows of m per step
constexpr int LDK = TK + 8;     // padded

// 8x8 bf16 transpose in registers: in[r] holds 8 columns of row r (4 dwords); out[c] holds 8 rows
// of column c.
__device__ __forceinline__ void transpose8x8(const u32x4 (&in)[8], u32x4 (&out)[8]) {
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    int w = c >> 1;                                   // dword holding column c
    unsigned sel = (c & 1) ? 0x07060302u : 0x05040100u;  // take high / low halves
    u32x4 o;
#pragma unroll
    for (int p = 0; p < 4; ++p) {                     // rows 2p, 2p+1 -> one dword
      unsigned lo = in[2 * p][w], hi = in[2 * p + 1][w];
      o[p] = __builtin_amdgcn_perm(hi, lo, sel);
    }
    out[c] = o;
  }
}

__device__ __attribute__((aligned(16))) unsigned int g_zero16[4];

__global__ void __launch_bounds__(256, 2) gemm_tn_mfma_k(GemmTN g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* At = reinterpret_cast<bf16*>(smem);   // [2][128][LDK]
  bf16* Bt = At + 2 * 128 * LDK;              // [2][128][LDK]
  int i0 = blockIdx.x * 128, j0 = blockIdx.y * 128, s = blockIdx.z;
  long long per = (g.M + g.slabs - 1) / g.slabs;
  per = (per + TK - 1) / TK * TK;
  long long lo = (long long)s * per, hi = lo + per < g.M ? lo + per : g.M;
  const bf16* A = (const bf16*)g.A;
  const bf16* B = (const bf16*)g.B;
  int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int wm = wave >> 1, wn = wave & 1;
  // loader: threads 0..127 take A, 128..255 take B; each an 8(m) x 8(col) block per step.
  // 4 neighbouring lanes read 64 contiguous bytes of a row; the 8 row blocks vary next, so that the
  // 16-byte LDS stores of neighbouring lanes fall on different banks.
  int t = tid & 127;
  bool isB = tid >= 128;
  int mb = (t >> 2) & 7, cb = (t >> 5) * 4 + (t & 3);
  const bf16* src = isB ? B : A;
  long long ld = isB ? g.ldb : g.lda;
  RowMap map = isB ? g.bmap : g.amap;
  int cbase = (isB ? j0 : i0) + cb * 8;
  int ncols = isB ? g.N2 : g.N1;
  bool col_ok = cbase < ncols;  // N1, N2 are multiples of 8 (checked on the host)
  bf16* dst = (isB ? Bt : At) + (cb * 8) * LDK + mb * 8;

  // The 8 consecutive rows of a thread: no branch around the loads (they would be issued and waited for one by one)
  // and one 32-bit division per step instead of a 64-bit one per row: rows past the slab's end re-read its last
  // row and are zeroed afterwards; threads whose columns lie outside the matrix read a row of zeros with stride 0.
  const bf16* lbase = col_ok ? src + cbase : reinterpret_cast<const bf16*>(g_zero16);
  const long long lld = col_ok ? ld : 0;
  auto load = [&](long long mstep, u32x4 (&v)[8]) {
    long long m0 = mstep + mb * 8;
    long long mc = m0 < hi ? m0 : hi - 1;   // lo < hi here
    unsigned q = 0, rem = 0;
    if (map.g2) { q = (unsigned)mc / (unsigned)map.g2; rem = (unsigned)mc - q * (unsigned)map.g2; }
    long long row = map.g2 ? (long long)q * map.T + 1 + rem : mc;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      v[r] = ldg16(lbase + row * lld);
      if (m0 + r >= hi) v[r] = u32x4{0, 0, 0, 0};
      if (m0 + r + 1 < hi) {   // the next row exists: step the mapped index
        if (map.g2) {
          ++rem;
          if (rem == (unsigned)map.g2) { rem = 0; ++q; }
          row = (long long)q * map.T + 1 + rem;
        } else {
          ++row;
        }
      }
    }
  };
  auto store = [&](int buf, const u32x4 (&v)[8]) {
    u32x4 o[8];
    transpose8x8(v, o);
#pragma unroll
    for (int c = 0; c < 8; ++c) *reinterpret_cast<u32x4*>(dst + buf * 128 * LDK + c * LDK) = o[c];
  };

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // column sums of A (bias gradients) ride along in the workgroups of the first tile column
  bool do_cs = g.cs_part != nullptr && blockIdx.y == 0 && !isB;
  float cs[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) cs[c] = 0.f;
  auto add_cs = [&](const u32x4 (&v)[8]) {
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        cs[2 * w] += __uint_as_float(v[r][w] << 16);
        cs[2 * w + 1] += __uint_as_float(v[r][w] & 0xffff0000u);
      }
  };

  u32x4 v[8];
  if (lo < hi) {
    load(lo, v);
    if (do_cs) add_cs(v);
    store(0, v);
  }
  __syncthreads();
  int frow = lane & 31, fk = (lane >> 5) * 8;
  int it = 0;
  for (long long mstep = lo; mstep < hi; mstep += TK, ++it) {
    int cur = it & 1;
    bool more = mstep + TK < hi;
    if (more) load(mstep + TK, v);
    const bf16* as = At + cur * 128 * LDK + (wm * 64 + frow) * LDK + fk;
    const bf16* bs = Bt + cur * 128 * LDK + (wn * 64 + frow) * LDK + fk;
#pragma unroll
    for (int ks = 0; ks < TK / 16; ++ks) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        fa[i] = *reinterpret_cast<const bf16x8*>(as + i * 32 * LDK + ks * 16);
        fb[i] = *reinterpret_cast<const bf16x8*>(bs + i * 32 * LDK + ks * 16);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      if (do_cs) add_cs(v);
      store(cur ^ 1, v);
    }
    __syncthreads();
  }
  if (g.cs_part != nullptr && blockIdx.y == 0) {  // uniform per workgroup
    float* red = reinterpret_cast<float*>(smem);  // [8][128]; all LDS reads are behind the last barrier
    if (!isB) {
#pragma unroll
      for (int c = 0; c < 8; ++c) red[mb * 128 + cb * 8 + c] = cs[c];
    }
    __syncthreads();
    if (tid < 128 && i0 + tid < g.N1) {
      float a = 0.f;
#pragma unroll
      for (int m = 0; m < 8; ++m) a += red[m * 128 + tid];
      g.cs_part[(size_t)s * g.N1 + i0 + tid] = a;
    }
  }
  float* P = g.part + (size_t)s * g.N1 * g.N2;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int c = j0 + wn * 64 + j * 32 + (lane & 31);
      bool c_ok = c < g.N2;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int row = i0 + wm * 64 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (c_ok && row < g.N1) P[(size_t)row * g.N2 + c] = acc[i][j][r];
      }
    }
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

bool gemm_tn_mfma_ok(const GemmTN& g) {
  return g.N1 % 8 == 0 && g.N2 % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 && aligned16(g.A) && aligned16(g.B) &&
         g.M < (1LL << 31);   // row indices are mapped with 32-bit arithmetic
}

hipError_t launch_gemm_tn_mfma(const GemmTN& g, hipStream_t s) {
  static bool attr_done = false;
  size_t lds = (size_t)2 * 2 * 128 * LDK * sizeof(bf16);
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_tn_mfma_k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid((g.N1 + 127) / 128, (g.N2 + 127) / 128, g.slabs);
  hipLaunchKernelGGL(gemm_tn_mfma_k, grid, dim3(256), lds, s, g);
  return hipGetLastError();
}

}  // namespace sl
