// Internal declarations shared by the translation units of libslide (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace sl {

// ---- element types -------------------------------------------------------------------
typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Residual-stream element type of the bf16 path (activations that are summed layer after
// layer, forward x and backward dx): bf16, which halves the traffic of every kernel that touches the
// stream.  The one row per tile whose rounding decides the accuracy of the slide gradient (the CLS
// row) is carried in fp32 beside it (cls_lane.hip).
typedef bf16 rs_bf16path_t;

enum { DT_F32 = 0, DT_BF16 = 1 };

__host__ __device__ inline size_t elem_size(int dt) { return dt == DT_F32 ? 4 : 2; }
inline size_t rs_size(int dt) { return dt == DT_F32 ? 4 : sizeof(rs_bf16path_t); }

__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float v) { return (bf16)v; }  // RNE

// ---- wave / block reductions (wave = 64 lanes) ------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// erf(x) and exp(-x^2) together.  Rational approximation 7.1.26 of Abramowitz & Stegun,
// |error| <= 1.5e-7 (about one fp32 ulp of the result near 1): one reciprocal, one exponential
// and five fused multiply-adds instead of the library routine's long polynomial ladder; the
// GEMM epilogues that apply GELU run it once per output element.
__device__ __forceinline__ float erf_exp(float x, float* e_out) {
  float ax = fabsf(x);
  float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * ax);  // 1 ulp reciprocal
  float e = __expf(-ax * ax);
  float p = ((((1.061405429f * t - 1.453152027f) * t + 1.421413741f) * t - 0.284496736f) * t + 0.254829592f) * t;
  *e_out = e;
  return copysignf(1.0f - p * e, x);
}
__device__ __forceinline__ float gelu_f(float m) {
  float e;
  return 0.5f * m * (1.0f + erf_exp(m * 0.70710678118654752f, &e));
}
// gelu(m) and gelu'(m) from one erf/exp evaluation
__device__ __forceinline__ void gelu_both(float m, float* g, float* dg) {
  float e;
  float c = 0.5f * (1.0f + erf_exp(m * 0.70710678118654752f, &e));
  *g = m * c;
  *dg = c + m * e * 0.39894228040143268f;
}
__device__ __forceinline__ float gelu_grad_f(float m) {
  float e;  // exp(-m^2/2)
  float c = 0.5f * (1.0f + erf_exp(m * 0.70710678118654752f, &e));
  return c + m * e * 0.39894228040143268f;
}

// The GELU derivative the bf16 path keeps for the backward is one byte per element: gelu'(m) lies in
// [-0.1289, 1.1289] (extrema at m = -+sqrt(2)), and the code q = rne((gelu'(m) + DG8_OFF) * DG8_SCALE) in 0..254
// gives it back as q / DG8_SCALE - DG8_OFF with an error of at most 2.5e-3 (rms 1.4e-3, the size of the bf16
// rounding of a value near 1), in half the bytes of a bf16.  The fp32 path keeps the derivative as a float.
constexpr float DG8_OFF = 0.12890625f, DG8_SCALE = 202.0f;
// four values already in code space ((gelu' + DG8_OFF) * DG8_SCALE), a in byte 0
__device__ __forceinline__ unsigned dg8_pack4_code(float a, float b, float c, float d) {
  unsigned r = 0;
  r = __builtin_amdgcn_cvt_pk_u8_f32(a, 0, r);   // rounds to nearest even, clamps to 0..255
  r = __builtin_amdgcn_cvt_pk_u8_f32(b, 1, r);
  r = __builtin_amdgcn_cvt_pk_u8_f32(c, 2, r);
  r = __builtin_amdgcn_cvt_pk_u8_f32(d, 3, r);
  return r;
}
__device__ __forceinline__ float dg8_code(float dg) { return __builtin_fmaf(dg, DG8_SCALE, DG8_OFF * DG8_SCALE); }
__device__ __forceinline__ unsigned dg8_pack4(float a, float b, float c, float d) {
  return dg8_pack4_code(dg8_code(a), dg8_code(b), dg8_code(c), dg8_code(d));
}
__device__ __forceinline__ void dg8_unpack4(unsigned q, float (&v)[4]) {
  v[0] = (float)(q & 0xffu) * (1.0f / DG8_SCALE) - DG8_OFF;
  v[1] = (float)((q >> 8) & 0xffu) * (1.0f / DG8_SCALE) - DG8_OFF;
  v[2] = (float)((q >> 16) & 0xffu) * (1.0f / DG8_SCALE) - DG8_OFF;
  v[3] = (float)(q >> 24) * (1.0f / DG8_SCALE) - DG8_OFF;
}
// what one element of the stored derivative is, by element type of the path
template <typename T> struct dgelu_store;
template <> struct dgelu_store<float> {
  typedef float type;
  static __device__ __forceinline__ float put(float dg) { return dg; }
  static __device__ __forceinline__ float get(float q) { return q; }
};
template <> struct dgelu_store<bf16> {
  typedef unsigned char type;
  static __device__ __forceinline__ unsigned char put(float dg) { return (unsigned char)(dg8_pack4(dg, 0.f, 0.f, 0.f) & 0xffu); }
  static __device__ __forceinline__ float get(unsigned char q) { return (float)q * (1.0f / DG8_SCALE) - DG8_OFF; }
};
__host__ __device__ inline size_t dgelu_elem_size(int dt) { return dt == DT_F32 ? 4 : 1; }   // bytes per element of it

// Row map used where a GEMM operand lives in the token matrix but only patch-token rows
// take part: logical row r (tile r / g2, patch r % g2) -> token row (r / g2) * T + 1 + r % g2.
// g2 == 0 means identity.
struct RowMap {
  int g2, T;
  __host__ __device__ __forceinline__ long long operator()(long long r) const {
    return g2 ? (r / g2) * T + 1 + (r % g2) : r;
  }
  // same for row indices below 2^31 (32-bit division)
  __host__ __device__ __forceinline__ long long map32(unsigned r) const {
    if (!g2) return r;
    unsigned q = r / (unsigned)g2;
    return (long long)q * T + 1 + (r - q * (unsigned)g2);
  }
};

// ---- GEMM epilogues (C = A * B^T, A [M,K], B [N,K], both K-contiguous) ------------------
enum {
  EPI_PLAIN = 0,       // out(T)  = acc
  EPI_BIAS = 1,        // out(T)  = acc + bias[n]
  EPI_BIAS_RESID = 2,  // out(RS) = acc + bias[n] + resid(RS)[m][n]
  EPI_BIAS_GELU = 3,   // m = acc + bias[n];  out(T) = gelu(m);  out2 = gelu'(m) (float / one-byte code, dgelu_store<T>)
  EPI_DGELU = 4,       // out(T)  = acc * pre[m][n]   (pre holds the gelu'(m) the forward stored, same format)
  EPI_PATCH = 5,       // out(RS)[rowmap(m)] = acc + bias[n] + pos[1 + m % g2][n]
  EPI_ROWTAB = 6,      // out(RS) = acc + resid(RS)[m % rperiod][n]: a table of rperiod rows added periodically (large-M kernel only)
};

struct GemmNT {
  const void* A; long long lda;  // T
  RowMap amap;                   // row map applied to A rows
  const void* B; long long ldb;  // T (weights, [N,K])
  long long M; int N, K;
  int epi;
  const float* bias;
  const void* resid; long long ldr;
  int rperiod;                   // EPI_ROWTAB: rows of the table
  void* out; long long ldc;
  void* out2; long long ldc2;          // leading dimensions in elements of the stored-derivative format
  const void* pre; long long ldpre;
  const float* pos;  // [T, N] position table (EPI_PATCH)
  RowMap cmap;       // EPI_PATCH output rows
};

// C[N1,N2] (fp32) = sum_m A[m,N1]^T B[m,N2]; split over `slabs` ranges of m, partial s is
// written to part + s*N1*N2.  A rows go through amap.
struct GemmTN {
  const void* A; long long lda; RowMap amap;  // T [M, N1]
  const void* B; long long ldb; RowMap bmap;  // T [M, N2]
  long long M; int N1, N2;
  float* part; int slabs;
  float* cs_part;  // optional: column sums of A per slab, [slabs][N1] (only the MFMA kernels fill it)
  int big;         // use the large-M kernel (slabs was chosen by gemm_tn_big_slabs)
};
int gemm_tn_big_slabs(const GemmTN& g, int max_slabs);   // 0: the large-M kernel does not take this problem
hipError_t launch_gemm_tn_big(const GemmTN& g, hipStream_t s);

// All launchers enqueue on `s` and return the launch status.
hipError_t launch_gemm_nt(int dt, const GemmNT& g, bool use_mfma, hipStream_t s);
hipError_t launch_gemm_tn(int dt, const GemmTN& g, bool use_mfma, hipStream_t s);
int gemm_tn_pick_slabs(long long M, int N1, int N2, int max_slabs);
bool gemm_tn_fuses_colsum(int dt, const GemmTN& g, bool use_mfma);  // will launch_gemm_tn fill cs_part?

hipError_t launch_cast_transpose(int dt, const float* src, int R, int C, void* dstW, void* dstWT, hipStream_t s);
// patches: [n * (g*g + lead)][3 P P], every tile's g*g patch rows behind `lead` rows of zeros
hipError_t launch_patchify(int dt, const void* pixels, void* patches, long long n, int S, int P, hipStream_t s, int lead);
hipError_t launch_unpatchify(int dt, const void* dpatches, void* dpix, long long n, int S, int P, hipStream_t s);
hipError_t launch_cls_rows(int dt, void* x, const float* cls, const float* pos, long long n, int T, int D, hipStream_t s);
hipError_t launch_pos_table(void* tab, const float* cls, const float* pos, const float* bias, int T, int D, hipStream_t s);
bool gemm_nt_big_ok(const GemmNT& g);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_calib_copy(void* dst, const void* src, size_t bytes, hipStream_t s);
hipError_t launch_gelu(int dt, const void* m, void* a, long long count, hipStream_t s);
// part[s][c] = sum over rows of slab s of A[map(r)][c]; elem: DT_F32 / DT_BF16 element type of A
int colsum_slabs(long long M);
hipError_t launch_colsum_part(int elem, const void* A, long long lda, RowMap map, long long M, int N, float* part,
                              int slabs, hipStream_t s);
// out[i] = (accumulate ? out[i] : 0) + sum_s part[s*stride + i], i < len
hipError_t launch_reduce_partials(const float* part, int slabs, long long stride, long long len, float* out,
                                  int accumulate, hipStream_t s);

// LayerNorm.  x rows at x + r*x_stride (RS), out rows at out + r*out_stride (T, or fp32 when out_f32).
hipError_t launch_ln_fwd(int dt, const void* x, long long x_stride, const float* gam, const float* bet, void* out,
                         long long out_stride, long long rows, int D, float eps, bool out_f32, hipStream_t s);
// dx_out[r] (RS) = (dres ? dres[r] : 0) + LN-backward(dy[r] (T, or fp32 when dy_f32); x[r] (RS)); optional T copy of dx_out
// (only written when RS and T differ); dgamma/dbeta partials -> part[slab][2][D], ln_bwd_slabs(rows) slabs.
int ln_bwd_slabs(long long rows);
hipError_t launch_ln_bwd(int dt, const void* x, long long x_stride, const void* dy, long long dy_stride,
                         const float* gam, const void* dres, void* dx_out, void* dx_out_t, long long o_stride,
                         long long rows, int D, float eps, float* part, bool dy_f32, hipStream_t s,
                         const float* bet = nullptr, void* u_out = nullptr, long long u_stride = 0, int dres_period = 0);
// dres_period != 0: dres contributes on rows r % dres_period == 0 only (its other rows are not read); only where
// ln_bwd_periodic_ok says so
bool ln_bwd_periodic_ok(int dt, const void* x, long long x_stride, const void* dy, long long dy_stride, const float* gam,
                        const void* dres, const void* dx_out, long long o_stride, int D, bool dy_f32);
// u_out: also write the normalised rows x_hat * gamma + beta (bf16 [rows][u_stride]); only where ln_bwd_emits_u says so
bool ln_bwd_emits_u(int dt, const void* x, long long x_stride, const void* dy, long long dy_stride, const float* gam,
                    const void* dres, const void* dx_out, long long o_stride, int D, bool dy_f32, const float* bet,
                    const void* u_out, long long u_stride);

// Attention over qkv [n*T, 3D] (T): O [n*T, D] (T), lse [n,H,T] fp32.
// cls_only (bf16 MFMA kernels only, see attn_cls_only_ok): only query 0 of every tile is wanted (forward: the rest
// of O and lse beyond the first block of 32 queries is not written) / only query 0 carries an output gradient
// (backward: other rows of dO are not read; dqkv is complete: dQ is zero for every other query).
bool attn_cls_only_ok(int dt, int T, int dh, bool use_mfma);
hipError_t launch_attn_fwd(int dt, const void* qkv, void* O, float* lse, long long n, int T, int H, int dh,
                           bool use_mfma, hipStream_t s, bool cls_only = false);
hipError_t launch_attn_bwd(int dt, const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv,
                           long long n, int T, int H, int dh, bool use_mfma, hipStream_t s, bool cls_only = false,
                           float* delta_ws = nullptr);   // [n][H][T] floats, needed by the matrix-core kernels
size_t attn_lds_bytes(int T, int dh);

// Gated-attention MIL pool.
struct PoolArgs {
  const float* H; long long N; int D, Mh, C; int label;  // features are fp32 in both paths
  const float *VW, *Vb, *UW, *Ub, *w, *cW, *cb;
  float* a;     // [N] attention logits
  double* part; // [blocks][2 + D] forward partials {max, sum, weighted feature sum}
  float* scal;  // [4 + 2C + 3D]: m, Z, loss, z.dz, logits[C], dy[C], z[D], dz[D], zlo[D]
  int blocks;
  float *loss, *logits, *alpha;  // outputs, may be null
  float* G;                      // [N,D]
  float* grads;                  // flat gradient vector
  size_t ocW, ocb;               // offsets of head.W / head.b in it
  int accumulate;
  void* vub;     // 2 x [2 Mh][D] bf16: copy of [V;U] and room for its transpose (scratch of the matrix-core kernels), may be null
  int use_mfma;  // bf16 path: gate projections on the matrix cores where the shape is built
  // M_h = 256 taken as two halves of 128 gate units by the register-resident forward kernel: the first half only writes
  // its partial logits (partial = 1), the second adds them (a_in) and does everything else; w_other = the other half's w
  // (the softmax shift is a bound over all gate units).  a_tmp: [N] floats of scratch for the partial logits.
  const float* a_in; int partial; const float* w_other; float* a_tmp;
};
int pool_blocks(long long N);
bool pool_mfma_ok(const PoolArgs& p);
int pool_mfma_rows(const PoolArgs& p);
hipError_t launch_pool_gate_part_mfma(const PoolArgs& p, hipStream_t s);
hipError_t launch_pool_fwd(const PoolArgs& p, hipStream_t s);
hipError_t launch_pool_bwd_rows(const PoolArgs& p, float* Dp, hipStream_t s);
hipError_t launch_pool_head_grads(const PoolArgs& p, hipStream_t s);

// fp32 lane of the CLS rows (bf16 path, cls_lane.hip)
bool cls_lane_ok(int D, int F);
hipError_t launch_lane_init(const float* cls, const float* pos, float* xc, long long n, int D, hipStream_t s);
hipError_t launch_lane_ln(const float* x, long long xs, const float* gam, const float* bet, float* out, long long os,
                          long long rows, int D, float eps, hipStream_t s);
// out[n,N] (fp32) = A[n,K] W[N,K]^T + bias, then + resid (fp32) or, with gelu, gelu(.).  A: fp32, or bf16 with a_bf16;
// W: bf16.  copy (may be null): bf16 copy of the result rows (row stride ldcopy), residual mode only.
hipError_t launch_lane_gemm(bool gelu, bool a_bf16, const void* A, long long lda, const void* W, long long ldw, long long n,
                            int N, int K, const float* bias, const float* resid, long long ldr, float* out, long long ldc,
                            void* copy, long long ldcopy, hipStream_t s);

// theta, m, v updated in place (fp32, n elements); step counts from 1
hipError_t launch_adamw(float* theta, const float* g, float* m, float* v, size_t n, long long step, float lr, float b1,
                        float b2, float eps, float wd, hipStream_t s);
// matrix-core backward over the rows (bf16 path, D = 384, M_h = 128 or 256 = two halves of 128 gate units): per half
// Dp [N][256] bf16 (dpV | dpU of its units) and csp [pool_bwd_mfma_blocks][128] partial sums of da t s (dw), half after
// half; Hb16 [N][D] bf16 feature copy; writes p.G.  p.vub must have room for two bf16 copies of [V;U] (plain and
// transposed).
bool pool_bwd_mfma_ok(const PoolArgs& p);
int pool_bwd_mfma_blocks(const PoolArgs& p);
hipError_t launch_pool_bwd_mfma(const PoolArgs& p, void* Dp, void* Hb16, float* csp, hipStream_t s);

}  // namespace sl
