// libslide: C ABI, parameter layout, arena carving and the launch sequence of one slide step.
#include "../../include/slide.h"
#include "../../include/slide_prof.h"
#include "slide_internal.h"
#include "run_internal.h"

#include <string>
#include <vector>
#include <mutex>
#include <cstring>
#include <cstdio>

using namespace sl;

// Work space of mil_pool_fwd_static: one copy per device, part of the loaded code object (nothing is allocated for
// it at run time).  Host code never uses this name as an address: it asks the runtime for the device address once
// per device (static_scratch below) and passes that pointer on.
static __device__ __align__(256) unsigned char scratch[SLIDE_STATIC_POOL_BYTES];

thread_local int sl::g_last_hip = 0;

namespace {

// device address of `scratch` on the current device (looked up on the first call per device), or null with *err set
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

void* static_scratch(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    *err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

enum KernelId {
  K_GEMM_NT = 0, K_GEMM_TN, K_ATTN_FWD, K_ATTN_BWD, K_LN_FWD, K_LN_BWD, K_COLSUM, K_POOL_FWD, K_POOL_BWD,
  K_ELEMWISE, K_CLS_LANE, K_COUNT
};
const char* const kKernelNames[K_COUNT] = {
  "gemm_nt", "gemm_tn", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd", "colsum", "pool_fwd", "pool_bwd", "elementwise",
  "cls_lane"};

struct Tensor { std::string name; size_t off, len; };

struct LayerOff { size_t ln1g, ln1b, qkvW, qkvb, projW, projb, ln2g, ln2b, fc1W, fc1b, fc2W, fc2b; };

// shadow copies (element offsets inside the shadow region, in T elements)
struct ShadowMat { size_t w, wt; int R, C; size_t poff; };

struct Layout {
  size_t total = 0;
  // pool
  size_t p_a, p_part, p_scal, p_Dp, p_tn, p_cs, p_vub, p_H, p_G, pool_end;
  // shared reduction work space
  size_t w_wpart, w_cpart, w_lnpart;
  // encoder
  size_t enc_begin;
  size_t e_patches, e_x, e_qkv, e_O, e_lse, e_xmid, e_m;              // first instance
  size_t e_postab;                                                    // [T, D] rows the patch embedding adds (bf16 path)
  size_t e_dl;                                                        // [n][H][T] fp32 work space of the attention backward
  size_t s_x, s_qkv, s_O, s_lse, s_xmid, s_m, s_a;                    // per-layer strides (0 when not saved)
  size_t e_u1, e_u2, s_u1, s_u2;                                          // LayerNorm outputs of a block (inputs of its QKV / fc1 GEMMs)
  size_t e_a, e_dm, e_dxA, e_dxB, e_dxAt, e_dxBt, e_du, e_dqkv;
  // fp32 lane of the CLS rows: stream at the input of every block and behind the last [L + 1][n][D] (stride s_xc),
  // and one instance each of the stream behind the attention half, its LayerNorm and the MLP activation
  size_t l_xc, s_xc, l_xcm, l_u2c, l_ac;
};

}  // namespace

struct slide_ctx {
  slide_config cfg;
  int g, g2, T, D, F, Kp, dh, L, H, Mh, C, dt;
  std::vector<Tensor> tensors;
  size_t n_params = 0;
  size_t o_peW, o_peb, o_cls, o_pos, o_lnfg, o_lnfb, o_VW, o_Vb, o_UW, o_Ub, o_w, o_cW, o_cb;
  std::vector<LayerOff> lo;
  std::vector<ShadowMat> sh;  // 0 = pe.W, then per layer qkv, proj, fc1, fc2
  size_t shadow_bytes = 0;
  size_t max_w = 0;  // largest weight matrix (elements)
  const float* params = nullptr;
  float* grads = nullptr;
  char* arena = nullptr;
  size_t arena_bytes = 0;
  // state
  bool enc_saved = false;     // activations of enc_n tiles are in the arena
  long long enc_n = 0;
  Layout enc_layout;
  bool step_saved = false;    // slide_step_fwd state (features in arena, label)
  int step_label = 0;
  bool use_mfma = true;
  bool use_lane = false;      // bf16 path: the CLS rows' stream and row-wise work are repeated in fp32 (cls_lane.hip)
  bool pool_only = false;     // aggregator of another encoder family: only mil.* / head.* exist, encoder calls are refused
  Prof prof;
};

namespace {

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t add_tensor(slide_ctx* c, const std::string& name, size_t len) {
  size_t off = c->n_params;
  c->tensors.push_back({name, off, len});
  c->n_params += len;
  return off;
}

void add_shadow(slide_ctx* c, size_t poff, int R, int Cc) {
  ShadowMat m;
  m.R = R; m.C = Cc; m.poff = poff;
  size_t e = elem_size(c->dt);
  size_t n = (size_t)R * Cc;
  m.w = c->shadow_bytes;
  if (c->dt == DT_BF16) c->shadow_bytes += align256(n * e);
  m.wt = c->shadow_bytes;
  c->shadow_bytes += align256(n * e);
  c->sh.push_back(m);
  if (n > c->max_w) c->max_w = n;
}

// Carve the arena for an encoder call on n tiles (with or without saved activations) and a
// pool over pool_N rows.  Pure arithmetic; the same inputs always give the same layout.
// keep: 0 = nothing is saved (feature extraction), 1 = every block's activations, 2 = block inputs only
// (one set of block activations is shared by all blocks and re-created in the backward).
enum { KEEP_NONE = 0, KEEP_ALL = 1, KEEP_INPUTS = 2 };

Layout make_layout(const slide_ctx* c, long long n, long long pool_N, int keep) {
  Layout y;
  bool save = keep == KEEP_ALL;      // per-block instances of every saved activation
  bool bwd = keep != KEEP_NONE;      // backward work buffers
  size_t cur = align256(c->shadow_bytes);
  auto take = [&](size_t bytes) { size_t o = cur; cur = align256(cur + bytes); return o; };
  size_t e = elem_size(c->dt), rs = rs_size(c->dt);
  long long PN = pool_N > 0 ? pool_N : 0;
  int D = c->D, Mh = c->Mh, C = c->C;
  y.p_a = take((size_t)PN * 4);
  y.p_part = take((size_t)1024 * (2 + D) * 8);
  y.p_scal = take((size_t)(4 + 2 * C + 3 * D) * 4);
  y.p_Dp = take((size_t)PN * 3 * Mh * 4);
  y.p_tn = take((size_t)64 * 2 * Mh * D * 4);
  y.p_cs = take((size_t)1024 * 3 * Mh * 4);
  y.p_vub = take((size_t)2 * 2 * Mh * D * 2);
  y.p_H = take((size_t)PN * D * 4);
  y.p_G = take((size_t)PN * D * 4);
  y.pool_end = cur;
  long long nn = n > 0 ? n : 0;
  size_t M = (size_t)nn * c->T;
  size_t maxcols = (size_t)(c->F > 3 * D ? c->F : 3 * D);
  size_t tokcols = (size_t)c->T * D;
  y.w_wpart = take((size_t)64 * c->max_w * 4);
  y.w_cpart = take((size_t)128 * (maxcols > tokcols ? maxcols : tokcols) * 4);
  y.w_lnpart = take((size_t)1024 * 2 * D * 4);
  y.enc_begin = cur;
  y.s_xc = align256((size_t)nn * D * 4);
  y.l_xc = take(0); cur += (size_t)(c->L + 1) * y.s_xc;
  y.l_xcm = take((size_t)nn * D * 4);
  y.l_u2c = take((size_t)nn * D * 4);
  y.l_ac = take((size_t)nn * c->F * 4);
  int inst = save ? c->L : (c->L > 0 ? 1 : 0);
  y.e_postab = take((size_t)c->T * D * rs);
  y.e_patches = take((size_t)nn * c->T * c->Kp * e);   // one row per token: the CLS slot is a row of zeros
  y.s_x = bwd ? align256(M * D * rs) : 0;
  y.e_x = take(0);
  cur += (bwd ? (size_t)(c->L + 1) : 1) * align256(M * D * rs);
  y.s_qkv = save ? align256(M * 3 * D * e) : 0;
  y.e_qkv = take(0); cur += (size_t)inst * align256(M * 3 * D * e);
  y.s_O = save ? align256(M * D * e) : 0;
  y.e_O = take(0); cur += (size_t)inst * align256(M * D * e);
  y.s_lse = save ? align256((size_t)nn * c->H * c->T * 4) : 0;
  y.e_lse = take(0); cur += (size_t)inst * align256((size_t)nn * c->H * c->T * 4);
  y.e_dl = take(bwd ? (size_t)nn * c->H * c->T * 4 : 0);
  if (bwd) {
    y.s_xmid = save ? align256(M * D * rs) : 0;
    y.e_xmid = take(0); cur += (size_t)inst * align256(M * D * rs);
  } else {
    y.s_xmid = 0; y.e_xmid = y.e_x;  // residual adds run in place
  }
  const size_t dge = dgelu_elem_size(c->dt);   // gelu'(pre-activation): a float, or a one-byte code on the bf16 path
  y.s_m = save ? align256(M * c->F * dge) : 0;
  y.e_m = take(0); cur += (size_t)inst * align256(M * c->F * dge);
  // the two LayerNorm outputs of a block are kept like its other activations: the weight gradients of the GEMMs
  // behind them need them again, and a LayerNorm backward that re-creates them writes a fifth more than one that
  // does not (+2 D e bytes per token and block)
  y.s_u1 = save ? align256(M * D * e) : 0;
  y.e_u1 = take(0); cur += (size_t)inst * align256(M * D * e);
  y.s_u2 = save ? align256(M * D * e) : 0;
  y.e_u2 = take(0); cur += (size_t)inst * align256(M * D * e);
  size_t abytes = M * c->F * e, pbytes = (size_t)nn * c->g2 * c->Kp * e;
  y.s_a = save ? align256(abytes) : 0;
  y.e_a = take(0); cur += (size_t)inst * align256(abytes);
  if (bwd) {
    y.e_dm = take(abytes > pbytes ? abytes : pbytes);
    y.e_dxA = take(M * D * rs);
    y.e_dxB = take(M * D * rs);
    if (rs != e) { y.e_dxAt = take(M * D * e); y.e_dxBt = take(M * D * e); }
    else { y.e_dxAt = y.e_dxA; y.e_dxBt = y.e_dxB; }
    y.e_du = take(M * D * e);
    y.e_dqkv = take(M * 3 * D * e);
  } else {
    y.e_dm = y.e_dxA = y.e_dxB = y.e_dxAt = y.e_dxBt = y.e_du = y.e_dqkv = 0;
  }
  y.total = cur;
  return y;
}

typedef RunT<slide_ctx> Run;

const void* weight(const slide_ctx* c, int idx) {  // [out][in] in T
  const ShadowMat& m = c->sh[idx];
  return c->dt == DT_F32 ? (const void*)(c->params + m.poff) : (const void*)(c->arena + m.w);
}
const void* weight_t(const slide_ctx* c, int idx) { return c->arena + c->sh[idx].wt; }  // [in][out] in T

void cast_weights(Run& r) {
  slide_ctx* c = r.c;
  for (size_t i = 0; i < c->sh.size(); ++i) {
    const ShadowMat& m = c->sh[i];
    void* w = c->dt == DT_BF16 ? (void*)(c->arena + m.w) : nullptr;
    void* wt = c->arena + m.wt;
    launch(r, K_ELEMWISE, 0, (double)m.R * m.C * (4 + 2 * elem_size(c->dt)),
           [&] { return launch_cast_transpose(c->dt, c->params + m.poff, m.R, m.C, w, wt, r.s); });
  }
}

void gemm_nt(Run& r, const GemmNT& g) {
  size_t e = elem_size(r.c->dt);
  // every operand once: A, B, the output(s), and the residual / saved pre-activation the epilogue reads
  double bytes = (double)g.M * g.K * e + (double)g.N * g.K * e + (double)g.M * g.N * e;
  if (g.epi == EPI_BIAS_RESID) bytes += (double)g.M * g.N * rs_size(r.c->dt);
  if (g.epi == EPI_ROWTAB) bytes += (double)g.rperiod * g.N * rs_size(r.c->dt);
  if (g.epi == EPI_BIAS_GELU || g.epi == EPI_DGELU) bytes += (double)g.M * g.N * dgelu_elem_size(r.c->dt);
  launch(r, K_GEMM_NT, 2.0 * g.M * g.N * g.K, bytes, [&] { return launch_gemm_nt(r.c->dt, g, r.c->use_mfma, r.s); });
}

void colsum(Run& r, int elem, const void* A, long long lda, RowMap map, long long M, int N, float* part, float* out,
            int accumulate);

// dW (+)= A^T B through split partials; optionally also db (+)= column sums of A
void gemm_tn(Run& r, const void* A, long long lda, RowMap amap, const void* B, long long ldb, RowMap bmap, long long M,
             int N1, int N2, float* part, size_t part_floats, float* out, int accumulate, int dt_override = -1,
             float* bias_out = nullptr, float* cpart = nullptr, float* out2 = nullptr, float* bias_out2 = nullptr) {
  // part: room for part_floats floats of slab partials (at least 64 results).
  // out2 / bias_out2: the result rows N1/2 .. N1-1 (and their column sums) belong to a second tensor
  GemmTN g;
  int dt = dt_override >= 0 ? dt_override : r.c->dt;
  g.A = A; g.lda = lda; g.amap = amap; g.B = B; g.ldb = ldb; g.bmap = bmap; g.M = M; g.N1 = N1; g.N2 = N2;
  g.part = part;
  g.cs_part = nullptr;
  g.big = 0;
  size_t fit = part_floats / ((size_t)N1 * N2);
  int bs = (dt == DT_BF16 && r.c->use_mfma) ? gemm_tn_big_slabs(g, fit > 256 ? 256 : (int)fit) : 0;
  if (bs) { g.slabs = bs; g.big = 1; }
  else g.slabs = gemm_tn_pick_slabs(M, N1, N2, 32);
  bool fused = bias_out && gemm_tn_fuses_colsum(dt, g, r.c->use_mfma);
  if (fused) g.cs_part = cpart;
  if (bias_out && !fused) {
    if (bias_out2) {
      colsum(r, dt, A, lda, amap, M, N1 / 2, cpart, bias_out, accumulate);
      colsum(r, dt, (const char*)A + (size_t)(N1 / 2) * elem_size(dt), lda, amap, M, N1 / 2, cpart, bias_out2, accumulate);
    } else {
      colsum(r, dt, A, lda, amap, M, N1, cpart, bias_out, accumulate);
    }
  }
  size_t e = elem_size(dt);
  launch(r, K_GEMM_TN, 2.0 * M * N1 * N2, (double)M * (N1 + N2) * e + (double)g.slabs * N1 * N2 * 4,
         [&] { return launch_gemm_tn(dt, g, r.c->use_mfma, r.s); });
  const long long len = (long long)N1 * N2, len1 = out2 ? len / 2 : len;
  launch(r, K_ELEMWISE, 0, (double)(g.slabs + 1) * len1 * 4,
         [&] { return launch_reduce_partials(part, g.slabs, len, len1, out, accumulate, r.s); });
  if (out2)
    launch(r, K_ELEMWISE, 0, (double)(g.slabs + 1) * len1 * 4,
           [&] { return launch_reduce_partials(part + len1, g.slabs, len, len1, out2, accumulate, r.s); });
  if (fused) {
    const int n1 = bias_out2 ? N1 / 2 : N1;
    launch(r, K_ELEMWISE, 0, 0,
           [&] { return launch_reduce_partials(cpart, g.slabs, N1, n1, bias_out, accumulate, r.s); });
    if (bias_out2)
      launch(r, K_ELEMWISE, 0, 0,
             [&] { return launch_reduce_partials(cpart + n1, g.slabs, N1, n1, bias_out2, accumulate, r.s); });
  }
}

void colsum(Run& r, int elem, const void* A, long long lda, RowMap map, long long M, int N, float* part, float* out,
            int accumulate) {
  int slabs = colsum_slabs(M);
  launch(r, K_COLSUM, 0, (double)M * N * elem_size(elem),
         [&] { return launch_colsum_part(elem, A, lda, map, M, N, part, slabs, r.s); });
  launch(r, K_ELEMWISE, 0, (double)slabs * N * 4,
         [&] { return launch_reduce_partials(part, slabs, N, N, out, accumulate, r.s); });
}

void ln_fwd(Run& r, const void* x, long long xs, const float* g, const float* b, void* out, long long os, long long rows,
            bool out_f32 = false) {
  slide_ctx* c = r.c;
  launch(r, K_LN_FWD, 0, (double)rows * c->D * (rs_size(c->dt) + elem_size(c->dt)),
         [&] { return launch_ln_fwd(c->dt, x, xs, g, b, out, os, rows, c->D, c->cfg.ln_eps, out_f32, r.s); });
}

// u_out: the forward output of this LayerNorm (needed by the weight gradient of the linear map behind it, not kept by
// the forward) is produced as well: by the backward kernel itself where it can, else by a forward launch
void ln_bwd(Run& r, const void* x, long long xs, const void* dy, long long dys, size_t o_gam, size_t o_bet,
            const void* dres, void* dxo, void* dxo_t, long long os, long long rows, float* part, int accumulate,
            bool dy_f32 = false, void* u_out = nullptr, int dres_period = 0) {
  slide_ctx* c = r.c;
  size_t rs = rs_size(c->dt), e = elem_size(c->dt);
  bool emit = u_out && ln_bwd_emits_u(c->dt, x, xs, dy, dys, c->params + o_gam, dres, dxo, os, c->D, dy_f32,
                                      c->params + o_bet, u_out, c->D);
  if (u_out && !emit) ln_fwd(r, x, xs, c->params + o_gam, c->params + o_bet, u_out, c->D, rows);
  double bytes = (double)rows * c->D * (rs + e + (dres && !dres_period ? rs : 0) + rs + (rs != e ? e : 0) + (emit ? e : 0));
  launch(r, K_LN_BWD, 0, bytes, [&] {
    return launch_ln_bwd(c->dt, x, xs, dy, dys, c->params + o_gam, dres, dxo, dxo_t, os, rows, c->D, c->cfg.ln_eps, part,
                         dy_f32, r.s, c->params + o_bet, emit ? u_out : nullptr, c->D, dres_period);
  });
  int slabs = ln_bwd_slabs(rows);
  if (o_bet == o_gam + (size_t)c->D) {   // gain and shift are neighbours in the parameter vector, as in a slab's partials
    launch(r, K_ELEMWISE, 0, 0, [&] {
      return launch_reduce_partials(part, slabs, 2LL * c->D, 2LL * c->D, c->grads + o_gam, accumulate, r.s);
    });
    return;
  }
  launch(r, K_ELEMWISE, 0, 0, [&] {
    return launch_reduce_partials(part, slabs, 2LL * c->D, c->D, c->grads + o_gam, accumulate, r.s);
  });
  launch(r, K_ELEMWISE, 0, 0, [&] {
    return launch_reduce_partials(part + c->D, slabs, 2LL * c->D, c->D, c->grads + o_bet, accumulate, r.s);
  });
}

int check_bound(const slide_ctx* c) {
  if (!c) return SLIDE_EINVAL;
  if (!c->params || !c->grads || !c->arena) return SLIDE_ESTATE;
  return SLIDE_OK;
}

// One transformer block forward: x_in(l) -> x_in(l+1), leaving qkv, O, lse, x_mid, the MLP activation
// a = gelu(m) and gelu'(m) of block l in their (per-block or shared) arena slots.  `replay` (backward of the
// block-inputs-only policy): x_in(l+1) is already stored, so the fc2 GEMM is skipped.
// The last block's output is only read at the CLS rows (final LayerNorm of token 0), so everything of it that
// works row by row - projection, LN2, MLP - runs on those n rows alone (they are rows 0, T, 2T, ... of the token
// matrices: leading dimension T * D), and its attention needs query 0 only.  K and V still need every token, so LN1
// and the QKV GEMM stay dense.  Exact, not an approximation; taken where the attention kernels support it.
bool prune_last_block(const slide_ctx* c) {
  return attn_cls_only_ok(c->dt, c->T, c->dh, c->use_mfma) && rs_size(c->dt) == elem_size(c->dt);
}

// ---- fp32 lane of the CLS rows (bf16 path).  xc(l) is the lane's stream at the input of block l.
float* lane_xc(const slide_ctx* c, const Layout& y, int l) { return (float*)(c->arena + y.l_xc + (size_t)l * y.s_xc); }

// attention half: xcm = xc(l) + O[cls rows] Wo^T + bo, and its rounded copy over the CLS rows of x_mid
void lane_attn_half(Run& r, const Layout& y, int l, long long n, const void* O, void* xmid) {
  slide_ctx* c = r.c;
  if (!c->use_lane) return;
  const int D = c->D;
  const long long TD = (long long)c->T * D;
  const LayerOff& o = c->lo[l];
  float* xcm = (float*)(c->arena + y.l_xcm);
  launch(r, K_CLS_LANE, 2.0 * n * D * D, (double)n * D * 14, [&] {
    return launch_lane_gemm(false, true, O, TD, weight(c, 2 + 4 * l), D, n, D, D, c->params + o.projb, lane_xc(c, y, l), D,
                            xcm, D, xmid, TD, r.s);
  });
}

// MLP half: xc(l+1) = xcm + gelu(LN2(xcm) W1^T + b1) W2^T + b2, and its rounded copy over the CLS rows of x_out
void lane_mlp_half(Run& r, const Layout& y, int l, long long n, void* xout) {
  slide_ctx* c = r.c;
  if (!c->use_lane) return;
  const int D = c->D, F = c->F;
  const long long TD = (long long)c->T * D;
  const LayerOff& o = c->lo[l];
  float* xcm = (float*)(c->arena + y.l_xcm);
  float* u2c = (float*)(c->arena + y.l_u2c);
  float* ac = (float*)(c->arena + y.l_ac);
  launch(r, K_CLS_LANE, 0, (double)n * D * 8, [&] {
    return launch_lane_ln(xcm, D, c->params + o.ln2g, c->params + o.ln2b, u2c, D, n, D, c->cfg.ln_eps, r.s);
  });
  launch(r, K_CLS_LANE, 4.0 * n * D * F, (double)n * (D + F) * 4, [&] {
    return launch_lane_gemm(true, false, u2c, D, weight(c, 3 + 4 * l), D, n, F, D, c->params + o.fc1b, nullptr, 0, ac, F,
                            nullptr, 0, r.s);
  });
  launch(r, K_CLS_LANE, 4.0 * n * D * F, (double)n * (F * 4 + D * 10), [&] {
    return launch_lane_gemm(false, false, ac, F, weight(c, 4 + 4 * l), F, n, D, F, c->params + o.fc2b, xcm, D,
                            lane_xc(c, y, l + 1), D, xout, TD, r.s);
  });
}

void block_fwd(Run& r, const Layout& y, int l, long long n, bool replay) {
  slide_ctx* c = r.c;
  hipStream_t s = r.s;
  char* ar = c->arena;
  int D = c->D, T = c->T, F = c->F, dt = c->dt;
  long long M = n * T;
  const LayerOff& o = c->lo[l];
  char* xin = ar + y.e_x + (size_t)l * y.s_x;
  char* xout = ar + y.e_x + (size_t)(l + 1) * y.s_x;
  char* xmid = ar + y.e_xmid + (size_t)l * y.s_xmid;
  char* qkv = ar + y.e_qkv + (size_t)l * y.s_qkv;
  char* O = ar + y.e_O + (size_t)l * y.s_O;
  float* lse = (float*)(ar + y.e_lse + (size_t)l * y.s_lse);
  char* m = ar + y.e_m + (size_t)l * y.s_m;
  char* u1 = ar + y.e_u1 + (size_t)l * y.s_u1;
  char* u2 = ar + y.e_u2 + (size_t)l * y.s_u2;
  char* a = ar + y.e_a + (size_t)l * y.s_a;
  int wi = 1 + 4 * l;
  ln_fwd(r, xin, D, c->params + o.ln1g, c->params + o.ln1b, u1, D, M);
  {
    GemmNT g{};
    g.A = u1; g.lda = D; g.B = weight(c, wi + 0); g.ldb = D; g.M = M; g.N = 3 * D; g.K = D;
    g.epi = EPI_BIAS; g.bias = c->params + o.qkvb; g.out = qkv; g.ldc = 3 * D;
    gemm_nt(r, g);
  }
  if (l == c->L - 1 && !replay && prune_last_block(c)) {
    long long TD = (long long)T * D;
    launch(r, K_ATTN_FWD, 4.0 * n * c->H * (double)T * c->dh, (double)M * 2 * D * elem_size(dt),
           [&] { return launch_attn_fwd(dt, qkv, O, lse, n, T, c->H, c->dh, c->use_mfma, s, true); });
    {
      GemmNT g{};
      g.A = O; g.lda = TD; g.B = weight(c, wi + 1); g.ldb = D; g.M = n; g.N = D; g.K = D;
      g.epi = EPI_BIAS_RESID; g.bias = c->params + o.projb; g.resid = xin; g.ldr = TD; g.out = xmid; g.ldc = TD;
      gemm_nt(r, g);
    }
    lane_attn_half(r, y, l, n, O, xmid);
    ln_fwd(r, xmid, TD, c->params + o.ln2g, c->params + o.ln2b, u2, D, n);   // compact [n, D]
    {
      GemmNT g{};
      g.A = u2; g.lda = D; g.B = weight(c, wi + 2); g.ldb = D; g.M = n; g.N = F; g.K = D;
      g.epi = EPI_BIAS_GELU; g.bias = c->params + o.fc1b; g.out = a; g.ldc = F; g.out2 = m; g.ldc2 = F;
      gemm_nt(r, g);
    }
    {
      GemmNT g{};
      g.A = a; g.lda = F; g.B = weight(c, wi + 3); g.ldb = F; g.M = n; g.N = D; g.K = F;
      g.epi = EPI_BIAS_RESID; g.bias = c->params + o.fc2b; g.resid = xmid; g.ldr = TD; g.out = xout; g.ldc = TD;
      gemm_nt(r, g);
    }
    lane_mlp_half(r, y, l, n, xout);
    return;
  }
  launch(r, K_ATTN_FWD, 4.0 * n * c->H * (double)T * T * c->dh, (double)M * 4 * D * elem_size(dt),
         [&] { return launch_attn_fwd(dt, qkv, O, lse, n, T, c->H, c->dh, c->use_mfma, s); });
  {
    GemmNT g{};
    g.A = O; g.lda = D; g.B = weight(c, wi + 1); g.ldb = D; g.M = M; g.N = D; g.K = D;
    g.epi = EPI_BIAS_RESID; g.bias = c->params + o.projb; g.resid = xin; g.ldr = D; g.out = xmid; g.ldc = D;
    gemm_nt(r, g);
  }
  lane_attn_half(r, y, l, n, O, xmid);
  ln_fwd(r, xmid, D, c->params + o.ln2g, c->params + o.ln2b, u2, D, M);
  {
    GemmNT g{};
    g.A = u2; g.lda = D; g.B = weight(c, wi + 2); g.ldb = D; g.M = M; g.N = F; g.K = D;
    g.epi = EPI_BIAS_GELU; g.bias = c->params + o.fc1b; g.out = a; g.ldc = F;
    g.out2 = m; g.ldc2 = F;   // m slot: gelu'(pre-activation), all the backward needs of it
    gemm_nt(r, g);
  }
  if (!replay) {
    GemmNT g{};
    g.A = a; g.lda = F; g.B = weight(c, wi + 3); g.ldb = F; g.M = M; g.N = D; g.K = F;
    g.epi = EPI_BIAS_RESID; g.bias = c->params + o.fc2b; g.resid = xmid; g.ldr = D; g.out = xout; g.ldc = D;
    gemm_nt(r, g);
    lane_mlp_half(r, y, l, n, xout);   // a replay only re-creates x_mid: x_in(l + 1) is stored with the lane's row in it
  }
}

// ------------------------------------------------------------------------------------------
// encoder forward
// ------------------------------------------------------------------------------------------
int enc_fwd(slide_ctx* c, const void* pixels, long long n, void* feats_out, bool save, long long pool_N,
            hipStream_t s) {
  if (c->pool_only) return SLIDE_EUNSUPPORTED;
  int keep = !save ? KEEP_NONE : (c->cfg.recompute ? KEEP_INPUTS : KEEP_ALL);
  Layout y = make_layout(c, n, pool_N, keep);
  if (y.total > c->arena_bytes) return SLIDE_EARENA;
  c->enc_saved = false;
  c->step_saved = false;
  Run r{c, s};
  char* ar = c->arena;
  int D = c->D, T = c->T, dt = c->dt;
  cast_weights(r);
  launch(r, K_ELEMWISE, 0, 2.0 * n * 3 * c->cfg.tile * c->cfg.tile * elem_size(dt),
         [&] { return launch_patchify(dt, pixels, ar + y.e_patches, n, c->cfg.tile, c->cfg.patch, s, T - c->g2); });
  // the patch matrix has the token matrix's rows (a row of zeros in each tile's CLS slot): its weight gradient is
  // then a plain product of two row-aligned matrices and runs on the large-M kernel, and so does the forward where
  // that kernel takes the shape: every token row gets its row of a [T, D] table added (bias + position row; class
  // token + position row in the CLS slot, where the product is zero)
  GemmNT gt{};
  gt.A = ar + y.e_patches; gt.lda = c->Kp; gt.B = weight(c, 0); gt.ldb = c->Kp;
  gt.M = n * T; gt.N = D; gt.K = c->Kp;
  gt.epi = EPI_ROWTAB; gt.resid = ar + y.e_postab; gt.ldr = D; gt.rperiod = T;
  gt.out = ar + y.e_x; gt.ldc = D;
  if (dt == DT_BF16 && c->use_mfma && gemm_nt_big_ok(gt)) {
    launch(r, K_ELEMWISE, 0, 0, [&] {
      return launch_pos_table(ar + y.e_postab, c->params + c->o_cls, c->params + c->o_pos, c->params + c->o_peb, T, D, s);
    });
    gemm_nt(r, gt);
  } else {
    GemmNT g{};
    g.A = ar + y.e_patches; g.lda = c->Kp; g.amap = RowMap{c->g2, T};
    g.B = weight(c, 0); g.ldb = c->Kp;
    g.M = n * c->g2; g.N = D; g.K = c->Kp;
    g.epi = EPI_PATCH; g.bias = c->params + c->o_peb; g.pos = c->params + c->o_pos;
    g.out = ar + y.e_x; g.ldc = D; g.cmap = RowMap{c->g2, T};
    gemm_nt(r, g);
    launch(r, K_ELEMWISE, 0, 0,
           [&] { return launch_cls_rows(dt, ar + y.e_x, c->params + c->o_cls, c->params + c->o_pos, n, T, D, s); });
  }
  if (c->use_lane)
    launch(r, K_CLS_LANE, 0, (double)n * D * 4,
           [&] { return launch_lane_init(c->params + c->o_cls, c->params + c->o_pos, lane_xc(c, y, 0), n, D, s); });
  for (int l = 0; l < c->L; ++l) block_fwd(r, y, l, n, false);
  char* xL = ar + y.e_x + (size_t)c->L * y.s_x;
  if (c->use_lane)   // the features are the final LayerNorm of the lane's stream (its rounded copy is the CLS row of xL)
    launch(r, K_CLS_LANE, 0, (double)n * D * 8, [&] {
      return launch_lane_ln(lane_xc(c, y, c->L), D, c->params + c->o_lnfg, c->params + c->o_lnfb, (float*)feats_out, D, n, D,
                            c->cfg.ln_eps, s);
    });
  else
    ln_fwd(r, xL, (long long)T * D, c->params + c->o_lnfg, c->params + c->o_lnfb, feats_out, D, n, true);
  if (r.ok() && save) { c->enc_saved = true; c->enc_n = n; c->enc_layout = y; }
  return finish(r);
}

// ------------------------------------------------------------------------------------------
// encoder backward
// ------------------------------------------------------------------------------------------
int enc_bwd(slide_ctx* c, const void* dfeats, long long n, int accumulate, void* pixel_grad, hipStream_t s) {
  if (c->pool_only) return SLIDE_EUNSUPPORTED;
  if (!c->enc_saved || c->enc_n != n) return SLIDE_ESTATE;
  const Layout& y = c->enc_layout;
  Run r{c, s};
  char* ar = c->arena;
  int D = c->D, T = c->T, F = c->F, dt = c->dt;
  long long M = n * T;
  size_t rs = rs_size(dt), e = elem_size(dt);
  bool dual = rs != e;
  int rs_elem = rs == 4 ? DT_F32 : DT_BF16;
  float* wpart = (float*)(ar + y.w_wpart);
  const size_t wcap = (size_t)64 * c->max_w;   // floats of room behind wpart (make_layout)
  float* cpart = (float*)(ar + y.w_cpart);
  float* lnpart = (float*)(ar + y.w_lnpart);
  char *dxA = ar + y.e_dxA, *dxB = ar + y.e_dxB, *dxAt = ar + y.e_dxAt, *dxBt = ar + y.e_dxBt;
  char *du = ar + y.e_du, *dqkv = ar + y.e_dqkv, *dm = ar + y.e_dm;
  RowMap id{0, 0};
  float* G = c->grads;
  // all token rows of the output gradient start at zero, the CLS rows get the final LayerNorm's backward; where the
  // last block is pruned to its CLS rows nothing reads the other rows before that block's LN1 backward writes them
  const bool pruned = c->L > 0 && prune_last_block(c);
  if (!pruned) {
    launch(r, K_ELEMWISE, 0, (double)M * D * rs, [&] { return launch_fill_zero(dxA, (size_t)M * D * rs, s); });
    if (dual) launch(r, K_ELEMWISE, 0, (double)M * D * e, [&] { return launch_fill_zero(dxAt, (size_t)M * D * e, s); });
  }
  char* xL = ar + y.e_x + (size_t)c->L * y.s_x;
  ln_bwd(r, xL, (long long)T * D, dfeats, D, c->o_lnfg, c->o_lnfb, nullptr, dxA, dxAt, (long long)T * D, n, lnpart,
         accumulate, true);
  for (int l = c->L - 1; l >= 0; --l) {
    const LayerOff& o = c->lo[l];
    char* xin = ar + y.e_x + (size_t)l * y.s_x;
    char* xmid = ar + y.e_xmid + (size_t)l * y.s_xmid;
    char* qkv = ar + y.e_qkv + (size_t)l * y.s_qkv;
    char* O = ar + y.e_O + (size_t)l * y.s_O;
    float* lse = (float*)(ar + y.e_lse + (size_t)l * y.s_lse);
    char* m = ar + y.e_m + (size_t)l * y.s_m;
    char* u1 = ar + y.e_u1 + (size_t)l * y.s_u1;   // LN1(x_in), LN2(x_mid) as the forward (or its re-run) left them
    char* u2 = ar + y.e_u2 + (size_t)l * y.s_u2;
    int wi = 1 + 4 * l;
    // block inputs only were kept: re-create this block's activations in the shared slots (the
    // last block's are still there from the forward)
    if (c->cfg.recompute && l != c->L - 1) block_fwd(r, y, l, n, true);
    char* a = ar + y.e_a + (size_t)l * y.s_a;
    if (l == c->L - 1 && prune_last_block(c)) {
      // the gradient of the last block's output is zero away from the CLS rows: its MLP, LN2 and projection
      // work on those n rows (leading dimension T * D); dxB is zero elsewhere
      long long TD = (long long)T * D;
      // the LN1 backward below adds dxB to every row: it is zero away from the CLS rows, which the kernel can be
      // told (it then reads the CLS rows only); otherwise the buffer is cleared
      const bool periodic = ln_bwd_periodic_ok(dt, xin, D, du, D, c->params + o.ln1g, dxB, dxA, D, D, false);
      if (!periodic)
        launch(r, K_ELEMWISE, 0, (double)M * D * rs, [&] { return launch_fill_zero(dxB, (size_t)M * D * rs, s); });
      {
        GemmNT g{};
        g.A = dxAt; g.lda = TD; g.B = weight_t(c, wi + 3); g.ldb = D; g.M = n; g.N = F; g.K = D;
        g.epi = EPI_DGELU; g.pre = m; g.ldpre = F; g.out = dm; g.ldc = F;
        gemm_nt(r, g);
      }
      gemm_tn(r, dxAt, TD, id, a, F, id, n, D, F, wpart, wcap, G + o.fc2W, accumulate, -1, G + o.fc2b, cpart);
      gemm_tn(r, dm, F, id, u2, D, id, n, F, D, wpart, wcap, G + o.fc1W, accumulate, -1, G + o.fc1b, cpart);
      {
        GemmNT g{};
        g.A = dm; g.lda = F; g.B = weight_t(c, wi + 2); g.ldb = F; g.M = n; g.N = D; g.K = F;
        g.epi = EPI_PLAIN; g.out = du; g.ldc = D;   // compact [n, D]
        gemm_nt(r, g);
      }
      ln_bwd(r, xmid, TD, du, D, o.ln2g, o.ln2b, dxA, dxB, dxBt, TD, n, lnpart, accumulate);
      gemm_tn(r, dxBt, TD, id, O, TD, id, n, D, D, wpart, wcap, G + o.projW, accumulate, -1, G + o.projb, cpart);
      {
        GemmNT g{};
        g.A = dxBt; g.lda = TD; g.B = weight_t(c, wi + 1); g.ldb = D; g.M = n; g.N = D; g.K = D;
        g.epi = EPI_PLAIN; g.out = du; g.ldc = TD;   // the CLS rows of dO; the attention backward reads no other
        gemm_nt(r, g);
      }
      launch(r, K_ATTN_BWD, 10.0 * n * c->H * (double)T * c->dh, (double)M * 7 * D * e,
             [&] { return launch_attn_bwd(dt, qkv, O, lse, du, dqkv, n, T, c->H, c->dh, c->use_mfma, s, true, (float*)(ar + y.e_dl)); });
      gemm_tn(r, dqkv, 3 * D, id, u1, D, id, M, 3 * D, D, wpart, wcap, G + o.qkvW, accumulate, -1, G + o.qkvb, cpart);
      {
        GemmNT g{};
        g.A = dqkv; g.lda = 3 * D; g.B = weight_t(c, wi + 0); g.ldb = 3 * D; g.M = M; g.N = D; g.K = 3 * D;
        g.epi = EPI_PLAIN; g.out = du; g.ldc = D;
        gemm_nt(r, g);
      }
      ln_bwd(r, xin, D, du, D, o.ln1g, o.ln1b, dxB, dxA, dxAt, D, M, lnpart, accumulate, false, nullptr, periodic ? T : 0);
      continue;
    }
    // ---- MLP half: x_out = x_mid + gelu(LN2(x_mid) W1^T + b1) W2^T + b2
    {  // dm = (dx W2) * gelu'(m), gelu'(m) as stored by the forward
      GemmNT g{};
      g.A = dxAt; g.lda = D; g.B = weight_t(c, wi + 3); g.ldb = D; g.M = M; g.N = F; g.K = D;
      g.epi = EPI_DGELU; g.pre = m; g.ldpre = F; g.out = dm; g.ldc = F;
      gemm_nt(r, g);
    }
    gemm_tn(r, dxAt, D, id, a, F, id, M, D, F, wpart, wcap, G + o.fc2W, accumulate, -1, G + o.fc2b, cpart);
    {
      GemmNT g{};
      g.A = dm; g.lda = F; g.B = weight_t(c, wi + 2); g.ldb = F; g.M = M; g.N = D; g.K = F;
      g.epi = EPI_PLAIN; g.out = du; g.ldc = D;
      gemm_nt(r, g);
    }
    ln_bwd(r, xmid, D, du, D, o.ln2g, o.ln2b, dxA, dxB, dxBt, D, M, lnpart, accumulate);
    gemm_tn(r, dm, F, id, u2, D, id, M, F, D, wpart, wcap, G + o.fc1W, accumulate, -1, G + o.fc1b, cpart);
    // ---- attention half: x_mid = x_in + attn(LN1(x_in)) Wo^T + bo
    gemm_tn(r, dxBt, D, id, O, D, id, M, D, D, wpart, wcap, G + o.projW, accumulate, -1, G + o.projb, cpart);
    {
      GemmNT g{};
      g.A = dxBt; g.lda = D; g.B = weight_t(c, wi + 1); g.ldb = D; g.M = M; g.N = D; g.K = D;
      g.epi = EPI_PLAIN; g.out = du; g.ldc = D;
      gemm_nt(r, g);
    }
    launch(r, K_ATTN_BWD, 10.0 * n * c->H * (double)T * T * c->dh, (double)M * 9 * D * e,
           [&] { return launch_attn_bwd(dt, qkv, O, lse, du, dqkv, n, T, c->H, c->dh, c->use_mfma, s, false, (float*)(ar + y.e_dl)); });
    {
      GemmNT g{};
      g.A = dqkv; g.lda = 3 * D; g.B = weight_t(c, wi + 0); g.ldb = 3 * D; g.M = M; g.N = D; g.K = 3 * D;
      g.epi = EPI_PLAIN; g.out = du; g.ldc = D;
      gemm_nt(r, g);
    }
    ln_bwd(r, xin, D, du, D, o.ln1g, o.ln1b, dxB, dxA, dxAt, D, M, lnpart, accumulate);
    gemm_tn(r, dqkv, 3 * D, id, u1, D, id, M, 3 * D, D, wpart, wcap, G + o.qkvW, accumulate, -1, G + o.qkvb, cpart);
  }
  // ---- token assembly: x0[n,0] = cls + pos[0]; x0[n,1+j] = patch_j W_pe^T + b_pe + pos[1+j]
  {
    long long cols = (long long)T * D;
    int slabs = colsum_slabs(n);
    launch(r, K_COLSUM, 0, (double)M * D * rs,
           [&] { return launch_colsum_part(rs_elem, dxA, cols, id, n, (int)cols, cpart, slabs, s); });
    launch(r, K_ELEMWISE, 0, 0,
           [&] { return launch_reduce_partials(cpart, slabs, cols, cols, G + c->o_pos, accumulate, s); });
    launch(r, K_ELEMWISE, 0, 0,
           [&] { return launch_reduce_partials(cpart, slabs, cols, D, G + c->o_cls, accumulate, s); });
    // the patch-embedding bias sees every patch token: its gradient is this step's position gradient summed over the
    // patch positions (rows 1 .. T - 1), taken from the same partial sums
    launch(r, K_ELEMWISE, 0, 0, [&] { return launch_reduce_partials(cpart, slabs, cols, cols, wpart, 0, s); });
    launch(r, K_ELEMWISE, 0, 0,
           [&] { return launch_reduce_partials(wpart + D, T - 1, D, D, G + c->o_peb, accumulate, s); });
  }
  RowMap pm{c->g2, T};
  long long Mp = n * c->g2;
  // all token rows: the CLS rows meet rows of zeros in the patch matrix
  gemm_tn(r, dxAt, D, id, ar + y.e_patches, c->Kp, id, M, D, c->Kp, wpart, wcap, G + c->o_peW, accumulate);
  if (pixel_grad) {
    GemmNT g{};
    g.A = dxAt; g.lda = D; g.amap = pm; g.B = weight_t(c, 0); g.ldb = D; g.M = Mp; g.N = c->Kp; g.K = D;
    g.epi = EPI_PLAIN; g.out = dm; g.ldc = c->Kp;
    gemm_nt(r, g);
    launch(r, K_ELEMWISE, 0, 2.0 * Mp * c->Kp * e,
           [&] { return launch_unpatchify(dt, dm, pixel_grad, n, c->cfg.tile, c->cfg.patch, s); });
  }
  return finish(r);
}

// ------------------------------------------------------------------------------------------
// pool
// ------------------------------------------------------------------------------------------
PoolArgs pool_args(slide_ctx* c, const Layout& y, const void* feats, long long N, int label) {
  PoolArgs p{};
  char* ar = c->arena;
  p.H = (const float*)feats; p.N = N; p.D = c->D; p.Mh = c->Mh; p.C = c->C; p.label = label;
  p.VW = c->params + c->o_VW; p.Vb = c->params + c->o_Vb; p.UW = c->params + c->o_UW; p.Ub = c->params + c->o_Ub;
  p.w = c->params + c->o_w; p.cW = c->params + c->o_cW; p.cb = c->params + c->o_cb;
  p.a = (float*)(ar + y.p_a); p.part = (double*)(ar + y.p_part); p.scal = (float*)(ar + y.p_scal);
  p.blocks = pool_blocks(N);
  p.grads = c->grads; p.ocW = c->o_cW; p.ocb = c->o_cb;
  p.vub = ar + y.p_vub; p.use_mfma = c->use_mfma && c->dt == DT_BF16;
  p.a_tmp = (float*)(ar + y.p_Dp);   // the backward's work space is idle during the forward
  return p;
}

int pool_fwd(slide_ctx* c, const Layout& y, const void* feats, long long N, int label, float* loss, float* logits,
             float* alpha, hipStream_t s) {
  Run r{c, s};
  PoolArgs p = pool_args(c, y, feats, N, label);
  p.loss = loss; p.logits = logits; p.alpha = alpha;
  launch(r, K_POOL_FWD, 4.0 * N * c->D * c->Mh, (double)N * c->D * 4, [&] { return launch_pool_fwd(p, s); });
  return finish(r);
}

int pool_bwd(slide_ctx* c, const Layout& y, const void* feats, long long N, int label, void* G, int accumulate,
             hipStream_t s) {
  Run r{c, s};
  char* ar = c->arena;
  PoolArgs p = pool_args(c, y, feats, N, label);
  p.G = (float*)G; p.accumulate = accumulate;
  int D = c->D, Mh = c->Mh;
  launch(r, K_POOL_FWD, 4.0 * N * D * Mh, (double)N * D * 4, [&] { return launch_pool_fwd(p, s); });
  char* Dp = ar + y.p_Dp;
  RowMap id{0, 0};
  float* tn = (float*)(ar + y.p_tn);
  // room for 64 results of [2 M_h, D]; the column-sum partials behind it are laid out for 64 slabs, so a
  // weight gradient of half the gate units must not take more either
  const size_t tncap = (size_t)64 * (2 * Mh >= 256 ? 256 : 2 * Mh) * D;
  float* cs = (float*)(ar + y.p_cs);
  // the matrix-core path keeps [dpV dpU] and a feature copy as bf16 in the room of the fp32 [N, 3 Mh] array; db_V and
  // db_U come out of the weight-gradient GEMM as column sums of its first operand
  if (pool_bwd_mfma_ok(p) && (size_t)(2 * Mh + D) * 2 <= (size_t)3 * Mh * 4) {
    // M_h = 256 runs as two halves of 128 gate units: Dp is then [2][N][256], the dw partials [2][blocks][128]
    const int MHK = 128, halves = Mh / MHK;
    char* Hb16 = Dp + (size_t)N * 2 * Mh * 2;
    float* csw = cs + (size_t)64 * 2 * MHK;   // behind the column-sum partials of the GEMM (at most 64 slabs)
    int blocks = pool_bwd_mfma_blocks(p);
    launch(r, K_POOL_BWD, 12.0 * N * D * Mh, 2.0 * N * D * 4, [&] { return launch_pool_bwd_mfma(p, Dp, Hb16, csw, s); });
    launch(r, K_ELEMWISE, 0, 0, [&] { return launch_pool_head_grads(p, s); });
    for (int h = 0; h < halves; ++h) {
      launch(r, K_ELEMWISE, 0, 0, [&] {
        return launch_reduce_partials(csw + (size_t)h * blocks * MHK, blocks, MHK, MHK, c->grads + c->o_w + h * MHK,
                                      accumulate, s);
      });
      const size_t ow = (size_t)h * MHK * D;
      gemm_tn(r, Dp + (size_t)h * N * 2 * MHK * 2, 2 * MHK, id, Hb16, D, id, N, 2 * MHK, D, tn, tncap, c->grads + c->o_VW + ow,
              accumulate, DT_BF16, c->grads + c->o_Vb + h * MHK, cs, c->grads + c->o_UW + ow, c->grads + c->o_Ub + h * MHK);
    }
    return finish(r);
  }
  launch(r, K_POOL_BWD, 8.0 * N * D * Mh, 2.0 * N * D * 4, [&] { return launch_pool_bwd_rows(p, (float*)Dp, s); });
  gemm_tn(r, Dp, 3 * Mh, id, feats, D, id, N, Mh, D, tn, tncap, c->grads + c->o_VW, accumulate, DT_F32);
  gemm_tn(r, Dp + (size_t)Mh * 4, 3 * Mh, id, feats, D, id, N, Mh, D, tn, tncap, c->grads + c->o_UW, accumulate, DT_F32);
  int slabs = colsum_slabs(N);
  launch(r, K_COLSUM, 0, (double)N * 3 * Mh * 4,
         [&] { return launch_colsum_part(DT_F32, Dp, 3 * Mh, id, N, 3 * Mh, cs, slabs, s); });
  launch(r, K_ELEMWISE, 0, 0,
         [&] { return launch_reduce_partials(cs, slabs, 3 * Mh, Mh, c->grads + c->o_Vb, accumulate, s); });
  launch(r, K_ELEMWISE, 0, 0,
         [&] { return launch_reduce_partials(cs + Mh, slabs, 3 * Mh, Mh, c->grads + c->o_Ub, accumulate, s); });
  launch(r, K_ELEMWISE, 0, 0,
         [&] { return launch_reduce_partials(cs + 2 * Mh, slabs, 3 * Mh, Mh, c->grads + c->o_w, accumulate, s); });
  return finish(r);
}

}  // namespace

// A context that holds the aggregator alone (tensors mil.V.W, mil.V.b, mil.U.W, mil.U.b, mil.w, head.W, head.b in
// this order from offset 0): the other encoder families run mil_pool_fwd / mil_pool_bwd on it over their own features.
int sl::pool_ctx_create(int D, int Mh, int C, int dt, slide_ctx** out) {
  if (!out) return SLIDE_EINVAL;
  *out = nullptr;
  if (D <= 0 || Mh <= 0 || C <= 0 || (dt != DT_F32 && dt != DT_BF16)) return SLIDE_EINVAL;
  if (D > 2048 || C > 64 || Mh > 1024) return SLIDE_EUNSUPPORTED;   // 8 feature rows + gate rows must fit the LDS
  slide_ctx* c = new (std::nothrow) slide_ctx();
  if (!c) return SLIDE_EINVAL;
  c->cfg = slide_config{};
  c->cfg.dim = D; c->cfg.mil_hidden = Mh; c->cfg.n_classes = C; c->cfg.dtype = dt;
  c->g = 0; c->g2 = 0; c->T = 1; c->D = D; c->F = D; c->Kp = 0; c->dh = D; c->L = 0; c->H = 1;
  c->Mh = Mh; c->C = C; c->dt = dt;
  c->pool_only = true;
  c->o_VW = add_tensor(c, "mil.V.W", (size_t)Mh * D);
  c->o_Vb = add_tensor(c, "mil.V.b", Mh);
  c->o_UW = add_tensor(c, "mil.U.W", (size_t)Mh * D);
  c->o_Ub = add_tensor(c, "mil.U.b", Mh);
  c->o_w = add_tensor(c, "mil.w", Mh);
  c->o_cW = add_tensor(c, "head.W", (size_t)C * D);
  c->o_cb = add_tensor(c, "head.b", C);
  c->max_w = (size_t)Mh * D;
  c->use_mfma = true;
  c->use_lane = false;
  *out = c;
  return SLIDE_OK;
}

// ============================================================================================
// C ABI
// ============================================================================================
extern "C" {

int slide_ctx_create(const slide_config* cfg, slide_ctx** out) {
  if (!cfg || !out) return SLIDE_EINVAL;
  *out = nullptr;
  if (cfg->tile <= 0 || cfg->patch <= 0 || cfg->tile % cfg->patch) return SLIDE_EINVAL;
  if (cfg->dim <= 0 || cfg->heads <= 0 || cfg->dim % cfg->heads) return SLIDE_EINVAL;
  if (cfg->layers < 0 || cfg->mlp_ratio <= 0 || cfg->mil_hidden <= 0 || cfg->n_classes <= 0) return SLIDE_EINVAL;
  if (cfg->dtype != DT_F32 && cfg->dtype != DT_BF16) return SLIDE_EINVAL;
  if (!(cfg->ln_eps > 0.f)) return SLIDE_EINVAL;
  int dh = cfg->dim / cfg->heads;
  int g = cfg->tile / cfg->patch;
  int T = g * g + 1;
  if (dh != 8 && dh != 32 && dh != 64) return SLIDE_EUNSUPPORTED;
  if (cfg->dim > 1024 || cfg->n_classes > 64 || cfg->mil_hidden > 1024) return SLIDE_EUNSUPPORTED;
  if (attn_lds_bytes(T, dh) > 160 * 1024) return SLIDE_EUNSUPPORTED;
  if (cfg->recompute != 0 && cfg->recompute != 1) return SLIDE_EINVAL;
  if (cfg->reserved != 0) return SLIDE_EINVAL;
  slide_ctx* c = new (std::nothrow) slide_ctx();
  if (!c) return SLIDE_EINVAL;
  c->cfg = *cfg;
  c->g = g; c->g2 = g * g; c->T = T; c->D = cfg->dim; c->F = cfg->mlp_ratio * cfg->dim;
  c->Kp = 3 * cfg->patch * cfg->patch; c->dh = dh; c->L = cfg->layers; c->H = cfg->heads;
  c->Mh = cfg->mil_hidden; c->C = cfg->n_classes; c->dt = cfg->dtype;
  size_t D = c->D, F = c->F;
  c->o_peW = add_tensor(c, "pe.W", D * c->Kp);
  c->o_peb = add_tensor(c, "pe.b", D);
  c->o_cls = add_tensor(c, "cls", D);
  c->o_pos = add_tensor(c, "pos", (size_t)T * D);
  add_shadow(c, c->o_peW, (int)D, c->Kp);
  for (int l = 0; l < c->L; ++l) {
    std::string p = "l" + std::to_string(l) + ".";
    LayerOff o;
    o.ln1g = add_tensor(c, p + "ln1.g", D);
    o.ln1b = add_tensor(c, p + "ln1.b", D);
    o.qkvW = add_tensor(c, p + "qkv.W", 3 * D * D);
    o.qkvb = add_tensor(c, p + "qkv.b", 3 * D);
    o.projW = add_tensor(c, p + "proj.W", D * D);
    o.projb = add_tensor(c, p + "proj.b", D);
    o.ln2g = add_tensor(c, p + "ln2.g", D);
    o.ln2b = add_tensor(c, p + "ln2.b", D);
    o.fc1W = add_tensor(c, p + "fc1.W", F * D);
    o.fc1b = add_tensor(c, p + "fc1.b", F);
    o.fc2W = add_tensor(c, p + "fc2.W", D * F);
    o.fc2b = add_tensor(c, p + "fc2.b", D);
    c->lo.push_back(o);
    add_shadow(c, o.qkvW, (int)(3 * D), (int)D);
    add_shadow(c, o.projW, (int)D, (int)D);
    add_shadow(c, o.fc1W, (int)F, (int)D);
    add_shadow(c, o.fc2W, (int)D, (int)F);
  }
  c->o_lnfg = add_tensor(c, "lnf.g", D);
  c->o_lnfb = add_tensor(c, "lnf.b", D);
  c->o_VW = add_tensor(c, "mil.V.W", (size_t)c->Mh * D);
  c->o_Vb = add_tensor(c, "mil.V.b", c->Mh);
  c->o_UW = add_tensor(c, "mil.U.W", (size_t)c->Mh * D);
  c->o_Ub = add_tensor(c, "mil.U.b", c->Mh);
  c->o_w = add_tensor(c, "mil.w", c->Mh);
  c->o_cW = add_tensor(c, "head.W", (size_t)c->C * D);
  c->o_cb = add_tensor(c, "head.b", c->C);
  if ((size_t)c->Mh * D > c->max_w) c->max_w = (size_t)c->Mh * D;
  c->use_mfma = true;
  c->use_lane = c->dt == DT_BF16 && cls_lane_ok(c->D, c->F);
  *out = c;
  return SLIDE_OK;
}

void slide_ctx_destroy(slide_ctx* c) {
  if (!c) return;
  prof_destroy(c->prof);
  delete c;
}

size_t slide_param_count(const slide_ctx* c) { return c ? c->n_params : 0; }
int slide_param_tensors(const slide_ctx* c) { return c ? (int)c->tensors.size() : 0; }

int slide_param_name(const slide_ctx* c, int index, char* name_out, size_t name_cap, size_t* offset, size_t* length) {
  if (!c || index < 0 || index >= (int)c->tensors.size()) return SLIDE_EINVAL;
  const Tensor& t = c->tensors[index];
  if (name_out) {
    if (name_cap < t.name.size() + 1) return SLIDE_EINVAL;
    memcpy(name_out, t.name.c_str(), t.name.size() + 1);
  }
  if (offset) *offset = t.off;
  if (length) *length = t.len;
  return SLIDE_OK;
}

int slide_param_offset(const slide_ctx* c, const char* name, size_t* offset, size_t* length) {
  if (!c || !name) return SLIDE_EINVAL;
  for (const Tensor& t : c->tensors)
    if (t.name == name) {
      if (offset) *offset = t.off;
      if (length) *length = t.len;
      return SLIDE_OK;
    }
  return SLIDE_EINVAL;
}

size_t slide_arena_bytes(const slide_ctx* c, int64_t n_tiles) {
  if (!c || n_tiles <= 0) return 0;
  return make_layout(c, n_tiles, n_tiles, c->cfg.recompute ? KEEP_INPUTS : KEEP_ALL).total;
}

size_t slide_pool_arena_bytes(const slide_ctx* c, int64_t N) {
  if (!c || N <= 0) return 0;
  return make_layout(c, 0, N, KEEP_NONE).pool_end;
}

int slide_bind(slide_ctx* c, const float* params, float* grads, void* arena, size_t arena_bytes) {
  if (!c || !params || !grads || !arena) return SLIDE_EINVAL;
  if (((uintptr_t)arena & 255) != 0) return SLIDE_EINVAL;
  c->params = params; c->grads = grads; c->arena = (char*)arena; c->arena_bytes = arena_bytes;
  c->enc_saved = false; c->step_saved = false;
  return SLIDE_OK;
}

int encoder_fwd_tiles(slide_ctx* c, const void* pixels, int64_t n, void* feats_out, int save, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!pixels || !feats_out || n <= 0) return SLIDE_EINVAL;
  return enc_fwd(c, pixels, n, feats_out, save != 0, n, (hipStream_t)stream);
}

int encoder_bwd_tiles(slide_ctx* c, const void* dfeats, int64_t n, int accumulate, void* pixel_grad, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!dfeats || n <= 0) return SLIDE_EINVAL;
  return enc_bwd(c, dfeats, n, accumulate, pixel_grad, (hipStream_t)stream);
}

static int pool_check(slide_ctx* c, const void* feats, int64_t N, int32_t label, Layout* y) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!feats || N <= 0) return SLIDE_EINVAL;
  if (label < 0 || label >= (c->C == 1 ? 2 : c->C)) return SLIDE_EINVAL;
  *y = make_layout(c, 0, N, KEEP_NONE);
  if (y->pool_end > c->arena_bytes) return SLIDE_EARENA;
  // a pool over more rows than the saved encoder state was laid out for would overwrite it: its work space then
  // reaches into the encoder part, and already for any N beyond the saved step's it lies over that step's features
  // (the pool part is laid out front to back with sizes that grow with N)
  if (c->enc_saved && y->pool_end > c->enc_layout.enc_begin) { c->enc_saved = false; c->step_saved = false; }
  if (c->step_saved && N > c->enc_n) c->step_saved = false;
  return SLIDE_OK;
}

int mil_pool_fwd(slide_ctx* c, const void* feats, int64_t N, int32_t label, float* loss, float* logits, float* alpha,
                 void* stream) {
  Layout y;
  int rc = pool_check(c, feats, N, label, &y);
  if (rc) return rc;
  return pool_fwd(c, y, feats, N, label, loss, logits, alpha, (hipStream_t)stream);
}

int mil_pool_bwd(slide_ctx* c, const void* feats, int64_t N, int32_t label, void* dfeats_out, int accumulate,
                 void* stream) {
  Layout y;
  int rc = pool_check(c, feats, N, label, &y);
  if (rc) return rc;
  if (!dfeats_out) return SLIDE_EINVAL;
  return pool_bwd(c, y, feats, N, label, dfeats_out, accumulate, (hipStream_t)stream);
}

int mil_pool_fwd_static(const slide_ctx* c, const float* params, const void* feats, int64_t N, int32_t label,
                        float* loss, float* logits, float* alpha, void* stream) {
  if (!c || !params || !feats || N <= 0) return SLIDE_EINVAL;
  if (label < 0 || label >= (c->C == 1 ? 2 : c->C)) return SLIDE_EINVAL;
  if (N > SLIDE_STATIC_POOL_MAX_ROWS) return SLIDE_EARENA;
  // the forward's work space: logits a[N], per-workgroup partials, scalars, the bf16 copy of [V;U], partial logits
  size_t cur = 0;
  auto take = [&](size_t bytes) { size_t o = cur; cur = align256(cur + bytes); return o; };
  const int D = c->D, Mh = c->Mh, C = c->C;
  const size_t o_a = take((size_t)N * 4), o_part = take((size_t)1024 * (2 + D) * 8);
  const size_t o_scal = take((size_t)(4 + 2 * C + 3 * D) * 4), o_vub = take((size_t)2 * 2 * Mh * D * 2);
  const size_t o_tmp = take((size_t)N * 4);
  if (cur > SLIDE_STATIC_POOL_BYTES) return SLIDE_EARENA;
  hipError_t e;
  char* ws = (char*)static_scratch(&e);
  if (!ws) { g_last_hip = (int)e; return SLIDE_EHIP; }
  PoolArgs p{};
  p.H = (const float*)feats; p.N = N; p.D = D; p.Mh = Mh; p.C = C; p.label = label;
  p.VW = params + c->o_VW; p.Vb = params + c->o_Vb; p.UW = params + c->o_UW; p.Ub = params + c->o_Ub;
  p.w = params + c->o_w; p.cW = params + c->o_cW; p.cb = params + c->o_cb;
  p.a = (float*)(ws + o_a); p.part = (double*)(ws + o_part); p.scal = (float*)(ws + o_scal);
  p.blocks = pool_blocks(N);
  p.vub = ws + o_vub; p.use_mfma = c->use_mfma && c->dt == DT_BF16;
  p.a_tmp = (float*)(ws + o_tmp);
  p.loss = loss; p.logits = logits; p.alpha = alpha;
  (void)hipGetLastError();
  e = launch_pool_fwd(p, (hipStream_t)stream);
  if (e != hipSuccess) { g_last_hip = (int)e; return SLIDE_EHIP; }
  return SLIDE_OK;
}

int slide_step_fwd(slide_ctx* c, const void* pixels, int64_t N, int32_t label, float* loss, float* logits,
                   float* alpha, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!pixels || N <= 0) return SLIDE_EINVAL;
  if (label < 0 || label >= (c->C == 1 ? 2 : c->C)) return SLIDE_EINVAL;
  Layout y = make_layout(c, N, N, c->cfg.recompute ? KEEP_INPUTS : KEEP_ALL);
  if (y.total > c->arena_bytes) return SLIDE_EARENA;
  rc = enc_fwd(c, pixels, N, c->arena + y.p_H, true, N, (hipStream_t)stream);
  if (rc) return rc;
  rc = pool_fwd(c, y, c->arena + y.p_H, N, label, loss, logits, alpha, (hipStream_t)stream);
  if (rc) { c->enc_saved = false; return rc; }
  c->step_saved = true;
  c->step_label = label;
  return SLIDE_OK;
}

int slide_step_bwd(slide_ctx* c, int accumulate, void* pixel_grad, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!c->step_saved || !c->enc_saved) return SLIDE_ESTATE;
  const Layout y = c->enc_layout;
  long long N = c->enc_n;
  rc = pool_bwd(c, y, c->arena + y.p_H, N, c->step_label, c->arena + y.p_G, accumulate, (hipStream_t)stream);
  if (rc) return rc;
  rc = enc_bwd(c, c->arena + y.p_G, N, accumulate, pixel_grad, (hipStream_t)stream);
  c->step_saved = false;  // activations are consumed (work buffers were overwritten)
  c->enc_saved = false;
  return rc;
}

size_t slide_chunked_arena_bytes(const slide_ctx* c, int64_t N, int64_t chunk_tiles) {
  if (!c || N <= 0 || chunk_tiles <= 0) return 0;
  if (chunk_tiles > N) chunk_tiles = N;
  return make_layout(c, chunk_tiles, N, c->cfg.recompute ? KEEP_INPUTS : KEEP_ALL).total;
}

int slide_step_chunked(slide_ctx* c, const void* pixels, int64_t N, int64_t chunk_tiles, int32_t label, int accumulate,
                       float* loss, float* logits, float* alpha, void* pixel_grad, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!pixels || N <= 0 || chunk_tiles <= 0) return SLIDE_EINVAL;
  if (label < 0 || label >= (c->C == 1 ? 2 : c->C)) return SLIDE_EINVAL;
  if (chunk_tiles > N) chunk_tiles = N;
  hipStream_t s = (hipStream_t)stream;
  // the pool part of the layout (features H, feature gradients G, pool work space) depends on N only and lies in
  // front of the encoder part, so every chunk call below sees H and G at the same place
  Layout y = make_layout(c, chunk_tiles, N, c->cfg.recompute ? KEEP_INPUTS : KEEP_ALL);
  if (y.total > c->arena_bytes) return SLIDE_EARENA;
  const size_t tile_bytes = (size_t)3 * c->cfg.tile * c->cfg.tile * elem_size(c->dt);
  const size_t row_bytes = (size_t)c->D * 4;
  char* H = c->arena + y.p_H;
  char* G = c->arena + y.p_G;
  // pass 1: features of every tile, nothing kept
  for (int64_t t0 = 0; t0 < N; t0 += chunk_tiles) {
    int64_t n = N - t0 < chunk_tiles ? N - t0 : chunk_tiles;
    rc = enc_fwd(c, (const char*)pixels + t0 * tile_bytes, n, H + t0 * row_bytes, false, N, s);
    if (rc) return rc;
  }
  // aggregator and loss on the whole slide, then the gradient of every feature row
  rc = pool_fwd(c, y, H, N, label, loss, logits, alpha, s);
  if (rc) return rc;
  rc = pool_bwd(c, y, H, N, label, G, accumulate, s);
  if (rc) return rc;
  // pass 2: chunk by chunk, forward again with the activations kept, backward seeded with the chunk's rows of G
  for (int64_t t0 = 0; t0 < N; t0 += chunk_tiles) {
    int64_t n = N - t0 < chunk_tiles ? N - t0 : chunk_tiles;
    rc = enc_fwd(c, (const char*)pixels + t0 * tile_bytes, n, H + t0 * row_bytes, true, N, s);
    if (rc) return rc;
    rc = enc_bwd(c, G + t0 * row_bytes, n, (accumulate || t0 > 0) ? 1 : 0,
                 pixel_grad ? (char*)pixel_grad + t0 * tile_bytes : nullptr, s);
    if (rc) return rc;
  }
  c->enc_saved = false;
  c->step_saved = false;
  return SLIDE_OK;
}

const void* slide_features(const slide_ctx* c) {
  if (!c || !c->arena) return nullptr;
  return c->arena + c->enc_layout.p_H;
}
const void* slide_feature_grads(const slide_ctx* c) {
  if (!c || !c->arena) return nullptr;
  return c->arena + c->enc_layout.p_G;
}

int slide_last_hip_error(void) { return g_last_hip; }

int slide_prof_begin(slide_ctx* c, int kernel_id) {
  if (!c) return SLIDE_EINVAL;
  return prof_begin(c->prof, kernel_id, K_COUNT);
}

int slide_prof_end(slide_ctx* c, double* total_ms, int* launches, double* flops, double* bytes) {
  if (!c) return SLIDE_EINVAL;
  return prof_end(c->prof, total_ms, launches, flops, bytes);
}

int slide_prof_family(const slide_ctx* c, int kernel_id, double* total_ms, int* launches, double* flops, double* bytes) {
  if (!c) return SLIDE_EINVAL;
  return prof_family(c->prof, kernel_id, K_COUNT, total_ms, launches, flops, bytes);
}

int slide_adamw_step(float* params, const float* grads, float* m, float* v, size_t count, int64_t step, float lr,
                     float beta1, float beta2, float eps, float weight_decay, void* stream) {
  if (!params || !grads || !m || !v || count == 0 || step < 1) return SLIDE_EINVAL;
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f)) return SLIDE_EINVAL;
  if (!(lr >= 0.f) || !(eps >= 0.f) || !(weight_decay >= 0.f)) return SLIDE_EINVAL;
  (void)hipGetLastError();   // the launch status below must be this call's, not an older error left on the thread
  hipError_t e = launch_adamw(params, grads, m, v, count, step, lr, beta1, beta2, eps, weight_decay, (hipStream_t)stream);
  if (e != hipSuccess) { g_last_hip = (int)e; return SLIDE_EHIP; }
  return SLIDE_OK;
}

int slide_calib_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return SLIDE_EINVAL;
  hipError_t e = launch_calib_copy(dst, src, bytes, (hipStream_t)stream);
  if (e != hipSuccess) { g_last_hip = (int)e; return SLIDE_EHIP; }
  return SLIDE_OK;
}

const char* slide_kernel_name(int id) { return (id >= 0 && id < K_COUNT) ? kKernelNames[id] : nullptr; }

}  // extern "C"
