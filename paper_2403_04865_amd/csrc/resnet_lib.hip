// libslide, convolutional tile encoders: C ABI of resnet.h, parameter layout, arena carving and the launch sequence of
// one slide step with a ResNet encoder.  The aggregator is the one of slide.h, run through an aggregator-only context.
#include "../../include/resnet.h"
#include "run_internal.h"
#include "resnet_internal.h"

#include <string>
#include <vector>
#include <new>

using namespace sl;

namespace {

enum RKernelId { RK_CONV_FWD = 0, RK_CONV_DGRAD, RK_CONV_WGRAD, RK_BN_STATS, RK_BN_APPLY, RK_BN_BWD, RK_POOLING,
                 RK_ELEMWISE, RK_MIL_POOL, RK_COUNT };
const char* const kRKernelNames[RK_COUNT] = {"conv_fwd", "conv_dgrad", "conv_wgrad", "bn_stats", "bn_apply", "bn_bwd",
                                             "pooling", "elementwise", "mil_pool"};
static_assert(RK_COUNT <= PROF_FAMILIES, "family arrays");

struct Tensor { std::string name; size_t off, len; };

// an activation tensor [n * H * H][C] (bf16): per-tile element count and, once laid out, its arena offset
// bits: one bit per element, set where the stored value is positive (kept for ReLU outputs: the mask of the backward)
struct Act { int H, C; bool relu; size_t off = 0, bits = 0; };

// one convolution with its batch normalisation
struct ConvL {
  int Cin, Cout, K, stride, pad;   // as the network defines it
  int inH, outH;
  size_t oW, og, ob;               // parameter offsets
  int t_src, t_conv;               // activation ids: source rows, convolution output
  // what the kernels see: the stem is a 1x1 convolution with 256 columns read from the padded pixel image
  int kCs, kK, kstride, kpad, kinH;
  int ldk() const { return kK * kK * kCs; }
  bool need_wt;                    // an input gradient is taken through it
  size_t w = 0, wt = 0, stats = 0; // arena offsets
  size_t wf = 0, wtf = 0;          // fragment-order copies (3x3 stride-1 convolutions), 0 = none
};

struct BlockL {
  int nconv;
  int conv[3];
  int down;          // convolution id of the shortcut projection or -1
  int t_in;          // block input
  int t_r[2];        // ReLU outputs between the convolutions
  int t_out;
};

struct RLayout {
  size_t total = 0;
  size_t pool, pool_bytes, H, G, bnpart, tpart, coef, wpart, wpart_bytes, img, parg, gA, gB, gC;
};

}  // namespace

struct resnet_ctx {
  resnet_config cfg;
  int S, D, Mh, C, expansion;
  std::vector<Tensor> tensors;
  size_t n_params = 0, agg_off = 0;
  std::vector<Act> acts;
  std::vector<ConvL> convs;
  std::vector<BlockL> blocks;
  int t_r0, t_p0;              // stem ReLU output, max-pool output
  int Cmax = 0;
  size_t max_act = 0;          // largest activation, elements per tile
  slide_ctx* agg = nullptr;
  const float* params = nullptr;
  float* grads = nullptr;
  char* arena = nullptr;
  size_t arena_bytes = 0;
  bool enc_saved = false, step_saved = false;
  long long enc_n = 0;
  int step_label = 0;
  RLayout lay;
  Prof prof;
};

namespace {

typedef RunT<resnet_ctx> Run;

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

size_t add_tensor(resnet_ctx* c, const std::string& name, size_t len) {
  size_t off = c->n_params;
  c->tensors.push_back({name, off, len});
  c->n_params += len;
  return off;
}

int add_act(resnet_ctx* c, int H, int C, bool relu) {
  c->acts.push_back(Act{H, C, relu});
  size_t e = (size_t)H * H * C;
  if (e > c->max_act) c->max_act = e;
  return (int)c->acts.size() - 1;
}

int add_conv(resnet_ctx* c, const std::string& conv, const std::string& bn, int Cin, int Cout, int K, int stride, int pad,
             int inH, int t_src, bool need_wt) {
  ConvL L{};
  L.Cin = Cin; L.Cout = Cout; L.K = K; L.stride = stride; L.pad = pad; L.inH = inH;
  L.outH = (inH + 2 * pad - K) / stride + 1;
  L.oW = add_tensor(c, conv + ".W", (size_t)Cout * Cin * K * K);
  L.og = add_tensor(c, bn + ".g", Cout);
  L.ob = add_tensor(c, bn + ".b", Cout);
  L.t_src = t_src;
  L.t_conv = add_act(c, L.outH, Cout, false);
  L.kCs = Cin; L.kK = K; L.kstride = stride; L.kpad = pad; L.kinH = inH;
  L.need_wt = need_wt;
  if (Cout > c->Cmax) c->Cmax = Cout;
  c->convs.push_back(L);
  return (int)c->convs.size() - 1;
}

// Arena for n tiles: aggregator work space, H, G, weight copies and statistics, reduction work space, every activation,
// three gradient buffers of the largest activation.  Pure arithmetic; also fills the offsets kept in the context.
RLayout make_layout(resnet_ctx* c, long long n, bool commit) {
  RLayout y;
  size_t cur = 0;
  auto take = [&](size_t bytes) { size_t o = cur; cur = align256(cur + bytes); return o; };
  const size_t nn = n > 0 ? (size_t)n : 0;
  y.pool_bytes = align256(slide_pool_arena_bytes(c->agg, (int64_t)nn));
  y.pool = take(y.pool_bytes);
  y.H = take(nn * c->D * 4);
  y.G = take(nn * c->D * 4);
  size_t wmax = 0;
  for (ConvL& L : c->convs) {
    size_t wb = (size_t)L.Cout * L.ldk() * 2;
    size_t w = take(wb), wt = L.need_wt ? take(wb) : 0, st = take((size_t)4 * L.Cout * 4);
    const bool frag = L.kK == 3 && L.kstride == 1 && L.need_wt;
    size_t wf = frag ? take(wb) : 0, wtf = frag ? take(wb) : 0;
    if (commit) { L.w = w; L.wt = wt; L.stats = st; L.wf = wf; L.wtf = wtf; }
    // partial weight gradients: see wgrad_slabs
    if (wb * 2 > wmax) wmax = wb * 2;   // one slab in fp32
  }
  y.bnpart = take((size_t)4096 * 2 * c->Cmax * 4);
  // per-tile channel sums of a convolution's output: 8 bytes per channel and row tile of at least 128 rows
  size_t tp = 0;
  for (const ConvL& L : c->convs) {
    const size_t rows = nn * L.outH * L.outH, tiles = (rows + 127) / 128;
    if (tiles * L.Cout * 8 > tp) tp = tiles * L.Cout * 8;
  }
  y.tpart = take(tp);
  y.coef = take((size_t)2 * c->Cmax * 4);
  // room for the slab partials of any weight gradient: 1024 slabs of the small ones, at least 16 of the largest
  y.wpart_bytes = (size_t)512 << 20;
  if (y.wpart_bytes < 16 * wmax) y.wpart_bytes = 16 * wmax;
  y.wpart = take(y.wpart_bytes);
  for (Act& a : c->acts) {
    size_t o = take(nn * a.H * a.H * a.C * 2), b = a.relu ? take(nn * a.H * a.H * a.C / 8) : 0;
    if (commit) { a.off = o; a.bits = b; }
  }
  y.img = take(nn * (c->S + 6) * (c->S + 8) * 4 * 2);   // padded pixel image of the stem
  y.parg = take(nn * (c->S / 4) * (c->S / 4) * c->cfg.width);   // winning taps of the max pooling, one byte each
  y.gA = take(nn * c->max_act * 2);
  y.gB = take(nn * c->max_act * 2);
  y.gC = take(nn * c->max_act * 2);
  y.total = cur;
  return y;
}

bf16* act(const resnet_ctx* c, int id) { return (bf16*)(c->arena + c->acts[id].off); }
unsigned char* act_bits(const resnet_ctx* c, int id) { return (unsigned char*)(c->arena + c->acts[id].bits); }
long long rows_of(const resnet_ctx* c, int id, long long n) { return n * c->acts[id].H * c->acts[id].H; }
const float* stats_of(const resnet_ctx* c, int conv) { return (const float*)(c->arena + c->convs[conv].stats); }

bool is_stem(const ConvL& L) { return L.kK != L.K; }

ConvGeom geom_fwd(const ConvL& L) {
  ConvGeom g{};
  g.YO = g.XO = L.outH; g.YS = g.XS = L.kinH; g.KH = g.KW = L.kK; g.stride = L.kstride; g.pad = L.kpad; g.transposed = 0;
  if (is_stem(L)) { g.stem = 1; g.YS = L.inH + 6; g.XS = L.inH + 8; }
  return g;
}

const bf16* conv_src(const resnet_ctx* c, const ConvL& L) {
  return is_stem(L) ? (const bf16*)(c->arena + c->lay.img) : act(c, L.t_src);
}

// algorithmic bytes of a convolution's forward or weight gradient: output (gradient) rows once, source tensor once
double conv_bytes(const resnet_ctx* c, const ConvL& L, long long M, long long n) {
  const double src = is_stem(L) ? (double)n * (c->S + 6) * (c->S + 8) * 4 : (double)n * L.inH * L.inH * L.Cin;
  return ((double)M * L.Cout + src) * 2;
}

void cast_weights(Run& r) {
  resnet_ctx* c = r.c;
  for (const ConvL& L : c->convs) {
    launch(r, RK_ELEMWISE, 0, 0, [&] {
      if (is_stem(L)) return launch_stem_cast_w(c->params + L.oW, L.Cout, (bf16*)(c->arena + L.w), r.s);
      return launch_conv_cast_w(c->params + L.oW, L.Cout, L.kCs, L.kK * L.kK, L.ldk(), (bf16*)(c->arena + L.w),
                                L.need_wt ? (bf16*)(c->arena + L.wt) : nullptr, L.wf ? (bf16*)(c->arena + L.wf) : nullptr,
                                L.wtf ? (bf16*)(c->arena + L.wtf) : nullptr, r.s);
    });
  }
}

// convolution forward + batch statistics of its output
void conv_fwd(Run& r, int id, long long n) {
  resnet_ctx* c = r.c;
  const ConvL& L = c->convs[id];
  ConvNT p{};
  p.src = conv_src(c, L); p.Cs = L.kCs; p.W = (const bf16*)(c->arena + L.w);
  p.Wf = L.wf ? (const bf16*)(c->arena + L.wf) : nullptr;
  p.out = act(c, L.t_conv); p.N = L.Cout; p.M = rows_of(c, L.t_conv, n); p.g = geom_fwd(L); p.add = 0;
  p.stat_part = (float*)(c->arena + c->lay.tpart);
  const double K = (double)L.Cin * L.K * L.K;
  launch(r, RK_CONV_FWD, 2.0 * p.M * L.Cout * K, conv_bytes(c, L, p.M, n),
         [&] { return launch_conv_nt(p, r.s); });
  // the statistics come from the per-tile sums the convolution's epilogue left
  const int tiles = conv_nt_row_tiles(p);
  launch(r, RK_BN_STATS, 0, (double)tiles * L.Cout * 8, [&] {
    return launch_bn_stats_tiles(p.stat_part, tiles, p.M, L.Cout, c->params + L.og, c->params + L.ob, c->cfg.bn_eps,
                                 (float*)(c->arena + c->lay.bnpart), (float*)(c->arena + L.stats), r.s);
  });
}

void bn_apply(Run& r, int id, long long n, const bf16* resid, const float* rstats, int t_out) {
  resnet_ctx* c = r.c;
  const ConvL& L = c->convs[id];
  const long long M = rows_of(c, L.t_conv, n);
  launch(r, RK_BN_APPLY, 0, (double)M * L.Cout * 2 * (resid ? 3 : 2),
         [&] {
           return launch_bn_apply(act(c, L.t_conv), M, L.Cout, stats_of(c, id), resid, rstats, 1, act(c, t_out),
                                  act_bits(c, t_out), r.s);
         });
}

// dx (rows of the convolution's output) from dy through ReLU mask and batch normalisation; gain / shift gradients
void bn_bwd(Run& r, int id, long long n, const bf16* dy, const unsigned char* mask, bf16* dx, int accumulate) {
  resnet_ctx* c = r.c;
  const ConvL& L = c->convs[id];
  const long long M = rows_of(c, L.t_conv, n);
  launch(r, RK_BN_BWD, 0, (double)M * L.Cout * (2 * 5 + 0.25), [&] {
    return launch_bn_bwd(dy, mask, act(c, L.t_conv), M, L.Cout, stats_of(c, id), (float*)(c->arena + c->lay.bnpart),
                         (float*)(c->arena + c->lay.coef), c->grads + L.og, c->grads + L.ob, accumulate, dx, r.s);
  });
}

void conv_wgrad(Run& r, int id, long long n, const bf16* dout, int accumulate) {
  resnet_ctx* c = r.c;
  const ConvL& L = c->convs[id];
  ConvWG p{};
  p.dout = dout; p.Co = L.Cout; p.src = conv_src(c, L);
  p.Cs = is_stem(L) ? 64 : L.kCs;   // the stem's 256 columns are four groups of 64 handled like taps
  p.part = (float*)(c->arena + c->lay.wpart);
  p.M = rows_of(c, L.t_conv, n); p.g = geom_fwd(L);
  const long long tiles = (long long)(L.Cout / 64) * (p.Cs / 64);
  long long slabs = (4096 + tiles - 1) / tiles;
  const long long by_rows = (p.M + 255) / 256;
  const long long by_room = (long long)(c->lay.wpart_bytes / ((size_t)L.Cout * L.ldk() * 4));
  if (slabs > by_rows) slabs = by_rows;
  if (slabs > by_room) slabs = by_room;
  if (slabs > 1024) slabs = 1024;
  if (slabs < 1) slabs = 1;
  p.slabs = (int)slabs;
  p.per = ((p.M + slabs - 1) / slabs + 31) / 32 * 32;
  const double K = (double)L.Cin * L.K * L.K;
  launch(r, RK_CONV_WGRAD, 2.0 * p.M * L.Cout * K, conv_bytes(c, L, p.M, n),
         [&] { return launch_conv_wgrad(p, r.s); });
  launch(r, RK_ELEMWISE, 0, 0, [&] {
    if (is_stem(L)) return launch_stem_wgrad_reduce(p.part, p.slabs, L.Cout, c->grads + L.oW, accumulate, r.s);
    return launch_wgrad_reduce(p.part, p.slabs, L.Cout, L.kCs, L.kK * L.kK, L.ldk(), c->grads + L.oW, accumulate, r.s);
  });
}

// gradient with respect to the convolution's source rows; add != 0 adds to what dsrc holds; extra (with mask): also
// adds extra where mask > 0 (the gradient that reaches the block input through an identity shortcut)
void conv_dgrad(Run& r, int id, long long n, const bf16* dout, bf16* dsrc, int add, const bf16* extra = nullptr,
                const unsigned char* mask = nullptr) {
  resnet_ctx* c = r.c;
  const ConvL& L = c->convs[id];
  ConvNT p{};
  p.src = dout; p.Cs = L.Cout; p.W = (const bf16*)(c->arena + L.wt); p.out = dsrc; p.N = L.kCs;
  p.Wf = L.wtf ? (const bf16*)(c->arena + L.wtf) : nullptr;
  p.M = rows_of(c, L.t_src, n);
  p.g.YO = p.g.XO = L.kinH; p.g.YS = p.g.XS = L.outH; p.g.KH = p.g.KW = L.kK; p.g.stride = L.kstride; p.g.pad = L.kpad;
  p.g.transposed = 1;
  p.add = add; p.extra = extra; p.mask = mask;
  const double K = (double)L.Cin * L.K * L.K;
  const double flops = 2.0 * rows_of(c, L.t_conv, n) * L.Cout * K;
  const double bytes = ((double)p.M * L.kCs * (add ? 2 : (extra ? 3 : 1)) + (double)rows_of(c, L.t_conv, n) * L.Cout) * 2;
  if (L.kstride == 2) {
    // one launch per parity class of the input positions: each only sees the taps that reach an output position
    p.M /= 4;
    for (int cls = 1; cls <= 4; ++cls) {
      p.g.cls = cls;
      const int kh0 = (((cls - 1) >> 1) + L.kpad) & 1, kw0 = (((cls - 1) & 1) + L.kpad) & 1;
      const bool no_tap = kh0 >= L.kK || kw0 >= L.kK;
      if (no_tap && add && !extra) continue;   // nothing to add to what is there
      launch(r, RK_CONV_DGRAD, flops / 4, bytes / 4, [&] { return launch_conv_nt(p, r.s); });
    }
    return;
  }
  launch(r, RK_CONV_DGRAD, flops, bytes, [&] { return launch_conv_nt(p, r.s); });
}

int check_bound(const resnet_ctx* c) {
  if (!c) return SLIDE_EINVAL;
  if (!c->params || !c->grads || !c->arena) return SLIDE_ESTATE;
  return SLIDE_OK;
}

int enc_fwd(resnet_ctx* c, const void* pixels, long long n, void* feats_out, hipStream_t s) {
  c->enc_saved = false; c->step_saved = false;
  if (n >= (1LL << 31) / ((long long)(c->S / 2) * (c->S / 2))) return SLIDE_EUNSUPPORTED;   // 32-bit row indices
  c->lay = make_layout(c, n, true);
  if (c->lay.total > c->arena_bytes) return SLIDE_EARENA;
  Run r{c, s};
  cast_weights(r);
  // stem
  launch(r, RK_ELEMWISE, 0, (double)n * (3 * c->S * c->S + 4.0 * (c->S + 6) * (c->S + 8)) * 2,
         [&] { return launch_stem_pad_pixels((const bf16*)pixels, (bf16*)(c->arena + c->lay.img), n, c->S, s); });
  conv_fwd(r, 0, n);
  bn_apply(r, 0, n, nullptr, nullptr, c->t_r0);
  {
    const Act& a = c->acts[c->t_r0];
    launch(r, RK_POOLING, 0, (double)rows_of(c, c->t_r0, n) * a.C * 2 * 1.375,
           [&] {
             return launch_maxpool_fwd(act(c, c->t_r0), act(c, c->t_p0), (unsigned char*)(c->arena + c->lay.parg), n, a.H,
                                       a.H, a.C, s);
           });
  }
  for (const BlockL& b : c->blocks) {
    for (int k = 0; k < b.nconv; ++k) {
      conv_fwd(r, b.conv[k], n);
      if (k + 1 < b.nconv) bn_apply(r, b.conv[k], n, nullptr, nullptr, b.t_r[k]);
    }
    if (b.down >= 0) conv_fwd(r, b.down, n);
    bn_apply(r, b.conv[b.nconv - 1], n, b.down >= 0 ? act(c, c->convs[b.down].t_conv) : act(c, b.t_in),
             b.down >= 0 ? stats_of(c, b.down) : nullptr, b.t_out);
  }
  const int t_last = c->blocks.back().t_out;
  const Act& a = c->acts[t_last];
  launch(r, RK_POOLING, 0, (double)rows_of(c, t_last, n) * a.C * 2,
         [&] { return launch_avgpool_fwd(act(c, t_last), (float*)feats_out, n, a.H * a.H, a.C, s); });
  int rc = finish(r);
  if (rc == SLIDE_OK) { c->enc_saved = true; c->enc_n = n; }
  return rc;
}

int enc_bwd(resnet_ctx* c, const void* dfeats, long long n, int accumulate, hipStream_t s) {
  if (!c->enc_saved || c->enc_n != n) return SLIDE_ESTATE;
  Run r{c, s};
  bf16* gA = (bf16*)(c->arena + c->lay.gA);
  bf16* gB = (bf16*)(c->arena + c->lay.gB);
  bf16* gC = (bf16*)(c->arena + c->lay.gC);
  {
    const int t_last = c->blocks.back().t_out;
    const Act& a = c->acts[t_last];
    launch(r, RK_POOLING, 0, (double)rows_of(c, t_last, n) * a.C * 2,
           [&] { return launch_avgpool_bwd((const float*)dfeats, gA, n, a.H * a.H, a.C, s); });
  }
  for (int bi = (int)c->blocks.size() - 1; bi >= 0; --bi) {
    const BlockL& b = c->blocks[bi];
    const unsigned char* out = act_bits(c, b.t_out);   // where the block's output is positive
    // gA: gradient at the block's output (behind the ReLU)
    bn_bwd(r, b.conv[b.nconv - 1], n, gA, out, gB, accumulate);
    for (int k = b.nconv - 1; k >= 0; --k) {
      conv_wgrad(r, b.conv[k], n, gB, accumulate);
      // the last input gradient of a block with an identity shortcut takes the shortcut's gradient along (one rounding
      // of the sum, no pass of its own)
      if (k == 0 && b.down < 0) conv_dgrad(r, b.conv[k], n, gB, gC, 0, gA, out);
      else conv_dgrad(r, b.conv[k], n, gB, gC, 0);
      if (k > 0) bn_bwd(r, b.conv[k - 1], n, gC, act_bits(c, b.t_r[k - 1]), gB, accumulate);
    }
    // gC: gradient at the block's input through the residual branch; add the shortcut's
    if (b.down >= 0) {
      bn_bwd(r, b.down, n, gA, out, gB, accumulate);
      conv_wgrad(r, b.down, n, gB, accumulate);
      conv_dgrad(r, b.down, n, gB, gC, 1);
    }
    bf16* t = gA; gA = gC; gC = t;
  }
  // stem: max pooling, ReLU + batch normalisation, weight gradient (no pixel gradient)
  {
    const Act& a = c->acts[c->t_r0];
    launch(r, RK_POOLING, 0, (double)rows_of(c, c->t_r0, n) * a.C * 2 * 1.375, [&] {
      return launch_maxpool_bwd((const unsigned char*)(c->arena + c->lay.parg), gA, gB, n, a.H, a.H, a.C, s);
    });
    bn_bwd(r, 0, n, gB, act_bits(c, c->t_r0), gC, accumulate);
    conv_wgrad(r, 0, n, gC, accumulate);
  }
  return finish(r);
}

int agg_bind(resnet_ctx* c) {
  return slide_bind(c->agg, c->params + c->agg_off, c->grads + c->agg_off, c->arena + c->lay.pool, c->lay.pool_bytes);
}

}  // namespace

extern "C" {

int resnet_ctx_create(const resnet_config* cfg, resnet_ctx** out) {
  if (!cfg || !out) return SLIDE_EINVAL;
  *out = nullptr;
  if (cfg->tile <= 0 || cfg->tile % 32 || (cfg->block != 0 && cfg->block != 1)) return SLIDE_EINVAL;
  for (int s = 0; s < 4; ++s)
    if (cfg->depths[s] < 1 || cfg->depths[s] > 64) return SLIDE_EINVAL;
  if (cfg->width <= 0 || cfg->mil_hidden <= 0 || cfg->n_classes <= 0 || !(cfg->bn_eps > 0.f) || cfg->reserved != 0)
    return SLIDE_EINVAL;
  const int exp = cfg->block ? 4 : 1;
  if (cfg->width < 64 || (cfg->width & (cfg->width - 1)) || cfg->width * 8 * exp > 2048) return SLIDE_EUNSUPPORTED;
  resnet_ctx* c = new (std::nothrow) resnet_ctx();
  if (!c) return SLIDE_EINVAL;
  c->cfg = *cfg;
  c->S = cfg->tile; c->expansion = exp; c->D = cfg->width * 8 * exp; c->Mh = cfg->mil_hidden; c->C = cfg->n_classes;
  const int w = cfg->width;
  // stem: the kernels see a 1x1 convolution with 256 columns whose rows are read from the padded pixel image
  add_conv(c, "stem.conv", "stem.bn", 3, w, 7, 2, 3, c->S, -1, false);
  {
    ConvL& L = c->convs[0];
    L.kCs = 256; L.kK = 1; L.kstride = 1; L.kpad = 0; L.kinH = L.outH;
  }
  c->t_r0 = add_act(c, c->S / 2, w, true);
  c->t_p0 = add_act(c, c->S / 4, w, false);
  int t_in = c->t_p0, cin = w, H = c->S / 4;
  for (int s = 0; s < 4; ++s) {
    const int mid = w << s, cout = mid * exp;
    for (int bidx = 0; bidx < cfg->depths[s]; ++bidx) {
      const int stride = (bidx == 0 && s > 0) ? 2 : 1;
      const bool down = stride != 1 || cin != cout;
      const std::string p = "s" + std::to_string(s) + ".b" + std::to_string(bidx) + ".";
      BlockL b{};
      b.t_in = t_in; b.down = -1;
      if (!cfg->block) {
        b.nconv = 2;
        b.conv[0] = add_conv(c, p + "conv1", p + "bn1", cin, mid, 3, stride, 1, H, t_in, true);
        b.t_r[0] = add_act(c, c->convs[b.conv[0]].outH, mid, true);
        b.conv[1] = add_conv(c, p + "conv2", p + "bn2", mid, cout, 3, 1, 1, c->convs[b.conv[0]].outH, b.t_r[0], true);
      } else {
        b.nconv = 3;
        b.conv[0] = add_conv(c, p + "conv1", p + "bn1", cin, mid, 1, 1, 0, H, t_in, true);
        b.t_r[0] = add_act(c, H, mid, true);
        b.conv[1] = add_conv(c, p + "conv2", p + "bn2", mid, mid, 3, stride, 1, H, b.t_r[0], true);
        b.t_r[1] = add_act(c, c->convs[b.conv[1]].outH, mid, true);
        b.conv[2] = add_conv(c, p + "conv3", p + "bn3", mid, cout, 1, 1, 0, c->convs[b.conv[1]].outH, b.t_r[1], true);
      }
      if (down) b.down = add_conv(c, p + "down.conv", p + "down.bn", cin, cout, 1, stride, 0, H, t_in, true);
      H = c->convs[b.conv[b.nconv - 1]].outH;
      b.t_out = add_act(c, H, cout, true);
      c->blocks.push_back(b);
      t_in = b.t_out; cin = cout;
    }
  }
  c->agg_off = c->n_params;
  int rc = pool_ctx_create(c->D, c->Mh, c->C, DT_BF16, &c->agg);
  if (rc != SLIDE_OK) { delete c; return rc; }
  const int na = slide_param_tensors(c->agg);
  for (int i = 0; i < na; ++i) {
    char nm[64];
    size_t off = 0, len = 0;
    if (slide_param_name(c->agg, i, nm, sizeof nm, &off, &len) != SLIDE_OK || off != c->n_params - c->agg_off) {
      slide_ctx_destroy(c->agg);
      delete c;
      return SLIDE_EINVAL;
    }
    add_tensor(c, nm, len);
  }
  *out = c;
  return SLIDE_OK;
}

void resnet_ctx_destroy(resnet_ctx* c) {
  if (!c) return;
  prof_destroy(c->prof);
  slide_ctx_destroy(c->agg);
  delete c;
}

size_t resnet_param_count(const resnet_ctx* c) { return c ? c->n_params : 0; }
int resnet_param_tensors(const resnet_ctx* c) { return c ? (int)c->tensors.size() : 0; }
int resnet_feature_dim(const resnet_ctx* c) { return c ? c->D : 0; }

int resnet_param_name(const resnet_ctx* c, int index, char* name_out, size_t name_cap, size_t* offset, size_t* length) {
  if (!c || index < 0 || index >= (int)c->tensors.size()) return SLIDE_EINVAL;
  const Tensor& t = c->tensors[index];
  if (name_out && name_cap) {
    size_t k = t.name.size() < name_cap - 1 ? t.name.size() : name_cap - 1;
    for (size_t i = 0; i < k; ++i) name_out[i] = t.name[i];
    name_out[k] = 0;
  }
  if (offset) *offset = t.off;
  if (length) *length = t.len;
  return SLIDE_OK;
}

size_t resnet_arena_bytes(const resnet_ctx* c, int64_t n_tiles) {
  if (!c || n_tiles <= 0) return 0;
  return make_layout(const_cast<resnet_ctx*>(c), n_tiles, false).total;
}

int resnet_bind(resnet_ctx* c, const float* params, float* grads, void* arena, size_t arena_bytes) {
  if (!c || !params || !grads || !arena) return SLIDE_EINVAL;
  if (((uintptr_t)arena & 255) != 0) return SLIDE_EINVAL;
  c->params = params; c->grads = grads; c->arena = (char*)arena; c->arena_bytes = arena_bytes;
  c->enc_saved = false; c->step_saved = false;
  return SLIDE_OK;
}

int resnet_encoder_fwd_tiles(resnet_ctx* c, const void* pixels, int64_t n, void* feats_out, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!pixels || !feats_out || n <= 0) return SLIDE_EINVAL;
  return enc_fwd(c, pixels, n, feats_out, (hipStream_t)stream);
}

int resnet_encoder_bwd_tiles(resnet_ctx* c, const void* dfeats, int64_t n, int accumulate, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!dfeats || n <= 0) return SLIDE_EINVAL;
  return enc_bwd(c, dfeats, n, accumulate, (hipStream_t)stream);
}

int resnet_slide_step_fwd(resnet_ctx* c, const void* pixels, int64_t N, int32_t label, float* loss, float* logits,
                          float* alpha, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!pixels || N <= 0) return SLIDE_EINVAL;
  if (label < 0 || label >= (c->C == 1 ? 2 : c->C)) return SLIDE_EINVAL;
  // the layout only depends on N: the feature matrix can be named before the encoder runs
  RLayout y = make_layout(c, N, false);
  if (y.total > c->arena_bytes) return SLIDE_EARENA;
  rc = enc_fwd(c, pixels, N, c->arena + y.H, (hipStream_t)stream);
  if (rc) return rc;
  rc = agg_bind(c);
  if (rc) return rc;
  Run r{c, (hipStream_t)stream};
  launch(r, RK_MIL_POOL, 4.0 * N * c->D * c->Mh, (double)N * c->D * 4, [&] {
    rc = mil_pool_fwd(c->agg, c->arena + c->lay.H, N, label, loss, logits, alpha, stream);
    return rc == SLIDE_OK ? hipSuccess : hipErrorUnknown;
  });
  if (rc) return rc;
  c->step_saved = true; c->step_label = label;
  return finish(r);
}

int resnet_slide_step_bwd(resnet_ctx* c, int accumulate, void* stream) {
  int rc = check_bound(c);
  if (rc) return rc;
  if (!c->step_saved || !c->enc_saved) return SLIDE_ESTATE;
  const long long N = c->enc_n;
  rc = agg_bind(c);
  if (rc) return rc;
  Run r{c, (hipStream_t)stream};
  launch(r, RK_MIL_POOL, 16.0 * N * c->D * c->Mh, 3.0 * N * c->D * 4, [&] {
    rc = mil_pool_bwd(c->agg, c->arena + c->lay.H, N, c->step_label, c->arena + c->lay.G, accumulate, stream);
    return rc == SLIDE_OK ? hipSuccess : hipErrorUnknown;
  });
  if (rc) return rc;
  rc = finish(r);
  if (rc) return rc;
  return enc_bwd(c, c->arena + c->lay.G, N, accumulate, (hipStream_t)stream);
}

const void* resnet_features(const resnet_ctx* c) {
  if (!c || !c->arena || !c->step_saved) return nullptr;
  return c->arena + c->lay.H;
}
const void* resnet_feature_grads(const resnet_ctx* c) {
  if (!c || !c->arena || !c->step_saved) return nullptr;
  return c->arena + c->lay.G;
}

int resnet_prof_begin(resnet_ctx* c, int kernel_id) {
  if (!c) return SLIDE_EINVAL;
  return prof_begin(c->prof, kernel_id, RK_COUNT);
}
int resnet_prof_end(resnet_ctx* c, double* total_ms, int* launches, double* flops, double* bytes) {
  if (!c) return SLIDE_EINVAL;
  return prof_end(c->prof, total_ms, launches, flops, bytes);
}
int resnet_prof_family(const resnet_ctx* c, int kernel_id, double* total_ms, int* launches, double* flops, double* bytes) {
  if (!c) return SLIDE_EINVAL;
  return prof_family(c->prof, kernel_id, RK_COUNT, total_ms, launches, flops, bytes);
}
int resnet_saved_activations(const resnet_ctx* c) { return c ? (int)c->acts.size() : 0; }

int resnet_saved_activation(const resnet_ctx* c, int index, const void** ptr, int32_t* side, int32_t* channels) {
  if (!c || !ptr || !side || !channels || index < 0 || index >= (int)c->acts.size()) return SLIDE_EINVAL;
  if (!c->arena || !c->enc_saved) return SLIDE_ESTATE;
  const Act& a = c->acts[index];
  *ptr = c->arena + a.off; *side = a.H; *channels = a.C;
  return SLIDE_OK;
}

const char* resnet_kernel_name(int id) { return (id >= 0 && id < RK_COUNT) ? kRKernelNames[id] : nullptr; }

}  // extern "C"
