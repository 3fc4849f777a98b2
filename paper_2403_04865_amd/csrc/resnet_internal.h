// Internal declarations of the convolutional (ResNet) tile encoder of libslide (gfx950 only).
// Activations are bf16, channels-last: a tensor is a matrix [n * H * W][C] whose row is one position of one tile.
#pragma once
#include "slide_internal.h"

namespace sl {

// How the rows of a convolution's source tensor are found from the rows being produced.
//   transposed == 0 (forward, weight gradient): produced row (n, y, x), tap (kh, kw) -> source position
//       (y * stride + kh - pad, x * stride + kw - pad), absent outside the source grid (zero padding).
//   transposed == 1 (input gradient): produced row (n, y, x) is an INPUT position, the source is the output
//       gradient: tap (kh, kw) -> ((y + pad - kh) / stride, (x + pad - kw) / stride), absent unless both
//       divisions are exact and the result lies in the source grid.
//   stem != 0: the 7x7 stride-2 pad-3 convolution of the network's input read from the padded pixel image
//       [n][YS = S + 6][XS = S + 8][4] (three channels and a zero, a zero border of three pixels): eight consecutive
//       pixels of one image row are 64 contiguous bytes = one kernel row of taps (kw 0..7, the eighth with zero
//       weights), so the contraction index is kh * 32 + kw * 4 + channel, 256 columns (kh = 7: zero weights), and no
//       row is ever absent.  The kernels see KH = KW = 1 and Cs = 256; produced row (n, y, x), column chunk of 8 at
//       column k reads image row 2 y + min(k / 32, 6), pixel 2 x + (k % 32) / 4.
struct ConvGeom {
  int YO, XO;   // grid of the produced rows
  int YS, XS;   // grid of the source rows
  int KH, KW, stride, pad;
  int transposed;
  int stem;
  // cls != 0 (input gradient of a stride-2 convolution only): the launch produces the positions of one parity class,
  // (y % 2, x % 2) = ((cls - 1) / 2, (cls - 1) % 2), i.e. M = n * (YO / 2) * (XO / 2) rows.  Only the taps whose offset
  // has the parity of the class reach a source position at all (kh = (y + pad) % 2 + 2 i): the contraction runs over
  // those (a quarter of KH * KW on average) instead of multiplying zeros for the rest.
  int cls;
};

// out[M][N] (bf16) = sum over taps of src_tap[M][Cs] * W[N][tap * Cs .. + Cs]^T
//                    (+ out when add != 0)  (+ (mask bit ? extra : 0) when extra is not null; extra: [M][N], mask: one
//                    bit per element of [M][N], bit e of byte i = element 8 i + e, as launch_bn_apply writes them).
// The sums are formed in fp32 and rounded once.  M = n * YO * XO < 2^31, Cs % 64 == 0, N % 64 == 0; W row stride =
// KH * KW * Cs.
struct ConvNT {
  const bf16* src; int Cs;
  const bf16* W;
  const bf16* Wf;           // optional: the same matrix in fragment order (launch_conv_cast_w), used by the 3x3 stride-1 kernel
  bf16* out; int N;
  long long M;
  ConvGeom g;
  int add;
  const bf16* extra; const unsigned char* mask;
  // optional: per row tile of the launch, the sums over the tile's rows of every output channel's stored value and of
  // its square: stat_part[tile][2][N] (conv_nt_row_tiles(p) tiles); the statistics of the batch normalisation behind
  // the convolution are built from these instead of a pass over the output
  float* stat_part;
};
hipError_t launch_conv_nt(const ConvNT& p, hipStream_t s);
int conv_nt_row_tiles(const ConvNT& p);

// part[slab][Co][KH * KW * Cs] (fp32) = sum over the slab's rows m of dout[m][co] * src_tap(m)[ci]; the rows
// (n, y, x) run over the OUTPUT grid of the convolution (geometry not transposed).  Co % 64 == 0, Cs % 64 == 0,
// KH * KW is 1 or 9.  Slab s covers rows [s * per, (s + 1) * per), per % 32 == 0.
struct ConvWG {
  const bf16* dout; int Co;
  const bf16* src; int Cs;
  float* part;
  long long M;
  ConvGeom g;
  int slabs; long long per;
};
hipError_t launch_conv_wgrad(const ConvWG& p, hipStream_t s);

// dW[co][ci][kh][kw] (fp32, the parameter's own layout) = (accumulate ? dW : 0) + sum_s part[s][co][tap * Cin + ci],
// part row stride ldk (>= taps * Cin)
hipError_t launch_wgrad_reduce(const float* part, int slabs, int Co, int Cin, int taps, int ldk, float* dW, int accumulate,
                               hipStream_t s);
// fp32 W[co][ci][kh][kw] -> bf16 Wk[co][ldk] (column tap * Cin + ci, zero beyond taps * Cin) and, if Wt is not null,
// Wt[ci][tap * Co + co]; Wf / Wtf (optional): the same two matrices in fragment order: for every block of 32 rows and
// 16 columns, the 64 MFMA lanes' operands (row l % 32, columns 8 (l / 32) .. + 7) back to back
hipError_t launch_conv_cast_w(const float* W, int Co, int Cin, int taps, int ldk, bf16* Wk, bf16* Wt, bf16* Wf, bf16* Wtf,
                              hipStream_t s);
// planar pixels [n][3][S][S] (bf16) -> padded image [n][S + 6][S + 8][4] (see ConvGeom::stem), borders and the fourth
// channel zero
hipError_t launch_stem_pad_pixels(const bf16* pixels, bf16* img, long long n, int S, hipStream_t s);
// fp32 W[co][3][7][7] -> bf16 Wk[co][256], column kh * 32 + kw * 4 + channel, zero elsewhere
hipError_t launch_stem_cast_w(const float* W, int Co, bf16* Wk, hipStream_t s);
// dW[co][3][7][7] = (accumulate ? dW : 0) + sum_s part[s][co][kh * 32 + kw * 4 + channel]
hipError_t launch_stem_wgrad_reduce(const float* part, int slabs, int Co, float* dW, int accumulate, hipStream_t s);

// ---- batch normalisation over all rows of [M][C] (C % 8 == 0, C <= 2048) --------------------------------------------
// stats: [4][C] floats: mean, 1 / sqrt(var + eps), a = gamma * rstd, b = beta - mean * a
int bn_blocks(long long M, int C);
// from per-tile sums tile_part[tiles][2][C] (as ConvNT::stat_part) over M rows in all
hipError_t launch_bn_stats_tiles(const float* tile_part, int tiles, long long M, int C, const float* gamma, const float* beta,
                                 float eps, float* part, float* stats, hipStream_t s);
// y = a x + b  (+ resid, or + ra resid + rb when rstats is not null), then max(., 0) when relu.  bits (may be null):
// one bit per element, set where the stored y is positive (bit e of byte i = element 8 i + e): the ReLU mask of the
// backward, a sixteenth of the bytes of y
hipError_t launch_bn_apply(const bf16* x, long long M, int C, const float* stats, const bf16* resid, const float* rstats,
                           int relu, bf16* y, unsigned char* bits, hipStream_t s);
// dz = (mask == null || mask bit) ? dy : 0;  dgamma = sum dz x_hat, dbeta = sum dz (written or added to the
// parameter gradients); dx = a (dz - dbeta / M - x_hat dgamma / M)
hipError_t launch_bn_bwd(const bf16* dy, const unsigned char* mask, const bf16* x, long long M, int C, const float* stats,
                         float* part, float* coef, float* dgamma, float* dbeta, int accumulate, bf16* dx, hipStream_t s);

// 3x3 stride-2 pad-1 max pooling on [n][H][W][C]; of equal maxima the first in (kh, kw) order takes the gradient.
// arg: one byte per output element (the winning tap), written by the forward, read by the backward
hipError_t launch_maxpool_fwd(const bf16* x, bf16* y, unsigned char* arg, long long n, int H, int W, int C, hipStream_t s);
hipError_t launch_maxpool_bwd(const unsigned char* arg, const bf16* dy, bf16* dx, long long n, int H, int W, int C,
                              hipStream_t s);
// global average over the HW positions of each tile: feats [n][C] fp32; and its gradient
hipError_t launch_avgpool_fwd(const bf16* x, float* feats, long long n, int HW, int C, hipStream_t s);
hipError_t launch_avgpool_bwd(const float* dfeats, bf16* dx, long long n, int HW, int C, hipStream_t s);
}  // namespace sl
