/*
 * resnet.h - C ABI of libslide for slides encoded by a residual convolutional network: the same end-to-end
 * training step as slide.h (every tile through the tile encoder, gated-attention MIL aggregator, slide-level
 * criterion, loss back-propagated to the feature matrix and from there through the encoder), with the encoder family
 * the paper's experiments train (Results: ResNet50 in the gradient-equivalence and EGFR experiments, ResNet18 on
 * 4,096 tiles of 224 px per device in the whole-slide breast experiment).
 *
 * Network: 7x7 stride-2 convolution, batch normalisation, ReLU, 3x3 stride-2 max pooling; four stages of residual
 * blocks (basic: 3x3, 3x3; bottleneck: 1x1, 3x3 carrying the stride, 1x1 with four-fold expansion), a 1x1
 * convolution + batch normalisation on the shortcut wherever stride or width changes; global average pooling gives
 * the tile's feature row.  Convolutions carry no bias.  Batch normalisation uses the statistics of the batch it sees:
 * over every tile and position of the call (Results, gradient equivalence: the normalisation layers were
 * synchronised, i.e. the statistics are those of all tiles of the slide).  Because of that the tiles of a call are
 * coupled: there is no chunked variant of this step, and one call must hold the whole slide.
 *
 * Conventions as in slide.h: device pointers unless a comment says "host"; `hip_stream` is a hipStream_t passed as
 * void*; every call only enqueues work and returns; the library never allocates device memory (the caller owns the
 * parameter vector, the gradient vector and the arena); return value 0 or a negative SLIDE_E* code; calls on one
 * context must not overlap in time.  Pixels are bfloat16, planar [n,3,S,S], already normalised; activations are
 * bfloat16 with float32 accumulation, parameters and gradients float32, tile features and feature gradients float32.
 * Pixel gradients are not computed (the input is data).
 */
#ifndef SLIDE_RESNET_H_
#define SLIDE_RESNET_H_

#include "slide.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Plain data; copied by resnet_ctx_create. */
typedef struct resnet_config {
  int32_t tile;         /* S: tile side in pixels, a multiple of 32 (224) */
  int32_t block;        /* 0 = basic block (ResNet18/34), 1 = bottleneck block (ResNet50/101/152) */
  int32_t depths[4];    /* residual blocks per stage: {2,2,2,2} = ResNet18, {3,4,6,3} with block 1 = ResNet50 */
  int32_t width;        /* channels of the stem and of the first stage (64); a power of two >= 64 */
  int32_t mil_hidden;   /* M_h of the gated-attention aggregator */
  int32_t n_classes;    /* C: 1 = one logit with binary cross-entropy; >1 = softmax cross-entropy */
  float   bn_eps;       /* batch-normalisation epsilon (1e-5) */
  int32_t reserved;     /* must be 0 */
} resnet_config;

typedef struct resnet_ctx resnet_ctx;

/* Validate `cfg` (host pointer) and build the host-side description.  Touches no device memory. */
int  resnet_ctx_create(const resnet_config* cfg, resnet_ctx** out);
void resnet_ctx_destroy(resnet_ctx* ctx);

/* Flat float32 parameter vector.  Layout, in order (convolution weights are [out][in][kh][kw]):
 *   stem.conv.W[w,3,7,7], stem.bn.g[w], stem.bn.b[w];
 *   per stage s, block b (prefix "s{s}.b{b}."):
 *     basic:      conv1.W[mid,in,3,3], bn1.g, bn1.b, conv2.W[out,mid,3,3], bn2.g, bn2.b
 *     bottleneck: conv1.W[mid,in,1,1], bn1.g, bn1.b, conv2.W[mid,mid,3,3], bn2.g, bn2.b, conv3.W[out,mid,1,1], bn3.g, bn3.b
 *     then, where stride or width changes: down.conv.W[out,in,1,1], down.bn.g, down.bn.b;
 *   mil.V.W[M_h,D], mil.V.b, mil.U.W[M_h,D], mil.U.b, mil.w[M_h], head.W[C,D], head.b[C]   (D = feature width).
 * resnet_param_name enumerates the tensors in layout order (host buffers). */
size_t resnet_param_count(const resnet_ctx* ctx);
int    resnet_param_tensors(const resnet_ctx* ctx);
int    resnet_param_name(const resnet_ctx* ctx, int index, char* name_out, size_t name_cap, size_t* offset, size_t* length);
int    resnet_feature_dim(const resnet_ctx* ctx);   /* D = 8 * width (basic) or 32 * width (bottleneck) */

/* Bytes of arena needed for a step over n_tiles tiles (every activation the backward needs, gradient work space,
 * low-precision weight copies, the aggregator's work space).  0 for n_tiles <= 0. */
size_t resnet_arena_bytes(const resnet_ctx* ctx, int64_t n_tiles);

/* Attach device buffers: params_fp32 [resnet_param_count] (read), grads_fp32 [resnet_param_count] (written by the
 * backward calls), arena (256-byte aligned).  May be called again to re-bind. */
int  resnet_bind(resnet_ctx* ctx, const float* params_fp32, float* grads_fp32, void* arena, size_t arena_bytes);

/* Tile encoder forward over all n_tiles tiles of the call (paper, Method: the encoder's forward step; batch
 * statistics over these tiles).  pixels: [n_tiles,3,S,S] bfloat16.  feats_out: [n_tiles,D] float32.  The
 * activations stay in the arena for one resnet_encoder_bwd_tiles on the same tiles. */
int  resnet_encoder_fwd_tiles(resnet_ctx* ctx, const void* pixels, int64_t n_tiles, void* feats_out, void* hip_stream);

/* Encoder backward seeded with the feature-gradient rows of these tiles (paper, Method: pseudo-loss equation, without
 * the rank factor).  dfeats: [n_tiles,D] float32.  Encoder slices of grads_fp32 are overwritten (accumulate == 0) or
 * added to.  SLIDE_ESTATE unless the last encoder forward on this context was over n_tiles tiles. */
int  resnet_encoder_bwd_tiles(resnet_ctx* ctx, const void* dfeats, int64_t n_tiles, int accumulate, void* hip_stream);

/* Whole-slide forward = resnet_encoder_fwd_tiles on all N tiles + aggregator, logits and loss (paper, appendix
 * listing: the aggregator rank's forward and criterion).  Outputs (device, float32; any may be NULL): loss[1],
 * logits[C], alpha[N].  label: 0/1 for C == 1, class index for C > 1. */
int  resnet_slide_step_fwd(resnet_ctx* ctx, const void* pixels, int64_t N, int32_t label, float* loss, float* logits,
                           float* alpha, void* hip_stream);

/* Whole-slide backward = aggregator backward + resnet_encoder_bwd_tiles on the state left by resnet_slide_step_fwd:
 * afterwards grads_fp32 holds d loss / d parameter for every parameter.  SLIDE_ESTATE without a preceding forward. */
int  resnet_slide_step_bwd(resnet_ctx* ctx, int accumulate, void* hip_stream);

/* Device pointers into the arena, valid after resnet_slide_step_fwd / _bwd until the next forward: features H [N,D]
 * and feature gradients G [N,D], float32. */
const void* resnet_features(const resnet_ctx* ctx);
const void* resnet_feature_grads(const resnet_ctx* ctx);

/* The activations the last encoder forward left in the arena, for inspection (the tests replay the backward on them).
 * They are bfloat16, channels-last: tensor `index` is [n_tiles][side][side][channels].  Order: stem convolution
 * output, stem ReLU output, max-pooling output, then per residual block: per convolution its output and (except the
 * last) the ReLU output behind its normalisation, the projection's output where the block has one, the block output.
 * resnet_saved_activations: how many there are.  SLIDE_ESTATE without a saved forward. */
int  resnet_saved_activations(const resnet_ctx* ctx);
int  resnet_saved_activation(const resnet_ctx* ctx, int index, const void** ptr, int32_t* side, int32_t* channels);

/* Measurement hooks, as slide_prof_begin / slide_prof_end / slide_prof_family / slide_kernel_name of slide_prof.h,
 * over this context type's kernel families. */
int         resnet_prof_begin(resnet_ctx* ctx, int kernel_id);
int         resnet_prof_end(resnet_ctx* ctx, double* total_ms, int* launches, double* flops, double* bytes);
int         resnet_prof_family(const resnet_ctx* ctx, int kernel_id, double* total_ms, int* launches, double* flops,
                               double* bytes);
const char* resnet_kernel_name(int kernel_id);

#ifdef __cplusplus
}
#endif
#endif /* SLIDE_RESNET_H_ */
