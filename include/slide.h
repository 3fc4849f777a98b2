/*
 * slide.h - C ABI of libslide: one end-to-end training step over all tiles of a
 * pathology slide on one MI355X (gfx950).
 *
 * The step is the one-device counterpart of the scheme in the paper's Method
 * section and appendix listing: every tile goes through a tile encoder, the
 * feature matrix goes through a gated-attention MIL aggregator and a slide-level
 * criterion, the loss is back-propagated to the feature matrix and from there
 * through the encoder (the pseudo-loss of the Method section, whose gradient is
 * J^T g; no rank factor on one device).
 *
 * Conventions common to every call
 *  - All data pointers are DEVICE pointers unless a comment says "host".
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the null stream).
 *    Every call only enqueues work on that stream and returns; scalar results
 *    (`loss`, `logits`) are device memory, the caller synchronises.
 *  - The library never allocates or frees device memory.  The caller owns the
 *    parameter vector, the gradient vector, the arena and every input/output
 *    buffer, and must keep them alive until the enqueued work has finished.
 *  - Element type of pixels and pixel gradients ("T") follows slide_config.dtype:
 *    0 = float32, 1 = bfloat16 (float32 accumulation, float32 master parameters,
 *    float32 gradients).  Tile features and feature gradients ([N,D]) are float32 on
 *    both paths: the softmax-over-tiles backward depends on differences between
 *    nearly equal feature rows, and the matrix is small.
 *  - Return value: 0 on success, a negative SLIDE_E* code otherwise.  No call
 *    aborts, throws or prints.
 *  - Calls on one context must not overlap in time (they share the arena).
 */
#ifndef SLIDE_H_
#define SLIDE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLIDE_OK            0
#define SLIDE_EINVAL       -1  /* null pointer, bad dimension, label out of range, n <= 0 */
#define SLIDE_EARENA       -2  /* arena missing or too small for n_tiles */
#define SLIDE_EUNSUPPORTED -3  /* shape outside what the kernels are built for */
#define SLIDE_ESTATE       -4  /* backward without a matching saved forward, or not bound */
#define SLIDE_EHIP         -5  /* a HIP call failed; see slide_last_hip_error() */

/* Plain data; copied by slide_ctx_create. */
typedef struct slide_config {
  int32_t tile;        /* S: tile side in pixels (224) */
  int32_t patch;       /* P: patch side (16); S % P == 0 */
  int32_t dim;         /* D: encoder width (384); D % heads == 0 */
  int32_t layers;      /* L: transformer blocks (12); 0 is allowed */
  int32_t heads;       /* H (6); head width D/H must be 8, 32 or 64 */
  int32_t mlp_ratio;   /* F = mlp_ratio * D (4) */
  int32_t mil_hidden;  /* M_h: gated-attention hidden width (128 / 256) */
  int32_t n_classes;   /* C: 1 = one logit with binary cross-entropy; >1 = softmax cross-entropy */
  int32_t dtype;       /* 0 = float32 path, 1 = bfloat16 storage / float32 accumulate */
  int32_t recompute;   /* 0 = keep every block's activations; 1 = keep block inputs, re-run blocks in backward */
  float   ln_eps;      /* LayerNorm epsilon (1e-6) */
  int32_t reserved;    /* must be 0 (pixel gradients are requested per call by a non-null pointer) */
} slide_config;

typedef struct slide_ctx slide_ctx;

/* Validate `cfg` (host pointer) and build the host-side description (parameter
 * layout, kernel shapes).  Touches no device memory. */
int  slide_ctx_create(const slide_config* cfg, slide_ctx** out);
void slide_ctx_destroy(slide_ctx* ctx);

/* Flat float32 parameter vector: length, and offset/length of one named tensor.
 * Layout (row-major, W is [out][in]):
 *   pe.W[D,3P^2] (in-index = c*P*P + py*P + px), pe.b[D], cls[D], pos[T,D],
 *   per block i: l{i}.ln1.g, l{i}.ln1.b, l{i}.qkv.W[3D,D] (rows: q heads, k heads, v heads),
 *   l{i}.qkv.b[3D], l{i}.proj.W[D,D], l{i}.proj.b, l{i}.ln2.g, l{i}.ln2.b,
 *   l{i}.fc1.W[F,D], l{i}.fc1.b, l{i}.fc2.W[D,F], l{i}.fc2.b,
 *   lnf.g, lnf.b, mil.V.W[M_h,D], mil.V.b, mil.U.W[M_h,D], mil.U.b, mil.w[M_h],
 *   head.W[C,D], head.b[C].
 * slide_param_name(ctx, i, ...) enumerates the tensors in layout order (host buffers). */
size_t slide_param_count(const slide_ctx* ctx);
int    slide_param_tensors(const slide_ctx* ctx);
int    slide_param_name(const slide_ctx* ctx, int index, char* name_out, size_t name_cap,
                        size_t* offset, size_t* length);
int    slide_param_offset(const slide_ctx* ctx, const char* name, size_t* offset, size_t* length);

/* Bytes of arena needed to run `n_tiles` tiles through one call (saved
 * activations, backward work space, low-precision weight copies).  Monotone in
 * n_tiles.  Returns 0 for n_tiles <= 0. */
size_t slide_arena_bytes(const slide_ctx* ctx, int64_t n_tiles);

/* Bytes of arena needed by mil_pool_fwd / mil_pool_bwd alone over N feature rows. */
size_t slide_pool_arena_bytes(const slide_ctx* ctx, int64_t N);

/* Attach device buffers: params_fp32 [slide_param_count] (read), grads_fp32
 * [slide_param_count] (written by the backward calls), arena (256-byte aligned).
 * May be called again to re-bind. */
int  slide_bind(slide_ctx* ctx, const float* params_fp32, float* grads_fp32,
                void* arena, size_t arena_bytes);

/* Tile encoder forward (paper, appendix listing: the encoder ranks' forward step; Method, first paragraph).
 * pixels: [n_tiles,3,S,S] of T, planar, already normalised.  feats_out: [n_tiles,D] float32.
 * save_for_bwd != 0 keeps this call's activations in the arena for one
 * encoder_bwd_tiles on the same tiles; 0 keeps nothing (feature extraction). */
int  encoder_fwd_tiles(slide_ctx* ctx, const void* pixels, int64_t n_tiles,
                       void* feats_out, int save_for_bwd, void* hip_stream);

/* Encoder backward seeded with the feature-gradient rows of these tiles (paper, Method:
 * pseudo-loss equation; appendix listing: the encoder ranks' backward step), without the
 * rank factor.  dfeats: [n_tiles,D] float32.  Encoder slices of grads_fp32 are overwritten
 * (accumulate == 0) or added to (accumulate != 0; chunk gradients SUM to the slide
 * gradient).  pixel_grad_or_null: [n_tiles,3,S,S] of T or NULL.
 * SLIDE_ESTATE unless the last encoder forward on this context saved n_tiles tiles. */
int  encoder_bwd_tiles(slide_ctx* ctx, const void* dfeats, int64_t n_tiles, int accumulate,
                       void* pixel_grad_or_null, void* hip_stream);

/* Gated-attention MIL pooling, class logits and slide loss (paper, appendix listing: the
 * aggregator rank's forward and criterion; Method, paragraph on the aggregator).
 * feats: [N,D] float32.  label: 0/1 for C == 1, class index for C > 1.
 * Outputs (device, float32; any may be NULL): loss[1], logits[C], alpha[N] (attention weights). */
int  mil_pool_fwd(slide_ctx* ctx, const void* feats, int64_t N, int32_t label,
                  float* loss, float* logits, float* alpha, void* hip_stream);

/* mil_pool_fwd for callers that cannot allocate device memory or hand over work space: code under HIP graph capture,
 * tight serving loops (slide-level prediction from stored features), harnesses that forbid hipMalloc.  Same
 * kernels, same results; the kernels' work space (attention logits, per-workgroup softmax partials, scalars, the
 * low-precision copy of the gate weights) is a fixed array of SLIDE_STATIC_POOL_BYTES inside the library's device
 * code, one copy per device, held until the process ends.  The context supplies the shapes only and need not be
 * bound; params_fp32 is the flat parameter vector (device).  The call allocates nothing and frees nothing.
 * SLIDE_EARENA if N > SLIDE_STATIC_POOL_MAX_ROWS or the work space for (N, D, M_h, C) exceeds the array; other
 * errors as mil_pool_fwd.  All calls on one device share the array: calls that overlap in time on one device race
 * (also on different streams or contexts); the array keeps the last call's contents, nothing in it needs clearing. */
#define SLIDE_STATIC_POOL_BYTES    (12u << 20)
#define SLIDE_STATIC_POOL_MAX_ROWS 65536
int  mil_pool_fwd_static(const slide_ctx* ctx, const float* params_fp32, const void* feats, int64_t N, int32_t label,
                         float* loss, float* logits, float* alpha, void* hip_stream);

/* Aggregator backward (paper, appendix listing: the aggregator rank's backward step, which yields
 * the gradient of the loss with respect to the gathered feature matrix).
 * Recomputes the forward from `feats` and `label` (no state is shared with mil_pool_fwd),
 * writes dfeats_out = G [N,D] float32 and the aggregator slices (mil.*, head.*) of grads_fp32
 * (overwrite, or add when accumulate != 0). */
int  mil_pool_bwd(slide_ctx* ctx, const void* feats, int64_t N, int32_t label,
                  void* dfeats_out, int accumulate, void* hip_stream);

/* Whole-slide forward = encoder_fwd_tiles(save) on all N tiles + mil_pool_fwd.
 * Features and everything the backward needs stay in the arena. */
int  slide_step_fwd(slide_ctx* ctx, const void* pixels, int64_t N, int32_t label,
                    float* loss, float* logits, float* alpha, void* hip_stream);

/* Whole-slide backward = mil_pool_bwd + encoder_bwd_tiles on the state left by
 * slide_step_fwd: afterwards grads_fp32 holds d loss / d parameter for every
 * parameter (overwrite or add).  SLIDE_ESTATE without a preceding slide_step_fwd. */
int  slide_step_bwd(slide_ctx* ctx, int accumulate, void* pixel_grad_or_null, void* hip_stream);

/* The same step for a slide whose activations do not fit the arena (the paper's resource-constrained setting;
 * Results, gradient equivalence: the gradients of a slide are the sum over any partition of its tiles once the
 * feature gradients are known).  The tiles go through the encoder in chunks of at most chunk_tiles: first every
 * chunk forward without keeping anything (features only), then aggregator, loss and feature gradients on all N
 * rows, then chunk by chunk a second forward with the activations kept and the backward seeded with that chunk's
 * feature gradients, accumulating the parameter gradients.  One call does forward and backward; it costs one extra
 * encoder forward.  Arguments as slide_step_fwd / slide_step_bwd; pixel_grad_or_null: [N,3,S,S] of T.
 * The arena must hold slide_chunked_arena_bytes(N, chunk_tiles).  Errors as slide_step_fwd. */
size_t slide_chunked_arena_bytes(const slide_ctx* ctx, int64_t N, int64_t chunk_tiles);
int  slide_step_chunked(slide_ctx* ctx, const void* pixels, int64_t N, int64_t chunk_tiles, int32_t label,
                        int accumulate, float* loss_out, float* logits_out_or_null, float* alpha_out_or_null,
                        void* pixel_grad_or_null, void* hip_stream);

/* Device pointers into the arena, valid after slide_step_fwd / slide_step_bwd until
 * the next forward: features H [N,D] and feature gradients G [N,D], float32. */
const void* slide_features(const slide_ctx* ctx);
const void* slide_feature_grads(const slide_ctx* ctx);

/* One AdamW update of `count` fp32 parameters in place (paper, Experiments: the optimiser both training set-ups
 * use; Adam with decoupled weight decay as in the work cited there):
 *   m = beta1 m + (1 - beta1) g;  v = beta2 v + (1 - beta2) g^2;
 *   params -= lr * ((m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) + weight_decay * params)
 * params, exp_avg (m) and exp_avg_sq (v) are device pointers to `count` floats each, read and written; grads is read.
 * The caller owns all four and zero-fills m and v before step 1.  step counts from 1.  After slide_step_bwd the
 * arguments are the buffers given to slide_bind (the next forward reads the updated parameters).
 * SLIDE_EINVAL: null pointer, count == 0, step < 1, beta outside [0,1), lr or eps or weight_decay negative. */
int  slide_adamw_step(float* params, const float* grads, float* exp_avg, float* exp_avg_sq, size_t count,
                      int64_t step, float lr, float beta1, float beta2, float eps, float weight_decay,
                      void* hip_stream);

/* hipError_t of the most recent failing HIP call on this thread (0 if none). */
int  slide_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SLIDE_H_ */
