/*
 * vitenc — packed vision-transformer image encoder for MI355X (gfx950), C ABI.
 *
 * The operation: the image-encoding stage of a large multimodal model served as its
 * own instance (paper Sec. 2 "Image Encoding"; Sec. 4 "Image Instances").  Uniform-size
 * image tiles go in, image-token embeddings come out.  Images of a request do not
 * attend to each other (paper Sec. 1; Sec. 3.1 "Compute Characteristics"), so the images
 * of many requests are packed into one launch; attention is confined to a tile (local
 * layers) or to the tiles of one image (global layers) and never crosses images.
 *
 * All functions return a status and never throw or abort across the ABI.
 * The message for the last failure on the calling thread is vit_last_error().
 */
#ifndef VITENC_H
#define VITENC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif
#pragma GCC visibility push(default)

typedef struct vit_encoder vit_encoder_t; /* opaque; owned by the library */

typedef enum {
  VIT_OK = 0,
  VIT_EINVAL = -1,    /* bad argument or inconsistent shapes; nothing was launched        */
  VIT_ENOMEM = -2,    /* host or device allocation failed (create only)                   */
  VIT_ECAPACITY = -3, /* output or workspace buffer too small; nothing was launched       */
  VIT_EDEVICE = -4,   /* a HIP call failed; vit_last_error() carries the HIP error string */
  VIT_ENOTREADY = -5  /* hand-off: not every image of the request has been published yet   */
} vit_status_t;

enum { VIT_DTYPE_FP32 = 0, VIT_DTYPE_BF16 = 1 };

/*
 * Encoder shape.  Tokens per tile T = floor(image_size/patch_size)^2 + has_cls
 * (paper Table 1: 560/14 with CLS -> 1601; 384/14 without -> 729).  Output tokens per tile
 * T_out = T, or (floor(image_size/patch_size) / token_merge)^2 with token down-sampling
 * (Table 1: 448/14 = 32, merged 2 x 2 -> 256).
 */
typedef struct {
  int32_t image_size;    /* S: tiles are S x S pixels; floor(S / p) <= 512                      */
  int32_t patch_size;    /* p <= 256                                                            */
  int32_t channels;      /* C (3); <= 16                                                        */
  int32_t hidden;        /* D, divisible by heads                                               */
  int32_t heads;         /* H; head dim D/H must be <= 128 and a multiple of 8                  */
  int32_t mlp;           /* M: width of the block MLP, a multiple of 8, <= 65536                */
  int32_t layers_local;  /* blocks whose attention segment is one tile (each count <= 1024)     */
  int32_t layers_global; /* following blocks whose attention segment is all tiles of one image  */
  int32_t has_cls;       /* 1: a learned CLS row precedes the patches of every tile             */
  int32_t final_ln;      /* 1: LayerNorm after the last block                                   */
  float ln_eps;          /* added to the biased variance                                        */
  int32_t proj_layers;   /* 0, 1 or 2 linear layers after the encoder, GELU between them        */
  int32_t proj_dims[2];  /* output width of each projector layer, multiples of 8, <= 65536      */
  int32_t dtype;         /* VIT_DTYPE_FP32: fp32 arithmetic and output;                         */
                         /* VIT_DTYPE_BF16: bf16 matrix operands, fp32 accumulation and         */
                         /* residual stream, bf16 output                                        */
  int32_t token_merge;   /* 0 or 1: every token is output.  m > 1: token down-sampling after    */
                         /* the final LayerNorm (paper Table 1: 448-px tiles -> 256 tokens): the */
                         /* CLS row is dropped and every m x m block of neighbouring patch       */
                         /* tokens becomes one token of m*m*D channels, the block's tokens one   */
                         /* after the other in (row, column) order; floor(S/p) must be a         */
                         /* multiple of m.  The projector (if any) then takes m*m*D inputs.      */
} vit_config_t;

/*
 * Number of fp32 values vit_encoder_create expects for `cfg` (0 if cfg is invalid).
 * Order of the flat buffer, every matrix row-major [out_features, in_features]:
 *   patch_w [D, C*p*p] (index c*p*p + py*p + px), patch_b [D], cls [D] (if has_cls),
 *   pos [T, D];
 *   per block: ln1_g, ln1_b [D]; wqkv [3D, D] (rows: all of Q, then K, then V; head h is
 *   rows h*dh..), bqkv [3D]; wo [D, D], bo [D]; ln2_g, ln2_b [D]; w1 [M, D], b1 [M];
 *   w2 [D, M], b2 [D];
 *   lnf_g, lnf_b [D] (if final_ln); per projector layer: w [out, in], b [out]; the first
 *   projector layer has in = D, or token_merge^2 * D with token down-sampling.
 */
size_t vit_weight_count(const vit_config_t* cfg);

/*
 * Build an encoder on HIP device `device`: one Image Instance's model (paper Sec. 4, "Image
 * Instances": the image encoder is deployed and scaled on its own, apart from the language model;
 * Sec. 2 "Image Encoding": a vision transformer that turns preprocessed tiles into image tokens).
 *   weights   HOST pointer, n_weights fp32 values in the order above.  The library
 *             converts (round-to-nearest-even to bf16 when dtype is bf16), pads and uploads
 *             them; the caller keeps ownership and may free the buffer on return.
 *   out       receives the handle; release it with vit_encoder_destroy.
 * Errors: VIT_EINVAL (null pointers, invalid cfg, n_weights != vit_weight_count),
 *         VIT_ENOMEM, VIT_EDEVICE.  *out is NULL on failure.
 */
vit_status_t vit_encoder_create(const vit_config_t* cfg, const float* weights, size_t n_weights,
                                int device, vit_encoder_t** out);

/*
 * Pure host function: what a launch over n_tiles tiles grouped into n_images images
 * produces and needs.  The token count is a function of the tile count alone (paper Sec. 2 and
 * Table 1: tiles of a fixed size yield a fixed number of tokens each, e.g. 4 x 1601 or
 * 10 x 729 or 5 x 256 per image), which is what lets a router account for image-token load
 * before any pixel is encoded (Sec. 4.3).  n_tokens = n_tiles * T_out; out_dim = last projector width, or D
 * (token_merge^2 * D with token down-sampling and no projector);
 * workspace_bytes is an upper bound valid for any grouping of n_tiles tiles into
 * n_images >= 1 images.  Any output pointer may be NULL.
 */
vit_status_t vit_encoder_query(const vit_encoder_t* enc, int32_t n_tiles, int32_t n_images,
                               int64_t* n_tokens, int32_t* out_dim, size_t* out_bytes,
                               size_t* workspace_bytes);

/*
 * Encode one packed batch (patchify + position add, all blocks, final LN, projector).
 *   pixels              DEVICE, [n_tiles, C, S, S] fp32, already normalised (preprocessing
 *                       is the stage before this one, paper Sec. 2; vit_preprocess_tiles
 *                       below writes this layout).
 *   images_per_request  HOST, [n_requests], each >= 0 (0 = text-only request, which owns
 *                       an empty token range); sum = n_images.
 *   tile_offsets        HOST, [n_images + 1], prefix sum of tiles per image:
 *                       [0] = 0, strictly increasing, last = n_tiles.
 *   out_tokens          DEVICE, [n_tiles * T_out, out_dim] row-major, bf16 or fp32 per dtype,
 *                       in input tile order; out_capacity_bytes is its size.
 *   request_token_offsets  HOST, optional [n_requests + 1]: first token row of each request.
 *   workspace           DEVICE scratch of at least vit_encoder_query's workspace_bytes,
 *                       256-byte aligned; contents are undefined before and after.
 *   stream              hipStream_t (NULL = default stream).
 * The call is asynchronous on `stream`: host arrays are consumed before it returns, device
 * buffers must stay valid until the stream has drained.  The library keeps no reference to
 * caller buffers afterwards and never frees them.  One handle may have any number of
 * launches queued on ONE stream; concurrent use from several threads or streams is not
 * supported.  n_requests = 0 or n_tiles = 0 is a successful no-op.
 * Errors: VIT_EINVAL (null pointers, negative counts, an image with no tiles),
 *         VIT_ECAPACITY (nothing launched), VIT_EDEVICE.
 */
vit_status_t vit_encode_packed(vit_encoder_t* enc, const float* pixels,
                               const int32_t* images_per_request, int32_t n_requests,
                               const int32_t* tile_offsets, void* out_tokens,
                               size_t out_capacity_bytes, int64_t* request_token_offsets,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * vit_encode_packed for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as vit_encode_packed
 * minus the workspace: the call carves its workspace out of a static device array of
 * VIT_STATIC_SCRATCH_BYTES that each GPU the library runs on holds until the process ends, writes
 * its attention work lists with a small kernel (no pinned staging buffer, no host-to-device copy),
 * and calls no hipMalloc / hipHostMalloc / hipFree / hipEventCreate or other allocating routine;
 * per-kernel timing (vit_profile_enable) does not cover it.
 * Limits: the batch's vit_encoder_query workspace_bytes must not exceed VIT_STATIC_SCRATCH_BYTES
 * (128 MiB: eight 336-px images of a ViT-L/14 encoder) and it may hold at most
 * VIT_STATIC_MAX_IMAGES images; beyond either the call returns VIT_ECAPACITY and launches nothing.
 * All calls on one GPU, from any handle, share that GPU's array: calls whose device work overlaps
 * (different streams or threads) race; calls queued on one stream do not.  The array keeps the
 * previous call's contents; every call rewrites all it reads.
 */
#define VIT_STATIC_SCRATCH_BYTES ((size_t)128 << 20)
#define VIT_STATIC_MAX_IMAGES 256
vit_status_t vit_encode_packed_static(vit_encoder_t* enc, const float* pixels,
                                      const int32_t* images_per_request, int32_t n_requests,
                                      const int32_t* tile_offsets, void* out_tokens,
                                      size_t out_capacity_bytes, int64_t* request_token_offsets,
                                      void* stream);

/*
 * vit_encode_packed for small, launch-bound batches: the paper's image requests mostly carry one
 * or a few images (Sec. 3.3 "Workload Characteristics": heavy-tailed images per request) and their
 * encode time sits on the path to the first token (Sec. 3.2), while one 336-px ViT-L image is
 * some 270 kernel launches that together run shorter than the host needs to issue them.  Same
 * arguments, results (bit for bit) and errors as vit_encode_packed.  The kernels' arguments are part
 * of a graph, so a launch sequence is kept per (pixels, out_tokens, workspace, tile_offsets
 * contents): the first call with a key runs like vit_encode_packed, the second records the sequence
 * into a HIP graph (on a stream of the library's own, so `stream` may be the default stream), every
 * later one replays it with one graph launch on `stream`.  The buffers' CONTENTS may change between
 * calls; a caller that cycles through a fixed pool of buffers hits after the second round.  Eight
 * sequences are kept per handle, the least recently used is replaced.  Only kernels are recorded:
 * the attention work lists are written on the device from tile offsets that travel as a kernel
 * argument, which limits a graphed batch to VIT_STATIC_MAX_IMAGES images; a larger batch runs as
 * vit_encode_packed does.  Per-kernel timing (vit_profile_*) does not cover these calls.  The first
 * two calls with a key allocate (key, graph); replays do not.
 */
vit_status_t vit_encode_packed_graph(vit_encoder_t* enc, const float* pixels,
                                     const int32_t* images_per_request, int32_t n_requests,
                                     const int32_t* tile_offsets, void* out_tokens,
                                     size_t out_capacity_bytes, int64_t* request_token_offsets,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Free device weights and the handle (an Image Instance scaled in by the pool manager, paper
 * Sec. 4.2, releases its encoder this way).  NULL is allowed.  The caller must have drained
 * every stream the handle was used on. */
void vit_encoder_destroy(vit_encoder_t* enc);

/* Message of the last failure on this thread (static storage, never NULL). */
const char* vit_last_error(void);

/*
 * Timing aid: device time in milliseconds of each kernel family over all vit_encode_packed
 * calls since the last reset, measured with HIP events on the launch stream.  Off by default
 * (it adds events to the stream); enable != 0 switches it on and resets the counters.
 * vit_profile_read synchronises the recorded events and fills ms[VIT_PROF_COUNT] and
 * launches[VIT_PROF_COUNT] with total milliseconds and number of kernel launches per family.
 * Every matrix product of the path has a family of its own.
 */
enum {
  VIT_PROF_PATCHIFY = 0,   /* patch gather, CLS rows, token down-sampling            */
  VIT_PROF_GEMM_PATCH = 1, /* patch-embedding product (+bias +pos)                   */
  VIT_PROF_LAYERNORM = 2,
  VIT_PROF_ATTENTION = 3,
  VIT_PROF_GEMM_QKV = 4,   /* h Wqkv^T + b                                           */
  VIT_PROF_GEMM_OUT = 5,   /* attention output projection, + bias, added to x        */
  VIT_PROF_GEMM_FC1 = 6,   /* first MLP product, + bias, GELU                        */
  VIT_PROF_GEMM_FC2 = 7,   /* second MLP product, + bias, added to x                 */
  VIT_PROF_GEMM_PROJ = 8,  /* projector layers                                       */
  VIT_PROF_COUNT = 9
};
vit_status_t vit_profile_enable(vit_encoder_t* enc, int enable);
vit_status_t vit_profile_read(vit_encoder_t* enc, double* ms, int64_t* launches);

/*
 * Measurement aid: where the persistent matrix-product kernel (the one that runs every large
 * product) spends its time.  While enabled, each workgroup stamps the first 64 tiles it computes
 * in every launch: a constant-rate device clock at the tile's start, after its k-loop and after
 * its epilogue, and the shader clocks the tile took.  vit_profile_tiles_read fills, per family of
 * VIT_PROF_* (arrays of VIT_PROF_COUNT; zero for families that ran no such kernel), the means
 * over the stamped tiles of the LAST launch of that family: microseconds in the k-loop,
 * microseconds in the epilogue, the shader clock in MHz (the chip is power-limited: this is what
 * it held), and the number of tiles stamped.  Enabling allocates 4.5 MiB of pinned host memory
 * (freed by disabling or by vit_encoder_destroy) and both calls synchronise the device; stamps
 * are taken only by vit_encode_packed, not by vit_encode_packed_static.
 * Errors: VIT_EINVAL (NULL, read while disabled), VIT_EDEVICE.
 */
vit_status_t vit_profile_tiles_enable(vit_encoder_t* enc, int enable);
vit_status_t vit_profile_tiles_read(vit_encoder_t* enc, double* main_loop_us, double* epilogue_us,
                                    double* clock_mhz, int64_t* tiles);

/*
 * Pull-style hand-off of finished image tokens (paper Sec. 4.3, "Image Token Transfer": the
 * transfer is deferred until all image tokens of a request are ready; the consumer then pulls
 * them from the producers' addresses).  Host-side table of device pointers and events; the
 * only device work is the copy queued by vit_handoff_pull.  All functions are thread-safe.
 *
 *   vit_handoff_expect   announces request `request_id` with n_images (1 ... 65536) images.
 *   vit_handoff_publish  image `image_index` of the request lies at `tokens` (device memory,
 *                        `bytes` > 0 long) once the work queued so far on `stream` (hipStream_t;
 *                        NULL = null stream) has finished: an event is recorded there.  The
 *                        memory stays the producer's; it must stay valid and unchanged until
 *                        vit_handoff_release and until any pull that was queued has run.
 *   vit_handoff_complete 1 when every image has been published (device work may still be in
 *                        flight), else 0; writes the byte total so far to *total_bytes if not NULL.
 *   vit_handoff_pull     queues on `stream` the copies of all images' tokens, in image order,
 *                        packed back to back into `dst` (device, `capacity` bytes), each behind
 *                        its producer's event; the host does not wait.  *bytes (may be NULL)
 *                        receives the total.  VIT_ENOTREADY if an image is missing,
 *                        VIT_ECAPACITY if dst is too small; nothing is queued then.
 *   vit_handoff_release  forgets the request and destroys its events.
 * Errors: VIT_EINVAL for NULL / unknown request / index out of range / duplicate publish or
 * expect, VIT_ENOMEM, VIT_EDEVICE.  `device` is made current by publish and pull.
 */
typedef struct vit_handoff vit_handoff_t; /* opaque; owned by the library */
vit_status_t vit_handoff_create(int device, vit_handoff_t** out);
void vit_handoff_destroy(vit_handoff_t* h); /* NULL allowed; pending pulls must have run */
vit_status_t vit_handoff_expect(vit_handoff_t* h, int64_t request_id, int32_t n_images);
vit_status_t vit_handoff_publish(vit_handoff_t* h, int64_t request_id, int32_t image_index, const void* tokens,
                                 size_t bytes, void* stream);
int32_t vit_handoff_complete(vit_handoff_t* h, int64_t request_id, size_t* total_bytes);
vit_status_t vit_handoff_pull(vit_handoff_t* h, int64_t request_id, void* dst, size_t capacity, void* stream,
                              size_t* bytes);
vit_status_t vit_handoff_release(vit_handoff_t* h, int64_t request_id);

/*
 * Image preprocessing on the GPU (paper Sec. 2, "Image Preprocessing": resize, rescale and
 * normalise the raw image, segment it into tiles), producing exactly the `pixels` operand of
 * vit_encode_packed.
 *   image       DEVICE, [height, width, channels] uint8, channels interleaved, 1 <= channels <= 4.
 *   The image is resized to (grid_rows * tile_size) x (grid_cols * tile_size) by bilinear
 *   interpolation (pixel centres at half-integers: source coordinate (o + 0.5) * in/out - 0.5,
 *   clamped below at 0, last pixel repeated at the far edge; no low-pass filter when shrinking),
 *   scaled by 1/255, normalised per channel as (v - mean[c]) / std[c], and cut into
 *   grid_rows * grid_cols tiles in row-major tile order.  thumbnail != 0 appends one more tile:
 *   the whole image resized to tile_size x tile_size.
 *   mean, std   HOST, [channels]; std > 0.
 *   out_pixels  DEVICE, [n_tiles, channels, tile_size, tile_size] fp32, n_tiles = grid_rows *
 *               grid_cols (+ 1), 4-byte aligned; out_capacity_bytes is its size.
 *   stream      hipStream_t (NULL = default stream); the call is asynchronous on it and runs on the
 *               calling thread's current device, where both buffers must live.
 * Choosing the tile grid from the image size, padding and tile-level augmentation stay with the caller.
 * Errors: VIT_EINVAL (NULL, non-positive sizes, channels > 4, more than 65534 tiles, std <= 0),
 *         VIT_ECAPACITY (nothing launched), VIT_EDEVICE.
 */
vit_status_t vit_preprocess_tiles(const uint8_t* image, int32_t height, int32_t width, int32_t channels,
                                  int32_t tile_size, int32_t grid_rows, int32_t grid_cols, int32_t thumbnail,
                                  const float* mean, const float* std, float* out_pixels,
                                  size_t out_capacity_bytes, void* stream);

/*
 * Measurement aid (no part of the encode path): runs a register-only bf16 MFMA loop
 * (v_mfma_f32_32x32x16_bf16, two waves per SIMD, no memory traffic) on `device` for about
 * `seconds` (0 < seconds <= 2) on the null stream and writes the sustained rate in TFLOP/s
 * to *tflops (host pointer).  random_operands != 0: the operands are seeded uniform [-1, 1)
 * values, as the products of the encoder have; 0: one constant.  The chip is power-limited
 * and the clock it holds depends on the operand data, so the two differ widely; the random
 * figure is the practical ceiling of the matrix cores for real data, printed by the
 * benchmark beside the nominal peak that every reported fraction uses.  Allocates and frees
 * 65 KiB of device memory; synchronises the device's null stream.
 * Errors: VIT_EINVAL (NULL / range), VIT_EDEVICE.
 */
vit_status_t vit_mfma_ceiling(int device, double seconds, int32_t random_operands, double* tflops);

#pragma GCC visibility pop
#ifdef __cplusplus
}
#endif
#endif /* VITENC_H */
