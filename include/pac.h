/*
 * libpac -- cached Parallel-Adapter training step on one MI355X (gfx950).
 *
 * The library implements the epoch >= 2 phase of PAC+ (arXiv 2408.10746):
 * the frozen backbone's per-layer hidden states are stored once
 * (pac_cache_fill; paper Sec. 4.2, "activation cache") and every later
 * training step runs forward and backward through the side adapter network
 * only (pac_adapter_step; paper Sec. 4.1 "Parallel Adapters", Sec. 5.2
 * "data-parallel fine-tuning for Parallel Adapters").  No backbone forward or
 * backward is ever executed here and no gradient flows into the cache.
 *
 * The network (linear down/up-projection adapters, Sec. 4.1; gate initialised
 * to 0.5, Sec. 4.1; zero-initialised up-projection, Sec. 4.3), with L cached
 * layers b_1..b_L, hidden size d, adapter width r, C classes:
 *
 *     s_0 = 0
 *     x_l   = lambda_l * b_l + (1 - lambda_l) * s_{l-1}
 *     pre_l = x_l W_down^l + c_down^l          h_l = GELU_erf(pre_l)
 *     s_l   = s_{l-1} + h_l W_up^l + c_up^l
 *     y = b_L + s_L ;  p = mean over valid tokens ;  z = p W_cls + c_cls
 *     loss = mean over the batch of softmax cross-entropy(z, label)
 *
 * followed by the exact gradients and one AdamW update.
 *
 * CONVENTIONS
 *  - Every pointer is marked HOST or DEVICE.  The caller allocates and frees
 *    every device buffer; the library allocates only the host-side pac_ctx and
 *    keeps no device pointer between calls.
 *  - All device work is enqueued on the HIP stream passed in (`hip_stream` is
 *    a hipStream_t cast to void*, NULL = the default stream).  No call blocks
 *    on the device; outputs are valid once the caller synchronises the stream.
 *  - Every entry point returns a pac_status.  Argument errors are detected on
 *    the host before anything is launched and leave device memory untouched.
 *    Nothing throws, aborts or prints.
 *  - Threads: a pac_ctx may be used by one host thread at a time (pac_cache_fill records sample
 *    positions in it, the profiling calls keep their events in it).  Different contexts may be used
 *    from different host threads at once; the library's only process-wide state is the one-time
 *    kernel attribute set-up, which is done under std::call_once.  pac_adapter_step_static calls
 *    additionally share one per-device scratch array (see there).
 *  - Arithmetic follows the cache dtype: a bf16 cache runs the contractions on
 *    bf16 MFMA with fp32 accumulation (side state, gradients, optimizer and
 *    master weights stay fp32); an fp32 cache runs everything in fp32.
 *
 * PARAMETER VECTOR (flat fp32, P = L*(2dr + r + d + 1) + dC + C entries)
 *    per layer  [ W_down (d x r, r contiguous) | c_down (r) | W_up (r x d, d contiguous)
 *                 | c_up (d) | lambda (1) ]
 *    then       [ W_cls (d x C, C contiguous) | c_cls (C) ]
 *
 * CACHE (paper Sec. 5.2: tokens x hidden x layers elements per sequence)
 *    sample s owns one block [layer][token][d], d contiguous, holding only its
 *    len_s valid tokens; blocks are packed in fill order.  Element size is 2
 *    (bf16, round-to-nearest-even at fill) or 4 (fp32, copied unchanged).
 */
#ifndef PAC_H
#define PAC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pac_ctx pac_ctx; /* opaque host object; owns no device memory */

typedef enum {
    PAC_OK = 0,
    PAC_ERR_NULL = 1,        /* a required pointer is NULL */
    PAC_ERR_SHAPE = 2,       /* a dimension is non-positive or inconsistent */
    PAC_ERR_RANGE = 3,       /* an index/length/count is outside its range */
    PAC_ERR_ALIGN = 4,       /* a device pointer is not aligned as required */
    PAC_ERR_UNSUPPORTED = 5, /* a valid shape this build has no kernel for */
    PAC_ERR_WORKSPACE = 6,   /* workspace or cache buffer too small */
    PAC_ERR_DEVICE = 7,      /* the HIP runtime reported an error */
    PAC_ERR_STATE = 8        /* a sample that was never filled is referenced */
} pac_status;

typedef enum { PAC_BF16 = 0, PAC_F32 = 1 } pac_dtype;

/*
 * L      cached layers (>= 1)                d      hidden size (multiple of 32)
 * n_max  longest sequence (>= 1)             r      adapter width (multiple of 32)
 * C      classes (1..16)                     B_max  largest batch of one step (1..64)
 * N      samples the cache can index (>= 1)  cache_dtype  PAC_BF16 or PAC_F32
 * flags  see PAC_FLAG_* below
 */
typedef struct {
    int32_t L, d, n_max, r, C, B_max;
    int64_t N;
    int32_t cache_dtype;
    int32_t flags; /* 0, or PAC_FLAG_* or-ed together */
} pac_config;

/* Run the step with the per-layer kernels even where the faster Gram-matrix
 * formulation applies (same results up to rounding; kept for cross-checking). */
#define PAC_FLAG_PER_LAYER 1
/* Measurement aid: launch every part of the fused multi-part launches on its own, so that
 * pac_profile_end reports one class per part (slower; results unchanged). */
#define PAC_FLAG_SPLIT_LAUNCH 2
/* On the Gram-matrix path, run the two chains over the layers layer by layer (groups of layers: one
 * wide contraction per group, one short one per layer; the form used where a 16-token tile's history
 * of all layers does not fit a compute unit's LDS, e.g. r > 128) even where the single-launch chains
 * apply (same results up to rounding). */
#define PAC_FLAG_LAYER_CHAIN 4

typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
} pac_adamw;

/* Fixes the shape of the side network and of its cache (paper Sec. 4.1: one adapter per backbone layer,
 * width d / reduction factor; Table "model" and Sec. 6.1 for the shapes the paper trains) and builds the
 * host context: validation, the parameter layout, the workspace plan, the per-sample position table.
 * No device work.  PAC_ERR_NULL / PAC_ERR_SHAPE / PAC_ERR_UNSUPPORTED on bad input; *out untouched then. */
pac_status pac_create(const pac_config *cfg /*HOST*/, pac_ctx **out /*HOST*/);
/* Frees the host context (the cache and every other device buffer belong to the caller: Sec. 4.2's cache
 * outlives any one training run).  NULL is allowed. */
void pac_destroy(pac_ctx *ctx);
/* Text of a status code (static storage); every entry point of Sec. 4.2 / 5.2's two phases reports through it. */
const char *pac_status_str(pac_status s);

/* P, the number of trainable values: the adapters of Sec. 4.1 (down- and up-projection with biases and the gate
 * lambda per layer) plus the classification head; the backbone contributes none (it is frozen, Sec. 4.1).
 * Layout above.  -1 if ctx is NULL. */
int64_t pac_param_count(const pac_ctx *ctx);

/* Where each tensor of Sec. 4.1's adapter l sits in the flat vector (offsets in elements).  layer in [0, L):
 * out[0..4] = W_down, c_down, W_up, c_up, lambda.  layer = -1: out[0..1] = W_cls, c_cls (out[2..4] = -1).
 * PAC_ERR_NULL, PAC_ERR_RANGE. */
pac_status pac_param_offsets(const pac_ctx *ctx, int32_t layer, int64_t out[5] /*HOST*/);

/* Bytes of cache needed for `count` samples with the given valid lengths
 * (paper Sec. 5.2: len x d x L elements each).  lens HOST, count entries, or
 * NULL = every sample has n_max tokens.  -1 on bad arguments. */
int64_t pac_cache_bytes(const pac_ctx *ctx, const int32_t *lens /*HOST*/, int64_t count);

/* Bytes of device workspace pac_adapter_step / pac_adapter_loss_grad need for a batch of up to B_max samples
 * of up to n_max tokens: what the cached phase of Sec. 5.2 keeps per step besides the cache (r-wide
 * activations of the side network, compute-dtype copies of the projections, partial sums of the token
 * reductions; no d-wide per-token state on the Gram-matrix path).  -1 if ctx is NULL. */
int64_t pac_workspace_bytes(const pac_ctx *ctx);

/* Which formulation of the step (paper Sec. 4.1, 5.2: the same function of the same inputs in each)
 * this configuration runs on: 0 the per-layer kernels; 1 the Gram-matrix formulation with the chains
 * over the layers as one launch per direction; 2 the Gram-matrix formulation with the chains launched
 * layer by layer.  Decided by pac_create from the shape, cache dtype and flags.  -1 if ctx is NULL. */
int32_t pac_step_path(const pac_ctx *ctx);

/*
 * Store one backbone forward's per-layer activations (paper Sec. 4.2: during
 * the first epoch everything the adapters consume is cached).
 *   cache       DEVICE, cache_bytes long, 256-byte aligned.
 *   sample_ids  HOST, count entries in [0, N), no repeats within a call.
 *   acts        DEVICE, [count][L][n_max][d] of acts_dtype, d contiguous, 16-byte aligned.
 *   lens        HOST, count entries in [1, n_max], or NULL = n_max for all.
 * A sample filled for the first time is appended after the blocks filled so
 * far; a sample filled again must keep its length and is overwritten in
 * place.  Rows t >= len of acts are never read.  bf16 storage rounds to
 * nearest-even, NaN stays NaN, infinities pass through.
 * Errors: NULL, RANGE (id/len/count), STATE (length changed), WORKSPACE (cache
 * too small), ALIGN, DEVICE.  On error nothing is recorded or written.
 */
pac_status pac_cache_fill(pac_ctx *ctx, void *cache /*DEVICE*/, int64_t cache_bytes,
                          const int64_t *sample_ids /*HOST*/, int32_t count,
                          const void *acts /*DEVICE*/, int32_t acts_dtype,
                          const int32_t *lens /*HOST*/, void *hip_stream);

/* Where a filled sample lives: element offset of its block ([layer][token][d], Sec. 5.2's tokens x hidden x
 * layers elements) and its length.  PAC_ERR_NULL, PAC_ERR_RANGE; PAC_ERR_STATE if it was never filled. */
pac_status pac_cache_lookup(const pac_ctx *ctx, int64_t sample_id,
                            int64_t *offset_elems /*HOST*/, int32_t *len /*HOST*/);

/*
 * Loss and gradients of one batch read from the cache, without an update: the forward pass through the side
 * network of Sec. 4.1 on cached activations (Sec. 4.2), the loss, and the exact gradients with respect to
 * the adapters and the head only (Sec. 4.1: no gradient enters the backbone).  Same forward/backward as
 * pac_adapter_step; used for evaluation and parity.
 *   cache       DEVICE (const: the backbone is frozen, nothing is written to it)
 *   sample_ids  HOST, B entries, each filled before; 1 <= B <= B_max
 *   labels      DEVICE, int32[B], each in [0, C) (out-of-range labels give a NaN loss)
 *   params      DEVICE, fp32[P]
 *   workspace   DEVICE, >= pac_workspace_bytes(), 256-byte aligned; contents are scratch
 *   loss_out    DEVICE, fp32[1]
 *   logits_out  DEVICE, fp32[B][C], or NULL
 *   grads_out   DEVICE, fp32[P], or NULL (then only the forward pass runs)
 */
pac_status pac_adapter_loss_grad(pac_ctx *ctx, const void *cache /*DEVICE*/,
                                 const int64_t *sample_ids /*HOST*/, int32_t B,
                                 const int32_t *labels /*DEVICE*/, const float *params /*DEVICE*/,
                                 void *workspace /*DEVICE*/, int64_t workspace_bytes,
                                 float *loss_out /*DEVICE*/, float *logits_out /*DEVICE*/,
                                 float *grads_out /*DEVICE*/, void *hip_stream);

/*
 * One optimizer step driven by the cache (paper Sec. 5.2: after the first
 * epoch only the adapters are trained, from cached activations): forward,
 * loss, backward, AdamW (decoupled decay on W_down, W_up, W_cls; bias-corrected;
 * eps added to the root of the corrected second moment).
 *   params, m, v  DEVICE, fp32[P], updated in place
 *   step          HOST, in/out: number of updates applied so far (incremented)
 *   grads_out     DEVICE fp32[P] or NULL (then the gradient lives in the workspace)
 * Other arguments as in pac_adapter_loss_grad.
 */
pac_status pac_adapter_step(pac_ctx *ctx, const void *cache /*DEVICE*/,
                            const int64_t *sample_ids /*HOST*/, int32_t B,
                            const int32_t *labels /*DEVICE*/,
                            float *params /*DEVICE*/, float *m /*DEVICE*/, float *v /*DEVICE*/,
                            int64_t *step /*HOST*/, const pac_adamw *hp /*HOST*/,
                            void *workspace /*DEVICE*/, int64_t workspace_bytes,
                            float *loss_out /*DEVICE*/, float *grads_out /*DEVICE*/,
                            void *hip_stream);

/*
 * The same step for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation): the workspace is a file-scope device
 * array inside the library, PAC_STATIC_WORKSPACE_BYTES long, which every GPU the library runs on holds
 * from the first such call until the process ends.  Nothing is allocated or freed, by the library or
 * through any other library, and nothing is recorded for the profiling calls.
 * Limits: pac_workspace_bytes(ctx) must not exceed PAC_STATIC_WORKSPACE_BYTES (PAC_ERR_WORKSPACE otherwise,
 * before anything is launched).  Every call on one GPU uses that GPU's one array, whose contents are scratch
 * between calls: calls that overlap on one GPU (two streams, two host threads, two contexts) race; calls
 * ordered on one stream are safe.  Other arguments, results and errors as in pac_adapter_step, which shares
 * its kernels.
 */
#define PAC_STATIC_WORKSPACE_BYTES (64ll << 20)
pac_status pac_adapter_step_static(pac_ctx *ctx, const void *cache /*DEVICE*/,
                                   const int64_t *sample_ids /*HOST*/, int32_t B,
                                   const int32_t *labels /*DEVICE*/,
                                   float *params /*DEVICE*/, float *m /*DEVICE*/, float *v /*DEVICE*/,
                                   int64_t *step /*HOST*/, const pac_adamw *hp /*HOST*/,
                                   float *loss_out /*DEVICE*/, float *grads_out /*DEVICE*/,
                                   void *hip_stream);

/*
 * Measurement aids for the two rooflines the step is set against (Sec. 5.2 calls the cached phase
 * lightweight: it is bound by how fast the cache streams from memory and, for wide adapters, by the matrix
 * units).  Neither is part of the training path.
 *   pac_probe_hbm_read   reads `bytes` (a multiple of 16) of `buf` once with every compute unit busy and
 *                        nothing else to do (16-byte loads, several in flight per lane, xor-folded into
 *                        sink[0..255] so that the loads cannot be dropped): bytes / duration is the read rate
 *                        this chip sustains on that buffer, e.g. the resident cache slice of one step.
 *   pac_probe_mfma_bf16  runs `iters` rounds of four independent 32x32x16 bf16 matrix instructions per
 *                        wavefront on register operands, four wavefronts per SIMD on every compute unit:
 *                        pac_probe_mfma_flops(iters) / duration is the matrix rate this chip sustains.
 *   pac_probe_hbm_update reads four arrays of n floats and writes three of them back (p, m, v in place; g read
 *                        only), one multiply-add per element: the access mix of the optimizer update (Sec. 5.2's
 *                        step ends with it) without its arithmetic; 28 n / duration is the rate this chip sustains
 *                        on that mix, which a read-only figure overstates.  n a multiple of 4, arrays 16-byte aligned.
 * sink: DEVICE, 256 floats, scratch.  The caller times the call with events on the same stream.
 * Errors: NULL, RANGE (bytes or iters not positive, bytes not a multiple of 16), ALIGN (buf not 16-byte
 * aligned), DEVICE.
 */
pac_status pac_probe_hbm_read(const void *buf /*DEVICE*/, int64_t bytes, float *sink /*DEVICE*/, void *hip_stream);
pac_status pac_probe_mfma_bf16(int64_t iters, float *sink /*DEVICE*/, void *hip_stream);
double pac_probe_mfma_flops(int64_t iters); /* flops one pac_probe_mfma_bf16(iters) call executes */
pac_status pac_probe_hbm_update(float *p /*DEVICE*/, float *m /*DEVICE*/, float *v /*DEVICE*/, const float *g /*DEVICE*/,
                                int64_t n, void *hip_stream);

/*
 * Measurement aid (not part of the training path): per-kernel timing with HIP
 * events recorded on the caller's stream around every kernel the library
 * launches, so the duration of each kernel class can be set against its
 * roofline (HBM bytes for the cache stream, MFMA flops for the adapter
 * contractions; paper Sec. 5.2 calls the cached phase lightweight, which makes
 * it bandwidth- and latency-sensitive).
 *   pac_profile_begin  starts recording for later calls on this context.
 *   pac_profile_end    waits for the recorded events, adds up elapsed time and
 *                      launch counts per kernel class into ms[]/launches[]
 *                      (HOST, max_classes entries each), stores the number of
 *                      classes in *n_classes and stops recording.
 *   pac_profile_class_name  name of class i, NULL past the end.
 * Errors: NULL, STATE (end without begin), WORKSPACE (max_classes too small), DEVICE.
 */
pac_status pac_profile_begin(pac_ctx *ctx);
pac_status pac_profile_end(pac_ctx *ctx, int32_t max_classes, float *ms /*HOST*/,
                           int32_t *launches /*HOST*/, int32_t *n_classes /*HOST*/);
const char *pac_profile_class_name(int32_t cls);

#ifdef __cplusplus
}
#endif
#endif /* PAC_H */
