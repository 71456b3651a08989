/*
 * libpac -- activation cache larger than device memory (arXiv 2408.10746, Sec. 5.2, storage cost analysis: the cache
 * is kept on the slower, larger storage tier and reloaded per micro-batch while training proceeds).
 *
 * Here the large tier is pinned host memory and the reload is a per-batch prefetch into a small device window:
 * the host cache has exactly the layout of a device cache (sample blocks [layer][token][d] at the offsets the
 * context records), a window holds the blocks of one batch packed in batch order, and the step kernels read the
 * window as they would read a resident cache.  The caller owns every buffer (host cache: pinned; windows: device)
 * and orders the copy stream against the compute stream with its own events: two windows and two streams give the
 * overlap of the next batch's reload with the current step.
 *
 * Nothing is allocated; every call only enqueues copies / kernels on the stream it is given.
 */
#ifndef PAC_TIER_H
#define PAC_TIER_H

#include <stdint.h>
#include "pac.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes a window needs for any batch of up to B_max samples of up to n_max tokens.  -1 if ctx is NULL. */
int64_t pac_tier_window_bytes(const pac_ctx *ctx);

/* pac_cache_fill for a host-resident cache (Sec. 4.2: the first epoch stores what the adapters consume; Sec. 5.2: on
 * the large tier): the activations are converted into `window` (packed in call order) and each sample's block is then
 * copied to its place in the host cache; samples are registered in ctx exactly as pac_cache_fill registers them.
 *   host_cache  HOST, pinned, host_bytes long, 256-byte aligned
 *   window      DEVICE, window_bytes long, 256-byte aligned, scratch; count <= B_max
 * Other arguments and errors as pac_cache_fill; WORKSPACE also when the window is too small. */
pac_status pac_tier_fill(pac_ctx *ctx, void *host_cache /*HOST pinned*/, int64_t host_bytes,
                         const int64_t *sample_ids /*HOST*/, int32_t count, const void *acts /*DEVICE*/,
                         int32_t acts_dtype, const int32_t *lens /*HOST*/, void *window /*DEVICE*/,
                         int64_t window_bytes, void *hip_stream);

/* Reload of one batch (Sec. 5.2: the cache is reloaded per micro-batch): copies the blocks of `sample_ids`, in that
 * order, from the host cache into `window`, back to back.  Errors: NULL, RANGE, STATE (a sample never filled),
 * ALIGN, WORKSPACE (window too small), DEVICE. */
pac_status pac_tier_stage(const pac_ctx *ctx, const void *host_cache /*HOST pinned*/,
                          const int64_t *sample_ids /*HOST*/, int32_t B, void *window /*DEVICE*/,
                          int64_t window_bytes, void *copy_stream);

/* pac_adapter_loss_grad / pac_adapter_step on a staged batch (Sec. 5.2: adapter-only training from the reloaded
 * cache): `window` must hold the blocks of exactly these sample_ids in this order (pac_tier_stage).  Same kernels,
 * same results bit for bit as the calls on a resident cache.  Arguments and errors as those calls. */
pac_status pac_adapter_loss_grad_staged(pac_ctx *ctx, const void *window /*DEVICE*/,
                                        const int64_t *sample_ids /*HOST*/, int32_t B,
                                        const int32_t *labels /*DEVICE*/, const float *params /*DEVICE*/,
                                        void *workspace /*DEVICE*/, int64_t workspace_bytes,
                                        float *loss_out /*DEVICE*/, float *logits_out /*DEVICE*/,
                                        float *grads_out /*DEVICE*/, void *hip_stream);
pac_status pac_adapter_step_staged(pac_ctx *ctx, const void *window /*DEVICE*/,
                                   const int64_t *sample_ids /*HOST*/, int32_t B,
                                   const int32_t *labels /*DEVICE*/,
                                   float *params /*DEVICE*/, float *m /*DEVICE*/, float *v /*DEVICE*/,
                                   int64_t *step /*HOST*/, const pac_adamw *hp /*HOST*/,
                                   void *workspace /*DEVICE*/, int64_t workspace_bytes,
                                   float *loss_out /*DEVICE*/, float *grads_out /*DEVICE*/,
                                   void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PAC_TIER_H */
