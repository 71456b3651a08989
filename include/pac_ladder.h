/*
 * libpac -- the paper's default Parallel-Adapter architecture trained from the activation cache
 * (arXiv 2408.10746, Sec. 4.1 and Fig. "pa-detail", Sec. 6.1; cached phase Sec. 4.2 / 5.2).
 *
 * Where pac_adapter_step trains the linear down/up-projection variant with a d-wide side state, these calls
 * train the r-wide ladder: with w = pac_config.r the adapter width (d over the paper's reduction factor),
 *
 *     u_l = b_l W_down^l + c_down^l                  x_l = lambda_l u_l + (1 - lambda_l) a_{l-1},  a_0 = 0
 *     a_l = Block_l(x_l)      a pre-norm transformer layer at width w (`heads` heads, FFN width 4 w, GELU_erf,
 *                             LayerNorm eps 1e-5): the first operation of the path that mixes tokens
 *     y = b_L + a_L W_up + c_up ;  p = mean over valid tokens ;  z = p W_cls + c_cls ;  mean cross-entropy
 *
 * followed by the exact gradients and AdamW (decoupled decay on the matrices only).  The cache, the context and
 * the conventions are those of pac.h: the same pac_ctx (created with r = w) addresses the same cache.
 * Arithmetic is fp32 throughout (fp32 matrix instructions); a bf16 cache is widened exactly.
 *
 * PARAMETER VECTOR (flat fp32; every tensor starts 16-byte aligned)
 *   per layer [ W_down d x w | c_down w | ln1_g w | ln1_b w | W_qkv w x 3w | b_qkv 3w | W_o w x w | b_o w | ln2_g w |
 *               ln2_b w | W_1 w x 4w | b_1 4w | W_2 4w x w | b_2 w | lambda, 3 unused zeros ]
 *   then      [ W_up w x d | c_up d | W_cls d x C | c_cls C ]
 *
 * Supported: w a multiple of 32 up to 256, w / heads in {4, 8, 16, 32, 64}, n_max * (w / heads) <= 4096
 * (one head of one sample is kept on chip).  Otherwise PAC_ERR_UNSUPPORTED.
 */
#ifndef PAC_LADDER_H
#define PAC_LADDER_H

#include <stdint.h>
#include "pac.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Length of the parameter vector above (Sec. 4.1: one adapter per backbone layer, one final up-projection, the head);
 * -1 if ctx is NULL. */
int64_t pac_ladder_param_count(const pac_ctx *ctx);

/* Bytes of device workspace the two calls below need (the r-wide activations of every layer kept for the reverse
 * pass, one layer's cache rows widened to fp32, split sums of the token reductions); -1 on bad arguments. */
int64_t pac_ladder_workspace_bytes(const pac_ctx *ctx, int32_t heads);

/* Loss, logits and gradients of one batch read from the cache (Sec. 4.2: the cached activations are all the ladder
 * consumes; no gradient enters the backbone).  Arguments as pac_adapter_loss_grad, plus `heads`.
 * grads_out NULL: forward only. */
pac_status pac_ladder_loss_grad(pac_ctx *ctx, const void *cache /*DEVICE*/, const int64_t *sample_ids /*HOST*/,
                                int32_t B, const int32_t *labels /*DEVICE*/, int32_t heads,
                                const float *params /*DEVICE*/, void *workspace /*DEVICE*/, int64_t workspace_bytes,
                                float *loss_out /*DEVICE*/, float *logits_out /*DEVICE*/, float *grads_out /*DEVICE*/,
                                void *hip_stream);

/* One optimizer step of the ladder from the cache (Sec. 5.2).  Arguments as pac_adapter_step, plus `heads`. */
pac_status pac_ladder_step(pac_ctx *ctx, const void *cache /*DEVICE*/, const int64_t *sample_ids /*HOST*/, int32_t B,
                           const int32_t *labels /*DEVICE*/, int32_t heads, float *params /*DEVICE*/,
                           float *m /*DEVICE*/, float *v /*DEVICE*/, int64_t *step /*HOST*/,
                           const pac_adamw *hp /*HOST*/, void *workspace /*DEVICE*/, int64_t workspace_bytes,
                           float *loss_out /*DEVICE*/, float *grads_out /*DEVICE*/, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PAC_LADDER_H */
