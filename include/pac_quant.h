/*
 * libpac -- storage side of the first epoch (arXiv 2408.10746, "Further memory efficiency through fine-tuning
 * with quantized LLMs", Eq. "quan" / "dequan", Fig. "quan"): the frozen backbone is kept in a low-bit storage type
 * and its linear layers run in a higher-precision computation type; their outputs are what the activation cache
 * stores (Sec. 4.2).
 *
 *   quantise    per contiguous block of `block` values:  c = qmax / absmax(block)  (a 32-bit constant; qmax = 127
 *               for 8 bits, 7 for 4 bits; an all-zero block has c = 1),  q = round(c * x)  (32-bit product, round to
 *               nearest, ties to even)
 *   dequantise  x' = q / c  (32-bit division)
 *   linear      y[m][n] = sum_k x[m][k] * q[n][k] / c[n][k / block]: the integer codes enter the matrix cores as bf16
 *               (every code is exactly representable), products and sums are fp32, and the block's constant is
 *               applied to the block's partial sum, so nothing but fp32 summation order separates the result from
 *               the exact one
 *
 * 4-bit codes are two's-complement nibbles, two per byte, the even index in the low nibble.
 * Every pointer is HOST or DEVICE as marked; device work is enqueued on `hip_stream`; argument errors are detected
 * on the host before any launch; nothing is allocated.
 */
#ifndef PAC_QUANT_H
#define PAC_QUANT_H

#include <stdint.h>
#include "pac.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Eq. "quan", block-wise.  x DEVICE fp32[n]; codes DEVICE int8[n] (bits = 8) or packed, (n + 1) / 2 bytes (bits = 4);
 * consts DEVICE fp32[ceil(n / block)].  block >= 1 (even for bits = 4).  Errors: NULL, RANGE (n < 0, block),
 * SHAPE (bits), ALIGN (x, consts not 4-byte aligned), DEVICE. */
pac_status pac_quant_blockwise(const float *x /*DEVICE*/, int64_t n, int32_t block, int32_t bits,
                               int8_t *codes /*DEVICE*/, float *consts /*DEVICE*/, void *hip_stream);

/* Eq. "dequan": out[i] = q[i] / c[i / block].  out DEVICE fp32[n].  Errors as above. */
pac_status pac_dequant_blockwise(const int8_t *codes /*DEVICE*/, const float *consts /*DEVICE*/, int64_t n,
                                 int32_t block, int32_t bits, float *out /*DEVICE*/, void *hip_stream);

/* The frozen backbone's linear layer on the stored form (Fig. "quan"): y = x dequant(W)^T.
 *   x      DEVICE bf16 [M][K], 16-byte aligned rows (K a multiple of 32)
 *   codes  DEVICE [N][K] codes of W, each row quantised in blocks of `block` along K (block a multiple of 32 that
 *          divides K); consts DEVICE fp32 [N][K / block]
 *   y      DEVICE fp32 [M][N]
 * Errors: NULL, SHAPE (M, N, K, bits), RANGE (block), ALIGN, DEVICE. */
pac_status pac_dequant_linear(const void *x /*DEVICE*/, int32_t M, int32_t K, const int8_t *codes /*DEVICE*/,
                              const float *consts /*DEVICE*/, int32_t N, int32_t block, int32_t bits,
                              float *y /*DEVICE*/, void *hip_stream);

/* The same layer with the cache fill fused into its epilogue (Sec. 4.2: during the first epoch everything the
 * adapters consume is cached): the output rows of cached layer `layer` of `count` samples go, rounded to the cache
 * dtype, straight to their place in the cache; no dense output exists.
 *   x       DEVICE bf16 [count][n_max][K]; rows t >= len are never read
 *   N       must equal the context's hidden size d
 *   samples are registered as pac_cache_fill registers them: a sample seen for the first time is appended after the
 *   blocks placed so far (its whole block, all layers), a known one must keep its length.
 * Errors: as pac_cache_fill and pac_dequant_linear, RANGE also for layer outside [0, L). */
pac_status pac_dequant_linear_to_cache(pac_ctx *ctx, void *cache /*DEVICE*/, int64_t cache_bytes,
                                       const int64_t *sample_ids /*HOST*/, int32_t count, const int32_t *lens /*HOST*/,
                                       int32_t layer, const void *x /*DEVICE*/, int32_t K,
                                       const int8_t *codes /*DEVICE*/, const float *consts /*DEVICE*/, int32_t block,
                                       int32_t bits, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PAC_QUANT_H */
