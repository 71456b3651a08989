/*
 * CPU oracle for the storage side of the first epoch: block-wise absmax quantisation of the frozen
 * backbone's weights, its inverse, and the mixed-precision linear layer that runs on the stored form
 * (paper: "Further memory efficiency through fine-tuning with quantized LLMs", Eq. "quan" and "dequan",
 * Fig. "quan").
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE: only the tests may build, load or call it.  It shares no code
 * with the HIP path.
 *
 *   quantise      the tensor is cut into contiguous blocks of `block` values; per block
 *                 c = qmax / absmax(block)   (qmax = 127 for 8 bits, 7 for 4 bits; the quantisation constant
 *                                             is a 32-bit float, as the paper writes it)
 *                 q = round(c * x)           (32-bit product, round to nearest, ties to even)
 *                 an all-zero block has c = 1 and q = 0.
 *                 The integer q is decided in 32-bit arithmetic because the paper's constant and input are
 *                 32-bit: both sides of a parity test take that decision in the same precision.
 *   dequantise    x' = q / c                 (32-bit division)
 *   linear layer  y[m][n] = sum_k x[m][k] * (q[n][k] / c[n][k / block]), accumulated in double; the storage
 *                 type is the integer code, the computation type a float (here: as exact as doubles allow)
 *
 * 4-bit codes are two's-complement nibbles, two per byte, the even index in the low nibble.
 *
 * Pins (tests/test_quant_oracle.py): hand cases incl. a tie, the rounding-error bound absmax / (2 qmax) per
 * element, the largest element mapping to +-qmax, block independence (an outlier spoils only its own block),
 * a library rounding routine, and the linear layer against a library matrix product of the dequantised weights.
 * The paper prints no numeric example of Eq. "quan": against its own numbers "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static float block_constant(const float *x, int64_t n, int qmax)
{
    float amax = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        float a = fabsf(x[i]);
        if (a > amax) amax = a;
    }
    if (amax == 0.0f) return 1.0f;
    return (float)qmax / amax;
}

/* x[n] -> codes (int8 per value for bits = 8; packed nibbles, (n + 1) / 2 bytes, for bits = 4) and one
 * constant per block (ceil(n / block) of them).  Returns 0, -1 on bad arguments. */
int orc_quant_blockwise(const float *x, int64_t n, int32_t block, int32_t bits, int8_t *codes, float *consts)
{
    if (!x || !codes || !consts || n < 0 || block < 1 || (bits != 8 && bits != 4)) return -1;
    const int qmax = bits == 8 ? 127 : 7;
    if (bits == 4) memset(codes, 0, (size_t)((n + 1) / 2));
    for (int64_t b0 = 0, bi = 0; b0 < n; b0 += block, ++bi) {
        const int64_t len = n - b0 < block ? n - b0 : block;
        const float c = block_constant(x + b0, len, qmax);
        consts[bi] = c;
        for (int64_t i = b0; i < b0 + len; ++i) {
            const float scaled = c * x[i];              /* 32-bit product */
            const int q = (int)rintf(scaled);           /* nearest, ties to even (default rounding mode) */
            if (bits == 8) {
                codes[i] = (int8_t)q;
            } else {
                const uint8_t nib = (uint8_t)(q & 0xf);
                uint8_t *byte = (uint8_t *)codes + i / 2;
                *byte = (i & 1) ? (uint8_t)((*byte & 0x0f) | (nib << 4)) : (uint8_t)((*byte & 0xf0) | nib);
            }
        }
    }
    return 0;
}

static int code_at(const int8_t *codes, int64_t i, int32_t bits)
{
    if (bits == 8) return codes[i];
    const uint8_t byte = ((const uint8_t *)codes)[i / 2];
    const int nib = (i & 1) ? (byte >> 4) : (byte & 0xf);
    return nib >= 8 ? nib - 16 : nib;
}

int orc_dequant_blockwise(const int8_t *codes, const float *consts, int64_t n, int32_t block, int32_t bits, float *out)
{
    if (!codes || !consts || !out || n < 0 || block < 1 || (bits != 8 && bits != 4)) return -1;
    for (int64_t i = 0; i < n; ++i) out[i] = (float)code_at(codes, i, bits) / consts[i / block];
    return 0;
}

/* y[M][N] (double) = x[M][K] (float) times the dequantised W[N][K]; W's rows are quantised independently in
 * blocks of `block` along K (K a multiple of block), consts[N][K / block]. */
int orc_dequant_linear(const float *x, int32_t M, int32_t K, const int8_t *codes, const float *consts, int32_t N,
                       int32_t block, int32_t bits, double *y)
{
    if (!x || !codes || !consts || !y || M < 0 || N < 0 || K < 1 || block < 1 || K % block || (bits != 8 && bits != 4))
        return -1;
    const int64_t bpr = K / block;
    for (int32_t m = 0; m < M; ++m)
        for (int32_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int32_t k = 0; k < K; ++k) {
                const float w = (float)code_at(codes, (int64_t)n * K + k, bits) / consts[(int64_t)n * bpr + k / block];
                acc += (double)x[(int64_t)m * K + k] * (double)w;
            }
            y[(int64_t)m * N + n] = acc;
        }
    return 0;
}
