/*
 * CPU oracle for the cached Parallel-Adapter training step.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may build, load or call it.  It
 * shares no code with the HIP path and is deliberately plain: scalar loops,
 * double precision everywhere, no blocking, no fusion, no reordering beyond
 * what the definitions below state.
 *
 * What is computed (paper: Parallel Adapters, Sec. 4.1; activation cache,
 * Sec. 4.2; zero-initialised up-projection, Sec. 4.3; data-parallel cached
 * phase, Sec. 5.2).  The adapter block is the linear down/up-projection
 * variant the paper declares compatible (Sec. 4.1), with a d-wide side state:
 *
 *   s_0 = 0
 *   for l = 1..L, every valid token t:
 *     x   = lambda_l * b_l[t] + (1 - lambda_l) * s_{l-1}[t]        (gate, Sec. 4.1)
 *     pre = x W_down^l + c_down^l                                  (d -> r)
 *     h   = GELU(pre) = 0.5 pre (1 + erf(pre / sqrt 2))
 *     s_l[t] = s_{l-1}[t] + h W_up^l + c_up^l                      (r -> d)
 *   y[t] = b_L[t] + s_L[t]                 (side output summed with backbone output)
 *   p    = mean over the valid tokens of y
 *   z    = p W_cls + c_cls ;  loss = mean over the batch of  logsumexp(z) - z[label]
 *
 * Gradients are the exact chain rule of the above with respect to every
 * parameter; nothing flows into the cached activations b (frozen backbone,
 * Sec. 4.1/4.2).  The optimizer is AdamW with decoupled decay on the matrices.
 *
 * Parameter vector layout (one flat array, P = L*(2dr + r + d + 1) + dC + C):
 *   per layer  [ W_down (d x r, row-major) | c_down (r) | W_up (r x d) | c_up (d) | lambda (1) ]
 *   then       [ W_cls (d x C) | c_cls (C) ]
 *
 * Cache layout: sample s owns a block of L*len_s*d values, [layer][token][d],
 * d contiguous, starting at element offset off[s].
 *
 * Pins (see tests, all CPU-only): finite differences, autograd of an
 * independently typed forward, the zero-init identity, loss = ln C for a zero
 * head, permutation / padding / batch-split invariants, AdamW closed forms and
 * a library AdamW, bf16 rounding against hand cases and a library cast.
 * No value printed in the paper covers this path, so against the paper's own
 * numbers this oracle is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef M_PI
#define M_PI 3.14159265358979323846
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int64_t orc_layer_block(int32_t d, int32_t r)
{
    return 2 * (int64_t)d * r + r + d + 1;
}

int64_t orc_param_count(int32_t L, int32_t d, int32_t r, int32_t C)
{
    return (int64_t)L * orc_layer_block(d, r) + (int64_t)d * C + C;
}

/* ---- bf16 storage format: 1 sign, 8 exponent, 7 mantissa bits = the top half
 * of an IEEE binary32.  Conversion rounds to nearest, ties to even; NaN stays
 * NaN (quiet bit forced so the payload cannot round to infinity), infinities
 * pass through. ---- */
uint16_t orc_f32_to_bf16_bits(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u && (u & 0x007fffffu) != 0u)
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

float orc_bf16_bits_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* Cache storage cost of one sequence: tokens x hidden x layers elements
 * (paper Sec. 5.2, storage cost analysis). */
int64_t orc_cache_elems_per_sample(int32_t L, int32_t len, int32_t d)
{
    return (int64_t)L * len * d;
}

/*
 * Store one backbone forward's per-layer activations into the cache
 * (paper Sec. 4.2: everything the adapters consume is kept once).
 * acts: [count][L][n_max][d] fp32.  lens[count] (NULL = all n_max).
 * Output block of sample i starts at off[i] (filled here, append order from 0)
 * and holds [L][len_i][d].  as_bf16 != 0: out is uint16 bf16 bits; else out is
 * float (copied unchanged).  Returns total elements written.
 */
int64_t orc_cache_fill(const float *acts, int32_t count, int32_t L, int32_t n_max, int32_t d,
                       const int32_t *lens, int as_bf16, void *out, int64_t *off)
{
    int64_t pos = 0;
    for (int32_t i = 0; i < count; ++i) {
        int32_t len = lens ? lens[i] : n_max;
        off[i] = pos;
        for (int32_t l = 0; l < L; ++l)
            for (int32_t t = 0; t < len; ++t)
                for (int32_t j = 0; j < d; ++j) {
                    float a = acts[(((int64_t)i * L + l) * n_max + t) * d + j];
                    int64_t o = pos + ((int64_t)l * len + t) * d + j;
                    if (as_bf16) ((uint16_t *)out)[o] = orc_f32_to_bf16_bits(a);
                    else ((float *)out)[o] = a;
                }
        pos += orc_cache_elems_per_sample(L, len, d);
    }
    return pos;
}

void orc_bf16_to_f32_array(const uint16_t *in, int64_t n, float *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = orc_bf16_bits_to_f32(in[i]);
}

static double gelu(double u)
{
    return 0.5 * u * (1.0 + erf(u / sqrt(2.0)));
}

/* d/du [u Phi(u)] = Phi(u) + u phi(u), Phi/phi the standard normal cdf/pdf */
static double gelu_deriv(double u)
{
    double Phi = 0.5 * (1.0 + erf(u / sqrt(2.0)));
    double phi = exp(-0.5 * u * u) / sqrt(2.0 * M_PI);
    return Phi + u * phi;
}

/*
 * Loss, logits and gradients of one batch.
 *   cache : float values (bf16 values widened exactly, or fp32), packed layout
 *   off[B], lens[B] : block offset (elements) and valid length of each batch sample
 *   labels[B]
 *   params[P]  (double)
 * out: *loss, logits[B*C] (may be NULL), pooled[B*d] (may be NULL),
 *      grads[P] (may be NULL; overwritten),
 *      glam_abs[L] (may be NULL; overwritten; needs grads): the cancellation scale of each gate
 *      gradient, sum over tokens and channels of |(b_l - s_{l-1}) * dx|, i.e. the same terms as
 *      dlambda_l with their signs dropped.  It bounds |dlambda_l| from above, with equality when
 *      all terms share one sign, and is the size against which a rounding error of that sum is
 *      to be judged (the gate of Sec. 4.1 mixes two d-wide streams, so its gradient is a sum of
 *      tokens x d signed terms that may cancel).
 * Returns 0, or -1 on allocation failure / bad label / bad length.
 */
int orc_loss_grad(int32_t L, int32_t d, int32_t r, int32_t C, int32_t B,
                  const float *cache, const int64_t *off, const int32_t *lens,
                  const int32_t *labels, const double *params,
                  double *loss, double *logits, double *pooled, double *grads, double *glam_abs)
{
    const int64_t PL = orc_layer_block(d, r);
    const int64_t P = orc_param_count(L, d, r, C);
    const double *Wcls = params + (int64_t)L * PL;
    const double *ccls = Wcls + (int64_t)d * C;
    double *gWcls = NULL, *gccls = NULL;
    if (grads) {
        memset(grads, 0, (size_t)P * sizeof(double));
        gWcls = grads + (int64_t)L * PL;
        gccls = gWcls + (int64_t)d * C;
        if (glam_abs) memset(glam_abs, 0, (size_t)L * sizeof(double));
    }
    double total = 0.0;

    for (int32_t sidx = 0; sidx < B; ++sidx) {
        const int32_t len = lens[sidx];
        if (len <= 0 || labels[sidx] < 0 || labels[sidx] >= C) return -1;
        const float *blk = cache + off[sidx];
        const size_t nd = (size_t)len * d, nr = (size_t)len * r;
        /* S[l] = side state after l layers, l = 0..L ; PRE[l], H[l] of layer l+1 */
        double *S = (double *)calloc((size_t)(L + 1) * nd, sizeof(double));
        double *PRE = (double *)malloc((size_t)L * nr * sizeof(double));
        double *H = (double *)malloc((size_t)L * nr * sizeof(double));
        double *p = (double *)calloc((size_t)d, sizeof(double));
        double *z = (double *)malloc((size_t)C * sizeof(double));
        if (!S || !PRE || !H || !p || !z) { free(S); free(PRE); free(H); free(p); free(z); return -1; }

        /* ---- forward through the side network ---- */
        for (int32_t l = 0; l < L; ++l) {
            const double *Wd = params + (int64_t)l * PL;
            const double *cd = Wd + (int64_t)d * r;
            const double *Wu = cd + r;
            const double *cu = Wu + (int64_t)r * d;
            const double lam = cu[d];
            const float *b = blk + (int64_t)l * nd;
            const double *Sp = S + (size_t)l * nd;
            double *Sn = S + (size_t)(l + 1) * nd;
            double *pre = PRE + (size_t)l * nr;
            double *h = H + (size_t)l * nr;
#pragma omp parallel for schedule(static)
            for (int32_t t = 0; t < len; ++t) {
                for (int32_t k = 0; k < r; ++k) pre[(size_t)t * r + k] = cd[k];
                for (int32_t j = 0; j < d; ++j) {
                    double x = lam * (double)b[(size_t)t * d + j] + (1.0 - lam) * Sp[(size_t)t * d + j];
                    for (int32_t k = 0; k < r; ++k) pre[(size_t)t * r + k] += x * Wd[(int64_t)j * r + k];
                }
                for (int32_t k = 0; k < r; ++k) h[(size_t)t * r + k] = gelu(pre[(size_t)t * r + k]);
                for (int32_t j = 0; j < d; ++j) Sn[(size_t)t * d + j] = Sp[(size_t)t * d + j] + cu[j];
                for (int32_t k = 0; k < r; ++k) {
                    double hk = h[(size_t)t * r + k];
                    for (int32_t j = 0; j < d; ++j) Sn[(size_t)t * d + j] += hk * Wu[(int64_t)k * d + j];
                }
            }
        }
        /* ---- y = b_L + s_L, mean pool over the valid tokens ---- */
        {
            const float *bL = blk + (int64_t)(L - 1) * nd;
            const double *SL = S + (size_t)L * nd;
            for (int32_t t = 0; t < len; ++t)
                for (int32_t j = 0; j < d; ++j) p[j] += (double)bL[(size_t)t * d + j] + SL[(size_t)t * d + j];
            for (int32_t j = 0; j < d; ++j) p[j] /= (double)len;
        }
        /* ---- classifier and cross-entropy ---- */
        double zmax = -INFINITY;
        for (int32_t c = 0; c < C; ++c) {
            double acc = ccls[c];
            for (int32_t j = 0; j < d; ++j) acc += p[j] * Wcls[(int64_t)j * C + c];
            z[c] = acc;
            if (acc > zmax) zmax = acc;
        }
        double se = 0.0;
        for (int32_t c = 0; c < C; ++c) se += exp(z[c] - zmax);
        const double lse = zmax + log(se);
        total += lse - z[labels[sidx]];
        if (logits) for (int32_t c = 0; c < C; ++c) logits[(int64_t)sidx * C + c] = z[c];
        if (pooled) for (int32_t j = 0; j < d; ++j) pooled[(int64_t)sidx * d + j] = p[j];

        if (grads) {
            /* ---- backward: head ---- */
            double *dz = (double *)malloc((size_t)C * sizeof(double));
            double *DS = (double *)malloc(nd * sizeof(double));
            double *DX = (double *)malloc(nd * sizeof(double));
            double *DPRE = (double *)malloc(nr * sizeof(double));
            if (!dz || !DS || !DX || !DPRE) { free(dz); free(DS); free(DX); free(DPRE); free(S); free(PRE); free(H); free(p); free(z); return -1; }
            for (int32_t c = 0; c < C; ++c)
                dz[c] = (exp(z[c] - lse) - (c == labels[sidx] ? 1.0 : 0.0)) / (double)B;
            for (int32_t c = 0; c < C; ++c) gccls[c] += dz[c];
            for (int32_t j = 0; j < d; ++j) {
                double dpj = 0.0;
                for (int32_t c = 0; c < C; ++c) {
                    gWcls[(int64_t)j * C + c] += p[j] * dz[c];
                    dpj += dz[c] * Wcls[(int64_t)j * C + c];
                }
                /* the mean pool hands every valid token the same share */
                for (int32_t t = 0; t < len; ++t) DS[(size_t)t * d + j] = dpj / (double)len;
            }
            /* ---- backward: layers L..1 ---- */
            for (int32_t l = L - 1; l >= 0; --l) {
                const double *Wd = params + (int64_t)l * PL;
                const double *cd = Wd + (int64_t)d * r;
                const double *Wu = cd + r;
                const double *cu = Wu + (int64_t)r * d;
                const double lam = cu[d];
                double *gWd = grads + (int64_t)l * PL;
                double *gcd = gWd + (int64_t)d * r;
                double *gWu = gcd + r;
                double *gcu = gWu + (int64_t)r * d;
                double *glam = gcu + d;
                const float *b = blk + (int64_t)l * nd;
                const double *Sp = S + (size_t)l * nd;
                const double *pre = PRE + (size_t)l * nr;
                const double *h = H + (size_t)l * nr;
                (void)cd; (void)cu;
                /* token-wise: dh = ds W_up^T ; dpre = dh * GELU'(pre) ; dx = dpre W_down^T */
#pragma omp parallel for schedule(static)
                for (int32_t t = 0; t < len; ++t) {
                    for (int32_t k = 0; k < r; ++k) {
                        double dh = 0.0;
                        for (int32_t j = 0; j < d; ++j) dh += DS[(size_t)t * d + j] * Wu[(int64_t)k * d + j];
                        DPRE[(size_t)t * r + k] = dh * gelu_deriv(pre[(size_t)t * r + k]);
                    }
                    for (int32_t j = 0; j < d; ++j) {
                        double dx = 0.0;
                        for (int32_t k = 0; k < r; ++k) dx += DPRE[(size_t)t * r + k] * Wd[(int64_t)j * r + k];
                        DX[(size_t)t * d + j] = dx;
                    }
                }
                /* parameter gradients: sums over the tokens */
#pragma omp parallel for schedule(static)
                for (int32_t k = 0; k < r; ++k) {
                    for (int32_t t = 0; t < len; ++t) {
                        double hk = h[(size_t)t * r + k];
                        for (int32_t j = 0; j < d; ++j) gWu[(int64_t)k * d + j] += hk * DS[(size_t)t * d + j];
                    }
                    double acc = 0.0;
                    for (int32_t t = 0; t < len; ++t) acc += DPRE[(size_t)t * r + k];
                    gcd[k] += acc;
                }
#pragma omp parallel for schedule(static)
                for (int32_t j = 0; j < d; ++j) {
                    double accu = 0.0;
                    for (int32_t t = 0; t < len; ++t) {
                        double x = lam * (double)b[(size_t)t * d + j] + (1.0 - lam) * Sp[(size_t)t * d + j];
                        for (int32_t k = 0; k < r; ++k) gWd[(int64_t)j * r + k] += x * DPRE[(size_t)t * r + k];
                        accu += DS[(size_t)t * d + j];
                    }
                    gcu[j] += accu;
                }
                {
                    double acc = 0.0, acc_abs = 0.0;
                    for (int32_t t = 0; t < len; ++t)
                        for (int32_t j = 0; j < d; ++j) {
                            double term = ((double)b[(size_t)t * d + j] - Sp[(size_t)t * d + j]) * DX[(size_t)t * d + j];
                            acc += term;
                            acc_abs += fabs(term);
                        }
                    *glam += acc;
                    if (glam_abs) glam_abs[l] += acc_abs;
                }
                /* ds_{l-1} = ds_l + (1 - lambda) dx */
#pragma omp parallel for schedule(static)
                for (int32_t t = 0; t < len; ++t)
                    for (int32_t j = 0; j < d; ++j) DS[(size_t)t * d + j] += (1.0 - lam) * DX[(size_t)t * d + j];
            }
            free(dz); free(DS); free(DX); free(DPRE);
        }
        free(S); free(PRE); free(H); free(p); free(z);
    }
    *loss = total / (double)B;
    return 0;
}

/*
 * AdamW (decoupled weight decay, bias-corrected moments, epsilon added to the
 * root of the corrected second moment).  t is the step number AFTER the
 * increment (first step: t = 1).  Decay applies to W_down, W_up and W_cls only.
 */
void orc_adamw(int32_t L, int32_t d, int32_t r, int32_t C,
               double *p, double *m, double *v, int64_t t, const double *g,
               double lr, double beta1, double beta2, double eps, double weight_decay)
{
    const int64_t PL = orc_layer_block(d, r);
    const int64_t P = orc_param_count(L, d, r, C);
    const double bc1 = 1.0 - pow(beta1, (double)t);
    const double bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < P; ++i) {
        int decayed;
        if (i < (int64_t)L * PL) {
            int64_t o = i % PL;
            decayed = (o < (int64_t)d * r) ||
                      (o >= (int64_t)d * r + r && o < 2 * (int64_t)d * r + r);
        } else {
            decayed = (i - (int64_t)L * PL) < (int64_t)d * C;
        }
        m[i] = beta1 * m[i] + (1.0 - beta1) * g[i];
        v[i] = beta2 * v[i] + (1.0 - beta2) * g[i] * g[i];
        double mhat = m[i] / bc1;
        double vhat = v[i] / bc2;
        if (decayed) p[i] -= lr * weight_decay * p[i];
        p[i] -= lr * mhat / (sqrt(vhat) + eps);
    }
}
