/*
 * libpac -- planner for the first (hybrid-parallel) epoch of PAC+ (arXiv 2408.10746, Sec. 5.1).
 *
 * A host-only program: no device work, nothing here touches a GPU.  It is the paper's planning step for the
 * epoch that fills the activation cache: split the L transformer layers into consecutive pipeline stages, give
 * each stage a group of consecutive devices of the ordered device list (the stage model is replicated inside
 * a group and a micro-batch's samples are dealt over the group's devices), and pick the number of stages.
 *
 *   sample dispatch   H_{x->y}(b, G_n) = min_{0<=i<=b} max{ H_{x->y}(b-i, G_n \ {d_{n-1}}),
 *                                                           sum_{l=x..y} [t_f^{d_{n-1},l}(i) + t_b^{d_{n-1},l}(i)] }
 *                     (Eq. "dp2"); a device whose memory footprint exceeds its budget counts as +infinity;
 *                     T(x->y, G) = H_{x->y}(B, G), B the micro-batch size.
 *   stage partition   W(0->y, D_n, s) = min_q min_m max{ W(0->q, D_{n-m}, s-1), T(q+1->y, {d_{n-m}..d_{n-1}}) }
 *                     (Eq. "dp-main"), W(0->y, D_n, 1) = T(0->y, D_n).
 *   stage count       L_b = sum_{i<s} [e_f(i) + c_f(i)],  L_e = M (e_f(s) + e_b(s)),
 *                     L_n = max_i ( AR(i) + sum_{j=i}^{s-1} (e_b(j) + c_b(j)) ),  sigma = argmin_s (L_b + L_e + L_n)
 *                     (Eq. "Lb", "Ln", "sigma"; Algorithm 1).
 *
 * Readings where the paper leaves a choice (all stated in the design notes as well):
 *  - memory footprint of a device holding layers x..y with i samples: sum_l (mem_fixed[l] + i * mem_act[l]); the
 *    stage model is replicated on every device of a group, so the check also applies to a device that gets no sample;
 *  - group sizes m range over 1 .. n - (s - 1) (every earlier stage keeps at least one device), cuts q over
 *    s - 2 .. y - 1 (every earlier stage keeps at least one layer);
 *  - e_f(i) / e_b(i): the slowest device of stage i under the recorded sample dispatch;
 *  - c_f(i) = B * act_bytes[last layer of stage i] / bandwidth, c_b(i) = B * grad_bytes[that layer] / bandwidth;
 *  - AR(i): ring all-reduce of the stage's trainable bytes over its g devices, 2 (g-1)/g * bytes / bandwidth;
 *  - the unbalanced parenthesis of Eq. "Ln" is closed after the inner sum; ties in sigma go to the smaller s.
 */
#ifndef PAC_PLAN_H
#define PAC_PLAN_H

#include <stdint.h>
#include "pac.h"

#ifdef __cplusplus
extern "C" {
#endif

/* All arrays HOST.  Times in seconds, sizes in bytes. */
typedef struct {
    int32_t L;       /* layers (>= 1) */
    int32_t n_dev;   /* devices, in the order groups are cut from (>= 1) */
    int32_t B;       /* micro-batch size (>= 1) */
    int32_t M;       /* micro-batches per mini-batch (>= 1) */
    const double *t_f;        /* [n_dev][L][B+1]: forward time of layer l on device d with beta samples (beta = 0: 0) */
    const double *t_b;        /* [n_dev][L][B+1]: backward time */
    const double *mem_fixed;  /* [L]: parameters + parameter gradients of layer l */
    const double *mem_act;    /* [L]: activations of layer l per sample */
    const double *mem_budget; /* [n_dev] */
    const double *act_bytes;  /* [L]: output activation of layer l per sample (forward inter-stage transfer) */
    const double *grad_bytes; /* [L]: gradient w.r.t. that activation per sample (backward transfer) */
    const double *train_bytes;/* [L]: trainable (adapter) bytes of layer l, all-reduced inside a group */
    double bandwidth;         /* bytes per second between devices (> 0) */
} pac_plan_problem;

/* Result for the chosen stage count sigma.  The caller provides arrays of at least min(L, n_dev) (stage_*),
 * n_dev (samples) and min(L, n_dev) + 1 (latency_by_stage_count) entries. */
typedef struct {
    int32_t sigma;               /* chosen number of stages; 0 if no stage count is feasible */
    int32_t *stage_first_layer;  /* [sigma] */
    int32_t *stage_last_layer;   /* [sigma] inclusive */
    int32_t *stage_first_dev;    /* [sigma] */
    int32_t *stage_n_dev;        /* [sigma] */
    int32_t *samples;            /* [n_dev]: samples of a micro-batch dispatched to each device */
    double slowest_stage;        /* W(0 -> L-1, D, sigma) */
    double L_b, L_e, L_n;        /* of the chosen configuration */
    double *latency_by_stage_count; /* [s] = L_b + L_e + L_n of W_s for s = 1 .. min(L, n_dev) (index 0 unused); +inf if infeasible */
    double *slowest_by_stage_count; /* same indexing: W(0 -> L-1, D, s) */
} pac_plan_result;

/* Runs Algorithm 1.  PAC_ERR_NULL / PAC_ERR_SHAPE / PAC_ERR_RANGE (negative or NaN time or size) on bad input;
 * PAC_OK with sigma = 0 when no configuration fits the memory budgets.  Allocates host memory only. */
pac_status pac_plan_hybrid(const pac_plan_problem *prob /*HOST*/, pac_plan_result *out /*HOST*/);

/* T(x -> y, {d_first .. d_first + n - 1}) of Eq. "dp2" alone, with the dispatch that attains it
 * (samples: n entries, or NULL).  Returns +infinity when the group cannot hold the stage; NaN on bad arguments. */
double pac_plan_stage_time(const pac_plan_problem *prob /*HOST*/, int32_t x, int32_t y, int32_t d_first, int32_t n,
                           int32_t *samples /*HOST*/);

#ifdef __cplusplus
}
#endif
#endif /* PAC_PLAN_H */
