// Planner of the hybrid-parallel first epoch (declared in include/pac_plan.h): host code only.
// Dynamic programs of Sec. 5.1: sample dispatch inside a device group (Eq. "dp2"), balanced stage partition
// (Eq. "dp-main"), stage count by the three-phase latency model (Eq. "Lb", "Ln", "sigma"; Algorithm 1).
#include "../../include/pac_plan.h"

#include <cmath>
#include <limits>
#include <vector>

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

struct Planner {
    const pac_plan_problem &P;
    int L, N, B;
    explicit Planner(const pac_plan_problem &p) : P(p), L(p.L), N(p.n_dev), B(p.B) {}

    double tf(int d, int l, int beta) const { return P.t_f[((size_t)d * L + l) * (B + 1) + beta]; }
    double tb(int d, int l, int beta) const { return P.t_b[((size_t)d * L + l) * (B + 1) + beta]; }

    // forward + backward time of device d on layers x..y with i samples, +inf when the footprint exceeds its budget
    void device_times(int d, int x, int y, int i, double &f, double &b) const
    {
        double mem = 0.0;
        f = b = 0.0;
        for (int l = x; l <= y; ++l) {
            mem += P.mem_fixed[l] + (double)i * P.mem_act[l];
            f += tf(d, l, i);
            b += tb(d, l, i);
        }
        if (mem > P.mem_budget[d]) f = b = kInf;
    }

    // Eq. "dp2": H[k][b] over the first k devices of the group; returns H[n][B] and the dispatch
    double stage_time(int x, int y, int d0, int n, int32_t *samples) const
    {
        std::vector<double> cost((size_t)n * (B + 1));
        for (int k = 0; k < n; ++k)
            for (int i = 0; i <= B; ++i) {
                double f, b;
                device_times(d0 + k, x, y, i, f, b);
                cost[(size_t)k * (B + 1) + i] = f + b;
            }
        std::vector<double> H((size_t)(n + 1) * (B + 1), kInf);
        std::vector<int> pick((size_t)(n + 1) * (B + 1), -1);
        H[0] = 0.0; // no device, no sample
        for (int k = 1; k <= n; ++k)
            for (int b = 0; b <= B; ++b) {
                double best = kInf;
                int bi = -1;
                for (int i = 0; i <= b; ++i) {
                    const double rest = H[(size_t)(k - 1) * (B + 1) + (b - i)];
                    const double mine = cost[(size_t)(k - 1) * (B + 1) + i];
                    const double v = rest > mine ? rest : mine;
                    if (v < best) { best = v; bi = i; }
                }
                H[(size_t)k * (B + 1) + b] = best;
                pick[(size_t)k * (B + 1) + b] = bi;
            }
        const double res = H[(size_t)n * (B + 1) + B];
        if (samples) {
            for (int k = 0; k < n; ++k) samples[k] = 0;
            if (res < kInf) {
                int b = B;
                for (int k = n; k >= 1; --k) {
                    const int i = pick[(size_t)k * (B + 1) + b];
                    samples[k - 1] = i;
                    b -= i;
                }
            }
        }
        return res;
    }
};

bool bad(double v) { return !(v >= 0.0); } // negative or NaN

} // namespace

extern "C" {

double pac_plan_stage_time(const pac_plan_problem *prob, int32_t x, int32_t y, int32_t d_first, int32_t n, int32_t *samples)
{
    const double nan = std::numeric_limits<double>::quiet_NaN();
    if (!prob || !prob->t_f || !prob->t_b || !prob->mem_fixed || !prob->mem_act || !prob->mem_budget) return nan;
    if (prob->L < 1 || prob->n_dev < 1 || prob->B < 1) return nan;
    if (x < 0 || y < x || y >= prob->L || d_first < 0 || n < 1 || d_first + n > prob->n_dev) return nan;
    return Planner(*prob).stage_time(x, y, d_first, n, samples);
}

pac_status pac_plan_hybrid(const pac_plan_problem *prob, pac_plan_result *out)
{
    if (!prob || !out) return PAC_ERR_NULL;
    const pac_plan_problem &P = *prob;
    if (!P.t_f || !P.t_b || !P.mem_fixed || !P.mem_act || !P.mem_budget || !P.act_bytes || !P.grad_bytes || !P.train_bytes)
        return PAC_ERR_NULL;
    if (!out->stage_first_layer || !out->stage_last_layer || !out->stage_first_dev || !out->stage_n_dev || !out->samples ||
        !out->latency_by_stage_count || !out->slowest_by_stage_count)
        return PAC_ERR_NULL;
    if (P.L < 1 || P.n_dev < 1 || P.B < 1 || P.M < 1) return PAC_ERR_SHAPE;
    if (!(P.bandwidth > 0.0)) return PAC_ERR_RANGE;
    const int L = P.L, N = P.n_dev, B = P.B;
    for (size_t i = 0; i < (size_t)N * L * (B + 1); ++i)
        if (bad(P.t_f[i]) || bad(P.t_b[i])) return PAC_ERR_RANGE;
    for (int l = 0; l < L; ++l)
        if (bad(P.mem_fixed[l]) || bad(P.mem_act[l]) || bad(P.act_bytes[l]) || bad(P.grad_bytes[l]) || bad(P.train_bytes[l]))
            return PAC_ERR_RANGE;
    for (int d = 0; d < N; ++d)
        if (bad(P.mem_budget[d])) return PAC_ERR_RANGE;

    Planner pl(P);
    const int S = L < N ? L : N;
    // T(x -> y, {d0 .. d0 + m - 1}) for every layer range and device range, once
    auto tidx = [&](int x, int y, int d0, int m) { return (((size_t)x * L + y) * N + d0) * (N + 1) + m; };
    std::vector<double> T((size_t)L * L * N * (N + 1), kInf);
    for (int x = 0; x < L; ++x)
        for (int y = x; y < L; ++y)
            for (int d0 = 0; d0 < N; ++d0)
                for (int m = 1; d0 + m <= N; ++m) T[tidx(x, y, d0, m)] = pl.stage_time(x, y, d0, m, nullptr);

    // W[s][y][n]: slowest stage of the best split of layers 0..y over the first n devices into s stages
    auto widx = [&](int s, int y, int n) { return ((size_t)s * L + y) * (N + 1) + n; };
    std::vector<double> W((size_t)(S + 1) * L * (N + 1), kInf);
    std::vector<int> cut((size_t)(S + 1) * L * (N + 1), -1), grp((size_t)(S + 1) * L * (N + 1), -1);
    for (int y = 0; y < L; ++y)
        for (int n = 1; n <= N; ++n) W[widx(1, y, n)] = T[tidx(0, y, 0, n)];
    for (int s = 2; s <= S; ++s)
        for (int y = s - 1; y < L; ++y)
            for (int n = s; n <= N; ++n) {
                double best = kInf;
                int bq = -1, bm = -1;
                for (int q = s - 2; q < y; ++q)
                    for (int m = 1; m <= n - (s - 1); ++m) {
                        const double a = W[widx(s - 1, q, n - m)];
                        const double b = T[tidx(q + 1, y, n - m, m)];
                        const double v = a > b ? a : b;
                        if (v < best) { best = v; bq = q; bm = m; }
                    }
                W[widx(s, y, n)] = best;
                cut[widx(s, y, n)] = bq;
                grp[widx(s, y, n)] = bm;
            }

    // stage count: three-phase latency of every W_s
    double best_total = kInf;
    int sigma = 0;
    out->latency_by_stage_count[0] = out->slowest_by_stage_count[0] = kInf;
    std::vector<int> fl(S), ll(S), fd(S), nd(S);
    std::vector<int32_t> smp(N);
    for (int s = 1; s <= S; ++s) {
        const double w = W[widx(s, L - 1, N)];
        out->slowest_by_stage_count[s] = w;
        out->latency_by_stage_count[s] = kInf;
        if (!(w < kInf)) continue;
        // walk the recorded configuration back from the last stage
        int y = L - 1, n = N;
        for (int st = s; st >= 1; --st) {
            if (st == 1) { fl[0] = 0; ll[0] = y; fd[0] = 0; nd[0] = n; break; }
            const int q = cut[widx(st, y, n)], m = grp[widx(st, y, n)];
            fl[st - 1] = q + 1; ll[st - 1] = y; fd[st - 1] = n - m; nd[st - 1] = m;
            y = q; n -= m;
        }
        std::vector<double> ef(s), eb(s), cf(s), cb(s), ar(s);
        std::vector<int32_t> alloc(N, 0);
        for (int i = 0; i < s; ++i) {
            pl.stage_time(fl[i], ll[i], fd[i], nd[i], alloc.data() + fd[i]);
            double mf = 0.0, mb = 0.0, bytes = 0.0;
            for (int k = 0; k < nd[i]; ++k) {
                double f, b;
                pl.device_times(fd[i] + k, fl[i], ll[i], alloc[fd[i] + k], f, b);
                mf = f > mf ? f : mf;
                mb = b > mb ? b : mb;
            }
            for (int l = fl[i]; l <= ll[i]; ++l) bytes += P.train_bytes[l];
            ef[i] = mf; eb[i] = mb;
            cf[i] = (double)B * P.act_bytes[ll[i]] / P.bandwidth;
            cb[i] = (double)B * P.grad_bytes[ll[i]] / P.bandwidth;
            ar[i] = nd[i] > 1 ? 2.0 * (nd[i] - 1) / nd[i] * bytes / P.bandwidth : 0.0;
        }
        double Lb = 0.0;
        for (int i = 0; i + 1 < s; ++i) Lb += ef[i] + cf[i];
        const double Le = (double)P.M * (ef[s - 1] + eb[s - 1]);
        double Ln = 0.0;
        for (int i = 0; i < s; ++i) {
            double v = ar[i];
            for (int j = i; j + 1 < s; ++j) v += eb[j] + cb[j];
            Ln = v > Ln ? v : Ln;
        }
        const double total = Lb + Le + Ln;
        out->latency_by_stage_count[s] = total;
        if (total < best_total) {
            best_total = total;
            sigma = s;
            out->slowest_stage = w;
            out->L_b = Lb; out->L_e = Le; out->L_n = Ln;
            for (int i = 0; i < s; ++i) {
                out->stage_first_layer[i] = fl[i]; out->stage_last_layer[i] = ll[i];
                out->stage_first_dev[i] = fd[i]; out->stage_n_dev[i] = nd[i];
            }
            for (int d = 0; d < N; ++d) out->samples[d] = alloc[d];
        }
    }
    out->sigma = sigma;
    if (sigma == 0) { out->slowest_stage = kInf; out->L_b = out->L_e = out->L_n = kInf; }
    return PAC_OK;
}

} // extern "C"
