// The paper's (alpha, beta) cost model on the library side (section 3.6) and what it is used for there
// (section 5.5): choosing, per input size, among several algorithms for the same collective.  Host only.
#include <cmath>
#include <utility>

#include "plan.hpp"

extern "C" {

// S * alpha + (R / C) * L * beta with L = C * chunk_bytes the input bytes of a node.
sccl_status_t sccl_plan_cost(const sccl_plan_t* plan, double alpha, double beta, double* out_seconds) {
    if (!plan || !out_seconds || !(alpha >= 0.0) || !(beta >= 0.0)) return SCCL_ERR_INVALID_ARG;
    const sccl_stats_t& st = plan->stats;
    const double L = (double)st.chunks_per_node * (double)st.chunk_bytes;
    double t = 0.0;
    for (int32_t r : plan->rounds) t += alpha + ((double)r / (double)st.chunks_per_node) * L * beta;   // per step
    *out_seconds = t;
    return SCCL_OK;
}

sccl_status_t sccl_select_plan(const sccl_plan_t* const* plans, int32_t num_plans, double alpha, double beta,
                               int32_t* out_best) {
    if (!plans || num_plans < 1 || !out_best) return SCCL_ERR_INVALID_ARG;
    int32_t best = -1;
    double best_t = 0.0;
    for (int32_t i = 0; i < num_plans; i++) {
        double t;
        const sccl_status_t st = sccl_plan_cost(plans[i], alpha, beta, &t);
        if (st != SCCL_OK) return st;
        if (best < 0 || t < best_t) { best = i; best_t = t; }     // ties go to the earlier plan
    }
    *out_best = best;
    return SCCL_OK;
}

// Least squares for t_i = a_i * alpha + b_i * beta (no intercept): the normal equations of a 2-column system.
sccl_status_t sccl_cost_fit(int32_t n, const double* a, const double* b, const double* t, double* out_alpha,
                            double* out_beta) {
    if (n < 2 || !a || !b || !t || !out_alpha || !out_beta) return SCCL_ERR_INVALID_ARG;
    double saa = 0, sab = 0, sbb = 0, sat = 0, sbt = 0;
    for (int32_t i = 0; i < n; i++) {
        saa += a[i] * a[i]; sab += a[i] * b[i]; sbb += b[i] * b[i];
        sat += a[i] * t[i]; sbt += b[i] * t[i];
    }
    const double det = saa * sbb - sab * sab;
    if (!(std::fabs(det) > 1e-300 * (saa * sbb + 1e-300)) || !std::isfinite(det)) return SCCL_ERR_INVALID_ARG;   // collinear samples
    *out_alpha = (sat * sbb - sbt * sab) / det;
    *out_beta = (saa * sbt - sab * sat) / det;
    return SCCL_OK;
}

// Weighted least squares for t_i = t0 + a_i * alpha + b_i * beta: minimises the sum of (w_i * residual_i)^2.  The
// three columns differ by many orders of magnitude (1, steps, bytes), so each is scaled by its largest magnitude
// before the 3 x 3 normal equations are solved by elimination with partial pivoting.
sccl_status_t sccl_cost_fit_intercept(int32_t n, const double* a, const double* b, const double* t, const double* weights,
                                      double* out_t0, double* out_alpha, double* out_beta) {
    if (n < 3 || !a || !b || !t || !out_t0 || !out_alpha || !out_beta) return SCCL_ERR_INVALID_ARG;
    if (weights)
        for (int32_t i = 0; i < n; i++)
            if (!(weights[i] >= 0.0) || !std::isfinite(weights[i])) return SCCL_ERR_INVALID_ARG;
    double sa = 0, sb = 0;
    for (int32_t i = 0; i < n; i++) {
        if (!std::isfinite(a[i]) || !std::isfinite(b[i]) || !std::isfinite(t[i])) return SCCL_ERR_INVALID_ARG;
        sa = std::fmax(sa, std::fabs(a[i])); sb = std::fmax(sb, std::fabs(b[i]));
    }
    if (!(sa > 0) || !(sb > 0)) return SCCL_ERR_INVALID_ARG;
    double m[3][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    for (int32_t i = 0; i < n; i++) {
        const double w = weights ? weights[i] : 1.0;
        const double x[3] = {w, w * a[i] / sa, w * b[i] / sb};
        for (int r = 0; r < 3; r++) {
            for (int c = 0; c < 3; c++) m[r][c] += x[r] * x[c];
            m[r][3] += x[r] * w * t[i];
        }
    }
    for (int col = 0; col < 3; col++) {
        int piv = col;
        for (int r = col + 1; r < 3; r++) if (std::fabs(m[r][col]) > std::fabs(m[piv][col])) piv = r;
        if (!(std::fabs(m[piv][col]) > 1e-12 * (double)n)) return SCCL_ERR_INVALID_ARG;     // the columns are dependent
        for (int c = 0; c < 4; c++) std::swap(m[col][c], m[piv][c]);
        for (int r = 0; r < 3; r++) {
            if (r == col) continue;
            const double f = m[r][col] / m[col][col];
            for (int c = col; c < 4; c++) m[r][c] -= f * m[col][c];
        }
    }
    *out_t0 = m[0][3] / m[0][0];
    *out_alpha = m[1][3] / m[1][1] / sa;
    *out_beta = m[2][3] / m[2][2] / sb;
    return SCCL_OK;
}

}  // extern "C"
