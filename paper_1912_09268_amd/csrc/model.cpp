// Host helpers around the planner: where a and b come from (Table 2, or a fit to measured all-reduce
// times as in Sec. 6.2), and the worker-count sweep of Sec. 6.4 built from the planner and evaluator.
#include <cmath>
#include <cstdint>
#include <vector>

#include "mgwfbp.h"

extern "C" int mgwfbp_allreduce_ab(int32_t algorithm, int32_t n_workers, double alpha_s, double beta_s_per_byte,
                                   double gamma_s_per_byte, double* a_out, double* b_out) {
    if (a_out == nullptr || b_out == nullptr || n_workers < 1) return MGWFBP_EINVAL;
    const double al = alpha_s, be = beta_s_per_byte, ga = gamma_s_per_byte;
    if (!(std::isfinite(al) && std::isfinite(be) && std::isfinite(ga)) || al < 0 || be < 0 || ga < 0)
        return MGWFBP_EINVAL;
    const double N = static_cast<double>(n_workers);
    const double lg = std::log2(N);
    switch (algorithm) {
        case MGWFBP_AR_BINARY_TREE:
            *a_out = 2.0 * al * lg;
            *b_out = (2.0 * be + ga) * lg;
            break;
        case MGWFBP_AR_RECURSIVE_DOUBLING:
            *a_out = al * lg;
            *b_out = (be + ga) * lg;
            break;
        case MGWFBP_AR_HALVING_DOUBLING:
            *a_out = 2.0 * al * lg;
            *b_out = 2.0 * be - (1.0 / N) * (2.0 * be + ga) + ga;
            break;
        case MGWFBP_AR_DOUBLE_BINARY_TREES:
            *a_out = 2.0 * al * lg;
            *b_out = be + ga;
            break;
        case MGWFBP_AR_RING:
            *a_out = 2.0 * (N - 1.0) * al;
            *b_out = (2.0 * (N - 1.0) / N) * be + ((N - 1.0) / N) * ga;
            break;
        default:
            return MGWFBP_EINVAL;
    }
    return MGWFBP_OK;
}

extern "C" int mgwfbp_fit_ab(const uint64_t* message_bytes, const double* seconds, int32_t n, double* a_out,
                             double* b_out) {
    if (message_bytes == nullptr || seconds == nullptr || a_out == nullptr || b_out == nullptr || n < 2)
        return MGWFBP_EINVAL;
    // ordinary least squares on centred data (keeps the normal equations well conditioned for sizes
    // that span many orders of magnitude)
    long double mx = 0, my = 0;
    for (int32_t i = 0; i < n; ++i) {
        if (!std::isfinite(seconds[i])) return MGWFBP_EINVAL;
        mx += static_cast<long double>(message_bytes[i]);
        my += seconds[i];
    }
    mx /= n;
    my /= n;
    long double sxx = 0, sxy = 0;
    for (int32_t i = 0; i < n; ++i) {
        const long double dx = static_cast<long double>(message_bytes[i]) - mx;
        sxx += dx * dx;
        sxy += dx * (seconds[i] - my);
    }
    if (!(sxx > 0)) return MGWFBP_EINVAL;      // all sizes equal: the slope is undetermined
    const long double b = sxy / sxx;
    *b_out = static_cast<double>(b);
    *a_out = static_cast<double>(my - b * mx);
    return MGWFBP_OK;
}

extern "C" int mgwfbp_simulate(const uint64_t* size_bytes, const double* t_backward_s, int32_t L, double t_forward_s,
                               int32_t algorithm, double alpha_s, double beta_s_per_byte, double gamma_s_per_byte,
                               const int32_t* worker_counts, int32_t n_counts, double* t_wfbp_out,
                               double* t_single_out, double* t_mgwfbp_out, int32_t* groups_out) {
    if (worker_counts == nullptr || n_counts < 0 || !std::isfinite(t_forward_s) || t_forward_s < 0) return MGWFBP_EINVAL;
    if (L < 0) return MGWFBP_EINVAL;
    std::vector<uint8_t> normal(static_cast<size_t>(L), 0), single(static_cast<size_t>(L), 1), plan(static_cast<size_t>(L), 0);
    if (L > 0) single[0] = 0;
    for (int32_t k = 0; k < n_counts; ++k) {
        double a = 0, b = 0, t = 0;
        int rc = mgwfbp_allreduce_ab(algorithm, worker_counts[k], alpha_s, beta_s_per_byte, gamma_s_per_byte, &a, &b);
        if (rc != MGWFBP_OK) return rc;
        int32_t G = 0;
        rc = mgwfbp_plan(size_bytes, t_backward_s, L, a, b, plan.data(), nullptr, &G);
        if (rc != MGWFBP_OK) return rc;
        if (groups_out) groups_out[k] = G;
        if (t_wfbp_out) {
            rc = mgwfbp_eval(normal.data(), size_bytes, t_backward_s, L, a, b, &t);
            if (rc != MGWFBP_OK) return rc;
            t_wfbp_out[k] = t_forward_s + t;
        }
        if (t_single_out) {
            rc = mgwfbp_eval(single.data(), size_bytes, t_backward_s, L, a, b, &t);
            if (rc != MGWFBP_OK) return rc;
            t_single_out[k] = t_forward_s + t;
        }
        if (t_mgwfbp_out) {
            rc = mgwfbp_eval(plan.data(), size_bytes, t_backward_s, L, a, b, &t);
            if (rc != MGWFBP_OK) return rc;
            t_mgwfbp_out[k] = t_forward_s + t;
        }
    }
    return MGWFBP_OK;
}
