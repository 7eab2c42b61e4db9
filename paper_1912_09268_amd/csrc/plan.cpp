// Host side of the MG-WFBP library: the layer-merge planner (Algorithm 1) and the timeline
// evaluator (Eq. 6-8 with the merged-layer properties Eq. 12-14).  No GPU code in this file.
//
// Indexing here is 0-based in forward order: tensor i is the paper's layer i+1.  Backpropagation
// produces gradients in the order L-1, ..., 0, so every loop below walks downwards.
#include <cmath>
#include <cstdint>
#include <vector>

#include "mgwfbp.h"

namespace {

bool valid_time(double x) { return std::isfinite(x) && x >= 0.0; }

bool valid_inputs(const uint64_t* size_bytes, const double* t_b, int32_t L, double a, double b) {
    if (L < 0 || !valid_time(a) || !valid_time(b)) return false;
    if (L > 0 && (size_bytes == nullptr || t_b == nullptr)) return false;
    uint64_t total = 0;
    for (int32_t i = 0; i < L; ++i) {
        if (!valid_time(t_b[i])) return false;
        if (size_bytes[i] > UINT64_MAX - total) return false;  // merged sizes must not wrap
        total += size_bytes[i];
    }
    return true;
}

// Eq. 10
inline double message_time(double a, double b, uint64_t bytes) { return a + b * static_cast<double>(bytes); }

// Time at which the gradient of tensor i exists: tau_b^(l) + t_b^(l) with tau_b from Eq. 6
// (tau_b of the last layer is 0, as Algorithm 1 initialises it).
void gradient_ready_times(const double* t_b, int32_t L, std::vector<double>& ready) {
    ready.resize(static_cast<size_t>(L));
    double tau_b = 0.0;
    for (int32_t i = L - 1; i >= 0; --i) {
        ready[static_cast<size_t>(i)] = tau_b + t_b[i];
        if (i > 0) tau_b = tau_b + t_b[i];
    }
}

}  // namespace

extern "C" int mgwfbp_plan(const uint64_t* size_bytes, const double* t_backward_s, int32_t L,
                           double a, double b, uint8_t* merged_out, int32_t* group_first_out,
                           int32_t* n_groups_out) {
    if (!valid_inputs(size_bytes, t_backward_s, L, a, b)) return MGWFBP_EINVAL;
    if (L > 0 && merged_out == nullptr) return MGWFBP_EINVAL;
    if (L == 0) {
        if (n_groups_out) *n_groups_out = 0;
        if (group_first_out) group_first_out[0] = -1;
        return MGWFBP_OK;
    }
    std::vector<double> ready;
    gradient_ready_times(t_backward_s, L, ready);

    // State of the layer under test (paper's l), given every decision taken above it:
    //   bytes_l : its own bytes plus everything merged into it so far      (Eq. 13)
    //   t_c_l   : its message time a + b*bytes_l                             (Eq. 10)
    //   tau_c_l : when that message could start                              (Eq. 7 / Eq. 14)
    // A merge only changes t_c of l and l-1, and tau_c of layers >= l does not depend on either,
    // so carrying tau_c downwards reproduces the full recomputation of Algorithm 1 exactly.
    uint64_t bytes_l = size_bytes[L - 1];
    double t_c_l = message_time(a, b, bytes_l);
    double tau_c_l = ready[static_cast<size_t>(L - 1)];
    for (int32_t i = L - 1; i >= 1; --i) {
        const double ready_below = ready[static_cast<size_t>(i - 1)];
        const bool merge = (ready_below - tau_c_l) < a;   // Algorithm 1's test, strict
        merged_out[i] = merge ? 1 : 0;
        if (merge) {
            bytes_l = size_bytes[i - 1] + bytes_l;                       // Eq. 13
            const double end_l = tau_c_l + 0.0;                          // Eq. 12: t_c of l is 0
            tau_c_l = end_l > ready_below ? end_l : ready_below;         // Eq. 14
        } else {
            const double end_l = tau_c_l + t_c_l;
            bytes_l = size_bytes[i - 1];
            tau_c_l = end_l > ready_below ? end_l : ready_below;         // Eq. 7
        }
        t_c_l = message_time(a, b, bytes_l);
    }
    merged_out[0] = 0;

    int32_t G = 0;
    for (int32_t i = L - 1; i >= 0; --i) {
        const bool opens_group = (i == L - 1) || merged_out[i + 1] == 0;
        if (opens_group) {
            if (group_first_out) group_first_out[G] = i;
            ++G;
        }
    }
    if (group_first_out) group_first_out[G] = -1;
    if (n_groups_out) *n_groups_out = G;
    return MGWFBP_OK;
}

// Eq. 6: group k's merge buffer is full when the gradient of its lowest layer exists.
extern "C" int mgwfbp_group_ready_times(const uint8_t* merged, const double* t_backward_s, int32_t L,
                                        double* ready_out, int32_t* n_groups_out) {
    if (L < 0 || (L > 0 && (merged == nullptr || t_backward_s == nullptr || merged[0] != 0))) return MGWFBP_EINVAL;
    for (int32_t i = 0; i < L; ++i)
        if (merged[i] > 1 || !valid_time(t_backward_s[i])) return MGWFBP_EINVAL;
    std::vector<double> ready;
    gradient_ready_times(t_backward_s, L, ready);
    int32_t G = 0;
    for (int32_t i = L - 1; i >= 0; --i) {
        if (merged[i] == 0) {                      // a normal layer closes the group it arrives in
            if (ready_out) ready_out[G] = ready[static_cast<size_t>(i)];
            ++G;
        }
    }
    if (n_groups_out) *n_groups_out = G;
    return MGWFBP_OK;
}

extern "C" int mgwfbp_eval(const uint8_t* merged, const uint64_t* size_bytes,
                           const double* t_backward_s, int32_t L, double a, double b,
                           double* t_iter_out) {
    if (t_iter_out == nullptr || !valid_inputs(size_bytes, t_backward_s, L, a, b)) return MGWFBP_EINVAL;
    if (L == 0) {
        *t_iter_out = 0.0;
        return MGWFBP_OK;
    }
    if (merged == nullptr || merged[0] != 0) return MGWFBP_EINVAL;
    for (int32_t i = 0; i < L; ++i)
        if (merged[i] > 1) return MGWFBP_EINVAL;
    std::vector<double> ready;
    gradient_ready_times(t_backward_s, L, ready);

    // Walk the messages in the order they are sent.  `carried` = bytes handed down by merged layers.
    uint64_t carried = 0;
    double prev_end = 0.0;   // tau_c + t_c of the layer above; nothing precedes layer L
    double finish = 0.0;
    for (int32_t i = L - 1; i >= 0; --i) {
        const double tau_c = (i == L - 1) ? ready[static_cast<size_t>(i)]
                                          : (prev_end > ready[static_cast<size_t>(i)] ? prev_end
                                                                                      : ready[static_cast<size_t>(i)]);
        const uint64_t bytes = size_bytes[i] + carried;
        double t_c;
        if (merged[i]) {
            t_c = 0.0;
            carried = bytes;
        } else {
            t_c = message_time(a, b, bytes);
            carried = 0;
        }
        prev_end = tau_c + t_c;
        finish = prev_end;   // after i = 0 this is tau_c^(1) + t_c^(1), Eq. 8 without t_f
    }
    *t_iter_out = finish;
    return MGWFBP_OK;
}

// Exact minimiser of Eq. 8 over all plans (Algorithm 1 is a greedy and can miss it).
//
// Arrival position k = 1..L is tensor L-k.  best_end[k] is the earliest time at which the messages of
// the first k arrivals can all have ended; the last of them carries arrivals i+1..k for some cut i:
//     best_end[k] = min_i  max(best_end[i], ready[k]) + (a + b * bytes(i+1..k)),   best_end[0] = 0.
// The end of a message never gets earlier when the message before it ends later, so taking the
// minimum at every k is exact.  Ties keep the smallest i.  O(L^2) time, O(L) memory.
extern "C" int mgwfbp_plan_opt(const uint64_t* size_bytes, const double* t_backward_s, int32_t L,
                               double a, double b, uint8_t* merged_out, int32_t* group_first_out,
                               int32_t* n_groups_out, double* t_iter_out) {
    if (!valid_inputs(size_bytes, t_backward_s, L, a, b)) return MGWFBP_EINVAL;
    if (L > 0 && merged_out == nullptr) return MGWFBP_EINVAL;
    if (L == 0) {
        if (n_groups_out) *n_groups_out = 0;
        if (group_first_out) group_first_out[0] = -1;
        if (t_iter_out) *t_iter_out = 0.0;
        return MGWFBP_OK;
    }
    std::vector<double> ready_by_tensor;
    gradient_ready_times(t_backward_s, L, ready_by_tensor);
    const size_t n = static_cast<size_t>(L);
    std::vector<double> best_end(n + 1, 0.0);
    std::vector<uint64_t> bytes_upto(n + 1, 0);     // bytes of arrivals 1..k
    std::vector<int32_t> cut(n + 1, 0);
    for (size_t k = 1; k <= n; ++k) bytes_upto[k] = bytes_upto[k - 1] + size_bytes[n - k];
    for (size_t k = 1; k <= n; ++k) {
        const double ready_k = ready_by_tensor[n - k];
        double best = 0.0;
        int32_t best_i = -1;
        for (size_t i = 0; i < k; ++i) {
            const double start = best_end[i] > ready_k ? best_end[i] : ready_k;
            const double end = start + message_time(a, b, bytes_upto[k] - bytes_upto[i]);
            if (best_i < 0 || end < best) {
                best = end;
                best_i = static_cast<int32_t>(i);
            }
        }
        best_end[k] = best;
        cut[k] = best_i;
    }
    for (int32_t i = 0; i < L; ++i) merged_out[i] = 1;
    for (size_t k = n; k > 0; k = static_cast<size_t>(cut[k])) merged_out[n - k] = 0;   // last arrival of a group closes it

    int32_t G = 0;
    for (int32_t i = L - 1; i >= 0; --i) {
        if (i == L - 1 || merged_out[i + 1] == 0) {
            if (group_first_out) group_first_out[G] = i;
            ++G;
        }
    }
    if (group_first_out) group_first_out[G] = -1;
    if (n_groups_out) *n_groups_out = G;
    if (t_iter_out) *t_iter_out = best_end[n];
    return MGWFBP_OK;
}
