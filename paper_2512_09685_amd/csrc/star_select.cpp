// Host-only: STAR-H, the heuristic choice of the synchronization mode
// (Section 4.3.1), producing the worker groups that feed star_group_update.
//
// Given the predicted iteration times T_k of a job's N workers, the
// pre-conditioned gradient noise scale phi of the current step and the total
// batch size M:
//   straggler test   d_i = (T_i - min T) / min T > threshold            (Section 2)
//   static x-order   T_x = (1 + phi/(x M/N)) * t_x                       (Eq. 1)
//   dynamic x-order  T_d = 1 / sum_i 1/((1 + phi/(n_ci M/N)) * t_ci)     (Eq. 2)
//   all-reduce       T_a = (1 + phi/((N-x+q) M/N)) * (t_ring + t_w)      (Eq. 3)
// and the mode with the least time wins.
//
// Readings where the paper is silent:
//  * t_x.  The paper says t_x, the expected time of one parameter update,
//    follows from the predicted iteration times without giving the rule.
//    Here t_x is the time by which x gradient reports have arrived: the x-th
//    smallest predicted iteration time.  x = N gives max T (SSGD waits for
//    the slowest worker), x = 1 gives min T.  (Summing update rates over
//    groups instead, as Eq. 2 does over clusters, would make the smallest
//    groups win for every input: the noise factor 1 + phi/B charges B + phi
//    samples per unit of progress, least for the smallest batch B.)
//  * Groups of a static mode handed back to the caller: the workers in
//    ascending iteration time, cut into consecutive groups of x (the order in
//    which reports arrive; the last group is smaller when x does not divide N).
//  * Clustering.  Agglomerative, complete linkage on the one-dimensional
//    times: the two clusters whose union has the smallest range are merged
//    while that range, relative to the union's fastest member, stays within
//    cluster_threshold (the straggler threshold by default, so no member of a
//    cluster is a straggler with respect to its own cluster).
//  * Ties go to the higher order (more gradients per update converge to a
//    higher accuracy, Section 4.2); the dynamic mode must be strictly faster.
//  * Without a straggler the job stays in SSGD (the mode is only reconsidered
//    when a straggler is predicted, Section 4.1).
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "star.h"

namespace {

bool finite_pos(double x) { return std::isfinite(x) && x > 0.0; }

double noise_factor(double phi, double n, double M, double N) { return 1.0 + phi / (n * M / N); }

}  // namespace

extern "C" {

star_status star_select_mode_ps(int32_t N, const double* iter_time, double phi, double batch_total,
                                double straggler_threshold, double cluster_threshold, star_mode_choice* choice,
                                double* time_static, double* time_dynamic, int32_t* group_offsets,
                                int32_t* group_members, int32_t* is_straggler) {
    if (!iter_time || !choice || !group_offsets || !group_members) return STAR_ERR_NULL;
    if (N < 1 || N > STAR_MAX_WORKERS) return STAR_ERR_SHAPE;
    if (!std::isfinite(phi) || phi < 0.0 || !finite_pos(batch_total) || !(straggler_threshold >= 0.0) ||
        !(cluster_threshold >= 0.0))
        return STAR_ERR_HPARAM;
    for (int32_t k = 0; k < N; ++k)
        if (!finite_pos(iter_time[k])) return STAR_ERR_HPARAM;

    const double Nd = (double)N, M = batch_total;
    std::vector<int32_t> order(N);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return iter_time[a] < iter_time[b]; });
    std::vector<double> t(N);
    for (int32_t i = 0; i < N; ++i) t[i] = iter_time[order[i]];
    const double tmin = t[0];

    int32_t n_strag = 0;
    for (int32_t k = 0; k < N; ++k) {
        const bool s = (iter_time[k] - tmin) / tmin > straggler_threshold;
        if (is_straggler) is_straggler[k] = s ? 1 : 0;
        n_strag += s ? 1 : 0;
    }

    // static x-order, x = 1..N
    std::vector<double> Tx(N + 1, 0.0);
    for (int32_t x = 1; x <= N; ++x) {
        Tx[x] = noise_factor(phi, (double)x, M, Nd) * t[x - 1];
        if (time_static) time_static[x - 1] = Tx[x];
    }

    // dynamic x-order: clusters as [begin, end) ranges of the sorted workers
    std::vector<int32_t> cut;  // cluster start positions
    for (int32_t i = 0; i < N; ++i) cut.push_back(i);
    cut.push_back(N);
    for (;;) {
        const int32_t nc = (int32_t)cut.size() - 1;
        if (nc <= 1) break;
        int32_t best = -1;
        double best_range = 0.0;
        for (int32_t c = 0; c + 1 < nc; ++c) {
            const double range = t[cut[c + 2] - 1] - t[cut[c]];
            if (best < 0 || range < best_range) {
                best = c;
                best_range = range;
            }
        }
        if (best_range / t[cut[best]] > cluster_threshold) break;
        cut.erase(cut.begin() + best + 1);
    }
    const int32_t n_clusters = (int32_t)cut.size() - 1;
    double rate_d = 0.0;
    for (int32_t c = 0; c < n_clusters; ++c)
        rate_d += 1.0 / (noise_factor(phi, (double)(cut[c + 1] - cut[c]), M, Nd) * t[cut[c + 1] - 1]);
    const double Td = 1.0 / rate_d;
    if (time_dynamic) *time_dynamic = Td;

    // the least time; ties to the higher order; dynamic only when strictly faster
    int32_t best_x = N;
    for (int32_t x = N - 1; x >= 1; --x)
        if (Tx[x] < Tx[best_x]) best_x = x;
    bool dynamic = Td < Tx[best_x];
    if (n_strag == 0) {
        best_x = N;
        dynamic = false;
    }

    choice->n_stragglers = n_strag;
    choice->n_clusters = n_clusters;
    if (dynamic) {
        choice->mode = STAR_MODE_DYNAMIC_X;
        choice->x = 0;
        choice->time_to_progress = Td;
        choice->n_groups = n_clusters;
        for (int32_t c = 0; c <= n_clusters; ++c) group_offsets[c] = cut[c];
    } else {
        choice->mode = best_x == N ? STAR_MODE_SSGD : (best_x == 1 ? STAR_MODE_ASGD : STAR_MODE_STATIC_X);
        choice->x = best_x;
        choice->time_to_progress = Tx[best_x];
        int32_t g = 0;
        for (int32_t lo = 0; lo < N; lo += best_x) group_offsets[g++] = lo;
        group_offsets[g] = N;
        choice->n_groups = g;
    }
    for (int32_t i = 0; i < N; ++i) group_members[i] = order[i];
    return STAR_OK;
}

star_status star_select_mode_ar(int32_t N, const double* iter_time, const double* child_time, double phi,
                                double batch_total, double straggler_threshold, int32_t n_wait,
                                const double* wait_candidates, int32_t* removed_out, double* wait_out,
                                double* time_out, double* time_table) {
    if (!iter_time || !child_time || !removed_out || !wait_out || !time_out) return STAR_ERR_NULL;
    if (n_wait > 0 && !wait_candidates) return STAR_ERR_NULL;
    if (N < 1 || N > STAR_MAX_WORKERS || n_wait < 0) return STAR_ERR_SHAPE;
    if (!std::isfinite(phi) || phi < 0.0 || !finite_pos(batch_total) || !(straggler_threshold >= 0.0))
        return STAR_ERR_HPARAM;
    for (int32_t k = 0; k < N; ++k)
        if (!finite_pos(iter_time[k]) || !(child_time[k] >= 0.0) || !std::isfinite(child_time[k])) return STAR_ERR_HPARAM;
    for (int32_t i = 0; i < n_wait; ++i)
        if (!(wait_candidates[i] >= 0.0) || !std::isfinite(wait_candidates[i])) return STAR_ERR_HPARAM;

    const double Nd = (double)N, M = batch_total;
    std::vector<int32_t> order(N);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return iter_time[a] < iter_time[b]; });
    const double tmin = iter_time[order[0]];
    int32_t X = 0;  // stragglers
    for (int32_t k = 0; k < N; ++k) X += (iter_time[k] - tmin) / tmin > straggler_threshold ? 1 : 0;

    // x = 0 (nobody removed, no waiting) is the plain ring; then the x slowest workers are removed, x <= X
    double best_T = noise_factor(phi, Nd, M, Nd) * iter_time[order[N - 1]];
    int32_t best_x = 0;
    double best_w = 0.0;
    if (time_table) time_table[0] = best_T;
    for (int32_t x = 1; x <= X && x < N; ++x) {
        const double t_ring = iter_time[order[N - 1 - x]];
        for (int32_t i = 0; i < n_wait; ++i) {
            const double tw = wait_candidates[i];
            int32_t q = 0;
            for (int32_t r = 0; r < x; ++r) q += child_time[order[N - 1 - r]] <= tw ? 1 : 0;
            const double Ta = noise_factor(phi, (double)(N - x + q), M, Nd) * (t_ring + tw);
            if (time_table) time_table[1 + (size_t)(x - 1) * n_wait + i] = Ta;
            if (Ta < best_T) {
                best_T = Ta;
                best_x = x;
                best_w = tw;
            }
        }
    }
    *removed_out = best_x;
    *wait_out = best_w;
    *time_out = best_T;
    return STAR_OK;
}

}  // extern "C"
