// The Solver's choice of the draft length for an active batch size (Section 5.2, "Solver:
// Offline Profiling Guided Search"), host code only.  The profile table is what an offline
// sweep of the verify step measures (batch size, draft length, step time, tokens emitted per
// sequence); the choice minimises Eq. 4's cost per produced token with the measured
// quantities in the place of its symbols.
#include "respec_common.hpp"

#include <algorithm>
#include <cmath>
#include <vector>

namespace respec {
namespace {

struct Row {
    double batch, step_us, emitted;
};

// Value at `b` of the piecewise-linear function through the rows (sorted by batch); the end
// values hold outside the profiled range.
double interpolate(const std::vector<Row> &rows, double b, double Row::*col) {
    if (b <= rows.front().batch) return rows.front().*col;
    if (b >= rows.back().batch) return rows.back().*col;
    for (size_t i = 0; i + 1 < rows.size(); ++i) {
        const Row &lo = rows[i], &hi = rows[i + 1];
        if (b <= hi.batch) {
            if (hi.batch == lo.batch) return lo.*col;
            const double w = (b - lo.batch) / (hi.batch - lo.batch);
            return lo.*col + w * (hi.*col - lo.*col);
        }
    }
    return rows.back().*col;
}

}  // namespace
}  // namespace respec

extern "C" respec_status_t respec_solver_pick(const respec_profile_point_t *points, int32_t n_points,
                                              int32_t active_batch, double draft_us_fixed,
                                              double draft_us_per_seq, int32_t *best_k, double *speedup,
                                              double *cost_us) {
    using namespace respec;
    if (!points || n_points <= 0 || !best_k)
        return fail(RESPEC_ERR_INVALID_ARG, "solver_pick: need a profile table and an output");
    if (active_batch <= 0 || !(draft_us_fixed >= 0.0) || !(draft_us_per_seq >= 0.0))
        return fail(RESPEC_ERR_INVALID_ARG, "solver_pick: need active_batch > 0 and drafter costs >= 0");
    std::vector<int32_t> ks;
    for (int32_t i = 0; i < n_points; ++i) {
        const respec_profile_point_t &p = points[i];
        if (p.batch <= 0 || p.k < 0 || !(p.step_us > 0.0) || !(p.emitted_per_seq > 0.0) ||
            !std::isfinite(p.step_us) || !std::isfinite(p.emitted_per_seq))
            return fail(RESPEC_ERR_INVALID_ARG, "solver_pick: profile point %d is not a measurement", i);
        if (std::find(ks.begin(), ks.end(), p.k) == ks.end()) ks.push_back(p.k);
    }
    std::sort(ks.begin(), ks.end());
    if (ks.front() != 0)
        return fail(RESPEC_ERR_INVALID_ARG, "solver_pick: the profile needs the plain-decoding points (k = 0)");
    const double b = (double)active_batch;
    const double draft = draft_us_fixed + draft_us_per_seq * b;
    double cost0 = 0.0, best_cost = 0.0;
    int32_t best = 0;
    for (const int32_t k : ks) {  // ascending, strict <: ties go to the smaller k
        std::vector<Row> rows;
        for (int32_t i = 0; i < n_points; ++i)
            if (points[i].k == k) rows.push_back({(double)points[i].batch, points[i].step_us, points[i].emitted_per_seq});
        std::stable_sort(rows.begin(), rows.end(), [](const Row &x, const Row &y) { return x.batch < y.batch; });
        const double t = interpolate(rows, b, &Row::step_us), e = interpolate(rows, b, &Row::emitted);
        const double cost = ((double)k * draft + t) / e;
        if (k == 0) cost0 = best_cost = cost;
        else if (cost < best_cost) {
            best_cost = cost;
            best = k;
        }
    }
    *best_k = best;
    if (speedup) *speedup = cost0 / best_cost;
    if (cost_us) *cost_us = best_cost;
    clear_error();
    return RESPEC_OK;
}
