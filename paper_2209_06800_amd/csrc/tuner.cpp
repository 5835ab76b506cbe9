// Run-time parameter search and analytical model (section 6 of the paper), host only.
//
// The search keeps the paper's order -- ps, then dist, then wpb, then the "retreat" of ps with
// a restarted wpb search, a lookup table of every trial, lowest latency wins -- and is exposed
// as a propose / report state machine so that the caller owns the measurement.  Internally
// there is no hidden state beyond the table: the next proposal is found by replaying the
// search against the table until it asks for a configuration that has not been measured.
#include <algorithm>
#include <limits>
#include <new>
#include <vector>

#include "mgg_internal.h"

struct mgg_tuner {
    int32_t limit[3] = {32, 16, 16};
    int32_t dim = 0;                 // > 0: the model's shared-memory constraint bounds the search space
    int64_t smem_limit = 0;
    std::vector<mgg_knobs_t> knobs;
    std::vector<double> latency;
    mgg_knobs_t pending{0, 0, 0};
    bool has_pending = false;
};

namespace {

bool same(const mgg_knobs_t &a, const mgg_knobs_t &b) { return a.ps == b.ps && a.dist == b.dist && a.wpb == b.wpb; }

// Latency of k if it has been measured; *made grows to the number of trials that had been
// made once k was known (the table is in trial order, and a replay meets trials in that order).
bool lookup(const mgg_tuner *t, const mgg_knobs_t &k, double *lat, size_t *made)
{
    for (size_t i = 0; i < t->knobs.size(); ++i)
        if (same(t->knobs[i], k)) { *lat = t->latency[i]; *made = std::max(*made, i + 1); return true; }
    return false;
}

// third-lowest latency among the first n_trials trials
double third_lowest(const mgg_tuner *t, size_t n_trials)
{
    if (n_trials == 0) return std::numeric_limits<double>::infinity();
    std::vector<double> v(t->latency.begin(), t->latency.begin() + n_trials);
    std::sort(v.begin(), v.end());
    return v[std::min<size_t>(2, v.size() - 1)];
}

// the model's constraint on shared memory (section 6): SMEM = ps wpb IntS + 2 wpb D FloatS <= limit
bool feasible(const mgg_tuner *t, const mgg_knobs_t &k)
{
    if (t->dim <= 0) return true;
    const int64_t smem = static_cast<int64_t>(k.ps) * k.wpb * 4 + 2 * static_cast<int64_t>(k.wpb) * t->dim * 4;
    return smem <= t->smem_limit;
}

// Replays the search.  Returns true when it has run to its end; otherwise *need is the
// configuration whose latency is missing.
bool replay(const mgg_tuner *t, mgg_knobs_t *need)
{
    // a configuration outside the model's constraints is never measured: slower than anything that was
#define MGG_MEASURE(k, var)                       \
    do {                                          \
        if (!feasible(t, (k))) (var) = std::numeric_limits<double>::infinity(); \
        else if (!lookup(t, (k), &(var), &made)) { *need = (k); return false; } \
    } while (0)

    int32_t cur[3] = {1, 1, 1};
    double best = 0.0, lat = 0.0, lat2 = 0.0;
    size_t made = 0;                                              // trials made so far in this replay
    MGG_MEASURE((mgg_knobs_t{cur[0], cur[1], cur[2]}), best);
    for (int axis = 0; axis < 3; ++axis) {                       // ps, then dist, then wpb
        while (cur[axis] * 2 <= t->limit[axis]) {
            int32_t trial[3] = {cur[0], cur[1], cur[2]};
            trial[axis] *= 2;
            MGG_MEASURE((mgg_knobs_t{trial[0], trial[1], trial[2]}), lat);
            if (lat >= best) break;                               // the increase did not pay
            cur[axis] = trial[axis];
            best = lat;
        }
    }
    int32_t ps = cur[0];
    const int32_t dist = cur[1];
    while (ps > 1) {                                              // retreat ps, restart wpb
        ps /= 2;
        int32_t wpb = 1;
        const mgg_knobs_t k0{ps, dist, wpb};
        MGG_MEASURE(k0, lat);
        if (lat > third_lowest(t, made)) return true;
        bool stop = false;
        while (wpb * 2 <= t->limit[2]) {
            const mgg_knobs_t k1{ps, dist, wpb * 2};
            MGG_MEASURE(k1, lat2);
            if (lat2 > third_lowest(t, made)) { stop = true; break; }
            if (lat2 >= lat) break;
            wpb *= 2;
            lat = lat2;
        }
        if (stop) return true;
    }
    return true;
#undef MGG_MEASURE
}

}  // namespace

using namespace mgg;

extern "C" {

mgg_status_t mgg_model_evaluate(int64_t n_local_partitions, int64_t n_remote_partitions, mgg_knobs_t k, int32_t dim,
                                int32_t num_units, int64_t smem_limit_bytes, mgg_model_t *out)
{
    if (!out || n_local_partitions < 0 || n_remote_partitions < 0 || k.ps < 1 || k.dist < 1 || k.wpb < 1 || dim < 1 || num_units < 1)
        return fail(MGG_ERR_INVALID_ARG, "bad argument");
    const int64_t int_s = 4, float_s = 4;
    out->wpw = 2 * static_cast<int64_t>(k.ps) * dim * k.dist;                                   // eq. (1)
    out->smem_bytes = static_cast<int64_t>(k.ps) * k.wpb * int_s + 2 * static_cast<int64_t>(k.wpb) * dim * float_s;
    const int64_t parts = std::max(n_local_partitions, n_remote_partitions);
    out->num_waves = (parts + k.dist - 1) / k.dist;                                             // eq. (2)
    out->num_blocks = (out->num_waves + k.wpb - 1) / k.wpb;                                     // eq. (3)
    out->blocks_per_unit = static_cast<double>(out->num_blocks) / num_units;
    out->feasible = out->smem_bytes <= smem_limit_bytes;
    return MGG_OK;
}

mgg_status_t mgg_tuner_create(int32_t ps_max, int32_t dist_max, int32_t wpb_max, mgg_tuner_t **out)
{
    if (!out) return fail(MGG_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (ps_max < 1 || ps_max > 64 || dist_max < 1 || dist_max > 1024 || wpb_max < 1 || wpb_max > 16)
        return fail(MGG_ERR_INVALID_ARG, "limits outside ps <= 64, dist <= 1024, wpb <= 16");
    mgg_tuner *t = new (std::nothrow) mgg_tuner;
    if (!t) return fail(MGG_ERR_ALLOC, "out of host memory");
    t->limit[0] = ps_max; t->limit[1] = dist_max; t->limit[2] = wpb_max;
    *out = t;
    return MGG_OK;
}

mgg_status_t mgg_tuner_set_constraint(mgg_tuner_t *t, int32_t dim, int64_t smem_limit_bytes)
{
    if (!t) return fail(MGG_ERR_INVALID_ARG, "tuner is NULL");
    if (dim < 0 || smem_limit_bytes < 0) return fail(MGG_ERR_INVALID_ARG, "dim %d, limit %lld", dim, (long long)smem_limit_bytes);
    if (!t->knobs.empty() || t->has_pending) return fail(MGG_ERR_INVALID_ARG, "the constraint has to be set before the first trial");
    t->dim = dim;
    t->smem_limit = smem_limit_bytes;
    return MGG_OK;
}

mgg_status_t mgg_tuner_next(mgg_tuner_t *t, mgg_knobs_t *next, int32_t *done)
{
    if (!t || !next || !done) return fail(MGG_ERR_INVALID_ARG, "NULL argument");
    mgg_knobs_t need{0, 0, 0};
    if (replay(t, &need)) { *done = 1; t->has_pending = false; *next = mgg_knobs_t{0, 0, 0}; return MGG_OK; }
    *done = 0;
    *next = need;
    t->pending = need;
    t->has_pending = true;
    return MGG_OK;
}

mgg_status_t mgg_tuner_report(mgg_tuner_t *t, double latency)
{
    if (!t) return fail(MGG_ERR_INVALID_ARG, "tuner is NULL");
    if (!t->has_pending) return fail(MGG_ERR_INVALID_ARG, "no proposal is waiting for a latency");
    if (!(latency >= 0.0)) return fail(MGG_ERR_INVALID_ARG, "latency must be a non-negative number");
    t->knobs.push_back(t->pending);
    t->latency.push_back(latency);
    t->has_pending = false;
    return MGG_OK;
}

mgg_status_t mgg_tuner_result(const mgg_tuner_t *t, mgg_knobs_t *best, double *best_latency, int32_t *n_trials)
{
    if (!t) return fail(MGG_ERR_INVALID_ARG, "tuner is NULL");
    if (t->knobs.empty()) return fail(MGG_ERR_INVALID_ARG, "no trial has been reported yet");
    const size_t i = std::min_element(t->latency.begin(), t->latency.end()) - t->latency.begin();
    if (best) *best = t->knobs[i];
    if (best_latency) *best_latency = t->latency[i];
    if (n_trials) *n_trials = static_cast<int32_t>(t->knobs.size());
    return MGG_OK;
}

mgg_status_t mgg_tuner_table(const mgg_tuner_t *t, int32_t capacity, mgg_knobs_t *knobs, double *latency, int32_t *n_trials)
{
    if (!t || capacity < 0) return fail(MGG_ERR_INVALID_ARG, "bad argument");
    const int32_t n = static_cast<int32_t>(t->knobs.size());
    if (n_trials) *n_trials = n;
    for (int32_t i = 0; i < std::min(n, capacity); ++i) {
        if (knobs) knobs[i] = t->knobs[i];
        if (latency) latency[i] = t->latency[i];
    }
    return MGG_OK;
}

void mgg_tuner_destroy(mgg_tuner_t *t) { delete t; }

mgg_status_t mgg_tune_aggregate(int64_t num_nodes, const int64_t *row_ptr, const int32_t *col_idx, int32_t num_parts,
                                int32_t part_id, const int64_t *bounds, const mgg_build_opts_t *base_opts,
                                mgg_agg_t mode, float eps, mgg_dtype_t x_dtype, const void *x_local, const void *x_halo,
                                int32_t dim, int64_t ld_x, float *out, int64_t ld_out, void *stream, int32_t iters,
                                mgg_tuner_t *tuner, mgg_knobs_t *best, double *best_ms)
{
    if (!tuner) return fail(MGG_ERR_INVALID_ARG, "tuner is NULL");
    // the model's resource constraint, evaluated for this width and the LDS of one compute unit
    if (tuner->dim <= 0 && tuner->knobs.empty() && !tuner->has_pending && dim > 0) { tuner->dim = dim; tuner->smem_limit = 160 * 1024; }
    mgg_build_opts_t o{};
    if (base_opts) o = *base_opts;
    o.host_only = 0;
    for (;;) {
        mgg_knobs_t k;
        int32_t done = 0;
        mgg_status_t s = mgg_tuner_next(tuner, &k, &done);
        if (s != MGG_OK) return s;
        if (done) break;
        o.ps = k.ps; o.dist = k.dist; o.wpb = k.wpb;
        mgg_partition_t *p = nullptr;
        s = mgg_build_partition(num_nodes, row_ptr, col_idx, num_parts, part_id, bounds, &o, &p);
        float ms = 0.f;
        if (s == MGG_OK) {
            s = mgg_partition_reserve(p, dim);
            if (s == MGG_OK) s = mgg_time_aggregate(p, mode, eps, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out, stream, iters, &ms);
            mgg_partition_destroy(p);
        }
        double latency = static_cast<double>(ms);
        if (s == MGG_ERR_ALLOC) {
            // The work items or their partial sums do not fit in memory: the resource constraint
            // of the model.  Such a trial counts as slower than any that fits, and the less so the
            // larger its work items, so the upward sweeps keep moving towards feasible ground.
            (void)hipGetLastError();
            latency = 1e30 / (static_cast<double>(k.ps) * k.dist * k.wpb);
        } else if (s != MGG_OK) {
            return s;
        }
        s = mgg_tuner_report(tuner, latency);
        if (s != MGG_OK) return s;
    }
    return mgg_tuner_result(tuner, best, best_ms, nullptr);
}

}  // extern "C"
