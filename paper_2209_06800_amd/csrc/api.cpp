// Argument checking and composition of the device entry points of libmgg.
#include <algorithm>
#include <atomic>
#include <cstring>

#include "mgg_internal.h"

namespace mgg {

static std::atomic<int32_t> g_lds_halo{0};
static std::atomic<int32_t> g_col_slab_bytes{0};
static std::atomic<int32_t> g_split_phases{0};
static std::atomic<int32_t> g_update_stream{1};
static std::atomic<int32_t> g_items_per_wave{0};
static std::atomic<int32_t> g_short_per_wave{0};
int32_t option_lds_halo() { return g_lds_halo.load(); }
int32_t option_col_slab_bytes() { return g_col_slab_bytes.load(); }
int32_t option_split_phases() { return g_split_phases.load(); }
int32_t option_update_stream() { return g_update_stream.load(); }
int32_t option_items_per_wave() { return g_items_per_wave.load(); }

void take_default_options(mgg_partition *p)
{
    p->opt_lds_halo = g_lds_halo.load(); p->opt_col_slab_bytes = g_col_slab_bytes.load();
    p->opt_split_phases = g_split_phases.load(); p->opt_items_per_wave = g_items_per_wave.load(); p->opt_short_per_wave = g_short_per_wave.load();
}

mgg_status_t check_option(const char *key, int32_t value)
{
    if (!key) return fail(MGG_ERR_INVALID_ARG, "key is NULL");
    if (!std::strcmp(key, "col_slab_bytes")) {
        // 0: automatic, 1: off, otherwise a power of two between 64 and 4096
        if (value != 0 && value != 1 && (value < 64 || value > 4096 || (value & (value - 1)))) return fail(MGG_ERR_INVALID_ARG, "col_slab_bytes must be 0, 1 or a power of two in [64, 4096]");
        return MGG_OK;
    }
    if (!std::strcmp(key, "short_per_wave")) {
        if (value < 0 || value > 64) return fail(MGG_ERR_INVALID_ARG, "short_per_wave must be 0 (automatic) or 1..64");
        return MGG_OK;
    }
    if (!std::strcmp(key, "items_per_wave")) {
        if (value < 0 || value > 64) return fail(MGG_ERR_INVALID_ARG, "items_per_wave must be 0 (automatic) or 1..64");
        return MGG_OK;
    }
    if (std::strcmp(key, "lds_halo") && std::strcmp(key, "split_phases") && std::strcmp(key, "update_stream")) return fail(MGG_ERR_INVALID_ARG, "unknown option '%s'", key);
    if (value != 0 && value != 1) return fail(MGG_ERR_INVALID_ARG, "option value must be 0 or 1");
    return MGG_OK;
}

static inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool dtype_ok(mgg_dtype_t t) { return t == MGG_F32 || t == MGG_BF16; }

static mgg_status_t check_aggregate(const mgg_partition *p, mgg_agg_t mode, mgg_dtype_t x_dtype, const void *x_local,
                                    const void *x_halo, int32_t dim, int64_t ld_x, const void *out, int64_t ld_out,
                                    mgg_dtype_t out_dtype = MGG_F32, bool bags_call = false)
{
    if (!p) return fail(MGG_ERR_INVALID_ARG, "partition is NULL");
    if (p->device < 0) return fail(MGG_ERR_INVALID_ARG, "partition was built host-only");
    if (p->bags != bags_call) return fail(MGG_ERR_INVALID_ARG, p->bags ? "a bag partition takes mgg_bag_sum" : "mgg_bag_sum needs a partition built by mgg_build_bags");
    if (mode != MGG_AGG_GCN_SYM && mode != MGG_AGG_GIN_SUM) return fail(MGG_ERR_INVALID_ARG, "unknown aggregation mode");
    if (!dtype_ok(x_dtype)) return fail(MGG_ERR_INVALID_ARG, "unknown dtype");
    if (dim < 1 || ld_x < dim || ld_out < dim) return fail(MGG_ERR_INVALID_ARG, "dim %d, ld_x %lld, ld_out %lld", dim, (long long)ld_x, (long long)ld_out);
    if (p->n_own > 0 && !out) return fail(MGG_ERR_INVALID_ARG, "out is NULL");
    if ((p->bags ? !p->local_col.empty() : p->n_own > 0) && !x_local) return fail(MGG_ERR_INVALID_ARG, "x_local is NULL");
    if (!p->halo_gid.empty() && !x_halo) return fail(MGG_ERR_INVALID_ARG, "x_halo is NULL but the partition has %zu halo rows", p->halo_gid.size());
    const size_t esz = x_dtype == MGG_BF16 ? 2 : 4;
    if (!dtype_ok(out_dtype)) return fail(MGG_ERR_INVALID_ARG, "unknown output dtype");
    if (reinterpret_cast<uintptr_t>(x_local) % esz || reinterpret_cast<uintptr_t>(x_halo) % esz ||
        reinterpret_cast<uintptr_t>(out) % (out_dtype == MGG_BF16 ? 2 : 4))
        return fail(MGG_ERR_INVALID_ARG, "pointer not aligned to its element size");
    int dev = -1;
    MGG_HIP_TRY(hipGetDevice(&dev));
    if (dev != p->device) return fail(MGG_ERR_INVALID_ARG, "partition lives on device %d, current device is %d", p->device, dev);
    return MGG_OK;
}

static mgg_status_t check_update(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
                                 mgg_dtype_t w_dtype, const void *w, int32_t d_out, mgg_act_t act, mgg_dtype_t out_dtype,
                                 const void *out, int64_t ld_out)
{
    if (n_rows < 0 || d_in < 1 || d_out < 1 || ld_a < d_in || ld_out < d_out)
        return fail(MGG_ERR_INVALID_ARG, "n_rows %lld, d_in %d, d_out %d, ld_a %lld, ld_out %lld", (long long)n_rows, d_in, d_out, (long long)ld_a, (long long)ld_out);
    if (!dtype_ok(a_dtype) || !dtype_ok(w_dtype) || !dtype_ok(out_dtype)) return fail(MGG_ERR_INVALID_ARG, "unknown dtype");
    if (act != MGG_ACT_NONE && act != MGG_ACT_RELU && act != MGG_ACT_SOFTMAX) return fail(MGG_ERR_INVALID_ARG, "unknown activation");
    if (w_dtype == MGG_F32 && a_dtype != MGG_F32) return fail(MGG_ERR_UNSUPPORTED, "fp32 weights need fp32 input");
    if (!w || (n_rows > 0 && (!a || !out))) return fail(MGG_ERR_INVALID_ARG, "NULL matrix pointer");
    if (reinterpret_cast<uintptr_t>(a) % (a_dtype == MGG_BF16 ? 2 : 4) || reinterpret_cast<uintptr_t>(w) % (w_dtype == MGG_BF16 ? 2 : 4) ||
        reinterpret_cast<uintptr_t>(out) % (out_dtype == MGG_BF16 ? 2 : 4))
        return fail(MGG_ERR_INVALID_ARG, "pointer not aligned to its element size");
    return MGG_OK;
}

struct LayerPlan {
    bool update_first = false;
    int64_t ld_agg = 0, ld_hid = 0;
    size_t agg_bytes = 0, hid_bytes = 0;        // aggregation result (width dims[0], or dims[1] when update_first), hidden activations
    size_t t_local_bytes = 0, t_halo_bytes = 0; // update_first: X w[0] of the two tables, leading dimension ld_agg
    size_t scratch_bytes = 0;                   // partial sums of rows cut into several work items (last in the workspace)
    mgg_dtype_t hid_dtype = MGG_F32;
    size_t total() const { return agg_bytes + hid_bytes + t_local_bytes + t_halo_bytes + scratch_bytes; }
    size_t scratch_offset() const { return agg_bytes + hid_bytes + t_local_bytes + t_halo_bytes; }
};

static bool plan_layer(const mgg_partition *p, const mgg_layer_desc_t *l, mgg_dtype_t x_dtype, mgg_dtype_t out_dtype, LayerPlan *pl)
{
    if (!p || !l || (l->n_linear != 1 && l->n_linear != 2)) return false;
    for (int i = 0; i <= l->n_linear; ++i)
        if (l->dims[i] < 1) return false;
    if (l->order != MGG_ORDER_AGG_FIRST && l->order != MGG_ORDER_UPDATE_FIRST && l->order != MGG_ORDER_AUTO) return false;
    // fp32 weights cannot take bf16 input, and a single linear hands its rows straight to `out`
    const bool supported = !(l->w_dtype == MGG_F32 && x_dtype == MGG_BF16) && (l->n_linear == 2 || out_dtype == MGG_F32);
    const int64_t in_bytes = static_cast<int64_t>(l->dims[0]) * (x_dtype == MGG_BF16 ? 2 : 4);
    pl->update_first = l->order == MGG_ORDER_UPDATE_FIRST ||
                       (l->order == MGG_ORDER_AUTO && supported && static_cast<int64_t>(l->dims[1]) * 4 * 4 <= in_bytes * 3);
    const int32_t agg_dim = pl->update_first ? l->dims[1] : l->dims[0];
    pl->ld_agg = static_cast<int64_t>(round_up(static_cast<size_t>(agg_dim), 8));      // rows start 32-byte aligned
    pl->agg_bytes = round_up(static_cast<size_t>(p->n_own) * pl->ld_agg * sizeof(float), 256);
    if (pl->update_first) {
        pl->t_local_bytes = pl->agg_bytes;
        pl->t_halo_bytes = round_up(p->halo_gid.size() * static_cast<size_t>(pl->ld_agg) * sizeof(float), 256);
        if (l->n_linear == 1) pl->agg_bytes = 0;       // aggregated rows are the layer's output
    }
    pl->scratch_bytes = round_up(scratch_bytes_for(p, static_cast<int32_t>(pl->ld_agg)), 256);
    if (l->n_linear == 2 && !pl->update_first) {
        pl->hid_dtype = l->w_dtype == MGG_BF16 ? MGG_BF16 : MGG_F32;
        pl->ld_hid = static_cast<int64_t>(round_up(static_cast<size_t>(l->dims[1]), 8));
        pl->hid_bytes = round_up(static_cast<size_t>(p->n_own) * pl->ld_hid * (pl->hid_dtype == MGG_BF16 ? 2 : 4), 256);
    }
    return true;
}

}  // namespace mgg

using namespace mgg;

extern "C" {

mgg_status_t mgg_aggregate(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                           const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x, float *out,
                           int64_t ld_out, void *stream)
{
    mgg_status_t s = check_aggregate(p, mode, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out);
    if (s != MGG_OK) return s;
    if (p->n_own == 0) return MGG_OK;
    return launch_aggregate(p, mode, eps, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out, static_cast<hipStream_t>(stream));
}

mgg_status_t mgg_aggregate_to(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype, const void *x_local,
                              const void *x_halo, int32_t dim, int64_t ld_x, mgg_dtype_t out_dtype, void *out, int64_t ld_out,
                              void *stream)
{
    mgg_status_t s = check_aggregate(p, mode, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out, out_dtype);
    if (s != MGG_OK) return s;
    if (p->n_own == 0) return MGG_OK;
    return launch_aggregate(p, mode, eps, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out, static_cast<hipStream_t>(stream), nullptr,
                            MGG_ACT_NONE, 0, out_dtype);
}

mgg_status_t mgg_aggregate_static(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype, const void *x_local,
                                  const void *x_halo, int32_t dim, int64_t ld_x, float *out, int64_t ld_out, void *stream)
{
    mgg_status_t s = check_aggregate(p, mode, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out);
    if (s != MGG_OK) return s;
    if (p->n_own == 0) return MGG_OK;
    size_t cap = 0;
    float *scratch = static_scratch(&cap);
    if (!scratch) return MGG_ERR_HIP;
    const size_t need = scratch_bytes_for(p, dim);
    if (need > cap)
        return fail(MGG_ERR_UNSUPPORTED, "partial sums of this partition at width %d take %zu bytes, the fixed scratch array holds %zu", dim, need, cap);
    return launch_aggregate(p, mode, eps, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out, static_cast<hipStream_t>(stream), nullptr, MGG_ACT_NONE, 0,
                            MGG_F32, scratch, cap);
}

size_t mgg_aggregate_scratch_bytes(const mgg_partition_t *p, int32_t dim)
{
    if (!p || dim < 1) return 0;
    return scratch_bytes_for(p, dim);
}

mgg_status_t mgg_partition_reserve(mgg_partition_t *p, int32_t dim)
{
    if (!p) return fail(MGG_ERR_INVALID_ARG, "partition is NULL");
    if (p->device < 0) return fail(MGG_ERR_INVALID_ARG, "partition was built host-only");
    if (dim < 1) return fail(MGG_ERR_INVALID_ARG, "dim %d", dim);
    int dev = -1;
    MGG_HIP_TRY(hipGetDevice(&dev));
    if (dev != p->device) return fail(MGG_ERR_INVALID_ARG, "partition lives on device %d, current device is %d", p->device, dev);
    const int64_t need_ld = scratch_ld_for(dim);
    if (p->reserved_dim < dim) p->reserved_dim = dim;
    if (p->n_split_items == 0 || p->d.scratch_ld >= need_ld) return MGG_OK;
    // work already enqueued may still use the old buffer
    MGG_HIP_TRY(hipDeviceSynchronize());
    if (p->d.scratch) { (void)hipFree(p->d.scratch); p->d.scratch = nullptr; p->d.scratch_ld = 0; }
    const size_t bytes = static_cast<size_t>(p->n_split_items) * static_cast<size_t>(need_ld) * sizeof(float);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&p->d.scratch), bytes);
    if (e != hipSuccess) { p->reserved_dim = 0; return fail(MGG_ERR_ALLOC, "hipMalloc(%zu bytes of scratch): %s", bytes, hipGetErrorString(e)); }
    p->d.scratch_ld = need_ld;
    return MGG_OK;
}

mgg_status_t mgg_bag_sum(const mgg_partition_t *p, mgg_dtype_t x_dtype, const void *table_local, const void *table_halo, int32_t dim,
                         int64_t ld_x, mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream)
{
    mgg_status_t s = check_aggregate(p, MGG_AGG_GIN_SUM, x_dtype, table_local, table_halo, dim, ld_x, out, ld_out, out_dtype, true);
    if (s != MGG_OK) return s;
    if (p->n_own == 0) return MGG_OK;
    // a kernel argument must not be NULL even when no bag looks into the local slice
    const void *tl = table_local ? table_local : (table_halo ? table_halo : out);
    return launch_aggregate(p, MGG_AGG_GIN_SUM, -1.f, x_dtype, tl, table_halo, dim, ld_x, out, ld_out, static_cast<hipStream_t>(stream),
                            nullptr, MGG_ACT_NONE, 0, out_dtype);
}

mgg_status_t mgg_update(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
                        mgg_dtype_t w_dtype, const void *w, const float *bias, int32_t d_out, mgg_act_t act,
                        mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream)
{
    mgg_status_t s = check_update(n_rows, a_dtype, a, ld_a, d_in, w_dtype, w, d_out, act, out_dtype, out, ld_out);
    if (s != MGG_OK) return s;
    return launch_update(n_rows, a_dtype, a, ld_a, d_in, w_dtype, w, bias, d_out, act, out_dtype, out, ld_out,
                         static_cast<hipStream_t>(stream));
}

size_t mgg_layer_workspace_bytes(const mgg_partition_t *p, const mgg_layer_desc_t *layer)
{
    // the largest need over the dtypes the call may be given (UPDATE_FIRST under AUTO depends on them)
    size_t need = 0;
    for (mgg_dtype_t xd : {MGG_F32, MGG_BF16})
        for (mgg_dtype_t od : {MGG_F32, MGG_BF16}) {
            LayerPlan pl;
            if (!plan_layer(p, layer, xd, od, &pl)) return 0;
            need = std::max(need, pl.total());
        }
    return need + 256;
}

mgg_status_t mgg_layer_forward(const mgg_partition_t *p, const mgg_layer_desc_t *layer, mgg_dtype_t x_dtype,
                               const void *x_local, const void *x_halo, int64_t ld_x, void *workspace,
                               size_t workspace_bytes, mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream)
{
    LayerPlan pl;
    if (!dtype_ok(x_dtype) || !dtype_ok(out_dtype)) return fail(MGG_ERR_INVALID_ARG, "unknown dtype");
    if (!plan_layer(p, layer, x_dtype, out_dtype, &pl)) return fail(MGG_ERR_INVALID_ARG, "bad layer description");
    if (!workspace || reinterpret_cast<uintptr_t>(workspace) % 256) return fail(MGG_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (workspace_bytes < pl.total()) return fail(MGG_ERR_INVALID_ARG, "workspace too small: %zu < %zu", workspace_bytes, pl.total());
    const int32_t d0 = layer->dims[0], d1 = layer->dims[1], d2 = layer->dims[2];
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t n_halo = static_cast<int64_t>(p->halo_gid.size());
    mgg_status_t s;

    if (pl.update_first) {
        // Aggregate(X) w[0] computed as Aggregate(X w[0]): transform both tables, gather the narrower rows
        if (layer->n_linear == 1 && out_dtype != MGG_F32) return fail(MGG_ERR_UNSUPPORTED, "UPDATE_FIRST with one linear needs fp32 output");
        char *ws = static_cast<char *>(workspace);
        float *t_local = reinterpret_cast<float *>(ws);
        float *t_halo = reinterpret_cast<float *>(ws + pl.t_local_bytes);
        float *agg = layer->n_linear == 1 ? static_cast<float *>(out) : reinterpret_cast<float *>(ws + pl.t_local_bytes + pl.t_halo_bytes);
        const int64_t ld_aggout = layer->n_linear == 1 ? ld_out : pl.ld_agg;
        if (layer->n_linear == 1 && ld_out < d1) return fail(MGG_ERR_INVALID_ARG, "ld_out %lld < %d", (long long)ld_out, d1);
        // validate everything before the first launch so that an error leaves no partial output
        if (n_halo > 0 && !x_halo) return fail(MGG_ERR_INVALID_ARG, "x_halo is NULL but the partition has %lld halo rows", (long long)n_halo);
        if (ld_x < d0) return fail(MGG_ERR_INVALID_ARG, "ld_x %lld < %d", (long long)ld_x, d0);
        s = check_aggregate(p, layer->mode, MGG_F32, t_local, t_halo, d1, pl.ld_agg, agg, ld_aggout);
        if (s == MGG_OK) s = check_update(p->n_own, x_dtype, x_local, ld_x, d0, layer->w_dtype, layer->w[0], d1, MGG_ACT_NONE, MGG_F32, t_local, pl.ld_agg);
        if (s == MGG_OK && n_halo > 0) s = check_update(n_halo, x_dtype, x_halo, ld_x, d0, layer->w_dtype, layer->w[0], d1, MGG_ACT_NONE, MGG_F32, t_halo, pl.ld_agg);
        if (s == MGG_OK && layer->n_linear == 2)
            s = check_update(p->n_own, MGG_F32, agg, pl.ld_agg, d1, layer->w_dtype, layer->w[1], d2, layer->act[1], out_dtype, out, ld_out);
        if (s == MGG_OK && layer->act[0] != MGG_ACT_NONE && layer->act[0] != MGG_ACT_RELU && layer->act[0] != MGG_ACT_SOFTMAX)
            s = fail(MGG_ERR_INVALID_ARG, "unknown activation");
        if (s != MGG_OK) return s;
        if (p->n_own == 0) return MGG_OK;
        s = launch_update(p->n_own, x_dtype, x_local, ld_x, d0, layer->w_dtype, layer->w[0], nullptr, d1, MGG_ACT_NONE, MGG_F32, t_local, pl.ld_agg, st);
        if (s != MGG_OK) return s;
        if (n_halo > 0) {
            s = launch_update(n_halo, x_dtype, x_halo, ld_x, d0, layer->w_dtype, layer->w[0], nullptr, d1, MGG_ACT_NONE, MGG_F32, t_halo, pl.ld_agg, st);
            if (s != MGG_OK) return s;
        }
        // the transformed tables are gathered at their width rounded up to whole 16-byte vectors (the
        // padding columns hold whatever the workspace held and only reach output columns that do not exist)
        const int32_t d1_padded = static_cast<int32_t>(std::min<int64_t>(round_up(static_cast<size_t>(d1), 4), pl.ld_agg));
        const bool softmax0 = layer->act[0] == MGG_ACT_SOFTMAX;     // not an elementwise epilogue: its own pass
        s = launch_aggregate(p, layer->mode, layer->eps, MGG_F32, t_local, n_halo > 0 ? t_halo : nullptr, d1_padded, pl.ld_agg, agg,
                             ld_aggout, st, layer->bias[0], softmax0 ? MGG_ACT_NONE : layer->act[0], d1, MGG_F32,
                             reinterpret_cast<float *>(ws + pl.scratch_offset()), pl.scratch_bytes);
        if (s == MGG_OK && softmax0) s = launch_row_softmax(p->n_own, d1, MGG_F32, agg, ld_aggout, st);
        if (s != MGG_OK || layer->n_linear == 1) return s;
        return launch_update(p->n_own, MGG_F32, agg, pl.ld_agg, d1, layer->w_dtype, layer->w[1], layer->bias[1], d2, layer->act[1],
                             out_dtype, out, ld_out, st);
    }

    // With bf16 weights the rows are rounded to bf16 on the way into the MFMA anyway; rounding them on the
    // way out of the aggregation gives the same bits and halves what is written and read back.
    void *agg = workspace;
    const mgg_dtype_t agg_dtype = layer->w_dtype == MGG_BF16 ? MGG_BF16 : MGG_F32;
    void *hid = static_cast<char *>(workspace) + pl.agg_bytes;
    // validate everything before the first launch so that an error leaves no partial output
    s = check_aggregate(p, layer->mode, x_dtype, x_local, x_halo, d0, ld_x, agg, pl.ld_agg, agg_dtype);
    if (s != MGG_OK) return s;
    if (layer->n_linear == 1)
        s = check_update(p->n_own, agg_dtype, agg, pl.ld_agg, d0, layer->w_dtype, layer->w[0], d1, layer->act[0], out_dtype, out, ld_out);
    else {
        s = check_update(p->n_own, agg_dtype, agg, pl.ld_agg, d0, layer->w_dtype, layer->w[0], d1, layer->act[0], pl.hid_dtype, hid, pl.ld_hid);
        if (s == MGG_OK)
            s = check_update(p->n_own, pl.hid_dtype, hid, pl.ld_hid, d1, layer->w_dtype, layer->w[1], d2, layer->act[1], out_dtype, out, ld_out);
    }
    if (s != MGG_OK) return s;
    if (p->n_own == 0) return MGG_OK;

    s = launch_aggregate(p, layer->mode, layer->eps, x_dtype, x_local, x_halo, d0, ld_x, agg, pl.ld_agg, st, nullptr, MGG_ACT_NONE, 0, agg_dtype,
                         reinterpret_cast<float *>(static_cast<char *>(workspace) + pl.scratch_offset()), pl.scratch_bytes);
    if (s != MGG_OK) return s;
    if (layer->n_linear == 1)
        return launch_update(p->n_own, agg_dtype, agg, pl.ld_agg, d0, layer->w_dtype, layer->w[0], layer->bias[0], d1,
                             layer->act[0], out_dtype, out, ld_out, st);
    return launch_update_mlp(p->n_own, agg_dtype, agg, pl.ld_agg, layer->dims, layer->w_dtype, layer->w[0], layer->bias[0], layer->act[0],
                             layer->w[1], layer->bias[1], layer->act[1], hid, pl.ld_hid, out_dtype, out, ld_out, st);
}

mgg_status_t mgg_update_mlp(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, const int32_t *dims, mgg_dtype_t w_dtype,
                            const void *w1, const float *bias1, mgg_act_t act1, const void *w2, const float *bias2, mgg_act_t act2,
                            void *hidden, int64_t ld_hidden, mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream)
{
    if (!dims) return fail(MGG_ERR_INVALID_ARG, "dims is NULL");
    const mgg_dtype_t hid_dtype = w_dtype == MGG_BF16 ? MGG_BF16 : MGG_F32;
    // Both products are checked as if they ran one after the other.  `hidden` may be NULL (the one-kernel
    // form needs none; launch_update_mlp refuses NULL when it has to fall back): `out` then stands in for it
    // in the checks, which only look at NULL-ness and alignment.
    const void *hid_probe = hidden ? hidden : out;
    const int64_t ld_probe = hidden ? ld_hidden : dims[1];
    mgg_status_t s = check_update(n_rows, a_dtype, a, ld_a, dims[0], w_dtype, w1, dims[1], act1, hid_dtype, hid_probe, ld_probe);
    if (s == MGG_OK) s = check_update(n_rows, hid_dtype, hid_probe, ld_probe, dims[1], w_dtype, w2, dims[2], act2, out_dtype, out, ld_out);
    if (s != MGG_OK) return s;
    return launch_update_mlp(n_rows, a_dtype, a, ld_a, dims, w_dtype, w1, bias1, act1, w2, bias2, act2, hidden, ld_hidden, out_dtype, out,
                             ld_out, static_cast<hipStream_t>(stream));
}

mgg_status_t mgg_set_option(const char *key, int32_t value)
{
    mgg_status_t s = check_option(key, value);
    if (s != MGG_OK) return s;
    if (!std::strcmp(key, "col_slab_bytes")) g_col_slab_bytes = value;
    else if (!std::strcmp(key, "items_per_wave")) g_items_per_wave = value;
    else if (!std::strcmp(key, "short_per_wave")) g_short_per_wave = value;
    else if (!std::strcmp(key, "lds_halo")) g_lds_halo = value;
    else if (!std::strcmp(key, "split_phases")) g_split_phases = value;
    else g_update_stream = value;
    return MGG_OK;
}

mgg_status_t mgg_get_option(const char *key, int32_t *value)
{
    if (!key || !value) return fail(MGG_ERR_INVALID_ARG, "NULL argument");
    if (!std::strcmp(key, "lds_halo")) { *value = g_lds_halo; return MGG_OK; }
    if (!std::strcmp(key, "col_slab_bytes")) { *value = g_col_slab_bytes; return MGG_OK; }
    if (!std::strcmp(key, "split_phases")) { *value = g_split_phases; return MGG_OK; }
    if (!std::strcmp(key, "update_stream")) { *value = g_update_stream; return MGG_OK; }
    if (!std::strcmp(key, "items_per_wave")) { *value = g_items_per_wave; return MGG_OK; }
    if (!std::strcmp(key, "short_per_wave")) { *value = g_short_per_wave; return MGG_OK; }
    return fail(MGG_ERR_INVALID_ARG, "unknown option '%s'", key);
}

mgg_status_t mgg_partition_set_option(mgg_partition_t *p, const char *key, int32_t value)
{
    if (!p) return fail(MGG_ERR_INVALID_ARG, "partition is NULL");
    mgg_status_t s = check_option(key, value);
    if (s != MGG_OK) return s;
    if (!std::strcmp(key, "col_slab_bytes")) p->opt_col_slab_bytes = value;
    else if (!std::strcmp(key, "items_per_wave")) p->opt_items_per_wave = value;
    else if (!std::strcmp(key, "short_per_wave")) p->opt_short_per_wave = value;
    else if (!std::strcmp(key, "lds_halo")) p->opt_lds_halo = value;
    else if (!std::strcmp(key, "split_phases")) p->opt_split_phases = value;
    else return fail(MGG_ERR_INVALID_ARG, "'%s' is not a switch of the aggregation", key);
    return MGG_OK;
}

mgg_status_t mgg_partition_get_option(const mgg_partition_t *p, const char *key, int32_t *value)
{
    if (!p || !key || !value) return fail(MGG_ERR_INVALID_ARG, "NULL argument");
    if (!std::strcmp(key, "lds_halo")) { *value = p->opt_lds_halo; return MGG_OK; }
    if (!std::strcmp(key, "col_slab_bytes")) { *value = p->opt_col_slab_bytes; return MGG_OK; }
    if (!std::strcmp(key, "split_phases")) { *value = p->opt_split_phases; return MGG_OK; }
    if (!std::strcmp(key, "items_per_wave")) { *value = p->opt_items_per_wave; return MGG_OK; }
    if (!std::strcmp(key, "short_per_wave")) { *value = p->opt_short_per_wave; return MGG_OK; }
    return fail(MGG_ERR_INVALID_ARG, "unknown option '%s'", key);
}

mgg_status_t mgg_probe_gather(int64_t table_bytes, int32_t row_bytes, int64_t n_gathers, int32_t iters, uint64_t seed, double *gbytes_per_s)
{
    return probe_gather(table_bytes, row_bytes, n_gathers, iters, seed, gbytes_per_s);
}

mgg_status_t mgg_time_aggregate(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                                const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x, float *out,
                                int64_t ld_out, void *stream, int32_t iters, float *ms_per_call)
{
    if (iters < 1 || !ms_per_call) return fail(MGG_ERR_INVALID_ARG, "iters < 1 or ms_per_call is NULL");
    hipStream_t st = static_cast<hipStream_t>(stream);
    // one untimed call first: it validates the arguments
    mgg_status_t s = mgg_aggregate(p, mode, eps, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out, stream);
    if (s != MGG_OK) return s;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    MGG_HIP_TRY(hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return hip_fail(e, "hipEventCreate"); }
    float ms = 0.f;
    e = hipEventRecord(e0, st);
    for (int32_t i = 0; i < iters && e == hipSuccess && s == MGG_OK; ++i)
        s = mgg_aggregate(p, mode, eps, x_dtype, x_local, x_halo, dim, ld_x, out, ld_out, stream);
    if (e == hipSuccess) e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (s != MGG_OK) return s;
    if (e != hipSuccess) return hip_fail(e, "event timing");
    *ms_per_call = ms / static_cast<float>(iters);
    return MGG_OK;
}

}  // extern "C"
