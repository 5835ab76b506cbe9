// Internal declarations shared by the translation units of libmgg (not installed).
#pragma once

#include <hip/hip_runtime_api.h>
#include <hip/hip_vector_types.h>

#include <cstdarg>
#include <cstdint>
#include <vector>

#include "mgg.h"

namespace mgg {

// One wavefront work item: a run of neighbour partitions of one owned row, from the local
// list and from the remote list (section 5.1: a warp handles pairs of local / remote
// partitions).  slot < 0: the item covers the whole row and writes the final value;
// slot >= 0: it writes a raw partial sum into scratch row `slot`.  row < 0: padding, nothing to do.
struct WorkItem {
    int32_t row;
    int32_t lbeg, lend;   // range in local_col
    int32_t rbeg, rend;   // range in remote_col
    int32_t slot;
    int32_t pad0, pad1;
};
static_assert(sizeof(WorkItem) == 32, "WorkItem is read as two 16-byte words");

// A row that was cut into several items: its partial sums sit in scratch rows
// [first_slot, first_slot + n_slots) and are combined in that order.
struct SplitRow {
    int32_t row;
    int32_t first_slot;
    int32_t n_slots;
    int32_t pad;
};

constexpr int kXcd = 8;             // accelerator complex dies of an MI355X, each with its own L2
constexpr int kDefaultWpb = 2;      // work items (wavefronts) per workgroup of the aggregation kernel
constexpr int kDefaultXcdMinDeg = 256;
constexpr int kDefaultHotPhases = 0;        // automatic choice between hash classes and popularity phases
constexpr int kAutoHotPhases = 4;           // phases when the automatic choice takes popularity classes
constexpr int kMaxHotPhases = 31;           // class index phase * 8 + XCD has to stay below kColdClass
constexpr int kDefaultMinPiece = 16;        // a class with fewer neighbours in a row joins the row's cold piece
constexpr int kDefaultHotMinCount = 8;      // table rows gathered fewer times than this are never hot
constexpr int kColdClass = 255;
constexpr int64_t kHotBytesPerXcd = 3 << 20;   // of the 4 MB L2 of one XCD, what the hot rows of a phase may fill

struct DeviceArrays {
    int32_t *local_row_ptr = nullptr, *local_col = nullptr;
    int32_t *remote_row_ptr = nullptr, *remote_col = nullptr;
    float *dinv_own = nullptr;
    float *w_local = nullptr, *w_remote = nullptr;   // 1/sqrt(deg+1) of the neighbour, per entry of the column arrays
    int4 *short_desc = nullptr;        // per short row: row, start in local_col, start in remote_col, counts (local | remote << 16)
    WorkItem *items = nullptr;
    SplitRow *split_rows = nullptr;
    float *scratch = nullptr;          // [n_split_items x scratch_ld] partial sums
    int64_t scratch_ld = 0;
};

}  // namespace mgg

struct mgg_partition {
    int64_t num_nodes = 0, lb = 0, ub = 0, n_own = 0;
    int64_t n_local_rows = 0;         // rows of the local table: n_own for a graph partition, the local slice for bags
    bool bags = false;                // built by mgg_build_bags: owned rows are bags, no self term, plain sums
    int32_t num_parts = 1, part_id = 0;
    int32_t ps = 64, dist = 8, short_max = 16, xcd_min_deg = -1, wpb = 4;
    int32_t hot_rows = 0, hot_phases = 0, n_phases = 0, min_piece = 0, hot_min_count = 0;
    int32_t class_mode = 0;           // 0: no source classes, 1: by hash, 2: by popularity
    std::vector<uint8_t> src_class;   // class of every table row (local rows, then halo slots); empty: no classes
    int device = -1;  // HIP device the arrays live on; -1 = host only
    std::vector<int32_t> local_row_ptr, local_col, remote_row_ptr, remote_col;
    std::vector<int32_t> sched_local_col, sched_remote_col;   // device order of the columns (empty: same as above)
    std::vector<int32_t> halo_gid, deg_own, deg_halo;
    std::vector<int64_t> halo_peer_ptr;
    std::vector<float> dinv_own, dinv_halo;
    std::vector<int32_t> short_rows;
    std::vector<mgg::WorkItem> items;
    std::vector<mgg::SplitRow> split_rows;
    int64_t n_split_items = 0;
    // run-time switches of this partition's aggregations: the process-wide defaults at build time, then mgg_partition_set_option
    int32_t opt_lds_halo = 0, opt_col_slab_bytes = 0, opt_split_phases = 0, opt_items_per_wave = 0, opt_short_per_wave = 0;
    int32_t reserved_dim = 0;         // widest aggregation the partition's own scratch buffer was sized for
    int64_t n_groups_local = 0, n_groups_remote = 0;
    mgg::DeviceArrays d;          // device copies; d.scratch is sized by mgg_partition_reserve (or at build)
};

namespace mgg {

mgg_status_t fail(mgg_status_t code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
mgg_status_t hip_fail(hipError_t e, const char *what);

#define MGG_HIP_TRY(expr)                                    \
    do {                                                     \
        hipError_t _e = (expr);                              \
        if (_e != hipSuccess) return ::mgg::hip_fail(_e, #expr); \
    } while (0)

int32_t option_lds_halo();
int32_t option_col_slab_bytes();
int32_t option_split_phases();
int32_t option_update_stream();
int32_t option_items_per_wave();
void take_default_options(mgg_partition *p);      // copies the four process-wide defaults above into a new partition
mgg_status_t check_option(const char *key, int32_t value);   // range check shared by both setters

// kernels (aggregate.hip / update.hip)
mgg_status_t launch_aggregate(const mgg_partition *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                              const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x,
                              void *out, int64_t ld_out, hipStream_t stream, const float *bias = nullptr,
                              mgg_act_t act = MGG_ACT_NONE, int32_t out_dim = 0, mgg_dtype_t out_dtype = MGG_F32,
                              float *scratch = nullptr, size_t scratch_bytes = 0);
// bias / act: optional epilogue of the final value.  out_dim (0 = dim): columns of `out` that exist
// when the tables carry padding columns beyond them (dim counts the padded width).  out_dtype BF16: the
// rows are rounded to bf16 (nearest even) on the way out -- what the bf16 MFMA would do on the way in.
// scratch / scratch_bytes: where the partial sums of rows cut into several items go; NULL = the partition's
// own buffer (mgg_partition_reserve).  The launch allocates nothing: too small a buffer is an error.
inline int64_t scratch_ld_for(int32_t dim) { return (static_cast<int64_t>(dim) + 7) / 8 * 8; }   // rows of partial sums start on 32-byte boundaries
inline size_t scratch_bytes_for(const mgg_partition *p, int32_t dim) { return static_cast<size_t>(p->n_split_items) * static_cast<size_t>(scratch_ld_for(dim)) * sizeof(float); }
// the library's fixed scratch array on the current device (aggregate.hip); NULL + error set on failure
float *static_scratch(size_t *bytes);
mgg_status_t launch_update(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
                           mgg_dtype_t w_dtype, const void *w, const float *bias, int32_t d_out,
                           mgg_act_t act, mgg_dtype_t out_dtype, void *out, int64_t ld_out,
                           hipStream_t stream);

// Two chained Updates; one kernel when the shape is covered, otherwise two launches through `hidden`
// ([n_rows x dims[1]], bf16 with bf16 weights, else fp32).
mgg_status_t launch_update_mlp(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, const int32_t dims[3],
                               mgg_dtype_t w_dtype, const void *w1, const float *b1, mgg_act_t act1, const void *w2, const float *b2,
                               mgg_act_t act2, void *hidden, int64_t ld_hidden, mgg_dtype_t out_dtype, void *out, int64_t ld_out,
                               hipStream_t stream);
mgg_status_t probe_gather(int64_t table_bytes, int32_t row_bytes, int64_t n_gathers, int32_t iters, uint64_t seed, double *gbs);
// in place: x[i][:] = softmax(x[i][:]) for every row (update.hip)
mgg_status_t launch_row_softmax(int64_t n_rows, int32_t d, mgg_dtype_t dtype, void *x, int64_t ld, hipStream_t stream);

}  // namespace mgg
