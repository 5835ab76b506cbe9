/*
 * mgg.h -- C ABI of the MI355X (gfx950) hot path of MGG's full-graph GNN layer
 * (arXiv 2209.06800): neighbour aggregation over N(v) U {v} from a local and a halo
 * embedding table, followed by the dense Update.
 *
 * One GPU, one node range.  The halo table stands in for the embedding slices that
 * other GPUs own (section 4.2); the library issues no inter-GPU traffic.
 *
 * Conventions
 *   - Every call returns an mgg_status_t; nothing throws or aborts.  On error no output
 *     is written and mgg_last_error() holds a message (thread-local).
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HBM of the current
 *     HIP device.  The caller owns every buffer it passes in; the library owns only what
 *     an mgg_partition_t holds and frees it in mgg_partition_destroy().
 *   - Device calls enqueue work on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and do not synchronise.  Calls that use the same partition must be
 *     ordered on one stream: they share the partition's scratch buffer.
 *   - Matrices are row-major with an explicit leading dimension counted in elements.
 *   - MGG_BF16 data are raw bfloat16 bit patterns (uint16_t).
 */
#ifndef MGG_H
#define MGG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MGG_OK = 0,
    MGG_ERR_INVALID_ARG = 1,   /* NULL / out-of-range argument, misaligned or too-small buffer */
    MGG_ERR_BAD_GRAPH = 2,     /* row_ptr not monotone from 0, or a column outside [0, N)      */
    MGG_ERR_UNSUPPORTED = 3,   /* a share with >= 2^31 - 1 neighbours, or > 2^31 - 1 nodes     */
    MGG_ERR_ALLOC = 4,         /* host or device allocation failed                             */
    MGG_ERR_HIP = 5            /* a HIP runtime call failed (message carries hipGetErrorString) */
} mgg_status_t;

typedef enum { MGG_F32 = 0, MGG_BF16 = 1 } mgg_dtype_t;
/* Weighting of N(v) U {v}.
 * GCN_SYM: section 7, GCN equation, A-hat = adjacency with self-loops, taken as
 *          D~^-1/2 (A+I) D~^-1/2 with d~ = (whole-graph degree) + 1.
 * GIN_SUM: section 7, GIN equation: (1+eps) h_v + sum_{u in N(v)} h_u.            */
typedef enum { MGG_AGG_GCN_SYM = 0, MGG_AGG_GIN_SUM = 1 } mgg_agg_t;
/* SOFTMAX: over each output row, exp(z_j) / sum_k exp(z_k) -- the last step of the 2-layer GCN of
 * section 7, Z = softmax(A-hat ReLU(A-hat X W0) W1).  Runs as a second, in-place pass over out. */
typedef enum { MGG_ACT_NONE = 0, MGG_ACT_RELU = 1, MGG_ACT_SOFTMAX = 2 } mgg_act_t;

typedef struct mgg_partition mgg_partition_t;   /* opaque, library-owned */

/* Knobs of the partition build.  They are the paper's tuning parameters (section 6):
 * ps = neighbours per neighbour partition (1..64), dist = how many (local, remote)
 * partition pairs one wavefront work item covers (1..1024), wpb = wavefronts per workgroup
 * (the paper's warps per block).  0 selects the default: ps 64 (one neighbour id per lane of a
 * 64-lane wavefront), dist 8, short_max 16, xcd_min_deg 256.  Rows with at most short_max
 * neighbours in total are handled several per wavefront; short_max < 0 disables that bin. */
typedef struct {
    int32_t ps;
    int32_t dist;
    int32_t short_max;
    int32_t host_only;   /* nonzero: build on the host only, never touch the GPU (for
                            checks of the integer structures); device calls on such a
                            partition fail with MGG_ERR_INVALID_ARG */
    int32_t wpb;         /* wavefronts (= work items) per workgroup of the aggregation kernel,
                            1..16; 0 = default 2 */
    int32_t xcd_min_deg; /* rows with at least this many neighbours have their neighbour lists
                            regrouped by source class (see hot_rows), one piece of work per
                            class; 0 = library default, negative = no classes at all */
    /* Source classes, two kinds.  By hash (hot_phases < 0): a table row's class is a hash of its
     * index, 8 classes, one per XCD.  By popularity (hot_phases >= 1): the rows of the two
     * embedding tables are ranked by how many owned rows gather them; the 8 * hot_rows most
     * gathered form phase 0 and are dealt round-robin to the 8 XCDs, the next 8 * hot_rows
     * phase 1, ...; the rest is cold.  Each XCD runs the work of its phase-0 class first, then
     * phase 1, ..., then cold work, so its L2 holds hot_rows table rows at a time, each gathered
     * many times.  hot_phases = 0 chooses: by popularity with 4 phases when the rows of phase 0
     * would receive less than half of all gathers (gathers spread evenly: plain LRU keeps little
     * of a hash class), by hash otherwise. */
    int32_t hot_row_bytes; /* bytes of one table row (or of one column slab of it) this schedule is
                              laid out for; sets hot_rows = 3 MB / (row bytes in whole 128-byte
                              lines) when hot_rows is 0; 0 = 256 */
    int32_t hot_rows;      /* table rows per XCD and phase; 0 = from hot_row_bytes */
    int32_t hot_phases;    /* most phases (1..31); negative = classes by a hash of the table row index, no
                              cold class: -1 gives 8 classes, one per XCD; -2, -4, ... -16 give 16, 32, ...
                              128, XCD x working through classes x, x + 8, ... in turn; 0 = automatic */
    int32_t min_piece;     /* a class with fewer neighbours than this in a row joins the row's
                              cold piece; 0 = default 16 */
    int32_t hot_min_count; /* table rows gathered fewer times than this are cold; 0 = default 8 */
    int32_t reserve_dim;   /* > 0: the build ends with mgg_partition_reserve(p, reserve_dim) */
} mgg_build_opts_t;

typedef struct {
    int64_t num_nodes, lb, ub, n_own;
    int64_t nnz_local, nnz_remote, num_halo;
    int32_t num_parts, part_id;
    int32_t ps, dist, short_max, on_device;
    int32_t xcd_min_deg, wpb;
    int32_t class_mode;                       /* source classes: 0 none, 1 by hash, 2 by popularity */
    int32_t hot_rows, n_phases;               /* table rows per XCD and phase; phases in use    */
    int32_t min_piece, hot_min_count;
    int64_t n_groups_local, n_groups_remote;  /* neighbour partitions of the two CSRs        */
    int64_t n_short_rows;                     /* rows handled several per wavefront          */
    int64_t n_items;                          /* wavefront work items incl. padding items     */
    int64_t n_split_rows, n_split_items;      /* rows cut into > 1 item, and those items     */
    int64_t n_local_rows;                     /* rows of the local table: n_own, or the local slice of a bag partition */
    int32_t is_bags;                          /* built by mgg_build_bags                      */
    int32_t reserved_dim;                     /* widest mgg_partition_reserve so far (0: none) */
} mgg_partition_info_t;

/* Caller-allocated HOST buffers for mgg_partition_export(); a NULL member is skipped.
 * Sizes come from mgg_partition_info(). */
typedef struct {
    int32_t *local_row_ptr;   /* [n_own+1]                                                   */
    int32_t *local_col;       /* [nnz_local]   neighbour id - lb                             */
    int32_t *remote_row_ptr;  /* [n_own+1]                                                   */
    int32_t *remote_col;      /* [nnz_remote]  position of the neighbour in halo_gid         */
    int32_t *halo_gid;        /* [num_halo]    global ids, strictly increasing               */
    int64_t *halo_peer_ptr;   /* [num_parts+1] halo_gid[ptr[q]..ptr[q+1]) is owned by part q */
    int32_t *deg_own;         /* [n_own]       whole-graph degree (self-loops not counted)   */
    int32_t *deg_halo;        /* [num_halo]                                                  */
    int32_t *grp_local_row, *grp_local_start, *grp_local_end;      /* [n_groups_local]       */
    int32_t *grp_remote_row, *grp_remote_start, *grp_remote_end;   /* [n_groups_remote]      */
    int32_t *short_rows;      /* [n_short_rows] owned-row indices of the short bin           */
    int32_t *sched_local_col; /* [nnz_local]  local_col in the order the kernel walks it: the  */
    int32_t *sched_remote_col;/* [nnz_remote] same rows, regrouped rows sorted by source class  */
    int32_t *item_row;        /* [n_items] owned row of each work item; -1 = padding item      */
    int32_t *item_lbeg, *item_lend;   /* [n_items] range in sched_local_col                  */
    int32_t *item_rbeg, *item_rend;   /* [n_items] range in sched_remote_col                 */
    int32_t *item_slot;       /* [n_items] -1: the item is the whole row; else partial slot  */
    int32_t *src_class_local; /* [n_own]    class of each local table row: phase * 8 + XCD, -1 = cold */
    int32_t *src_class_halo;  /* [num_halo] same for the halo table                                   */
} mgg_partition_arrays_t;

/* ---------------------------------------------------------------------------------------
 * mgg_build_partition -- section 4.1 Step-2 (local and remote CSR of one GPU's rows),
 * Step-3 (neighbour partitions of ps neighbours), section 4.2 / Fig. 4 (node-id range
 * [lb, ub) per GPU, embedding ids rebased to zero), section 5.1 (pairs of local/remote
 * partitions per wavefront).
 *
 * Host, synchronous.  row_ptr[num_nodes+1] (int64, row_ptr[0]==0), col_idx[nnz] (int32) and
 * bounds[num_parts+1] are HOST pointers, read only, not retained.  Row v lists the nodes
 * summed into v.  bounds==NULL selects the equal-node split bounds[p]=floor(N*p/P).
 * A neighbour equal to its own row id is dropped (the self term is added by the
 * aggregation mode); duplicates are kept.  Degrees are whole-graph row lengths.
 * opts may be NULL (defaults).  Unless opts->host_only, the partition's arrays are copied
 * to the current HIP device before the call returns.  *out receives the handle.
 * Errors: INVALID_ARG, BAD_GRAPH, UNSUPPORTED, ALLOC, HIP.
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_build_partition(int64_t num_nodes, const int64_t *row_ptr, const int32_t *col_idx,
                                 int32_t num_parts, int32_t part_id, const int64_t *bounds,
                                 const mgg_build_opts_t *opts, mgg_partition_t **out);

mgg_status_t mgg_partition_info(const mgg_partition_t *p, mgg_partition_info_t *out);

/* ---------------------------------------------------------------------------------------
 * mgg_partition_reserve -- sizes the partition's scratch buffer for aggregations up to `dim`
 * columns wide.  Rows with many neighbours are cut into several wavefront work items (section
 * 4.1 Step-3: neighbour partitions; section 5.1: a wavefront takes a few of them), whose partial
 * sums pass through this buffer: mgg_aggregate_scratch_bytes(p, dim) bytes, nothing when no row
 * is cut.  Host, synchronous (it may wait for the device and allocate); never shrinks.  The
 * device calls below allocate nothing: mgg_aggregate / mgg_aggregate_to / mgg_bag_sum /
 * mgg_time_aggregate on a width that was not reserved fail with MGG_ERR_INVALID_ARG.
 * mgg_layer_forward does not use this buffer (its workspace holds the partial sums).
 * Errors: INVALID_ARG, ALLOC, HIP.
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_partition_reserve(mgg_partition_t *p, int32_t dim);
size_t       mgg_aggregate_scratch_bytes(const mgg_partition_t *p, int32_t dim);   /* 0 on bad arguments */
mgg_status_t mgg_partition_export(const mgg_partition_t *p, mgg_partition_arrays_t *host_buffers);
void         mgg_partition_destroy(mgg_partition_t *p);   /* NULL is allowed */

/* ---------------------------------------------------------------------------------------
 * mgg_aggregate -- section 1 "GNN" equation (Aggregate over N(v) U {v}); section 4.1
 * (LR / LL / AC stages: remote rows, local rows, accumulation) run in ONE kernel launch
 * plus a small fix-up launch for rows cut into several work items.
 *
 *   GCN_SYM: out[v] = sum_u x_u / sqrt(d~_u d~_v) + x_v / d~_v
 *   GIN_SUM: out[v] = (1+eps) x_v + sum_u x_u              (eps is ignored for GCN_SYM)
 *
 * x_local [n_own x dim] holds the rows this GPU owns, x_halo [num_halo x dim] the rows of
 * the halo list in halo_gid order (may be NULL iff num_halo == 0); both DEVICE, same dtype
 * and leading dimension ld_x >= dim.  Both tables must be allocated as rows x ld_x elements:
 * when ld_x leaves room, rows are read up to the next multiple of 16 bytes (whatever the
 * padding holds is never used), so that a width like 602 or 47 still gets 16-byte loads.
 * out [n_own x dim] is DEVICE fp32, ld_out >= dim, fully overwritten (columns >= dim of a
 * padded out are not touched); it must not alias the inputs.  Accumulation is fp32.
 * Allocates nothing and never synchronises: the width must have been reserved
 * (mgg_partition_reserve, or reserve_dim at build) when the partition cuts rows into several items.
 * Errors: INVALID_ARG (NULL, dim < 1, ld < dim, host-only partition, width not reserved), HIP.
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_aggregate(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                           const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x,
                           float *out, int64_t ld_out, void *stream);

/* mgg_aggregate for callers that cannot allocate and hold no reserved partition: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and result as
 * mgg_aggregate; the partial sums of cut rows go to a fixed 64 MiB array inside the library's device
 * code (one copy per GPU, held until the process ends) instead of the partition's buffer, so the call
 * allocates nothing whatever was or was not reserved.  A partition whose partial sums at this width
 * (mgg_aggregate_scratch_bytes) exceed 64 MiB is refused with MGG_ERR_UNSUPPORTED.  The first call on
 * a device looks up the array's address (not capturable); every call on a GPU shares that GPU's array,
 * so calls that may overlap on one GPU -- two streams, two threads, two partitions -- race: order them
 * on one stream.  The array keeps the last call's contents; nothing needs clearing (every slot read
 * is written first by the same launch). */
mgg_status_t mgg_aggregate_static(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                                  const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x,
                                  float *out, int64_t ld_out, void *stream);

/* mgg_aggregate with a choice of output type: out_dtype MGG_F32 is mgg_aggregate; MGG_BF16 rounds
 * the fp32 sums to bf16 (nearest even) as they are written, out then being [n_own x dim] bf16.  A
 * bf16 MFMA rounds its input the same way, so feeding it the bf16 rows gives the bits it would
 * have computed from the fp32 rows, for half the bytes written and read back. */
mgg_status_t mgg_aggregate_to(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                              const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x,
                              mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream);

/* ---------------------------------------------------------------------------------------
 * mgg_build_bags / mgg_bag_sum -- section 8.3 ("Generality to other applications"): the embedding
 * lookup of a recommendation model, rows of a large table fetched and added element-wise, with
 * the table cut by rows over the GPUs.  The same path as the aggregation: a bag is an owned row
 * without an embedding of its own, its lookups into this GPU's slice [local_lo, local_hi) of the
 * table are the local neighbours, the others the remote ones, served from a halo table of the
 * distinct remote rows in ascending row order (what an exchange with the owners would fill).
 *
 * mgg_build_bags: host, synchronous.  bag_ptr[num_bags+1] (int64, bag_ptr[0]==0) and
 * bag_idx[bag_ptr[num_bags]] (int32 rows of the whole table, duplicates kept) are HOST pointers,
 * not retained.  The handle works with mgg_partition_info / export / destroy (n_own = num_bags,
 * lb / ub = the local slice, halo_gid = the remote rows) and with mgg_bag_sum only.  opts as for
 * mgg_build_partition, except that short_max defaults to 32 (bags of a few tens of lookups are taken
 * several per wavefront).
 *
 * mgg_bag_sum: out[b] = sum over the lookups of bag b of the table row, fp32 accumulation; empty
 * bags give zero rows.  table_local [(local_hi-local_lo) x dim] and table_halo [num_halo x dim]
 * DEVICE, same dtype and ld_x (either may be NULL when no lookup goes there); out [num_bags x dim]
 * DEVICE, F32 or BF16.  Asynchronous on `stream`.  Errors as mgg_aggregate.
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_build_bags(int64_t num_bags, const int64_t *bag_ptr, const int32_t *bag_idx, int64_t table_rows,
                            int64_t local_lo, int64_t local_hi, const mgg_build_opts_t *opts, mgg_partition_t **out);
mgg_status_t mgg_bag_sum(const mgg_partition_t *p, mgg_dtype_t x_dtype, const void *table_local, const void *table_halo,
                         int32_t dim, int64_t ld_x, mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream);

/* ---------------------------------------------------------------------------------------
 * mgg_update -- section 1 (Update = a fully-connected layer), section 7 (X W, ReLU, MLP):
 *     out = act(a . w + bias)        on MFMA, fp32 accumulation.
 * a [n_rows x d_in] DEVICE, a_dtype F32 or BF16.  w [d_in x d_out] DEVICE row-major,
 * w_dtype F32 or BF16.  F32 weights need F32 input and use the fp32 MFMA; BF16 weights use
 * the bf16 MFMA and an F32 input is rounded to bf16 (nearest even) on the way in.
 * bias [d_out] DEVICE fp32 or NULL.  out [n_rows x d_out] DEVICE, out_dtype F32 or BF16
 * (rounded nearest even).  out must not alias a.
 * Errors: INVALID_ARG, UNSUPPORTED (dtype combination; softmax over more than 512 columns), HIP.
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_update(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
                        mgg_dtype_t w_dtype, const void *w, const float *bias, int32_t d_out,
                        mgg_act_t act, mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream);

/* ---------------------------------------------------------------------------------------
 * mgg_update_mlp -- section 7, GIN: the Update is an MLP; two chained mgg_update calls,
 *     out = act2(act1(a . w1 + bias1) . w2 + bias2),      dims = {d_in, d_hidden, d_out}.
 * With bf16 weights, d_in 64 or 128, 33..128 hidden and output columns and
 * elementwise activations both products run in ONE kernel and the hidden activations stay
 * in registers (rounded to bf16, as the two-call form keeps them).  Any other shape runs as
 * two launches through `hidden`, a DEVICE buffer [n_rows x d_hidden] (bf16 with bf16
 * weights, fp32 otherwise), which may be NULL only when the one-kernel form applies
 * (else MGG_ERR_INVALID_ARG).  Other arguments and errors as in mgg_update.
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_update_mlp(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, const int32_t *dims,
                            mgg_dtype_t w_dtype, const void *w1, const float *bias1, mgg_act_t act1,
                            const void *w2, const float *bias2, mgg_act_t act2,
                            void *hidden, int64_t ld_hidden, mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream);

/* Order of the aggregation and of the first linear of the Update.  Aggregation is linear, so
 * Aggregate(X) W = Aggregate(X W) (section 7: A-hat X W is one product); when W narrows the rows
 * the second form gathers d_out-wide rows instead of d_in-wide ones.  Values agree within
 * rounding.  AUTO takes UPDATE_FIRST when the transformed rows are at most 3/4 the bytes of the
 * input rows and the combination is supported, AGG_FIRST otherwise. */
typedef enum { MGG_ORDER_AGG_FIRST = 0, MGG_ORDER_UPDATE_FIRST = 1, MGG_ORDER_AUTO = 2 } mgg_order_t;

/* One GNN layer: Aggregate, then n_linear (1 or 2) Updates (GCN: one; GIN's MLP: two). */
typedef struct {
    mgg_agg_t   mode;
    float       eps;
    int32_t     n_linear;      /* 1 or 2 */
    int32_t     dims[3];       /* d_in, then the output width of each linear */
    mgg_dtype_t w_dtype;       /* dtype of every weight matrix */
    const void *w[2];          /* DEVICE, [dims[i] x dims[i+1]] row-major */
    const float *bias[2];      /* DEVICE fp32 or NULL */
    mgg_act_t   act[2];
    mgg_order_t order;         /* 0 = AGG_FIRST, the paper's formulation */
} mgg_layer_desc_t;

/* Bytes of DEVICE workspace mgg_layer_forward needs (aggregation result, the partial sums of rows
 * cut into several work items and, for two linears, the hidden activations; with UPDATE_FIRST the
 * transformed local and halo tables).
 * Returns 0 on bad arguments. */
size_t mgg_layer_workspace_bytes(const mgg_partition_t *p, const mgg_layer_desc_t *layer);

/* ---------------------------------------------------------------------------------------
 * mgg_layer_forward -- section 1 "GNN" equation: h' = Update(Aggregate(...)), all on
 * `stream`, no host synchronisation between the kernels.
 * x_local / x_halo / ld_x as in mgg_aggregate with dim = layer->dims[0].  workspace is a
 * DEVICE buffer of at least mgg_layer_workspace_bytes() bytes, 256-byte aligned.
 * out [n_own x dims[n_linear]] DEVICE, out_dtype F32 or BF16.  With BF16 weights the hidden
 * activations of a 2-linear MLP are kept in bf16.
 * UPDATE_FIRST: T = X w[0] is computed for the local AND the halo table (fp32, no bias, no
 * activation), T is aggregated at width dims[1], and bias[0] / act[0] are applied to the
 * aggregated rows.  Transforming the halo rows here stands in for the GPUs that own them:
 * in a multi-GPU run each GPU transforms its own rows once and the exchange ships the
 * narrower rows.  Needs out_dtype F32 when n_linear is 1 (else MGG_ERR_UNSUPPORTED).
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_layer_forward(const mgg_partition_t *p, const mgg_layer_desc_t *layer,
                               mgg_dtype_t x_dtype, const void *x_local, const void *x_halo, int64_t ld_x,
                               void *workspace, size_t workspace_bytes,
                               mgg_dtype_t out_dtype, void *out, int64_t ld_out, void *stream);

/* ---------------------------------------------------------------------------------------
 * mgg_split_edge_balanced -- section 4.1 Step-1 / Algorithm 1: contiguous node ranges with
 * about ceil(E / num_parts) edges each.  Host only.  bounds_out has num_parts+1 entries,
 * bounds_out[0] = 0, bounds_out[num_parts] = num_nodes; interior point s is the first node
 * index n >= the previous point with row_ptr[n] >= min(row_ptr[previous] + ceil(E/P), E).
 * ------------------------------------------------------------------------------------- */
mgg_status_t mgg_split_edge_balanced(int64_t num_nodes, const int64_t *row_ptr, int32_t num_parts,
                                     int64_t *bounds_out);

/* ---------------------------------------------------------------------------------------
 * Analytical model and run-time parameter search -- section 6 ("Performance-Resource Analytical
 * Modeling", "Heuristic-based Cross Iteration Optimization").  Host only.
 *
 * mgg_model_evaluate: equations (1)-(3).  wpw = 2 ps D dist (workload per wavefront);
 * smem_bytes = ps wpb 4 + 2 wpb D 4 (the block-level layout of section 5.2: ids, partial
 * results, fetched rows); num_waves = ceil(max(local, remote partitions) / dist);
 * num_blocks = ceil(num_waves / wpb); blocks_per_unit = num_blocks / num_units (256 CUs on an
 * MI355X); feasible = smem_bytes <= smem_limit_bytes (160 KB of LDS per CU).
 *
 * mgg_tuner_*: the greedy search.  All knobs start at 1; ps is doubled while the latency falls,
 * then dist, then wpb; then ps is lowered step by step ("retreat") with the wpb search started
 * again from 1, until a trial is slower than the third-lowest latency seen; every trial is kept
 * in a lookup table and the lowest latency wins.  Usage: call mgg_tuner_next (it proposes a
 * configuration, or sets *done), measure it, call mgg_tuner_report with the latency (any unit),
 * repeat.  mgg_tuner_table copies up to `capacity` trials in the order they were made.
 * mgg_tuner_set_constraint (before the first trial; dim 0 = none) bounds the search space by the
 * model's constraint on shared memory: a configuration with smem_bytes(ps, wpb, dim) above the
 * limit is never proposed and counts as slower than anything measured (an upward step onto it does
 * not pay, a retreat trial on it ends the search).  mgg_tune_aggregate sets it to its `dim` and the
 * 160 KB of LDS per CU unless the caller has set one.
 *
 * mgg_tune_aggregate drives a tuner on the GPU: for every proposal it builds the partition with
 * base_opts (NULL = defaults) plus the proposed ps / dist / wpb, times `iters` aggregations on
 * `stream` with HIP events (synchronises), and reports the mean milliseconds.  Pointers as in
 * mgg_build_partition and mgg_aggregate; `out` is overwritten by every trial.
 * ------------------------------------------------------------------------------------- */
typedef struct { int32_t ps, dist, wpb; } mgg_knobs_t;
typedef struct {
    int64_t wpw, smem_bytes, num_waves, num_blocks;
    double  blocks_per_unit;
    int32_t feasible;
} mgg_model_t;
typedef struct mgg_tuner mgg_tuner_t;

mgg_status_t mgg_model_evaluate(int64_t n_local_partitions, int64_t n_remote_partitions, mgg_knobs_t knobs,
                                int32_t dim, int32_t num_units, int64_t smem_limit_bytes, mgg_model_t *out);
mgg_status_t mgg_tuner_create(int32_t ps_max, int32_t dist_max, int32_t wpb_max, mgg_tuner_t **out);
mgg_status_t mgg_tuner_set_constraint(mgg_tuner_t *t, int32_t dim, int64_t smem_limit_bytes);
mgg_status_t mgg_tuner_next(mgg_tuner_t *t, mgg_knobs_t *next, int32_t *done);
mgg_status_t mgg_tuner_report(mgg_tuner_t *t, double latency);
mgg_status_t mgg_tuner_result(const mgg_tuner_t *t, mgg_knobs_t *best, double *best_latency, int32_t *n_trials);
mgg_status_t mgg_tuner_table(const mgg_tuner_t *t, int32_t capacity, mgg_knobs_t *knobs, double *latency,
                             int32_t *n_trials);
void         mgg_tuner_destroy(mgg_tuner_t *t);   /* NULL is allowed */
mgg_status_t mgg_tune_aggregate(int64_t num_nodes, const int64_t *row_ptr, const int32_t *col_idx,
                                int32_t num_parts, int32_t part_id, const int64_t *bounds,
                                const mgg_build_opts_t *base_opts, mgg_agg_t mode, float eps,
                                mgg_dtype_t x_dtype, const void *x_local, const void *x_halo, int32_t dim,
                                int64_t ld_x, float *out, int64_t ld_out, void *stream, int32_t iters,
                                mgg_tuner_t *tuner, mgg_knobs_t *best, double *best_ms);

/* Run-time switches for experiments (ablations of section 7.2's kind).  The switches of the aggregation
 * belong to a partition: mgg_partition_set_option changes them for that partition only (not while a call
 * using it is running on another thread).  mgg_set_option sets the process-wide default that partitions
 * built afterwards start from -- existing partitions keep what they have -- and the one switch of the
 * Update kernels, which have no handle to carry it.  Keys:
 *   "lds_halo"    0/1  stage halo rows through LDS ahead of accumulation  (default 0)
 *   "split_phases" 0/1 aggregate the local lists and the remote lists in two launches, the
 *                      second adding to the first (no interleaving; default 0)
 *   "col_slab_bytes"   0 = automatic (default), 1 = off, or a power of two in [64, 4096]:
 *                      bytes of an embedding row handled per pass over the work items
 *   "items_per_wave"   0 = automatic (default), or 1..64: work items a wavefront takes one after
 *                      the other, the next one's ids and descriptor requested while it gathers
 *   "short_per_wave"   the same for the groups of short rows a wavefront takes
 *   "update_stream" 0/1 (process-wide only) the Update kernels added for streaming efficiency (whole-line
 *                      kernels, the one-kernel MLP, two W slabs in LDS) are used where they apply
 *                      (default 1; 0 = the plain register-resident and slab kernels everywhere)
 * Unknown key or bad value -> MGG_ERR_INVALID_ARG. */
mgg_status_t mgg_set_option(const char *key, int32_t value);
mgg_status_t mgg_get_option(const char *key, int32_t *value);
mgg_status_t mgg_partition_set_option(mgg_partition_t *p, const char *key, int32_t value);
mgg_status_t mgg_partition_get_option(const mgg_partition_t *p, const char *key, int32_t *value);

/* Time of the most recent kernel launches of this thread is not kept by the library; for
 * measurement the caller brackets calls with events on its stream.  This helper does that
 * with HIP events on `stream` around `iters` back-to-back calls of mgg_aggregate and returns
 * the mean milliseconds per call (synchronises). */
mgg_status_t mgg_time_aggregate(const mgg_partition_t *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                                const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x,
                                float *out, int64_t ld_out, void *stream, int32_t iters, float *ms_per_call);

/* Measurement aid for the roofline of the aggregation (section 3.1 of the paper frames the aggregation as
 * bound by irregular, fine-grained remote and local loads): gathers n_gathers rows of row_bytes (128, 256,
 * 512 or 1024) by seeded random ids from a zero-filled table of table_bytes that the call allocates on the
 * current device, with the aggregation kernel's load shape (16 bytes per lane, eight loads in flight) and no
 * other work, `iters` launches timed with HIP events on the default stream; returns gathered GB/s.  Host call,
 * synchronous, allocates and frees.  The table size decides where the rows come from: a few MB stay in one
 * XCD's L2, up to 256 MB in the Infinity Cache, beyond that in HBM.  Errors: INVALID_ARG, ALLOC, HIP. */
mgg_status_t mgg_probe_gather(int64_t table_bytes, int32_t row_bytes, int64_t n_gathers, int32_t iters, uint64_t seed,
                              double *gbytes_per_s);

const char *mgg_last_error(void);      /* thread-local, never NULL */
const char *mgg_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MGG_H */
