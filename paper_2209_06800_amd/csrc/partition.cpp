// Host side of libmgg: partition build (section 4.1 Steps 1-3, section 4.2), export of the
// integer structures, upload to HBM.  All integer work; the only floating-point values made
// here are the per-node factors 1/sqrt(deg+1) of the GCN normalisation.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "mgg_internal.h"

namespace mgg {

static thread_local char g_err[512] = "";

mgg_status_t fail(mgg_status_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

mgg_status_t hip_fail(hipError_t e, const char *what)
{
    return fail(MGG_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

const char *last_error() { return g_err; }

template <typename T>
static mgg_status_t upload(const std::vector<T> &h, T **d)
{
    *d = nullptr;
    // one element at least, so that kernels never receive a null table pointer
    size_t bytes = std::max<size_t>(h.size(), 1) * sizeof(T);
    hipError_t e = hipMalloc(reinterpret_cast<void **>(d), bytes);
    if (e != hipSuccess) return fail(MGG_ERR_ALLOC, "hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(e));
    if (!h.empty()) MGG_HIP_TRY(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return MGG_OK;
}

static void free_device(mgg_partition *p)
{
    if (p->device < 0) return;
    DeviceArrays &d = p->d;
    void *ptrs[] = {d.local_row_ptr, d.local_col, d.remote_row_ptr, d.remote_col, d.dinv_own, d.w_local,
                    d.w_remote,      d.short_desc, d.items,         d.split_rows, d.scratch};
    for (void *q : ptrs)
        if (q) (void)hipFree(q);
    d = DeviceArrays{};
}

static mgg_status_t upload_all(mgg_partition *p)
{
    int dev = 0;
    MGG_HIP_TRY(hipGetDevice(&dev));
    p->device = dev;
    mgg_status_t s;
    if ((s = upload(p->local_row_ptr, &p->d.local_row_ptr)) != MGG_OK) return s;
    if ((s = upload(p->sched_local_col.empty() ? p->local_col : p->sched_local_col, &p->d.local_col)) != MGG_OK) return s;
    if ((s = upload(p->remote_row_ptr, &p->d.remote_row_ptr)) != MGG_OK) return s;
    if ((s = upload(p->sched_remote_col.empty() ? p->remote_col : p->sched_remote_col, &p->d.remote_col)) != MGG_OK) return s;
    if ((s = upload(p->dinv_own, &p->d.dinv_own)) != MGG_OK) return s;
    {
        // the neighbour's factor, stored per edge in the order the kernel walks the columns: a
        // coalesced stream instead of a 4-byte gather per neighbour
        const std::vector<int32_t> &lc = p->sched_local_col.empty() ? p->local_col : p->sched_local_col;
        const std::vector<int32_t> &rc = p->sched_remote_col.empty() ? p->remote_col : p->sched_remote_col;
        std::vector<float> w(p->bags ? 0 : lc.size());      // a bag partition has no factors: plain sums only
        for (size_t i = 0; i < w.size(); ++i) w[i] = p->dinv_own[lc[i]];
        if ((s = upload(w, &p->d.w_local)) != MGG_OK) return s;
        w.resize(p->bags ? 0 : rc.size());
        for (size_t i = 0; i < w.size(); ++i) w[i] = p->dinv_halo[rc[i]];
        if ((s = upload(w, &p->d.w_remote)) != MGG_OK) return s;
    }
    {
        // one 16-byte record per short row, so that the kernel needs no dependent look-up of row pointers
        std::vector<int4> sd(p->short_rows.size());
        for (size_t i = 0; i < sd.size(); ++i) {
            const int32_t v = p->short_rows[i];
            const int32_t nl = p->local_row_ptr[v + 1] - p->local_row_ptr[v], nr = p->remote_row_ptr[v + 1] - p->remote_row_ptr[v];
            sd[i] = make_int4(v, p->local_row_ptr[v], p->remote_row_ptr[v], nl | (nr << 16));
        }
        if ((s = upload(sd, &p->d.short_desc)) != MGG_OK) return s;
    }
    if ((s = upload(p->items, &p->d.items)) != MGG_OK) return s;
    if ((s = upload(p->split_rows, &p->d.split_rows)) != MGG_OK) return s;
    return MGG_OK;
}

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Class of an embedding-table row (a multiplicative hash, so that classes are balanced even when
// hubs crowd the low ids).
static inline int source_class(int32_t row, int bits = 3) { return static_cast<int>((static_cast<uint32_t>(row) * 0x9E3779B1u) >> (32 - bits)); }

static void export_groups(const std::vector<int32_t> &rp, int32_t ps, int32_t *row, int32_t *start, int32_t *end)
{
    int64_t g = 0;
    for (size_t r = 0; r + 1 < rp.size(); ++r)
        for (int32_t s = rp[r]; s < rp[r + 1]; s += ps, ++g) {
            if (row) row[g] = static_cast<int32_t>(r);
            if (start) start[g] = s;
            if (end) end[g] = std::min<int32_t>(s + ps, rp[r + 1]);
        }
}

template <typename T>
static void copy_out(const std::vector<T> &v, T *dst)
{
    if (dst && !v.empty()) std::memcpy(dst, v.data(), v.size() * sizeof(T));
}


// The knobs of a build with the defaults filled in.
struct Knobs {
    int32_t ps = 64, dist = 8, short_max = 16, host_only = 0, xcd_min_deg = kDefaultXcdMinDeg, wpb = kDefaultWpb;
    int32_t hot_rows = 0, hot_phases = kDefaultHotPhases, min_piece = kDefaultMinPiece, hot_min_count = kDefaultHotMinCount;
    int32_t reserve_dim = 0;
};

static mgg_status_t parse_opts(const mgg_build_opts_t *opts, Knobs *k)
{
    int32_t &ps = k->ps, &dist = k->dist, &short_max = k->short_max, &host_only = k->host_only, &xcd_min_deg = k->xcd_min_deg, &wpb = k->wpb;
    int32_t hot_row_bytes = 256;
    int32_t &hot_rows = k->hot_rows, &hot_phases = k->hot_phases, &min_piece = k->min_piece, &hot_min_count = k->hot_min_count;
    if (opts) {
        if (opts->hot_row_bytes) hot_row_bytes = opts->hot_row_bytes;
        if (opts->hot_rows) hot_rows = opts->hot_rows;
        hot_phases = opts->hot_phases;
        if (opts->min_piece) min_piece = opts->min_piece;
        if (opts->hot_min_count) hot_min_count = opts->hot_min_count;
        if (opts->ps) ps = opts->ps;
        if (opts->dist) dist = opts->dist;
        if (opts->short_max) short_max = opts->short_max;
        host_only = opts->host_only;
        if (opts->xcd_min_deg) xcd_min_deg = opts->xcd_min_deg;
        if (opts->wpb) wpb = opts->wpb;
        k->reserve_dim = opts->reserve_dim;
    }
    if (ps < 1 || ps > 64) return fail(MGG_ERR_INVALID_ARG, "ps %d outside [1, 64]", ps);
    if (dist < 1 || dist > 1024) return fail(MGG_ERR_INVALID_ARG, "dist %d outside [1, 1024]", dist);
    if (short_max > 4096) return fail(MGG_ERR_INVALID_ARG, "short_max %d above 4096", short_max);
    if (wpb < 1 || wpb > 16) return fail(MGG_ERR_INVALID_ARG, "wpb %d outside [1, 16]", wpb);
    if (hot_row_bytes < 1 || hot_row_bytes > (1 << 20)) return fail(MGG_ERR_INVALID_ARG, "hot_row_bytes %d outside [1, 2^20]", hot_row_bytes);
    if (hot_rows == 0) {
        // as many table rows as fit kHotBytesPerXcd of one XCD's L2, rows counted in whole 128-byte lines
        const int64_t line_bytes = (static_cast<int64_t>(hot_row_bytes) + 127) / 128 * 128;
        hot_rows = static_cast<int32_t>(std::max<int64_t>(1, kHotBytesPerXcd / line_bytes));
    }
    if (hot_rows < 1 || hot_rows > (1 << 24)) return fail(MGG_ERR_INVALID_ARG, "hot_rows %d outside [1, 2^24]", hot_rows);
    if (hot_phases > kMaxHotPhases) return fail(MGG_ERR_INVALID_ARG, "hot_phases %d above %d", hot_phases, kMaxHotPhases);
    if (min_piece < 1) return fail(MGG_ERR_INVALID_ARG, "min_piece %d below 1", min_piece);
    if (hot_min_count < 1) return fail(MGG_ERR_INVALID_ARG, "hot_min_count %d below 1", hot_min_count);
    if (k->reserve_dim < 0) return fail(MGG_ERR_INVALID_ARG, "reserve_dim %d below 0", k->reserve_dim);
    return MGG_OK;
}

// Source classes, work items and the short-row bin of a partition whose two CSRs are in place
// (may throw std::bad_alloc).
static void build_schedule(mgg_partition *p, const Knobs &k)
{
    const int64_t n_own = p->n_own, num_halo = static_cast<int64_t>(p->halo_gid.size());
    const int64_t n_loc = p->n_local_rows;                  // rows of the local table (= n_own for a graph partition)
    const int32_t ps = k.ps, dist = k.dist, short_max = k.short_max, xcd_min_deg = k.xcd_min_deg, wpb = k.wpb;
    const int32_t hot_rows = k.hot_rows, min_piece = k.min_piece, hot_min_count = k.hot_min_count;
    int32_t hot_phases = k.hot_phases;
    p->ps = ps; p->dist = dist; p->short_max = short_max; p->xcd_min_deg = xcd_min_deg; p->wpb = wpb;
    p->hot_rows = hot_rows; p->hot_phases = hot_phases; p->min_piece = min_piece; p->hot_min_count = hot_min_count;

    // ---- source classes -------------------------------------------------------------
    // Every row of the two embedding tables gets a class.  hot_phases < 0: a hash of its index, 8
    // classes, one per XCD, no cold class.  With hot_phases >= 1 (0 chooses between the two) the class is
    // either (phase, XCD) -- "hot" -- or cold, and hot classes are filled in order of popularity (how many owned rows gather the
    // table row): the 8*hot_rows most gathered rows form phase 0, dealt round-robin to the
    // 8 XCDs, the next 8*hot_rows phase 1, and so on.  An XCD works through its phases in
    // order, so at any time its L2 only has to hold hot_rows table rows, all of which are
    // gathered many times.
    const bool use_classes = xcd_min_deg > 0;
    const int64_t n_tab = n_loc + num_halo;                  // local rows first, then halo slots
    int n_phase = 0;
    if (use_classes) {
        p->src_class.assign(static_cast<size_t>(n_tab), kColdClass);
        std::vector<int32_t> order;                          // table rows, most gathered first
        std::vector<int32_t> cnt;
        const int64_t per_phase = static_cast<int64_t>(kXcd) * hot_rows;
        if (hot_phases >= 0 && n_tab > 0) {
            cnt.assign(static_cast<size_t>(n_tab), 0);
            for (int32_t u : p->local_col) ++cnt[u];
            for (int32_t u : p->remote_col) ++cnt[n_loc + u];
            // counting sort by gather count (ties: lower index first)
            const int32_t max_cnt = *std::max_element(cnt.begin(), cnt.end());
            std::vector<int64_t> start(static_cast<size_t>(max_cnt) + 2, 0);
            for (int64_t i = 0; i < n_tab; ++i) ++start[max_cnt - cnt[i] + 1];
            for (size_t c = 1; c < start.size(); ++c) start[c] += start[c - 1];
            order.resize(static_cast<size_t>(n_tab));
            for (int64_t i = 0; i < n_tab; ++i) order[start[max_cnt - cnt[i]]++] = static_cast<int32_t>(i);
        }
        if (hot_phases == 0) {
            // Automatic.  The hash classes win while L2 can hold what matters of a class under plain LRU;
            // when gathers are spread so evenly that the most gathered rows of one phase get less than
            // half of them (measured: the 2.4 M-node R-MAT of the configs, 41 %, 4-8 % faster with
            // phases; the others, 69-86 %, 5-10 % slower), explicit hot phases do better.
            int64_t top = 0, all = static_cast<int64_t>(p->local_col.size()) + static_cast<int64_t>(p->remote_col.size());
            for (int64_t r = 0; r < std::min<int64_t>(n_tab, per_phase); ++r) top += cnt[order[r]];
            hot_phases = (all > 0 && 2 * top < all) ? kAutoHotPhases : -1;
        }
        p->class_mode = hot_phases < 0 ? 1 : 2;
        if (hot_phases < 0) {
            // -1: 8 hash classes, one per XCD; -2, -4, ...: 16, 32, ... hash classes, XCD x working through
            // classes x, x + 8, ... one after the other (each holds a smaller share of the table rows)
            int bits = 3;
            n_phase = 1;
            while (n_phase * 2 <= -hot_phases && n_phase * 2 <= 16) { n_phase *= 2; ++bits; }
            for (int64_t i = 0; i < n_loc; ++i) p->src_class[i] = static_cast<uint8_t>(source_class(static_cast<int32_t>(i), bits));
            for (int64_t i = 0; i < num_halo; ++i) p->src_class[n_loc + i] = static_cast<uint8_t>(source_class(static_cast<int32_t>(i), bits));
        } else if (n_tab > 0) {
            const int64_t limit = std::min<int64_t>(n_tab, per_phase * hot_phases);
            int64_t r = 0;
            for (; r < limit && cnt[order[r]] >= hot_min_count; ++r)
                p->src_class[order[r]] = static_cast<uint8_t>((r / per_phase) * kXcd + r % kXcd);
            n_phase = static_cast<int>(ceil_div(r, per_phase));
        }
    }
    p->n_phases = n_phase;
    const int n_hot = n_phase * kXcd;                        // hot classes; class index n_hot = cold

    // ---- work decomposition ----------------------------------------------------------
    // short rows: several per wavefront; whole rows: one item; long rows: cut at
    // multiples of dist neighbour partitions, item k pairing local run k with remote run k.
    // Rows with at least xcd_min_deg neighbours are first regrouped by source class: each
    // class with at least min_piece neighbours becomes a piece with its own items (the rest
    // joins the row's cold piece), and the launch order below hands the items of class
    // (phase, x) to XCD x, phase by phase.
    const int64_t run = static_cast<int64_t>(ps) * dist;   // neighbours per run
    if (use_classes) { p->sched_local_col = p->local_col; p->sched_remote_col = p->remote_col; }
    std::vector<std::vector<WorkItem>> bucket(static_cast<size_t>(std::max(n_hot, 1)));   // hot items by class
    std::vector<WorkItem> cold;                              // cold pieces and whole rows
    std::vector<std::vector<int32_t>> by_len(short_max >= 0 ? short_max + 1 : 0);
    auto item_work = [](const WorkItem &it) { return static_cast<int64_t>(it.lend - it.lbeg) + (it.rend - it.rbeg) + 8; };
    std::vector<int32_t> n_in(static_cast<size_t>(n_hot) + 1), lcut(static_cast<size_t>(n_hot) + 2), rcut(static_cast<size_t>(n_hot) + 2), pos(static_cast<size_t>(n_hot) + 1), tmp;
    std::vector<uint8_t> final_class(static_cast<size_t>(n_hot) + 1);
    // stable counting sort of col[b, e) by final class of the table row `base + col`; cut[c] = start of class c
    auto regroup = [&](std::vector<int32_t> &col, int32_t b, int32_t e, int64_t base, std::vector<int32_t> &cut) {
        std::fill(pos.begin(), pos.end(), 0);
        for (int32_t i = b; i < e; ++i) ++pos[final_class[std::min<int>(p->src_class[base + col[i]], n_hot)]];
        cut[0] = b;
        for (int c = 0; c <= n_hot; ++c) cut[c + 1] = cut[c] + pos[c];
        tmp.assign(col.begin() + b, col.begin() + e);
        for (int c = 0; c <= n_hot; ++c) pos[c] = cut[c];
        for (int32_t u : tmp) col[pos[final_class[std::min<int>(p->src_class[base + u], n_hot)]]++] = u;
    };
    std::vector<std::pair<WorkItem, int>> row_items;         // item, class (n_hot = cold)
    for (int64_t v = 0; v < n_own; ++v) {
        const int32_t l0 = p->local_row_ptr[v], l1 = p->local_row_ptr[v + 1];
        const int32_t r0 = p->remote_row_ptr[v], r1 = p->remote_row_ptr[v + 1];
        const int64_t dl = l1 - l0, dr = r1 - r0;
        p->n_groups_local += ceil_div(dl, ps);
        p->n_groups_remote += ceil_div(dr, ps);
        if (short_max >= 0 && dl + dr <= short_max) { by_len[dl + dr].push_back(static_cast<int32_t>(v)); continue; }
        // the pieces of this row: one per surviving class if it is regrouped, otherwise the whole row
        int first_piece = n_hot, n_piece_end = n_hot + 1;     // default: only the cold piece = the whole row
        if (use_classes && n_hot > 0 && dl + dr >= xcd_min_deg) {
            std::fill(n_in.begin(), n_in.end(), 0);
            for (int32_t i = l0; i < l1; ++i) ++n_in[std::min<int>(p->src_class[p->local_col[i]], n_hot)];
            for (int32_t i = r0; i < r1; ++i) ++n_in[std::min<int>(p->src_class[n_loc + p->remote_col[i]], n_hot)];
            for (int c = 0; c < n_hot; ++c) final_class[c] = static_cast<uint8_t>(n_in[c] >= min_piece ? c : n_hot);
            final_class[n_hot] = static_cast<uint8_t>(n_hot);
            regroup(p->sched_local_col, l0, l1, 0, lcut);
            regroup(p->sched_remote_col, r0, r1, n_loc, rcut);
            first_piece = 0;
        } else {
            lcut[n_hot] = l0; lcut[n_hot + 1] = l1; rcut[n_hot] = r0; rcut[n_hot + 1] = r1;
        }
        row_items.clear();
        for (int c = first_piece; c < n_piece_end; ++c) {
            const int64_t pl = lcut[c + 1] - lcut[c], pr = rcut[c + 1] - rcut[c];
            if (pl + pr == 0 && !(c == n_hot && row_items.empty())) continue;   // an empty row still needs its one item
            const int64_t n_it = std::max<int64_t>(1, std::max(ceil_div(pl, run), ceil_div(pr, run)));
            for (int64_t k = 0; k < n_it; ++k) {
                WorkItem it;
                it.row = static_cast<int32_t>(v);
                it.lbeg = static_cast<int32_t>(std::min<int64_t>(lcut[c] + k * run, lcut[c + 1]));
                it.lend = static_cast<int32_t>(std::min<int64_t>(lcut[c] + (k + 1) * run, lcut[c + 1]));
                it.rbeg = static_cast<int32_t>(std::min<int64_t>(rcut[c] + k * run, rcut[c + 1]));
                it.rend = static_cast<int32_t>(std::min<int64_t>(rcut[c] + (k + 1) * run, rcut[c + 1]));
                it.slot = -1;
                it.pad0 = it.pad1 = 0;
                row_items.emplace_back(it, c);
            }
        }
        if (row_items.size() > 1) {                      // partial sums + fix-up
            SplitRow sr{static_cast<int32_t>(v), static_cast<int32_t>(p->n_split_items), static_cast<int32_t>(row_items.size()), 0};
            p->split_rows.push_back(sr);
            for (auto &ri : row_items) ri.first.slot = static_cast<int32_t>(p->n_split_items++);
        }
        for (auto &ri : row_items) {
            if (ri.second < n_hot) bucket[ri.second].push_back(ri.first);
            else cold.push_back(ri.first);
        }
    }
    // heavy items first, so that the tail of the launch is made of small ones
    std::stable_sort(cold.begin(), cold.end(), [&](const WorkItem &a, const WorkItem &b) { return item_work(a) > item_work(b); });
    if (!use_classes) {
        p->items = std::move(cold);
    } else {
        // XCD x takes the hot items of classes (0, x), (1, x), ... in that order; cold items then
        // go, largest first, to whichever XCD has the least work so far (a gather that hits in L2
        // is taken as half the cost of one that does not)
        std::vector<std::vector<WorkItem>> queue(kXcd);
        std::vector<int64_t> queue_work(kXcd, 0);
        for (int c = 0; c < n_hot; ++c) {
            std::vector<WorkItem> &q = queue[c % kXcd];
            for (const WorkItem &it : bucket[c]) queue_work[c % kXcd] += item_work(it);
            q.insert(q.end(), bucket[c].begin(), bucket[c].end());
        }
        for (int c = 0; c < kXcd; ++c) queue_work[c] /= 2;
        for (const WorkItem &it : cold) {
            const int c = static_cast<int>(std::min_element(queue_work.begin(), queue_work.end()) - queue_work.begin());
            queue[c].push_back(it);
            queue_work[c] += item_work(it);
        }
        // launch order: workgroup b (wpb items) runs on XCD b mod kXcd; pad with empty items
        size_t longest = 0;
        for (auto &q : queue) longest = std::max(longest, q.size());
        longest = (longest + wpb - 1) / wpb * wpb;
        const WorkItem dummy{-1, 0, 0, 0, 0, -1, 0, 0};
        for (auto &q : queue) q.resize(longest, dummy);
        p->items.reserve(longest * kXcd);
        for (size_t g = 0; g < longest; g += wpb)
            for (int c = 0; c < kXcd; ++c)
                p->items.insert(p->items.end(), queue[c].begin() + g, queue[c].begin() + g + wpb);
    }
    for (int32_t len = short_max; len >= 0; --len)         // longest first, isolated rows last
        p->short_rows.insert(p->short_rows.end(), by_len[len].begin(), by_len[len].end());
}

}  // namespace mgg

using namespace mgg;

extern "C" {

const char *mgg_last_error(void) { return mgg::last_error(); }
const char *mgg_version(void) { return "mgg-mi355x 0.1 (gfx950)"; }

mgg_status_t mgg_build_partition(int64_t num_nodes, const int64_t *row_ptr, const int32_t *col_idx,
                                 int32_t num_parts, int32_t part_id, const int64_t *bounds,
                                 const mgg_build_opts_t *opts, mgg_partition_t **out)
{
    if (!out) return fail(MGG_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (num_nodes < 0 || !row_ptr) return fail(MGG_ERR_INVALID_ARG, "num_nodes < 0 or row_ptr is NULL");
    if (num_nodes > INT32_MAX - 1) return fail(MGG_ERR_UNSUPPORTED, "more than 2^31-2 nodes");
    if (num_parts < 1 || part_id < 0 || part_id >= num_parts)
        return fail(MGG_ERR_INVALID_ARG, "part_id %d outside [0, %d)", part_id, num_parts);
    Knobs knobs;
    {
        mgg_status_t st = parse_opts(opts, &knobs);
        if (st != MGG_OK) return st;
    }
    const int32_t host_only = knobs.host_only;

    // ---- validate the graph ------------------------------------------------------------
    if (row_ptr[0] != 0) return fail(MGG_ERR_BAD_GRAPH, "row_ptr[0] != 0");
    for (int64_t v = 0; v < num_nodes; ++v)
        if (row_ptr[v + 1] < row_ptr[v]) return fail(MGG_ERR_BAD_GRAPH, "row_ptr decreases at row %lld", (long long)v);
    const int64_t nnz = row_ptr[num_nodes];
    if (nnz > 0 && !col_idx) return fail(MGG_ERR_INVALID_ARG, "col_idx is NULL");
    for (int64_t e = 0; e < nnz; ++e)
        if (col_idx[e] < 0 || col_idx[e] >= num_nodes)
            return fail(MGG_ERR_BAD_GRAPH, "column %d at position %lld outside [0, %lld)", col_idx[e],
                        (long long)e, (long long)num_nodes);

    // ---- node range --------------------------------------------------------------------
    std::vector<int64_t> bnd(num_parts + 1);
    if (bounds) {
        for (int32_t q = 0; q <= num_parts; ++q) bnd[q] = bounds[q];
        if (bnd[0] != 0 || bnd[num_parts] != num_nodes)
            return fail(MGG_ERR_INVALID_ARG, "bounds must run from 0 to num_nodes");
        for (int32_t q = 0; q < num_parts; ++q)
            if (bnd[q + 1] < bnd[q]) return fail(MGG_ERR_INVALID_ARG, "bounds decrease at part %d", q);
    } else {
        for (int32_t q = 0; q <= num_parts; ++q) bnd[q] = (num_nodes * q) / num_parts;
    }
    const int64_t lb = bnd[part_id], ub = bnd[part_id + 1], n_own = ub - lb;
    if (row_ptr[ub] - row_ptr[lb] >= INT32_MAX)
        return fail(MGG_ERR_UNSUPPORTED, "this share holds 2^31-1 or more neighbours");

    mgg_partition *p = new (std::nothrow) mgg_partition;
    if (!p) return fail(MGG_ERR_ALLOC, "out of host memory");
    try {
        take_default_options(p);
        p->num_nodes = num_nodes; p->lb = lb; p->ub = ub; p->n_own = n_own; p->n_local_rows = n_own;
        p->num_parts = num_parts; p->part_id = part_id;

        // ---- pass 1: count local / remote per owned row, mark halo nodes -----------------
        std::vector<uint8_t> is_halo(static_cast<size_t>(num_nodes), 0);
        p->local_row_ptr.assign(n_own + 1, 0);
        p->remote_row_ptr.assign(n_own + 1, 0);
        for (int64_t v = 0; v < n_own; ++v) {
            const int64_t g = lb + v;
            int32_t nl = 0, nr = 0;
            for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) {
                const int64_t u = col_idx[e];
                if (u == g) continue;                       // self term comes from the mode
                if (u >= lb && u < ub) ++nl;
                else { ++nr; is_halo[u] = 1; }
            }
            p->local_row_ptr[v + 1] = p->local_row_ptr[v] + nl;
            p->remote_row_ptr[v + 1] = p->remote_row_ptr[v] + nr;
        }
        // ---- halo list in ascending global id and the id -> slot map ---------------------
        std::vector<int32_t> slot_of(static_cast<size_t>(num_nodes), -1);
        for (int64_t u = 0; u < num_nodes; ++u)
            if (is_halo[u]) { slot_of[u] = static_cast<int32_t>(p->halo_gid.size()); p->halo_gid.push_back(static_cast<int32_t>(u)); }
        is_halo.clear(); is_halo.shrink_to_fit();
        const int64_t num_halo = static_cast<int64_t>(p->halo_gid.size());
        p->halo_peer_ptr.assign(num_parts + 1, 0);
        for (int32_t q = 0; q <= num_parts; ++q)
            p->halo_peer_ptr[q] = std::lower_bound(p->halo_gid.begin(), p->halo_gid.end(), bnd[q],
                                                   [](int32_t gid, int64_t b) { return gid < b; }) - p->halo_gid.begin();

        // ---- pass 2: fill the two column arrays -----------------------------------------
        p->local_col.resize(p->local_row_ptr[n_own]);
        p->remote_col.resize(p->remote_row_ptr[n_own]);
        for (int64_t v = 0; v < n_own; ++v) {
            const int64_t g = lb + v;
            int32_t wl = p->local_row_ptr[v], wr = p->remote_row_ptr[v];
            for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) {
                const int64_t u = col_idx[e];
                if (u == g) continue;
                if (u >= lb && u < ub) p->local_col[wl++] = static_cast<int32_t>(u - lb);
                else p->remote_col[wr++] = slot_of[u];
            }
        }
        slot_of.clear(); slot_of.shrink_to_fit();

        // ---- whole-graph degrees and 1/sqrt(deg+1) ---------------------------------------
        auto degree_of = [&](int64_t g) {
            int32_t d = static_cast<int32_t>(row_ptr[g + 1] - row_ptr[g]);
            for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) d -= (col_idx[e] == g);
            return d;
        };
        p->deg_own.resize(n_own); p->dinv_own.resize(n_own);
        for (int64_t v = 0; v < n_own; ++v) {
            p->deg_own[v] = degree_of(lb + v);
            p->dinv_own[v] = static_cast<float>(1.0 / std::sqrt(static_cast<double>(p->deg_own[v]) + 1.0));
        }
        p->deg_halo.resize(num_halo); p->dinv_halo.resize(num_halo);
        for (int64_t h = 0; h < num_halo; ++h) {
            p->deg_halo[h] = degree_of(p->halo_gid[h]);
            p->dinv_halo[h] = static_cast<float>(1.0 / std::sqrt(static_cast<double>(p->deg_halo[h]) + 1.0));
        }

        build_schedule(p, knobs);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(MGG_ERR_ALLOC, "out of host memory while building the partition");
    }

    if (!host_only) {
        mgg_status_t s = upload_all(p);
        if (s == MGG_OK && knobs.reserve_dim > 0) s = mgg_partition_reserve(p, knobs.reserve_dim);
        if (s != MGG_OK) { free_device(p); delete p; return s; }
    }
    *out = p;
    return MGG_OK;
}

mgg_status_t mgg_build_bags(int64_t num_bags, const int64_t *bag_ptr, const int32_t *bag_idx, int64_t table_rows,
                            int64_t local_lo, int64_t local_hi, const mgg_build_opts_t *opts, mgg_partition_t **out)
{
    if (!out) return fail(MGG_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (num_bags < 0 || !bag_ptr || table_rows < 0) return fail(MGG_ERR_INVALID_ARG, "num_bags < 0, table_rows < 0 or bag_ptr is NULL");
    if (num_bags > INT32_MAX - 1 || table_rows > INT32_MAX - 1) return fail(MGG_ERR_UNSUPPORTED, "more than 2^31-2 bags or table rows");
    if (local_lo < 0 || local_hi < local_lo || local_hi > table_rows)
        return fail(MGG_ERR_INVALID_ARG, "local slice [%lld, %lld) outside the table", (long long)local_lo, (long long)local_hi);
    Knobs knobs;
    {
        mgg_status_t st = parse_opts(opts, &knobs);
        if (st != MGG_OK) return st;
    }
    // Bags of a recommendation batch hold one lookup per table, a few tens in all: up to 32 lookups they
    // are taken several per wavefront like short graph rows (26-lookup bags: 0.89 -> 0.68 ms per batch).
    if (!opts || !opts->short_max) knobs.short_max = 32;
    if (bag_ptr[0] != 0) return fail(MGG_ERR_BAD_GRAPH, "bag_ptr[0] != 0");
    for (int64_t b = 0; b < num_bags; ++b)
        if (bag_ptr[b + 1] < bag_ptr[b]) return fail(MGG_ERR_BAD_GRAPH, "bag_ptr decreases at bag %lld", (long long)b);
    const int64_t nnz = bag_ptr[num_bags];
    if (nnz >= INT32_MAX) return fail(MGG_ERR_UNSUPPORTED, "2^31-1 or more lookups");
    if (nnz > 0 && !bag_idx) return fail(MGG_ERR_INVALID_ARG, "bag_idx is NULL");
    for (int64_t e = 0; e < nnz; ++e)
        if (bag_idx[e] < 0 || bag_idx[e] >= table_rows)
            return fail(MGG_ERR_BAD_GRAPH, "table row %d at position %lld outside [0, %lld)", bag_idx[e], (long long)e, (long long)table_rows);

    mgg_partition *p = new (std::nothrow) mgg_partition;
    if (!p) return fail(MGG_ERR_ALLOC, "out of host memory");
    try {
        take_default_options(p);
        p->bags = true;
        p->num_nodes = table_rows; p->lb = local_lo; p->ub = local_hi; p->n_own = num_bags; p->n_local_rows = local_hi - local_lo;
        p->num_parts = 1; p->part_id = 0;
        // rows of the table outside the local slice that are looked up, in ascending order, and their slots
        std::vector<uint8_t> used(static_cast<size_t>(table_rows), 0);
        for (int64_t e = 0; e < nnz; ++e)
            if (bag_idx[e] < local_lo || bag_idx[e] >= local_hi) used[bag_idx[e]] = 1;
        std::vector<int32_t> slot_of(static_cast<size_t>(table_rows), -1);
        for (int64_t u = 0; u < table_rows; ++u)
            if (used[u]) { slot_of[u] = static_cast<int32_t>(p->halo_gid.size()); p->halo_gid.push_back(static_cast<int32_t>(u)); }
        p->halo_peer_ptr = {0, static_cast<int64_t>(p->halo_gid.size())};
        p->local_row_ptr.assign(num_bags + 1, 0);
        p->remote_row_ptr.assign(num_bags + 1, 0);
        for (int64_t b = 0; b < num_bags; ++b) {
            for (int64_t e = bag_ptr[b]; e < bag_ptr[b + 1]; ++e) {
                const int32_t u = bag_idx[e];
                if (u >= local_lo && u < local_hi) p->local_col.push_back(static_cast<int32_t>(u - local_lo));
                else p->remote_col.push_back(slot_of[u]);
            }
            p->local_row_ptr[b + 1] = static_cast<int32_t>(p->local_col.size());
            p->remote_row_ptr[b + 1] = static_cast<int32_t>(p->remote_col.size());
        }
        p->deg_own.resize(num_bags);
        for (int64_t b = 0; b < num_bags; ++b) p->deg_own[b] = static_cast<int32_t>(bag_ptr[b + 1] - bag_ptr[b]);
        p->deg_halo.assign(p->halo_gid.size(), 0);
        p->dinv_own.assign(num_bags, 1.f);
        p->dinv_halo.assign(p->halo_gid.size(), 1.f);
        build_schedule(p, knobs);
    } catch (const std::bad_alloc &) {
        delete p;
        return fail(MGG_ERR_ALLOC, "out of host memory while building the bag partition");
    }
    if (!knobs.host_only) {
        mgg_status_t s = upload_all(p);
        if (s == MGG_OK && knobs.reserve_dim > 0) s = mgg_partition_reserve(p, knobs.reserve_dim);
        if (s != MGG_OK) { free_device(p); delete p; return s; }
    }
    *out = p;
    return MGG_OK;
}

mgg_status_t mgg_partition_info(const mgg_partition_t *p, mgg_partition_info_t *o)
{
    if (!p || !o) return fail(MGG_ERR_INVALID_ARG, "NULL argument");
    std::memset(o, 0, sizeof *o);
    o->num_nodes = p->num_nodes; o->lb = p->lb; o->ub = p->ub; o->n_own = p->n_own;
    o->n_local_rows = p->n_local_rows; o->is_bags = p->bags ? 1 : 0;
    o->nnz_local = static_cast<int64_t>(p->local_col.size());
    o->nnz_remote = static_cast<int64_t>(p->remote_col.size());
    o->num_halo = static_cast<int64_t>(p->halo_gid.size());
    o->num_parts = p->num_parts; o->part_id = p->part_id;
    o->ps = p->ps; o->dist = p->dist; o->short_max = p->short_max; o->on_device = p->device >= 0;
    o->xcd_min_deg = p->xcd_min_deg; o->wpb = p->wpb;
    o->class_mode = p->class_mode;
    o->hot_rows = p->hot_rows; o->n_phases = p->n_phases; o->min_piece = p->min_piece; o->hot_min_count = p->hot_min_count;
    o->n_groups_local = p->n_groups_local; o->n_groups_remote = p->n_groups_remote;
    o->n_short_rows = static_cast<int64_t>(p->short_rows.size());
    o->n_items = static_cast<int64_t>(p->items.size());
    o->n_split_rows = static_cast<int64_t>(p->split_rows.size());
    o->n_split_items = p->n_split_items;
    o->reserved_dim = p->reserved_dim;
    return MGG_OK;
}

mgg_status_t mgg_partition_export(const mgg_partition_t *p, mgg_partition_arrays_t *a)
{
    if (!p || !a) return fail(MGG_ERR_INVALID_ARG, "NULL argument");
    copy_out(p->local_row_ptr, a->local_row_ptr);
    copy_out(p->local_col, a->local_col);
    copy_out(p->remote_row_ptr, a->remote_row_ptr);
    copy_out(p->remote_col, a->remote_col);
    copy_out(p->halo_gid, a->halo_gid);
    copy_out(p->halo_peer_ptr, a->halo_peer_ptr);
    copy_out(p->deg_own, a->deg_own);
    copy_out(p->deg_halo, a->deg_halo);
    if (a->grp_local_row || a->grp_local_start || a->grp_local_end)
        export_groups(p->local_row_ptr, p->ps, a->grp_local_row, a->grp_local_start, a->grp_local_end);
    if (a->grp_remote_row || a->grp_remote_start || a->grp_remote_end)
        export_groups(p->remote_row_ptr, p->ps, a->grp_remote_row, a->grp_remote_start, a->grp_remote_end);
    copy_out(p->short_rows, a->short_rows);
    copy_out(p->sched_local_col.empty() ? p->local_col : p->sched_local_col, a->sched_local_col);
    copy_out(p->sched_remote_col.empty() ? p->remote_col : p->sched_remote_col, a->sched_remote_col);
    if (a->src_class_local || a->src_class_halo) {
        // -1: cold (or no classes at all); otherwise phase * 8 + XCD
        const int64_t nl = p->n_local_rows, nh = static_cast<int64_t>(p->halo_gid.size());
        for (int64_t i = 0; i < nl && a->src_class_local; ++i)
            a->src_class_local[i] = p->src_class.empty() || p->src_class[i] == kColdClass ? -1 : p->src_class[i];
        for (int64_t i = 0; i < nh && a->src_class_halo; ++i)
            a->src_class_halo[i] = p->src_class.empty() || p->src_class[nl + i] == kColdClass ? -1 : p->src_class[nl + i];
    }
    for (size_t i = 0; i < p->items.size(); ++i) {
        const WorkItem &it = p->items[i];
        if (a->item_row) a->item_row[i] = it.row;
        if (a->item_lbeg) a->item_lbeg[i] = it.lbeg;
        if (a->item_lend) a->item_lend[i] = it.lend;
        if (a->item_rbeg) a->item_rbeg[i] = it.rbeg;
        if (a->item_rend) a->item_rend[i] = it.rend;
        if (a->item_slot) a->item_slot[i] = it.slot;
    }
    return MGG_OK;
}

void mgg_partition_destroy(mgg_partition_t *p)
{
    if (!p) return;
    if (p->device >= 0) {
        int cur = 0;
        bool switched = hipGetDevice(&cur) == hipSuccess && cur != p->device && hipSetDevice(p->device) == hipSuccess;
        free_device(p);
        if (switched) (void)hipSetDevice(cur);
    }
    delete p;
}

mgg_status_t mgg_split_edge_balanced(int64_t num_nodes, const int64_t *row_ptr, int32_t num_parts,
                                     int64_t *bounds_out)
{
    if (num_nodes < 0 || !row_ptr || num_parts < 1 || !bounds_out)
        return fail(MGG_ERR_INVALID_ARG, "bad argument");
    const int64_t e_total = row_ptr[num_nodes];
    const int64_t per_gpu = ceil_div(e_total, num_parts);
    const int64_t *first = row_ptr, *last = row_ptr + num_nodes + 1;
    int64_t prev = 0;
    bounds_out[0] = 0;
    for (int32_t s = 1; s < num_parts; ++s) {
        const int64_t target = std::min(row_ptr[prev] + per_gpu, e_total);
        // binary search restricted to [prev, N]: first node whose edge offset reaches target
        prev = std::lower_bound(first + prev, last, target) - first;
        prev = std::min(prev, num_nodes);
        bounds_out[s] = prev;
    }
    bounds_out[num_parts] = num_nodes;
    return MGG_OK;
}

}  // extern "C"
