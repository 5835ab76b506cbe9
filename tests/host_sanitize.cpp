// Host-side sanitizer run: the CPU oracle (oracle/mgg_oracle.c) and the host logic of the library
// (partition build, export, edge-balanced split, analytical model, search state machine) exercised on
// seeded graphs in one executable built with -fsanitize=address,undefined.  No GPU is touched: partitions
// are built host-only.  Besides running clean under the sanitizers, every integer structure of the library
// is compared with the oracle's (bit-exact).  Built and run by tests/test_host_sanitizers.py.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>

#include "mgg.h"

extern "C" {
int mgg_oracle_partition_sizes(int64_t n, const int64_t *row_ptr, const int32_t *col, int32_t parts, int32_t part_id,
                               const int64_t *bounds, int64_t *nnz_local, int64_t *nnz_remote, int64_t *num_halo);
int mgg_oracle_partition_fill(int64_t n, const int64_t *row_ptr, const int32_t *col, int32_t parts, int32_t part_id,
                              const int64_t *bounds, int64_t *local_row_ptr, int32_t *local_col, int64_t *remote_row_ptr,
                              int32_t *remote_col, int32_t *halo_gid, int64_t *halo_peer_ptr, int32_t *deg_own, int32_t *deg_halo);
int64_t mgg_oracle_groups(int64_t n_rows, const int64_t *row_ptr, int32_t ps, int32_t *grp_row, int64_t *grp_start, int64_t *grp_end);
int mgg_oracle_aggregate(int64_t n, const int64_t *row_ptr, const int32_t *col, int64_t lb, int64_t ub, int32_t mode, double eps,
                         int32_t x_dtype, const void *x_local, const void *x_halo, const int32_t *halo_gid, int64_t num_halo,
                         int32_t dim, int64_t ld_x, const int64_t *rows_sel, int64_t n_sel, double *out);
int mgg_oracle_update(int64_t n_rows, const double *a, int64_t ld_a, int32_t d_in, const double *w, const double *bias,
                      int32_t d_out, int32_t act, double *out, int64_t ld_out);
int mgg_oracle_bag_sum(int64_t num_bags, const int64_t *bag_ptr, const int32_t *bag_idx, int64_t table_rows, int32_t x_dtype,
                       const void *table, int64_t ld, int32_t dim, double *out);
int mgg_oracle_split_edge_balanced(int64_t n, const int64_t *row_ptr, int32_t parts, int64_t *bounds);
}

static int g_fail = 0;
#define CHECK(cond, ...)                                      \
    do {                                                      \
        if (!(cond)) {                                        \
            std::fprintf(stderr, "FAIL %s:%d: ", __FILE__, __LINE__); \
            std::fprintf(stderr, __VA_ARGS__);                \
            std::fprintf(stderr, "\n");                       \
            ++g_fail;                                         \
        }                                                     \
    } while (0)

struct Graph {
    int64_t n;
    std::vector<int64_t> row_ptr;
    std::vector<int32_t> col;
};

// hubs, empty rows, duplicates and self-loops, rows in ascending order
static Graph random_graph(std::mt19937_64 &rng, int64_t n)
{
    Graph g;
    g.n = n;
    g.row_ptr.assign(n + 1, 0);
    for (int64_t v = 0; v < n; ++v) {
        const int kind = static_cast<int>(rng() % 10);
        int64_t d = kind < 3 ? 0 : kind < 7 ? static_cast<int64_t>(rng() % 6) : kind < 9 ? static_cast<int64_t>(rng() % 60) : static_cast<int64_t>(rng() % (2 * n + 1));
        std::vector<int32_t> row(d);
        for (auto &u : row) u = static_cast<int32_t>(rng() % n);
        std::sort(row.begin(), row.end());
        g.col.insert(g.col.end(), row.begin(), row.end());
        g.row_ptr[v + 1] = static_cast<int64_t>(g.col.size());
    }
    return g;
}

static void check_partition(const Graph &g, int32_t parts, int32_t part_id, const std::vector<int64_t> &bounds, const mgg_build_opts_t &opts)
{
    int64_t nl = 0, nr = 0, nh = 0;
    int rc = mgg_oracle_partition_sizes(g.n, g.row_ptr.data(), g.col.data(), parts, part_id, bounds.data(), &nl, &nr, &nh);
    CHECK(rc == 0, "oracle sizes rc %d", rc);
    const int64_t n_own = bounds[part_id + 1] - bounds[part_id];
    std::vector<int64_t> o_lrp(n_own + 1), o_rrp(n_own + 1), o_peer(parts + 1);
    std::vector<int32_t> o_lc(nl), o_rc(nr), o_hg(nh), o_do(n_own), o_dh(nh);
    rc = mgg_oracle_partition_fill(g.n, g.row_ptr.data(), g.col.data(), parts, part_id, bounds.data(), o_lrp.data(), o_lc.data(),
                                   o_rrp.data(), o_rc.data(), o_hg.data(), o_peer.data(), o_do.data(), o_dh.data());
    CHECK(rc == 0, "oracle fill rc %d", rc);

    mgg_partition_t *p = nullptr;
    mgg_status_t st = mgg_build_partition(g.n, g.row_ptr.data(), g.col.empty() ? nullptr : g.col.data(), parts, part_id, bounds.data(), &opts, &p);
    CHECK(st == MGG_OK, "build: %s", mgg_last_error());
    if (st != MGG_OK) return;
    mgg_partition_info_t info;
    CHECK(mgg_partition_info(p, &info) == MGG_OK, "info");
    CHECK(info.n_own == n_own && info.nnz_local == nl && info.nnz_remote == nr && info.num_halo == nh, "sizes differ");
    std::vector<int32_t> lrp(n_own + 1), lc(nl), rrp(n_own + 1), rc_(nr), hg(nh), d_own(n_own), d_halo(nh);
    std::vector<int64_t> peer(parts + 1);
    std::vector<int32_t> gl_row(info.n_groups_local), gl_s(info.n_groups_local), gl_e(info.n_groups_local);
    std::vector<int32_t> gr_row(info.n_groups_remote), gr_s(info.n_groups_remote), gr_e(info.n_groups_remote);
    std::vector<int32_t> short_rows(info.n_short_rows), slc(nl), src(nr);
    std::vector<int32_t> it_row(info.n_items), it_lb(info.n_items), it_le(info.n_items), it_rb(info.n_items), it_re(info.n_items), it_slot(info.n_items);
    std::vector<int32_t> cl(info.n_local_rows), ch(nh);
    mgg_partition_arrays_t a;
    std::memset(&a, 0, sizeof a);
    a.local_row_ptr = lrp.data(); a.local_col = lc.data(); a.remote_row_ptr = rrp.data(); a.remote_col = rc_.data();
    a.halo_gid = hg.data(); a.halo_peer_ptr = peer.data(); a.deg_own = d_own.data(); a.deg_halo = d_halo.data();
    a.grp_local_row = gl_row.data(); a.grp_local_start = gl_s.data(); a.grp_local_end = gl_e.data();
    a.grp_remote_row = gr_row.data(); a.grp_remote_start = gr_s.data(); a.grp_remote_end = gr_e.data();
    a.short_rows = short_rows.data(); a.sched_local_col = slc.data(); a.sched_remote_col = src.data();
    a.item_row = it_row.data(); a.item_lbeg = it_lb.data(); a.item_lend = it_le.data(); a.item_rbeg = it_rb.data(); a.item_rend = it_re.data();
    a.item_slot = it_slot.data(); a.src_class_local = cl.data(); a.src_class_halo = ch.data();
    CHECK(mgg_partition_export(p, &a) == MGG_OK, "export: %s", mgg_last_error());
    for (int64_t i = 0; i <= n_own; ++i) CHECK(lrp[i] == o_lrp[i] && rrp[i] == o_rrp[i], "row pointers differ at %lld", (long long)i);
    CHECK(lc == o_lc && rc_ == o_rc && hg == o_hg && d_own == o_do && d_halo == o_dh, "column / halo / degree arrays differ");
    CHECK(peer == o_peer, "owner spans differ");
    // neighbour partitions against the oracle's cut of the same rows
    std::vector<int32_t> og_row(info.n_groups_local);
    std::vector<int64_t> og_s(info.n_groups_local), og_e(info.n_groups_local);
    const int64_t ng = mgg_oracle_groups(n_own, o_lrp.data(), info.ps, og_row.data(), og_s.data(), og_e.data());
    CHECK(ng == info.n_groups_local, "local partitions: %lld vs %lld", (long long)ng, (long long)info.n_groups_local);
    for (int64_t i = 0; i < ng && i < info.n_groups_local; ++i)
        CHECK(og_row[i] == gl_row[i] && og_s[i] == gl_s[i] && og_e[i] == gl_e[i], "local partition %lld differs", (long long)i);
    // every neighbour appears in exactly one work item or short row; items stay inside their row
    std::vector<int32_t> seen_l(nl, 0), seen_r(nr, 0);
    for (int64_t i = 0; i < info.n_items; ++i) {
        if (it_row[i] < 0) continue;
        const int32_t v = it_row[i];
        CHECK(v < n_own && it_lb[i] >= lrp[v] && it_le[i] <= lrp[v + 1] && it_rb[i] >= rrp[v] && it_re[i] <= rrp[v + 1], "item %lld leaves its row", (long long)i);
        for (int32_t e = it_lb[i]; e < it_le[i]; ++e) ++seen_l[e];
        for (int32_t e = it_rb[i]; e < it_re[i]; ++e) ++seen_r[e];
    }
    for (int32_t v : short_rows) {
        for (int32_t e = lrp[v]; e < lrp[v + 1]; ++e) ++seen_l[e];
        for (int32_t e = rrp[v]; e < rrp[v + 1]; ++e) ++seen_r[e];
    }
    for (int64_t e = 0; e < nl; ++e) CHECK(seen_l[e] == 1, "local neighbour %lld covered %d times", (long long)e, seen_l[e]);
    for (int64_t e = 0; e < nr; ++e) CHECK(seen_r[e] == 1, "remote neighbour %lld covered %d times", (long long)e, seen_r[e]);
    // the scheduled order is a permutation of every row
    for (int64_t v = 0; v < n_own; ++v) {
        std::vector<int32_t> x(slc.begin() + lrp[v], slc.begin() + lrp[v + 1]), y(lc.begin() + lrp[v], lc.begin() + lrp[v + 1]);
        std::sort(x.begin(), x.end()); std::sort(y.begin(), y.end());
        CHECK(x == y, "scheduled local row %lld is not a permutation", (long long)v);
    }
    CHECK(mgg_aggregate_scratch_bytes(p, 20) == static_cast<size_t>(info.n_split_items) * 24 * 4, "scratch bytes");
    mgg_partition_destroy(p);
}

int main()
{
    std::mt19937_64 rng(220906800);
    // ---- partitions, schedules and splits on random graphs -------------------------------------
    for (int trial = 0; trial < 24; ++trial) {
        const int64_t n = 1 + static_cast<int64_t>(rng() % 400);
        const Graph g = random_graph(rng, n);
        const int32_t parts = 1 + static_cast<int32_t>(rng() % 5);
        std::vector<int64_t> bounds(parts + 1), ob(parts + 1);
        CHECK(mgg_split_edge_balanced(g.n, g.row_ptr.data(), parts, bounds.data()) == MGG_OK, "split: %s", mgg_last_error());
        CHECK(mgg_oracle_split_edge_balanced(g.n, g.row_ptr.data(), parts, ob.data()) == 0, "oracle split");
        CHECK(bounds == ob, "edge-balanced bounds differ");
        if (trial % 2) for (int32_t q = 0; q <= parts; ++q) bounds[q] = g.n * q / parts;
        mgg_build_opts_t o;
        std::memset(&o, 0, sizeof o);
        o.host_only = 1;
        const int32_t ps_c[4] = {1, 7, 32, 64}, dist_c[3] = {1, 2, 16}, short_c[3] = {-1, 3, 16}, xcd_c[4] = {-1, 1, 20, 256}, hot_c[3] = {-1, 0, 2};
        o.ps = ps_c[rng() % 4]; o.dist = dist_c[rng() % 3]; o.short_max = short_c[rng() % 3]; o.xcd_min_deg = xcd_c[rng() % 4];
        o.hot_phases = hot_c[rng() % 3]; o.wpb = 1 + static_cast<int32_t>(rng() % 8); o.min_piece = 1 + static_cast<int32_t>(rng() % 16);
        o.hot_rows = static_cast<int32_t>(rng() % 40);
        for (int32_t q = 0; q < parts; ++q) check_partition(g, parts, q, bounds, o);
    }
    // ---- the oracle's arithmetic on one graph: aggregation in both modes and dtypes, update, bags ----
    {
        const Graph g = random_graph(rng, 300);
        const int32_t dim = 20;
        std::vector<float> x(g.n * dim);
        std::vector<uint16_t> xb(g.n * dim);
        for (size_t i = 0; i < x.size(); ++i) { x[i] = static_cast<float>((static_cast<double>(rng() % 2001) - 1000.0) / 500.0); uint32_t u; std::memcpy(&u, &x[i], 4); xb[i] = static_cast<uint16_t>(u >> 16); }
        const int64_t lb = 100, ub = 220;
        std::vector<int64_t> bounds = {0, lb, ub, g.n};
        int64_t nl, nr, nh;
        mgg_oracle_partition_sizes(g.n, g.row_ptr.data(), g.col.data(), 3, 1, bounds.data(), &nl, &nr, &nh);
        std::vector<int64_t> lrp(ub - lb + 1), rrp(ub - lb + 1), peer(4);
        std::vector<int32_t> lc(nl), rc(nr), hg(nh), d_own(ub - lb), d_halo(nh);
        mgg_oracle_partition_fill(g.n, g.row_ptr.data(), g.col.data(), 3, 1, bounds.data(), lrp.data(), lc.data(), rrp.data(), rc.data(), hg.data(),
                                  peer.data(), d_own.data(), d_halo.data());
        std::vector<float> xh(nh * dim);
        std::vector<uint16_t> xhb(nh * dim);
        for (int64_t h = 0; h < nh; ++h)
            for (int32_t k = 0; k < dim; ++k) { xh[h * dim + k] = x[hg[h] * dim + k]; xhb[h * dim + k] = xb[hg[h] * dim + k]; }
        std::vector<double> part(static_cast<size_t>(ub - lb) * dim), whole(static_cast<size_t>(g.n) * dim);
        for (int mode = 0; mode < 2; ++mode) {
            CHECK(mgg_oracle_aggregate(g.n, g.row_ptr.data(), g.col.data(), lb, ub, mode, 0.25, 0, x.data() + lb * dim, xh.data(), hg.data(), nh, dim, dim,
                                       nullptr, 0, part.data()) == 0, "aggregate share");
            CHECK(mgg_oracle_aggregate(g.n, g.row_ptr.data(), g.col.data(), 0, g.n, mode, 0.25, 0, x.data(), nullptr, nullptr, 0, dim, dim, nullptr, 0,
                                       whole.data()) == 0, "aggregate whole");
            for (size_t i = 0; i < part.size(); ++i) CHECK(part[i] == whole[lb * dim + i], "share and whole graph disagree at %zu", i);
            CHECK(mgg_oracle_aggregate(g.n, g.row_ptr.data(), g.col.data(), lb, ub, mode, 0.0, 1, xb.data() + lb * dim, xhb.data(), hg.data(), nh, dim, dim,
                                       nullptr, 0, part.data()) == 0, "aggregate bf16");
        }
        std::vector<double> w(dim * 7), b(7, 0.5), out(static_cast<size_t>(ub - lb) * 7);
        for (auto &v : w) v = static_cast<double>(rng() % 100) / 100.0 - 0.5;
        for (int act = 0; act < 3; ++act)
            CHECK(mgg_oracle_update(ub - lb, part.data(), dim, dim, w.data(), b.data(), 7, act, out.data(), 7) == 0, "update act %d", act);
        std::vector<int64_t> bag_ptr = {0, 0, 3, 4, 9};
        std::vector<int32_t> bag_idx = {5, 5, 299, 0, 1, 2, 3, 4, 4};
        std::vector<double> bag(4 * dim);
        CHECK(mgg_oracle_bag_sum(4, bag_ptr.data(), bag_idx.data(), g.n, 0, x.data(), dim, dim, bag.data()) == 0, "bag sum");
        for (int32_t k = 0; k < dim; ++k) CHECK(bag[k] == 0.0 && bag[dim + k] == 2.0 * x[5 * dim + k] + x[299 * dim + k], "bag values");
        // bags through the library's host path
        mgg_build_opts_t o;
        std::memset(&o, 0, sizeof o);
        o.host_only = 1;
        mgg_partition_t *p = nullptr;
        CHECK(mgg_build_bags(4, bag_ptr.data(), bag_idx.data(), g.n, 2, 6, &o, &p) == MGG_OK, "build bags: %s", mgg_last_error());
        mgg_partition_info_t info;
        if (p) { CHECK(mgg_partition_info(p, &info) == MGG_OK && info.is_bags == 1 && info.nnz_local + info.nnz_remote == 9, "bag partition info"); mgg_partition_destroy(p); }
    }
    // ---- analytical model and the search state machine ------------------------------------------
    {
        mgg_model_t m;
        CHECK(mgg_model_evaluate(1000, 800, mgg_knobs_t{16, 4, 4}, 64, 256, 160 * 1024, &m) == MGG_OK && m.wpw == 2 * 16 * 64 * 4, "model");
        mgg_tuner_t *t = nullptr;
        CHECK(mgg_tuner_create(32, 16, 16, &t) == MGG_OK, "tuner create");
        int trials = 0;
        for (;;) {
            mgg_knobs_t k;
            int32_t done = 0;
            CHECK(mgg_tuner_next(t, &k, &done) == MGG_OK, "tuner next");
            if (done || trials > 200) break;
            const double lat = 1.0 + std::abs(k.ps - 16) * 0.1 + std::abs(k.dist - 4) * 0.05 + std::abs(k.wpb - 2) * 0.02;
            CHECK(mgg_tuner_report(t, lat) == MGG_OK, "tuner report");
            ++trials;
        }
        mgg_knobs_t best;
        double lat;
        int32_t n;
        CHECK(mgg_tuner_result(t, &best, &lat, &n) == MGG_OK && n == trials && trials > 3 && trials < 60, "tuner result after %d trials", trials);
        std::vector<mgg_knobs_t> ks(n);
        std::vector<double> ls(n);
        CHECK(mgg_tuner_table(t, n, ks.data(), ls.data(), &n) == MGG_OK, "tuner table");
        mgg_tuner_destroy(t);
    }
    // ---- error paths ------------------------------------------------------------------------------
    {
        const int64_t rp_bad[3] = {0, 2, 1};
        const int32_t c[2] = {0, 1};
        mgg_partition_t *p = nullptr;
        mgg_build_opts_t o;
        std::memset(&o, 0, sizeof o);
        o.host_only = 1;
        CHECK(mgg_build_partition(2, rp_bad, c, 1, 0, nullptr, &o, &p) == MGG_ERR_BAD_GRAPH && p == nullptr, "bad graph accepted");
        CHECK(mgg_partition_reserve(nullptr, 4) == MGG_ERR_INVALID_ARG, "reserve(NULL)");
        mgg_partition_destroy(nullptr);
    }
    if (g_fail) { std::fprintf(stderr, "%d check(s) failed\n", g_fail); return 1; }
    std::printf("host sanitizer run: all checks passed\n");
    return 0;
}
