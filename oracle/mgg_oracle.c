/*
 * CPU oracle for the full-graph GNN layer of MGG (arXiv 2209.06800).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, double-precision
 * statement of what the layer computes.  It shares no code, header, table or
 * helper with the HIP library; only tests, the smoke check and the bench's
 * cpu_baseline leg may call it.  There is no blocking, fusion or reordering
 * here beyond what the definitions state, so it can be checked by eye.
 *
 * What is computed, and where the paper defines it:
 *   - Aggregate / Update split of a layer ............ section 1, the "GNN" equation
 *   - GCN:  A_hat X W with A_hat = adjacency + self-loops (section 7, eq. for Z),
 *           read as the symmetric normalisation D^-1/2 (A+I) D^-1/2, d = deg + 1
 *   - GIN:  (1+eps) h_v + sum over N(v) of h_u ........ section 7, the GIN equation
 *   - local / remote split into two CSRs per GPU ..... section 4.1, Step-2
 *   - fixed-size neighbour partitions of ps neighbours  section 4.1, Step-3
 *   - node-range ownership and ids rebased to zero .... section 4.2, Fig. 4
 *   - edge-balanced contiguous split ................. section 4.1, Step-1 / Algorithm 1
 *   - embedding-bag sum (lookup + element-wise addition) section 8.3, generality to DLRM
 *
 * Conventions: graph = CSR (row_ptr int64[N+1], col int32[nnz]); row v lists the
 * nodes whose embeddings are summed into v.  A neighbour equal to the row's own id
 * (a self-loop in the input) is ignored; the self term is added by the mode.
 * Duplicate neighbours count with multiplicity.  Degrees are always those of the
 * whole graph, never of a partition.
 *
 * Every function returns 0 on success, a negative code on bad input.
 * Pins: tests/test_oracle_pins.py (dense brute force, closed forms, invariants).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORA_F32 = 0, ORA_BF16 = 1, ORA_F64 = 2 };
enum { ORA_GCN = 0, ORA_GIN = 1 };
enum { ORA_ACT_NONE = 0, ORA_ACT_RELU = 1, ORA_ACT_SOFTMAX = 2 };

int mgg_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* value of element i of a table stored as f32, bf16 bit patterns or f64 */
static double load_elem(const void *base, int dtype, int64_t i)
{
    if (dtype == ORA_F32) return (double)((const float *)base)[i];
    if (dtype == ORA_F64) return ((const double *)base)[i];
    uint32_t bits = ((uint32_t)((const uint16_t *)base)[i]) << 16; /* bf16 = top half of f32 */
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

static int csr_ok(int64_t n, const int64_t *row_ptr, const int32_t *col)
{
    if (n < 0 || !row_ptr || row_ptr[0] != 0) return 0;
    for (int64_t v = 0; v < n; ++v)
        if (row_ptr[v + 1] < row_ptr[v]) return 0;
    if (row_ptr[n] > 0 && !col) return 0;
    for (int64_t e = 0; e < row_ptr[n]; ++e)
        if (col[e] < 0 || col[e] >= n) return 0;
    return 1;
}

/* deg[v] = number of neighbours of v other than v itself (whole graph). */
int mgg_oracle_degrees(int64_t n, const int64_t *row_ptr, const int32_t *col, int32_t *deg)
{
    if (!csr_ok(n, row_ptr, col) || !deg) return -1;
    for (int64_t v = 0; v < n; ++v) {
        int32_t d = 0;
        for (int64_t e = row_ptr[v]; e < row_ptr[v + 1]; ++e)
            if (col[e] != v) ++d;
        deg[v] = d;
    }
    return 0;
}

/* ------------------------------------------------------------------------- *
 * Partition build (section 4.1 Step-2, section 4.2): the rows [lb, ub) this
 * GPU owns, split into a local CSR (neighbour inside the range, id rebased by
 * -lb) and a remote CSR (neighbour outside; id replaced by its position in the
 * sorted list of distinct remote ids, the "halo").  Two calls: sizes, then fill.
 * ------------------------------------------------------------------------- */
static int cmp_i32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

static int bounds_ok(int64_t n, int32_t parts, int32_t part_id, const int64_t *bounds)
{
    if (parts < 1 || part_id < 0 || part_id >= parts || !bounds) return 0;
    if (bounds[0] != 0 || bounds[parts] != n) return 0;
    for (int32_t p = 0; p < parts; ++p)
        if (bounds[p + 1] < bounds[p]) return 0;
    return 1;
}

int mgg_oracle_partition_sizes(int64_t n, const int64_t *row_ptr, const int32_t *col,
                               int32_t parts, int32_t part_id, const int64_t *bounds,
                               int64_t *nnz_local, int64_t *nnz_remote, int64_t *num_halo)
{
    if (!csr_ok(n, row_ptr, col)) return -1;
    if (!bounds_ok(n, parts, part_id, bounds)) return -2;
    int64_t lb = bounds[part_id], ub = bounds[part_id + 1];
    int64_t nl = 0, nr = 0;
    for (int64_t g = lb; g < ub; ++g)
        for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) {
            int64_t u = col[e];
            if (u == g) continue;
            if (u >= lb && u < ub) ++nl; else ++nr;
        }
    int32_t *rem = (int32_t *)malloc((size_t)(nr > 0 ? nr : 1) * sizeof(int32_t));
    if (!rem) return -3;
    int64_t k = 0;
    for (int64_t g = lb; g < ub; ++g)
        for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) {
            int64_t u = col[e];
            if (u != g && (u < lb || u >= ub)) rem[k++] = (int32_t)u;
        }
    qsort(rem, (size_t)nr, sizeof(int32_t), cmp_i32);
    int64_t nh = 0;
    for (int64_t i = 0; i < nr; ++i)
        if (i == 0 || rem[i] != rem[i - 1]) ++nh;
    free(rem);
    *nnz_local = nl; *nnz_remote = nr; *num_halo = nh;
    return 0;
}

int mgg_oracle_partition_fill(int64_t n, const int64_t *row_ptr, const int32_t *col,
                              int32_t parts, int32_t part_id, const int64_t *bounds,
                              int64_t *local_row_ptr, int32_t *local_col,
                              int64_t *remote_row_ptr, int32_t *remote_col,
                              int32_t *halo_gid, int64_t *halo_peer_ptr,
                              int32_t *deg_own, int32_t *deg_halo)
{
    int64_t nl, nr, nh;
    int rc = mgg_oracle_partition_sizes(n, row_ptr, col, parts, part_id, bounds, &nl, &nr, &nh);
    if (rc) return rc;
    int64_t lb = bounds[part_id], ub = bounds[part_id + 1];

    /* halo = sorted distinct remote neighbour ids */
    int32_t *rem = (int32_t *)malloc((size_t)(nr > 0 ? nr : 1) * sizeof(int32_t));
    if (!rem) return -3;
    int64_t k = 0;
    for (int64_t g = lb; g < ub; ++g)
        for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) {
            int64_t u = col[e];
            if (u != g && (u < lb || u >= ub)) rem[k++] = (int32_t)u;
        }
    qsort(rem, (size_t)nr, sizeof(int32_t), cmp_i32);
    int64_t h = 0;
    for (int64_t i = 0; i < nr; ++i)
        if (i == 0 || rem[i] != rem[i - 1]) halo_gid[h++] = rem[i];
    free(rem);

    /* rows, in order; each neighbour goes to the local or the remote row */
    int64_t pl = 0, pr = 0;
    local_row_ptr[0] = 0; remote_row_ptr[0] = 0;
    for (int64_t g = lb; g < ub; ++g) {
        for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) {
            int64_t u = col[e];
            if (u == g) continue;
            if (u >= lb && u < ub) {
                local_col[pl++] = (int32_t)(u - lb);
            } else {
                int64_t lo = 0, hi = nh;              /* position of u in halo_gid */
                while (lo < hi) {
                    int64_t mid = (lo + hi) / 2;
                    if (halo_gid[mid] < u) lo = mid + 1; else hi = mid;
                }
                remote_col[pr++] = (int32_t)lo;
            }
        }
        local_row_ptr[g - lb + 1] = pl;
        remote_row_ptr[g - lb + 1] = pr;
    }

    /* owner spans of the halo list: halo ids below bounds[p] */
    for (int32_t p = 0; p <= parts; ++p) {
        int64_t c = 0;
        for (int64_t i = 0; i < nh; ++i)
            if (halo_gid[i] < bounds[p]) ++c;
        halo_peer_ptr[p] = c;
    }

    /* whole-graph degrees (self-loops not counted) */
    for (int64_t g = lb; g < ub; ++g) {
        int32_t d = 0;
        for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) if (col[e] != g) ++d;
        deg_own[g - lb] = d;
    }
    for (int64_t i = 0; i < nh; ++i) {
        int64_t u = halo_gid[i];
        int32_t d = 0;
        for (int64_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) if (col[e] != u) ++d;
        deg_halo[i] = d;
    }
    return 0;
}

/* ------------------------------------------------------------------------- *
 * Neighbour partitions (section 4.1 Step-3): every non-empty row of a CSR is
 * cut, front to back, into groups of ps neighbours; the last may be shorter.
 * Call with grp_row == NULL to count only.
 * ------------------------------------------------------------------------- */
int64_t mgg_oracle_groups(int64_t n_rows, const int64_t *row_ptr, int32_t ps,
                          int32_t *grp_row, int64_t *grp_start, int64_t *grp_end)
{
    if (ps < 1 || n_rows < 0 || !row_ptr) return -1;
    int64_t g = 0;
    for (int64_t r = 0; r < n_rows; ++r)
        for (int64_t s = row_ptr[r]; s < row_ptr[r + 1]; s += ps) {
            if (grp_row) {
                grp_row[g] = (int32_t)r;
                grp_start[g] = s;
                grp_end[g] = (s + ps < row_ptr[r + 1]) ? s + ps : row_ptr[r + 1];
            }
            ++g;
        }
    return g;
}

/* ------------------------------------------------------------------------- *
 * Aggregate (section 1 "GNN" equation; section 7 GCN and GIN equations).
 * For owned node g (output row g - lb), with N(g) the row of g without g itself
 * and d~ = |N(.)| + 1:
 *     GCN:  a_g = sum_{u in N(g)} x_u / sqrt(d~_u d~_g)  +  x_g / d~_g
 *     GIN:  a_g = (1 + eps) x_g + sum_{u in N(g)} x_u
 * x_u comes from x_local (row u - lb) when lb <= u < ub, otherwise from x_halo
 * at the position of u in halo_gid.  With lb = 0, ub = N there is no halo and
 * this is the plain whole-graph definition.
 * rows_sel (nullable): compute only these owned rows (indices relative to lb);
 * out then has n_sel rows.  out is double, row-major, leading dimension dim.
 * ------------------------------------------------------------------------- */
int mgg_oracle_aggregate(int64_t n, const int64_t *row_ptr, const int32_t *col,
                         int64_t lb, int64_t ub, int32_t mode, double eps,
                         int32_t x_dtype, const void *x_local, const void *x_halo,
                         const int32_t *halo_gid, int64_t num_halo,
                         int32_t dim, int64_t ld_x,
                         const int64_t *rows_sel, int64_t n_sel, double *out)
{
    if (!csr_ok(n, row_ptr, col)) return -1;
    if (lb < 0 || ub < lb || ub > n || dim < 1 || ld_x < dim || !out) return -2;
    if (mode != ORA_GCN && mode != ORA_GIN) return -2;
    if (ub > lb && !x_local) return -2;
    int64_t n_out = rows_sel ? n_sel : ub - lb;
    for (int64_t i = 0; rows_sel && i < n_sel; ++i)
        if (rows_sel[i] < 0 || rows_sel[i] >= ub - lb) return -2;

    int32_t *deg = (int32_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int32_t));
    if (!deg) return -3;
    mgg_oracle_degrees(n, row_ptr, col, deg);

    int bad = 0;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < n_out; ++i) {
        int64_t g = lb + (rows_sel ? rows_sel[i] : i);
        double *a = out + i * (int64_t)dim;
        double dg = (double)deg[g] + 1.0;
        double w_self = (mode == ORA_GCN) ? 1.0 / dg : 1.0 + eps;
        for (int32_t k = 0; k < dim; ++k)
            a[k] = w_self * load_elem(x_local, x_dtype, (g - lb) * ld_x + k);
        for (int64_t e = row_ptr[g]; e < row_ptr[g + 1]; ++e) {
            int64_t u = col[e];
            if (u == g) continue;
            const void *tab; int64_t r;
            if (u >= lb && u < ub) { tab = x_local; r = u - lb; }
            else {
                int64_t lo = 0, hi = num_halo;
                while (lo < hi) {
                    int64_t mid = (lo + hi) / 2;
                    if (halo_gid[mid] < u) lo = mid + 1; else hi = mid;
                }
                if (lo >= num_halo || halo_gid[lo] != u || !x_halo) { bad = 1; continue; }
                tab = x_halo; r = lo;
            }
            double w = (mode == ORA_GCN) ? 1.0 / sqrt(((double)deg[u] + 1.0) * dg) : 1.0;
            for (int32_t k = 0; k < dim; ++k)
                a[k] += w * load_elem(tab, x_dtype, r * ld_x + k);
        }
    }
    free(deg);
    return bad ? -4 : 0;
}

/* ------------------------------------------------------------------------- *
 * Update (section 1: "a fully-connected NN layer"; section 7: X W, ReLU, MLP):
 *     out[i][j] = act( bias[j] + sum_k a[i][k] * w[k][j] )
 * a, w, bias (nullable), out are double, row-major.  act = softmax is the last step of the
 * 2-layer GCN of section 7, Z = softmax(A_hat ReLU(A_hat X W0) W1), taken over each row:
 * softmax(z)_j = exp(z_j) / sum_k exp(z_k), evaluated as exp(z_j - max z) / sum_k exp(z_k - max z),
 * which is the same number and cannot overflow.
 * ------------------------------------------------------------------------- */
int mgg_oracle_update(int64_t n_rows, const double *a, int64_t ld_a, int32_t d_in,
                      const double *w, const double *bias, int32_t d_out, int32_t act,
                      double *out, int64_t ld_out)
{
    if (n_rows < 0 || d_in < 1 || d_out < 1 || ld_a < d_in || ld_out < d_out) return -2;
    if (n_rows > 0 && (!a || !w || !out)) return -2;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n_rows; ++i) {
        double *o = out + i * ld_out;
        for (int32_t j = 0; j < d_out; ++j) o[j] = bias ? bias[j] : 0.0;
        for (int32_t k = 0; k < d_in; ++k) {
            double aik = a[i * ld_a + k];
            for (int32_t j = 0; j < d_out; ++j) o[j] += aik * w[(int64_t)k * d_out + j];
        }
        if (act == ORA_ACT_RELU)
            for (int32_t j = 0; j < d_out; ++j) if (o[j] < 0.0) o[j] = 0.0;
        if (act == ORA_ACT_SOFTMAX) {
            double zmax = o[0], sum = 0.0;
            for (int32_t j = 1; j < d_out; ++j) if (o[j] > zmax) zmax = o[j];
            for (int32_t j = 0; j < d_out; ++j) { o[j] = exp(o[j] - zmax); sum += o[j]; }
            for (int32_t j = 0; j < d_out; ++j) o[j] /= sum;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- *
 * Embedding-bag sum (section 8.3, "Generality to other applications": embedding
 * lookup followed by element-wise addition):
 *     out[b][k] = sum over e in [bag_ptr[b], bag_ptr[b+1]) of table[bag_idx[e]][k]
 * over the WHOLE table (no local / remote split here: where a row is stored does
 * not change the sum).  Duplicates count with multiplicity, an empty bag gives zeros.
 * table is [table_rows x ld] of x_dtype, out is double [num_bags x dim].
 * ------------------------------------------------------------------------- */
int mgg_oracle_bag_sum(int64_t num_bags, const int64_t *bag_ptr, const int32_t *bag_idx, int64_t table_rows,
                       int32_t x_dtype, const void *table, int64_t ld, int32_t dim, double *out)
{
    if (num_bags < 0 || !bag_ptr || dim < 1 || ld < dim || (num_bags > 0 && !out)) return -2;
    if (bag_ptr[0] != 0) return -3;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t b = 0; b < num_bags; ++b) {
        double *o = out + b * dim;
        for (int32_t k = 0; k < dim; ++k) o[k] = 0.0;
        if (bag_ptr[b + 1] < bag_ptr[b]) { bad = 1; continue; }
        for (int64_t e = bag_ptr[b]; e < bag_ptr[b + 1]; ++e) {
            int64_t u = bag_idx[e];
            if (u < 0 || u >= table_rows) { bad = 1; continue; }
            for (int32_t k = 0; k < dim; ++k) o[k] += load_elem(table, x_dtype, u * ld + k);
        }
    }
    return bad ? -4 : 0;
}

/* ------------------------------------------------------------------------- *
 * Edge-balanced contiguous split (section 4.1 Step-1, Algorithm 1).  The
 * printed pseudo-code averages two edge offsets where it means to probe the
 * middle node and cannot terminate as written; what it states it computes is:
 * with ePerGPU = ceil(E / parts), split point s is the first node index
 * n >= previous split with row_ptr[n] >= min(row_ptr[previous] + ePerGPU, E).
 * Written here as that definition, by linear scan.  bounds has parts+1 entries.
 * ------------------------------------------------------------------------- */
int mgg_oracle_split_edge_balanced(int64_t n, const int64_t *row_ptr, int32_t parts,
                                   int64_t *bounds)
{
    if (n < 0 || parts < 1 || !row_ptr || !bounds) return -2;
    int64_t e_total = row_ptr[n];
    int64_t per = (e_total + parts - 1) / parts;
    int64_t last = 0;
    bounds[0] = 0;
    for (int32_t s = 1; s < parts; ++s) {
        int64_t target = row_ptr[last] + per;
        if (target > e_total) target = e_total;
        int64_t p = last;
        while (p < n && row_ptr[p] < target) ++p;
        bounds[s] = p;
        last = p;
    }
    bounds[parts] = n;
    return 0;
}
