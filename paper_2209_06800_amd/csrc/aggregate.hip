// Host side of the neighbour aggregation (launch geometry, column slabs, scratch for partial sums) and
// the fix-up kernel that combines the partial sums of rows cut into several work items.  The
// aggregation kernels themselves live in aggregate_kernels.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "aggregate_kernels.h"

namespace mgg {

namespace {

constexpr int kWavesPerBlock = 4;                   // fix-up kernel
constexpr int kBlock = kWave * kWavesPerBlock;

// Rows cut into several items: one wavefront per such row adds its partial sums slot by slot, front
// to back (a fixed order: results do not depend on scheduling), adds the self term and the row
// factor, and writes the row.  Scratch rows start on 32-byte boundaries, so every lane takes four
// consecutive columns with one 16-byte load per slot, several slots in flight; no LDS, no barrier.
template <bool BF16>
__global__ __launch_bounds__(kBlock) void fixup_kernel(const SplitRow *split_rows, int32_t n_split, int32_t dim, const float *scratch,
                                                       int64_t scratch_ld, const void *x_local, int64_t ld_x,
                                                       const float *dinv_own, int32_t gcn, float self_w, void *out_v, int32_t out_bf16,
                                                       int64_t ld_out, int32_t out_vec_ok, int32_t phase, const float *bias, int32_t relu,
                                                       int32_t no_self)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int r_id = static_cast<int>(blockIdx.x) * kWavesPerBlock + static_cast<int>(threadIdx.x / kWave);
    if (r_id >= n_split) return;
    const SplitRow sr = split_rows[r_id];
    const float dv = gcn ? dinv_own[sr.row] : 1.f;
    const float ws = gcn ? dv : self_w;
    const float *base = scratch + static_cast<int64_t>(sr.first_slot) * scratch_ld;
    for (int k = 4 * lane; k < dim; k += 4 * kWave) {
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        const float *src = base + k;                 // columns k .. k+3 exist in scratch (its rows are padded to 8)
        int i = 0;
        for (; i + 3 < sr.n_slots; i += 4) {
            const float4 v0 = *reinterpret_cast<const float4 *>(src + static_cast<int64_t>(i) * scratch_ld);
            const float4 v1 = *reinterpret_cast<const float4 *>(src + static_cast<int64_t>(i + 1) * scratch_ld);
            const float4 v2 = *reinterpret_cast<const float4 *>(src + static_cast<int64_t>(i + 2) * scratch_ld);
            const float4 v3 = *reinterpret_cast<const float4 *>(src + static_cast<int64_t>(i + 3) * scratch_ld);
            sum.x = (((sum.x + v0.x) + v1.x) + v2.x) + v3.x; sum.y = (((sum.y + v0.y) + v1.y) + v2.y) + v3.y;
            sum.z = (((sum.z + v0.z) + v1.z) + v2.z) + v3.z; sum.w = (((sum.w + v0.w) + v1.w) + v2.w) + v3.w;
        }
        for (; i < sr.n_slots; ++i) {
            const float4 v = *reinterpret_cast<const float4 *>(src + static_cast<int64_t>(i) * scratch_ld);
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        const float total[4] = {sum.x, sum.y, sum.z, sum.w};
        float *o = static_cast<float *>(out_v) + static_cast<int64_t>(sr.row) * ld_out + k;
        uint16_t *ob = static_cast<uint16_t *>(out_v) + static_cast<int64_t>(sr.row) * ld_out + k;
        float r[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            r[e] = 0.f;
            if (k + e < dim) {
                float xv = 0.f;
                if (no_self) {
                } else if constexpr (BF16)
                    xv = __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t *>(x_local)[static_cast<int64_t>(sr.row) * ld_x + k + e]) << 16);
                else
                    xv = static_cast<const float *>(x_local)[static_cast<int64_t>(sr.row) * ld_x + k + e];
                r[e] = phase == 2 ? o[e] + dv * total[e] : dv * (total[e] + ws * xv);
                if (phase != 1) {
                    if (bias) r[e] += bias[k + e];
                    if (relu) r[e] = fmaxf(r[e], 0.f);
                }
            }
        }
        if (out_bf16) {
            if (out_vec_ok && k + 3 < dim) {
                *reinterpret_cast<uint2 *>(ob) = make_uint2(f32_to_bf16_bits(r[0]) | (f32_to_bf16_bits(r[1]) << 16),
                                                            f32_to_bf16_bits(r[2]) | (f32_to_bf16_bits(r[3]) << 16));
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (k + e < dim) ob[e] = static_cast<uint16_t>(f32_to_bf16_bits(r[e]));
            }
        } else if (out_vec_ok && k + 3 < dim) {
            *reinterpret_cast<float4 *>(o) = make_float4(r[0], r[1], r[2], r[3]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (k + e < dim) o[e] = r[e];
        }
    }
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Measurement aid: rows of row_bytes gathered by pre-drawn random ids from a table of table_rows rows, 16-byte
// loads, eight in flight per lane, nothing but an add per element -- the rate at which the memory hierarchy
// delivers gathered rows to the CUs when the kernel around the gathers costs nothing.
template <int LPR>
__global__ __launch_bounds__(256) void probe_gather_kernel(const float4 *__restrict__ table, const int32_t *__restrict__ idx, int per_wave, float *sink)
{
    constexpr int NPW = kWave / LPR;
    const int lane = threadIdx.x & (kWave - 1), sub = lane / LPR, lis = lane % LPR;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (blockDim.x / kWave) + threadIdx.x / kWave;
    const int32_t *my = idx + wave * per_wave;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    int ids = my[lane];
    for (int g = 0; g < per_wave; g += kWave) {
        const int nxt = g + kWave < per_wave ? my[g + kWave + lane] : 0;
#pragma unroll
        for (int t0 = 0; t0 < kWave / NPW; t0 += 8) {
            float4 r[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int j = (t0 + u) * NPW + sub;
                const int id = NPW == 1 ? __builtin_amdgcn_readlane(ids, j) : __shfl(ids, j);
                r[u] = table[static_cast<int64_t>(id) * LPR + lis];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc.x += r[u].x; acc.y += r[u].y; acc.z += r[u].z; acc.w += r[u].w; }
        }
        ids = nxt;
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = acc.x;     // keeps the loads alive
}

}  // namespace

// A fixed scratch array for callers that must not allocate (mgg_aggregate_static).  Each GPU the
// library runs on holds its own copy; its device address is looked up once per device.
constexpr size_t kStaticScratchBytes = static_cast<size_t>(64) << 20;
static __device__ __align__(256) float g_static_scratch[kStaticScratchBytes / sizeof(float)];
constexpr int kMaxDevices = 64;
static float *g_static_scratch_ptr[kMaxDevices];      // per device; written once, under the mutex
static std::mutex g_static_scratch_mutex;

float *static_scratch(size_t *bytes)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { hip_fail(e, "hipGetDevice"); return nullptr; }
    if (dev < 0 || dev >= kMaxDevices) { fail(MGG_ERR_UNSUPPORTED, "device %d beyond the %d the static scratch is kept for", dev, kMaxDevices); return nullptr; }
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch_ptr[dev]) {
        float *ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(g_static_scratch));
        if (e != hipSuccess || !ptr) { hip_fail(e, "hipGetSymbolAddress(static scratch)"); return nullptr; }
        g_static_scratch_ptr[dev] = ptr;
    }
    if (bytes) *bytes = kStaticScratchBytes;
    return g_static_scratch_ptr[dev];
}

mgg_status_t probe_gather(int64_t table_bytes, int32_t row_bytes, int64_t n_gathers, int32_t iters, uint64_t seed, double *gbs)
{
    if (row_bytes != 128 && row_bytes != 256 && row_bytes != 512 && row_bytes != 1024)
        return fail(MGG_ERR_INVALID_ARG, "row_bytes must be 128, 256, 512 or 1024");
    constexpr int per_wave = 512, wpb = 4;
    if (table_bytes < row_bytes || table_bytes > (static_cast<int64_t>(8) << 30) || n_gathers < per_wave * wpb || n_gathers > (static_cast<int64_t>(1) << 28) ||
        iters < 1 || !gbs)
        return fail(MGG_ERR_INVALID_ARG, "probe sizes out of range");
    const int64_t rows = table_bytes / row_bytes;
    const int64_t waves = n_gathers / per_wave / wpb * wpb;
    n_gathers = waves * per_wave;
    float4 *table = nullptr;
    int32_t *idx = nullptr;
    float *sink = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    std::vector<int32_t> h(static_cast<size_t>(n_gathers));
    uint64_t x = seed * 0x9E3779B97F4A7C15ull + 1;
    for (auto &v : h) {                                   // splitmix64
        x += 0x9E3779B97F4A7C15ull;
        uint64_t z = x;
        z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull; z = (z ^ (z >> 27)) * 0x94D049BB133111EBull; z ^= z >> 31;
        v = static_cast<int32_t>(z % static_cast<uint64_t>(rows));
    }
    mgg_status_t st = MGG_OK;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&table), static_cast<size_t>(rows) * row_bytes);
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&idx), h.size() * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&sink), sizeof(float));
    if (e != hipSuccess) st = fail(MGG_ERR_ALLOC, "probe buffers: %s", hipGetErrorString(e));
    if (st == MGG_OK) {
        e = hipMemset(table, 0, static_cast<size_t>(rows) * row_bytes);
        if (e == hipSuccess) e = hipMemcpy(idx, h.data(), h.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        if (e == hipSuccess) e = hipEventCreate(&e0);
        if (e == hipSuccess) e = hipEventCreate(&e1);
        const dim3 grid(static_cast<unsigned>(waves / wpb)), block(kWave * wpb);
        for (int it = -2; it < iters && e == hipSuccess; ++it) {           // two untimed launches first
            if (it == 0) e = hipEventRecord(e0, nullptr);
            if (row_bytes == 128) hipLaunchKernelGGL(probe_gather_kernel<8>, grid, block, 0, nullptr, table, idx, per_wave, sink);
            else if (row_bytes == 256) hipLaunchKernelGGL(probe_gather_kernel<16>, grid, block, 0, nullptr, table, idx, per_wave, sink);
            else if (row_bytes == 512) hipLaunchKernelGGL(probe_gather_kernel<32>, grid, block, 0, nullptr, table, idx, per_wave, sink);
            else hipLaunchKernelGGL(probe_gather_kernel<64>, grid, block, 0, nullptr, table, idx, per_wave, sink);
            if (e == hipSuccess) e = hipGetLastError();
        }
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventRecord(e1, nullptr);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess) st = hip_fail(e, "gather probe");
        else *gbs = static_cast<double>(n_gathers) * row_bytes * iters / (ms * 1e-3) / 1e9;
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipFree(table); (void)hipFree(idx); (void)hipFree(sink);
    return st;
}

mgg_status_t launch_aggregate(const mgg_partition *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                              const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x, void *out,
                              int64_t ld_out, hipStream_t stream, const float *bias, mgg_act_t act, int32_t out_dim,
                              mgg_dtype_t out_dtype, float *scratch, size_t scratch_bytes)
{
    const bool bf16 = x_dtype == MGG_BF16;
    const size_t esz = bf16 ? 2 : 4;
    const void *xh = x_halo ? x_halo : x_local;   // never dereferenced when there is no halo

    // Widest vector the layout allows: it must keep every row start aligned, and the row must hold a
    // whole number of vectors -- counting the padding between dim and ld_x, which is read (its
    // values only reach output columns that do not exist) and never written.
    if (out_dim <= 0) out_dim = dim;
    int vec = 1;
    const int cand[3] = {bf16 ? 8 : 4, 2, 1};
    for (int c : cand) {
        const size_t bytes = c * esz;
        const int64_t padded = (static_cast<int64_t>(dim) + c - 1) / c * c;
        if (padded <= ld_x && ld_x % c == 0 && aligned(x_local, bytes) && aligned(xh, bytes)) { vec = c; dim = static_cast<int32_t>(padded); break; }
    }
    const int nvec = dim / vec;
    // Column slabs: when one XCD's share of the table rows does not fit its L2 at full width, the
    // launch walks the feature dimension slab by slab (grid.y), all work items of slab 0 first,
    // so that what stays in L2 between two uses of a table row is a slab of it, not the whole
    // row.  Costs one more pass over the ids per slab; output columns of different slabs are
    // disjoint, so nothing has to be combined.
    int slab_vecs = nvec;
    {
        const int64_t opt = p->opt_col_slab_bytes;
        const int64_t vec_bytes = static_cast<int64_t>(vec) * static_cast<int64_t>(esz);
        int64_t slab_bytes = 0;
        if (opt == 0) {
            // automatic: measured on MI355X, slabs pay (1.05-1.6x) when rows are at least 1 KB wide: what has to
            // survive in L2 between two uses of a table row is then a slab of it.  512-byte slabs, except that
            // 256-byte slabs are taken when they bring one XCD's share of the table rows within twice its 4 MB
            // L2 and 512-byte slabs do not (the 233 k x 2.4 KB table of the configs: 18.7 ms against 20.5 with
            // 512 and 20.4 with 128).  On tables far beyond the caches (2 M rows of 1 KB: 4.70 ms against 4.92
            // without slabs) the gain is small but still there; narrower rows lose to the extra passes.
            const int64_t table_rows = p->n_own + static_cast<int64_t>(p->halo_gid.size());
            const int64_t class_rows = (p->xcd_min_deg > 0 ? table_rows / kXcd : table_rows) + 1;
            if (static_cast<int64_t>(dim) * static_cast<int64_t>(esz) >= 1024) {
                if (class_rows * 512 > (8 << 20) && class_rows * 256 <= (8 << 20)) slab_bytes = 256;
                else slab_bytes = 512;
            }
        } else if (opt >= 64) {
            slab_bytes = opt;
        }
        if (slab_bytes > 0 && slab_bytes % vec_bytes == 0 && slab_bytes / vec_bytes < nvec) slab_vecs = static_cast<int>(slab_bytes / vec_bytes);
    }
    // a lane holds at most 4 chunks of a row: wider rows are always walked in slabs of 256 vectors
    if (slab_vecs > 64 * 4) slab_vecs = 64 * 4;
    const int n_slabs = (nvec + slab_vecs - 1) / slab_vecs;
    if (n_slabs > 65535) return fail(MGG_ERR_UNSUPPORTED, "dim %d too wide (at most %d)", dim, 65535 * 64 * 4 * vec);
    int lpr = 4;
    while (lpr < slab_vecs && lpr < 64) lpr <<= 1;
    const int ch = (slab_vecs + 63) / 64;

    // scratch rows for the partial sums of split rows: the caller's buffer, else the partition's own;
    // nothing is allocated here
    int64_t scratch_ld = 0;
    if (p->n_split_items > 0) {
        scratch_ld = scratch_ld_for(dim);
        const size_t need = static_cast<size_t>(p->n_split_items) * static_cast<size_t>(scratch_ld) * sizeof(float);
        if (scratch) {
            if (scratch_bytes < need) return fail(MGG_ERR_INVALID_ARG, "scratch of %zu bytes given, width %d needs %zu", scratch_bytes, dim, need);
            if (!aligned(scratch, 32)) return fail(MGG_ERR_INVALID_ARG, "scratch must be 32-byte aligned");
        } else {
            if (p->d.scratch_ld < scratch_ld)
                return fail(MGG_ERR_INVALID_ARG, "no scratch for width %d: call mgg_partition_reserve(p, %d) first (reserved: %lld columns)", dim, dim,
                            (long long)p->d.scratch_ld);
            scratch = p->d.scratch;
            scratch_ld = p->d.scratch_ld;
        }
    }

    AggArgs a{};
    a.local_row_ptr = p->d.local_row_ptr; a.local_col = p->d.local_col;
    a.remote_row_ptr = p->d.remote_row_ptr; a.remote_col = p->d.remote_col;
    a.dinv_own = p->d.dinv_own; a.w_local = p->d.w_local; a.w_remote = p->d.w_remote;
    a.short_desc = p->d.short_desc; a.items = p->d.items;
    a.x_local = x_local; a.x_halo = xh;
    a.out = out; a.scratch = scratch;
    a.ld_x = ld_x; a.ld_out = ld_out; a.scratch_ld = scratch_ld;
    a.nvec = nvec;
    a.slab_vecs = slab_vecs;
    a.n_items = static_cast<int32_t>(p->items.size());
    const int wpb = p->wpb;
    a.n_short = static_cast<int32_t>(p->short_rows.size());
    // Work per wavefront: M items (or groups of short rows) one after the other, pipelined.  More per
    // wavefront amortises its start-up latencies; fewer leaves more workgroups for the hardware to
    // balance.  Automatic: 2 where the launch still has about 8192 workgroups (measured on MI355X: 0.3-2.5 %
    // faster than 1 and than 8 on every workload tried), else 1.
    const int64_t n_groups = (a.n_items + wpb - 1) / wpb;
    const int64_t short_groups = (a.n_short + 64 / lpr - 1) / (64 / lpr);
    {
        auto pick = [&](int32_t opt, int64_t units, int64_t most) { return static_cast<int32_t>(opt > 0 ? opt : std::min<int64_t>(most, std::max<int64_t>(1, units * n_slabs / 8192))); };
        a.items_per_wave = pick(p->opt_items_per_wave, n_groups, 2);
        a.short_per_wave = pick(p->opt_short_per_wave, (short_groups + wpb - 1) / wpb, 2);
    }
    a.n_item_blocks = static_cast<int32_t>((n_groups + static_cast<int64_t>(kXcd) * a.items_per_wave - 1) / (static_cast<int64_t>(kXcd) * a.items_per_wave) * kXcd);
    a.ps = p->ps;
    const bool gcn = mode == MGG_AGG_GCN_SYM;
    // row offsets inside a table are 32-bit unless a table reaches beyond 4 GB
    {
        const uint64_t rows = static_cast<uint64_t>(std::max<int64_t>(p->n_local_rows, static_cast<int64_t>(p->halo_gid.size())));
        a.wide = rows * static_cast<uint64_t>(ld_x) * esz >= (1ull << 32) ? 1 : 0;
    }
    a.self_w = p->bags ? 0.f : 1.f + eps;
    a.no_self = p->bags ? 1 : 0;
    a.bias = bias;
    a.out_dim = out_dim;
    a.relu = act == MGG_ACT_RELU;
    a.out_bf16 = out_dtype == MGG_BF16;
    if (a.out_bf16) {           // one store of 2 * vec bytes per vector
        a.out_vec_ok = (ld_out % vec == 0) && aligned(out, static_cast<size_t>(vec) * 2);
    } else {                    // 16-byte stores at most (two per 8-element vector)
        const size_t out_bytes = (vec >= 4 ? 4 : vec) * sizeof(float);
        a.out_vec_ok = (ld_out % (vec >= 4 ? 4 : vec) == 0) && aligned(out, out_bytes);
    }

    // one launch for both neighbour lists (the default), or -- as the ablation of interleaving --
    // the local lists first and the remote lists in a second launch that adds to the result
    const bool two_phases = p->opt_split_phases != 0 && !p->halo_gid.empty() && !a.out_bf16;   // phase 2 reads `out` back
    for (int phase = two_phases ? 1 : 0; phase <= (two_phases ? 2 : 0); ++phase) {
        a.phase = phase;
        const int64_t short_waves = (short_groups + a.short_per_wave - 1) / a.short_per_wave;
        int grid_x = a.n_item_blocks + static_cast<int>((short_waves + wpb - 1) / wpb);
        if (n_slabs > 1) grid_x = (grid_x + kXcd - 1) / kXcd * kXcd;   // keeps workgroup x on XCD x mod 8 in every slab
        const dim3 grid(static_cast<unsigned>(grid_x), static_cast<unsigned>(n_slabs));
        const bool lds = p->opt_lds_halo != 0 && !p->halo_gid.empty();
        if (grid_x > 0) {
            hipError_t e;
            if (bf16) e = launch_aggregate_bf16(a, gcn, vec, grid, wpb, stream, lpr, ch, lds);
            else e = launch_aggregate_f32(a, gcn, vec, grid, wpb, stream, lpr, ch, lds);
            if (e != hipSuccess) return hip_fail(e, "aggregate kernel launch");
        }
        const int32_t n_split = static_cast<int32_t>(p->split_rows.size());
        if (n_split > 0) {
            const dim3 fgrid(static_cast<unsigned>((n_split + kWavesPerBlock - 1) / kWavesPerBlock));
            const int32_t fix_vec_ok = (ld_out % 4 == 0) && aligned(out, a.out_bf16 ? 8 : 16);
            if (bf16)
                hipLaunchKernelGGL(fixup_kernel<true>, fgrid, dim3(kBlock), 0, stream, p->d.split_rows, n_split, out_dim, scratch,
                                   scratch_ld, x_local, ld_x, p->d.dinv_own, gcn ? 1 : 0, a.self_w, out, a.out_bf16, ld_out, fix_vec_ok, a.phase, bias, a.relu, a.no_self);
            else
                hipLaunchKernelGGL(fixup_kernel<false>, fgrid, dim3(kBlock), 0, stream, p->d.split_rows, n_split, out_dim, scratch,
                                   scratch_ld, x_local, ld_x, p->d.dinv_own, gcn ? 1 : 0, a.self_w, out, a.out_bf16, ld_out, fix_vec_ok, a.phase, bias, a.relu, a.no_self);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return hip_fail(e, "fix-up kernel launch");
        }
    }
    return MGG_OK;
}

}  // namespace mgg
