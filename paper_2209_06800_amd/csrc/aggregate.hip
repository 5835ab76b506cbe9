// Neighbour aggregation for gfx950 (section 1 "GNN" equation; section 4.1 LR / LL / AC
// stages; section 5.1 warp-per-partition mapping with local and remote work interleaved).
//
// Mapping used here, per 64-lane wavefront:
//   - a row of the embedding table is spread over LPR lanes (LPR = 4..64, a power of two),
//     each lane owning VEC contiguous elements per chunk (16-byte loads when the layout
//     allows), so one load instruction fetches 64/LPR neighbour rows;
//   - a work item is a run of neighbour partitions (<= ps neighbours each) of ONE owned row,
//     local and remote partitions taken alternately, so every wavefront mixes both kinds;
//   - the 64/LPR sub-wave accumulators are combined with cross-lane shuffles at the end;
//   - short rows are handled one per sub-wave (several rows per wavefront);
//   - rows cut into several items leave raw partial sums in scratch rows, and a second
//     small kernel adds them in a fixed order (results do not depend on scheduling).
// Bound by memory traffic (about 0.5 flop per byte): no MFMA here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "mgg_internal.h"

namespace mgg {

namespace {

#ifndef MGG_AGG_INFLIGHT
#define MGG_AGG_INFLIGHT 8          // 16-byte loads a lane keeps in flight
#endif
constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;                   // fix-up kernel, and the LDS stage of the staged variant
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kMaxWpb = 16;                         // wavefronts per workgroup of the aggregation kernel

struct AggArgs {
    const int32_t *local_row_ptr, *local_col, *remote_row_ptr, *remote_col;
    const float *dinv_own;               // 1/sqrt(deg+1) of the owned rows (the row factor of GCN)
    const float *w_local, *w_remote;     // GCN: factor of the neighbour, one per entry of the column arrays
    const int32_t *short_rows;
    const WorkItem *items;
    const void *x_local, *x_halo;
    void *out;               // fp32, or bf16 when out_bf16 (rounded to nearest even)
    float *scratch;
    int64_t ld_x, ld_out, scratch_ld;
    int32_t nvec;            // vectors of VEC elements per row (dim / VEC)
    int32_t slab_vecs;       // vectors per column slab; blockIdx.y selects the slab (= nvec: one slab)
    int32_t n_items, n_item_blocks, n_short;
    int32_t ps;
    int32_t gcn;             // 1: symmetric normalisation, 0: plain sum
    float self_w;            // GIN: 1 + eps
    int32_t out_bf16;
    int32_t no_self;         // bags: the owned row has no embedding of its own, x_local is only a table
    int32_t out_vec_ok;      // out rows allow VEC-wide stores
    int32_t out_dim;         // columns of `out` that exist (<= nvec * VEC; the rest of the last vector is padding of the tables)
    int32_t phase;           // 0: local and remote lists in one launch; 1: local lists (+ self term) only;
                             // 2: remote lists only, added to what phase 1 left in out
    const float *bias;       // optional epilogue of the final value: + bias[column], then ReLU if relu != 0
    int32_t relu;            // (used when the Update's matrix product was applied before the aggregation)
};

// ---- element access ---------------------------------------------------------------------
template <bool BF16, int VEC> struct Raw;
template <> struct Raw<false, 4> { using type = float4; };
template <> struct Raw<false, 2> { using type = float2; };
template <> struct Raw<false, 1> { using type = float; };
template <> struct Raw<true, 8> { using type = uint4; };
template <> struct Raw<true, 2> { using type = uint32_t; };
template <> struct Raw<true, 1> { using type = uint16_t; };

__device__ __forceinline__ float bf16_lo(uint32_t d) { return __uint_as_float(d << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t d) { return __uint_as_float(d & 0xffff0000u); }

template <bool BF16, int VEC>
__device__ __forceinline__ void unpack(const typename Raw<BF16, VEC>::type &r, float (&f)[VEC])
{
    if constexpr (!BF16) {
        if constexpr (VEC == 4) { f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w; }
        else if constexpr (VEC == 2) { f[0] = r.x; f[1] = r.y; }
        else { f[0] = r; }
    } else {
        if constexpr (VEC == 8) {
            f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
            f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
        } else if constexpr (VEC == 2) { f[0] = bf16_lo(r); f[1] = bf16_hi(r); }
        else { f[0] = __uint_as_float(static_cast<uint32_t>(r) << 16); }
    }
}

template <typename R> __device__ __forceinline__ R zero_raw() { R z; __builtin_memset(&z, 0, sizeof z); return z; }

template <int VEC>
__device__ __forceinline__ void store_vec(float *dst, const float (&v)[VEC], bool vec_ok)
{
    if (vec_ok) {
        if constexpr (VEC == 8) {
            reinterpret_cast<float4 *>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
            reinterpret_cast<float4 *>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
        } else if constexpr (VEC == 4) {
            *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        } else if constexpr (VEC == 2) {
            *reinterpret_cast<float2 *>(dst) = make_float2(v[0], v[1]);
        } else {
            dst[0] = v[0];
        }
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) dst[e] = v[e];
    }
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);       // round to nearest, ties to even
    return u >> 16;
}

// bf16 output: the same VEC values, rounded, as one 2*VEC-byte store when the layout allows
template <int VEC>
__device__ __forceinline__ void store_vec_bf16(uint16_t *dst, const float (&v)[VEC], bool vec_ok)
{
    if (vec_ok && VEC >= 2) {
        uint32_t pk[VEC >= 2 ? VEC / 2 : 1];
#pragma unroll
        for (int e = 0; e < VEC / 2; ++e) pk[e] = f32_to_bf16_bits(v[2 * e]) | (f32_to_bf16_bits(v[2 * e + 1]) << 16);
        if constexpr (VEC == 8) *reinterpret_cast<uint4 *>(dst) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        else if constexpr (VEC == 4) *reinterpret_cast<uint2 *>(dst) = make_uint2(pk[0], pk[1]);
        else if constexpr (VEC == 2) *reinterpret_cast<uint32_t *>(dst) = pk[0];
    } else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) dst[e] = static_cast<uint16_t>(f32_to_bf16_bits(v[e]));
    }
}

// ---- one kernel configuration --------------------------------------------------------------
template <bool BF16_, int VEC_, int LPR_, int CH_>
struct Cfg {
    static constexpr bool BF16 = BF16_;
    static constexpr int VEC = VEC_, LPR = LPR_, CH = CH_;
    static constexpr int NPW = kWave / LPR;                 // neighbour rows per load instruction
    static constexpr int U = (MGG_AGG_INFLIGHT / CH) > 0 ? (MGG_AGG_INFLIGHT / CH) : 1;   // neighbour rows in flight per lane
    using elem = typename std::conditional<BF16, uint16_t, float>::type;
    using raw = typename Raw<BF16, VEC>::type;
};

template <class K>
struct Acc {
    float v[K::CH][K::VEC];
    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int c = 0; c < K::CH; ++c)
#pragma unroll
            for (int e = 0; e < K::VEC; ++e) v[c][e] = 0.f;
    }
};

// Final value of an owned row from its neighbour sum: adds the self term and the row factor.
template <class K>
__device__ __forceinline__ void write_final(const AggArgs &a, const Acc<K> &acc, int32_t row, int lis, int vend)
{
    const typename K::elem *xs = static_cast<const typename K::elem *>(a.x_local) + static_cast<int64_t>(row) * a.ld_x;
    float *o = static_cast<float *>(a.out) + static_cast<int64_t>(row) * a.ld_out;             // fp32 output
    uint16_t *ob = static_cast<uint16_t *>(a.out) + static_cast<int64_t>(row) * a.ld_out;     // bf16 output
    const float dv = a.gcn ? a.dinv_own[row] : 1.f;
    const float ws = a.gcn ? dv : a.self_w;     // GCN: dv * (sum + dv * x_v) = sum_u x_u/sqrt(du dv) + x_v/dv^2
#pragma unroll
    for (int c = 0; c < K::CH; ++c) {
        const int vi = c * K::LPR + lis;
        if (vi < vend) {
            float xv[K::VEC], r[K::VEC];
            if (a.no_self) {
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) xv[e] = 0.f;
            } else {
                unpack<K::BF16, K::VEC>(*reinterpret_cast<const typename K::raw *>(xs + static_cast<int64_t>(vi) * K::VEC), xv);
            }
            if (a.phase == 2) {                 // second of two launches: add to the first one's result
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) r[e] = (vi * K::VEC + e < a.out_dim ? o[vi * K::VEC + e] : 0.f) + dv * acc.v[c][e];
            } else {
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) r[e] = dv * (acc.v[c][e] + ws * xv[e]);
            }
            if (a.phase != 1) {                 // the value is final: optional bias and ReLU
                if (a.bias) {
#pragma unroll
                    for (int e = 0; e < K::VEC; ++e)
                        if (vi * K::VEC + e < a.out_dim) r[e] += a.bias[vi * K::VEC + e];
                }
                if (a.relu) {
#pragma unroll
                    for (int e = 0; e < K::VEC; ++e) r[e] = fmaxf(r[e], 0.f);
                }
            }
            const int col0 = vi * K::VEC;
            if (a.out_bf16) {                   // (never combined with phase 2, which reads `out` back)
                if (col0 + K::VEC <= a.out_dim) {
                    store_vec_bf16<K::VEC>(ob + col0, r, a.out_vec_ok);
                } else {
#pragma unroll
                    for (int e = 0; e < K::VEC; ++e)
                        if (col0 + e < a.out_dim) ob[col0 + e] = static_cast<uint16_t>(f32_to_bf16_bits(r[e]));
                }
            } else if (col0 + K::VEC <= a.out_dim) {
                store_vec<K::VEC>(o + col0, r, a.out_vec_ok);
            } else {                            // last vector reaches into the padding: store what exists
#pragma unroll
                for (int e = 0; e < K::VEC; ++e)
                    if (col0 + e < a.out_dim) o[col0 + e] = r[e];
            }
        }
    }
}

template <class K>
__device__ __forceinline__ void write_partial(const AggArgs &a, const Acc<K> &acc, int32_t slot, int lis, int vend)
{
    float *o = a.scratch + static_cast<int64_t>(slot) * a.scratch_ld;
#pragma unroll
    for (int c = 0; c < K::CH; ++c) {
        const int vi = c * K::LPR + lis;
        if (vi < vend) store_vec<K::VEC>(o + static_cast<int64_t>(vi) * K::VEC, acc.v[c], true);
    }
}

// Accumulate one neighbour partition: `len` (<= 64) neighbour ids are held one per lane in
// my_idx (weights in my_w); sub-wave `sub` takes neighbours sub, sub+NPW, ...
template <class K>
__device__ __forceinline__ void accumulate_partition(Acc<K> &acc, const typename K::elem *table, int64_t ld,
                                                     int my_idx, float my_w, int len, int sub, int lis, int nvec)
{
    const int steps = (len + K::NPW - 1) / K::NPW;
    for (int t0 = 0; t0 < steps; t0 += K::U) {
        typename K::raw r[K::U][K::CH];
        float w[K::U];
#pragma unroll
        for (int u = 0; u < K::U; ++u) {
            const int j = (t0 + u) * K::NPW + sub;
            const bool ok = j < len;
            int idx;
            if constexpr (K::NPW == 1) {           // j is wave-uniform: scalar broadcast
                idx = __builtin_amdgcn_readlane(my_idx, j & 63);
                const float wj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_w), j & 63));
                w[u] = ok ? wj : 0.f;
            } else {
                idx = __shfl(my_idx, j & 63);
                const float wj = __shfl(my_w, j & 63);
                w[u] = ok ? wj : 0.f;
            }
            const typename K::elem *rowp = table + static_cast<int64_t>(idx) * ld;
#pragma unroll
            for (int c = 0; c < K::CH; ++c) {
                const int vi = c * K::LPR + lis;
                if (ok && vi < nvec)
                    r[u][c] = *reinterpret_cast<const typename K::raw *>(rowp + static_cast<int64_t>(vi) * K::VEC);
                else
                    r[u][c] = zero_raw<typename K::raw>();
            }
        }
#pragma unroll
        for (int u = 0; u < K::U; ++u)
#pragma unroll
            for (int c = 0; c < K::CH; ++c) {
                float f[K::VEC];
                unpack<K::BF16, K::VEC>(r[u][c], f);
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) acc.v[c][e] = fmaf(w[u], f[e], acc.v[c][e]);
            }
    }
}

// Load the ids (and GCN factors) of the partition starting at `pos`, one per lane.  The factors
// are stored per edge, in the order of the column array, so both loads are coalesced.
__device__ __forceinline__ void load_partition_ids(const int32_t *col, const float *wts, int pos, int len, int lane,
                                                   bool gcn, int &idx, float &w)
{
    idx = 0; w = 0.f;
    if (lane < len) {
        idx = col[pos + lane];
        w = gcn ? wts[pos + lane] : 1.f;
    }
}

// Sub-wave walk over one short neighbour list (all lanes of the sub-wave read the same id).
template <class K>
__device__ __forceinline__ void accumulate_list(Acc<K> &acc, const typename K::elem *table, int64_t ld,
                                                const int32_t *col, const float *wts, int beg, int end,
                                                bool gcn, int lis, int nvec)
{
    for (int j0 = beg; j0 < end; j0 += K::U) {
        typename K::raw r[K::U][K::CH];
        float w[K::U];
#pragma unroll
        for (int u = 0; u < K::U; ++u) {
            const bool ok = j0 + u < end;
            const int idx = ok ? col[j0 + u] : 0;
            w[u] = ok ? (gcn ? wts[j0 + u] : 1.f) : 0.f;
            const typename K::elem *rowp = table + static_cast<int64_t>(idx) * ld;
#pragma unroll
            for (int c = 0; c < K::CH; ++c) {
                const int vi = c * K::LPR + lis;
                if (ok && vi < nvec)
                    r[u][c] = *reinterpret_cast<const typename K::raw *>(rowp + static_cast<int64_t>(vi) * K::VEC);
                else
                    r[u][c] = zero_raw<typename K::raw>();
            }
        }
#pragma unroll
        for (int u = 0; u < K::U; ++u)
#pragma unroll
            for (int c = 0; c < K::CH; ++c) {
                float f[K::VEC];
                unpack<K::BF16, K::VEC>(r[u][c], f);
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) acc.v[c][e] = fmaf(w[u], f[e], acc.v[c][e]);
            }
    }
}

// ---- optional LDS staging of halo rows (section 5.2, "pipelined memory operation") -----------
// The rows of a remote partition are requested with global_load_lds: the data go from memory
// straight into this wavefront's LDS stage, holding no registers while in flight.  The local
// partition of the same pair is then accumulated through registers, and only afterwards does
// the wavefront wait for the staged rows and add them.  One stage holds kStageInstr load
// instructions (1 KB each: 64/LPR rows).  Only for 16-byte vectors and one chunk per lane.
constexpr int kStageInstr = 8;

template <class K>
__device__ __forceinline__ void stage_halo_rows(uint4 (*stage)[kWave], const typename K::elem *table, int64_t ld,
                                                int my_idx, int len, int t0, int sub, int lis, int nvec)
{
#pragma unroll
    for (int u = 0; u < kStageInstr; ++u) {
        if ((t0 + u) * K::NPW >= len) break;                     // wave-uniform
        const int j = (t0 + u) * K::NPW + sub;
        const int idx = __shfl(my_idx, j & 63);
        const bool ok = j < len && lis < nvec;
        // lanes with nothing to fetch read the first bytes of the table (always valid memory)
        const typename K::elem *src = ok ? table + static_cast<int64_t>(idx) * ld + static_cast<int64_t>(lis) * K::VEC : table;
        typedef const __attribute__((address_space(1))) void *gptr_t;
        typedef __attribute__((address_space(3))) void *lptr_t;
        __builtin_amdgcn_global_load_lds((gptr_t)(const void *)src, (lptr_t)(void *)&stage[u][0], 16, 0, 0);
    }
}

template <class K>
__device__ __forceinline__ void consume_staged_rows(Acc<K> &acc, uint4 (*stage)[kWave], const typename K::elem *table,
                                                    int64_t ld, int my_idx, float my_w, int len, int sub, int lis,
                                                    int nvec, int lane)
{
    const int steps = (len + K::NPW - 1) / K::NPW;
    for (int t0 = 0; t0 < steps; t0 += kStageInstr) {
        if (t0 > 0) stage_halo_rows<K>(stage, table, ld, my_idx, len, t0, sub, lis, nvec);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // staged rows have landed in LDS
#pragma unroll
        for (int u = 0; u < kStageInstr; ++u) {
            if ((t0 + u) * K::NPW >= len) break;
            const int j = (t0 + u) * K::NPW + sub;
            const float wj = __shfl(my_w, j & 63);
            const bool ok = j < len && lis < nvec;
            uint4 q = stage[u][lane];
            if (!ok) q = make_uint4(0u, 0u, 0u, 0u);
            typename K::raw r;
            __builtin_memcpy(&r, &q, sizeof r);
            float f[K::VEC];
            unpack<K::BF16, K::VEC>(r, f);
            const float w = ok ? wj : 0.f;
#pragma unroll
            for (int e = 0; e < K::VEC; ++e) acc.v[0][e] = fmaf(w, f[e], acc.v[0][e]);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // stage is free for the next batch
    }
}

template <class K, bool LDSH>
__global__ __launch_bounds__(kWave * kMaxWpb) void aggregate_kernel(const AggArgs a)
{
    __shared__ uint4 stage_all[LDSH ? kWavesPerBlock : 1][LDSH ? kStageInstr : 1][LDSH ? kWave : 1];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int wpb = static_cast<int>(blockDim.x) / kWave;   // wavefronts (work items) per workgroup
    const int sub = lane / K::LPR;      // which neighbour row of a load instruction
    // first vector of the row this lane owns: lane inside the sub-wave, shifted to the column slab
    const int lis = lane % K::LPR + static_cast<int>(blockIdx.y) * a.slab_vecs;
    const int vend = min(a.nvec, (static_cast<int>(blockIdx.y) + 1) * a.slab_vecs);   // end of the slab
    const typename K::elem *xl = static_cast<const typename K::elem *>(a.x_local);
    const typename K::elem *xh = static_cast<const typename K::elem *>(a.x_halo);
    const bool gcn = a.gcn != 0;
    Acc<K> acc;
    acc.clear();

    if (static_cast<int>(blockIdx.x) < a.n_item_blocks) {
        // ---- one work item per wavefront ----------------------------------------------------
        const int item_id = __builtin_amdgcn_readfirstlane(static_cast<int>(blockIdx.x) * wpb + wave);
        if (item_id >= a.n_items) return;
        const WorkItem it = a.items[item_id];
        if (it.row < 0) return;                         // padding item
        const int ps = a.ps;
        const int n_l = a.phase == 2 ? 0 : it.lend - it.lbeg, n_r = a.phase == 1 ? 0 : it.rend - it.rbeg;
        const int g_l = (n_l + ps - 1) / ps, g_r = (n_r + ps - 1) / ps;
        const int g_n = g_l > g_r ? g_l : g_r;
        int idx_l, idx_r, nidx_l = 0, nidx_r = 0;
        float w_l, w_r, nw_l = 0.f, nw_r = 0.f;
        load_partition_ids(a.local_col, a.w_local, it.lbeg, min(ps, n_l), lane, gcn, idx_l, w_l);
        load_partition_ids(a.remote_col, a.w_remote, it.rbeg, min(ps, n_r), lane, gcn, idx_r, w_r);
        for (int g = 0; g < g_n; ++g) {
            // ids of the next pair are requested before this pair's rows are gathered
            const int off = (g + 1) * ps;
            load_partition_ids(a.local_col, a.w_local, it.lbeg + off, min(ps, n_l - off), lane, gcn, nidx_l, nw_l);
            load_partition_ids(a.remote_col, a.w_remote, it.rbeg + off, min(ps, n_r - off), lane, gcn, nidx_r, nw_r);
            const int len_l = min(ps, n_l - g * ps), len_r = min(ps, n_r - g * ps);
            if constexpr (LDSH) {
                uint4 (*stage)[kWave] = stage_all[wave];
                if (len_r > 0) stage_halo_rows<K>(stage, xh, a.ld_x, idx_r, len_r, 0, sub, lis, vend);
                if (len_l > 0) accumulate_partition<K>(acc, xl, a.ld_x, idx_l, w_l, len_l, sub, lis, vend);
                if (len_r > 0) consume_staged_rows<K>(acc, stage, xh, a.ld_x, idx_r, w_r, len_r, sub, lis, vend, lane);
            } else {
                if (len_l > 0) accumulate_partition<K>(acc, xl, a.ld_x, idx_l, w_l, len_l, sub, lis, vend);
                if (len_r > 0) accumulate_partition<K>(acc, xh, a.ld_x, idx_r, w_r, len_r, sub, lis, vend);
            }
            idx_l = nidx_l; w_l = nw_l; idx_r = nidx_r; w_r = nw_r;
        }
        // combine the sub-wave accumulators: lanes with equal `lis` hold the same columns
#pragma unroll
        for (int off = K::LPR; off < kWave; off <<= 1)
#pragma unroll
            for (int c = 0; c < K::CH; ++c)
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) acc.v[c][e] += __shfl_xor(acc.v[c][e], off);
        if (sub == 0) {
            if (it.slot < 0) write_final<K>(a, acc, it.row, lis, vend);
            else write_partial<K>(a, acc, it.slot, lis, vend);
        }
    } else {
        // ---- short rows: one per sub-wave -----------------------------------------------------
        const int w_id = (static_cast<int>(blockIdx.x) - a.n_item_blocks) * wpb + wave;
        const int s_id = w_id * K::NPW + sub;
        if (s_id >= a.n_short) return;
        const int32_t row = a.short_rows[s_id];
        if (a.phase != 2)
            accumulate_list<K>(acc, xl, a.ld_x, a.local_col, a.w_local, a.local_row_ptr[row], a.local_row_ptr[row + 1],
                               gcn, lis, vend);
        if (a.phase != 1)
            accumulate_list<K>(acc, xh, a.ld_x, a.remote_col, a.w_remote, a.remote_row_ptr[row], a.remote_row_ptr[row + 1],
                               gcn, lis, vend);
        write_final<K>(a, acc, row, lis, vend);
    }
}

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

template <class K>
hipError_t launch_cfg(const AggArgs &a, dim3 grid, int wpb, hipStream_t stream, bool lds_halo)
{
    if constexpr (K::CH == 1 && sizeof(typename K::raw) == 16) {
        if (lds_halo && wpb <= kWavesPerBlock) {
            hipLaunchKernelGGL((aggregate_kernel<K, true>), grid, dim3(kWave * wpb), 0, stream, a);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((aggregate_kernel<K, false>), grid, dim3(kWave * wpb), 0, stream, a);
    return hipGetLastError();
}

// LPR = smallest power of two >= nvec (at least 4, at most 64); CH = chunks per lane.
template <bool BF16, int VEC>
hipError_t dispatch_shape(const AggArgs &a, dim3 grid, int wpb, hipStream_t stream, int lpr, int ch, bool lds)
{
    if (lpr == 4) return launch_cfg<Cfg<BF16, VEC, 4, 1>>(a, grid, wpb, stream, lds);
    if (lpr == 8) return launch_cfg<Cfg<BF16, VEC, 8, 1>>(a, grid, wpb, stream, lds);
    if (lpr == 16) return launch_cfg<Cfg<BF16, VEC, 16, 1>>(a, grid, wpb, stream, lds);
    if (lpr == 32) return launch_cfg<Cfg<BF16, VEC, 32, 1>>(a, grid, wpb, stream, lds);
    if (ch == 1) return launch_cfg<Cfg<BF16, VEC, 64, 1>>(a, grid, wpb, stream, lds);
    if (ch == 2) return launch_cfg<Cfg<BF16, VEC, 64, 2>>(a, grid, wpb, stream, lds);
    if (ch <= 4) return launch_cfg<Cfg<BF16, VEC, 64, 4>>(a, grid, wpb, stream, lds);
    return launch_cfg<Cfg<BF16, VEC, 64, 8>>(a, grid, wpb, stream, lds);
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

mgg_status_t launch_aggregate(const mgg_partition *p, mgg_agg_t mode, float eps, mgg_dtype_t x_dtype,
                              const void *x_local, const void *x_halo, int32_t dim, int64_t ld_x, void *out,
                              int64_t ld_out, hipStream_t stream, const float *bias, mgg_act_t act, int32_t out_dim,
                              mgg_dtype_t out_dtype)
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
        const int64_t opt = option_col_slab_bytes();
        const int64_t vec_bytes = static_cast<int64_t>(vec) * static_cast<int64_t>(esz);
        int64_t slab_bytes = 0;
        if (opt == 0) {
            // automatic: measured on MI355X, slabs pay (1.1-1.5x) when rows are at least 1 KB wide and one
            // XCD's share of the table rows, at slab width, stays within a few times its 4 MB L2: 512-byte
            // slabs when that share is at most 8 MB, else 256-byte slabs if those get it there (the
            // 233 k x 2.4 KB table of the configs: 18.7 ms against 20.5 with 512 and 20.4 with 128), else
            // 512-byte slabs up to 16 MB; narrower slabs or larger tables lose to the extra passes
            const int64_t table_rows = p->n_own + static_cast<int64_t>(p->halo_gid.size());
            const int64_t class_rows = (p->xcd_min_deg > 0 ? table_rows / kXcd : table_rows) + 1;
            if (static_cast<int64_t>(dim) * static_cast<int64_t>(esz) >= 1024) {
                if (class_rows * 512 <= (8 << 20)) slab_bytes = 512;
                else if (class_rows * 256 <= (8 << 20)) slab_bytes = 256;
                else if (class_rows * 512 <= (16 << 20)) slab_bytes = 512;
            }
        } else if (opt >= 64) {
            slab_bytes = opt;
        }
        if (slab_bytes > 0 && slab_bytes % vec_bytes == 0 && slab_bytes / vec_bytes < nvec) slab_vecs = static_cast<int>(slab_bytes / vec_bytes);
    }
    // a lane holds at most 8 chunks of a row: wider rows are always walked in slabs of 512 vectors
    if (slab_vecs > 64 * 8) slab_vecs = 64 * 8;
    const int n_slabs = (nvec + slab_vecs - 1) / slab_vecs;
    if (n_slabs > 65535) return fail(MGG_ERR_UNSUPPORTED, "dim %d too wide (at most %d)", dim, 65535 * 64 * 8 * vec);
    int lpr = 4;
    while (lpr < slab_vecs && lpr < 64) lpr <<= 1;
    const int ch = (slab_vecs + 63) / 64;

    // scratch rows for the partial sums of split rows
    if (p->n_split_items > 0) {
        const int64_t need_ld = (static_cast<int64_t>(dim) + 7) / 8 * 8;
        if (p->d.scratch_ld < need_ld) {
            if (p->d.scratch) { MGG_HIP_TRY(hipDeviceSynchronize()); (void)hipFree(p->d.scratch); p->d.scratch = nullptr; p->d.scratch_ld = 0; }
            const size_t bytes = static_cast<size_t>(p->n_split_items) * need_ld * sizeof(float);
            hipError_t e = hipMalloc(reinterpret_cast<void **>(&p->d.scratch), bytes);
            if (e != hipSuccess) return fail(MGG_ERR_ALLOC, "hipMalloc(%zu bytes of scratch): %s", bytes, hipGetErrorString(e));
            p->d.scratch_ld = need_ld;
        }
    }

    AggArgs a{};
    a.local_row_ptr = p->d.local_row_ptr; a.local_col = p->d.local_col;
    a.remote_row_ptr = p->d.remote_row_ptr; a.remote_col = p->d.remote_col;
    a.dinv_own = p->d.dinv_own; a.w_local = p->d.w_local; a.w_remote = p->d.w_remote;
    a.short_rows = p->d.short_rows; a.items = p->d.items;
    a.x_local = x_local; a.x_halo = xh;
    a.out = out; a.scratch = p->d.scratch;
    a.ld_x = ld_x; a.ld_out = ld_out; a.scratch_ld = p->d.scratch_ld;
    a.nvec = nvec;
    a.slab_vecs = slab_vecs;
    a.n_items = static_cast<int32_t>(p->items.size());
    const int wpb = p->wpb;
    a.n_item_blocks = (a.n_items + wpb - 1) / wpb;
    a.n_short = static_cast<int32_t>(p->short_rows.size());
    a.ps = p->ps;
    a.gcn = mode == MGG_AGG_GCN_SYM;
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
    const bool two_phases = option_split_phases() != 0 && !p->halo_gid.empty() && !a.out_bf16;   // phase 2 reads `out` back
    for (int phase = two_phases ? 1 : 0; phase <= (two_phases ? 2 : 0); ++phase) {
        a.phase = phase;
        const int npw = 64 / lpr;
        const int short_waves = (a.n_short + npw - 1) / npw;
        int grid_x = a.n_item_blocks + (short_waves + wpb - 1) / wpb;
        if (n_slabs > 1) grid_x = (grid_x + kXcd - 1) / kXcd * kXcd;   // keeps workgroup x on XCD x mod 8 in every slab
        const dim3 grid(static_cast<unsigned>(grid_x), static_cast<unsigned>(n_slabs));
        const bool lds = option_lds_halo() != 0 && !p->halo_gid.empty();
        if (grid_x > 0) {
            hipError_t e;
            if (bf16) {
                if (vec == 8) e = dispatch_shape<true, 8>(a, grid, wpb, stream, lpr, ch, lds);
                else if (vec == 2) e = dispatch_shape<true, 2>(a, grid, wpb, stream, lpr, ch, lds);
                else e = dispatch_shape<true, 1>(a, grid, wpb, stream, lpr, ch, lds);
            } else {
                if (vec == 4) e = dispatch_shape<false, 4>(a, grid, wpb, stream, lpr, ch, lds);
                else if (vec == 2) e = dispatch_shape<false, 2>(a, grid, wpb, stream, lpr, ch, lds);
                else e = dispatch_shape<false, 1>(a, grid, wpb, stream, lpr, ch, lds);
            }
            if (e != hipSuccess) return hip_fail(e, "aggregate kernel launch");
        }
        const int32_t n_split = static_cast<int32_t>(p->split_rows.size());
        if (n_split > 0) {
            const dim3 fgrid(static_cast<unsigned>((n_split + kWavesPerBlock - 1) / kWavesPerBlock));
            const int32_t fix_vec_ok = (ld_out % 4 == 0) && aligned(out, a.out_bf16 ? 8 : 16);
            if (bf16)
                hipLaunchKernelGGL(fixup_kernel<true>, fgrid, dim3(kBlock), 0, stream, p->d.split_rows, n_split, out_dim, p->d.scratch,
                                   p->d.scratch_ld, x_local, ld_x, p->d.dinv_own, a.gcn, a.self_w, out, a.out_bf16, ld_out, fix_vec_ok, a.phase, bias, a.relu, a.no_self);
            else
                hipLaunchKernelGGL(fixup_kernel<false>, fgrid, dim3(kBlock), 0, stream, p->d.split_rows, n_split, out_dim, p->d.scratch,
                                   p->d.scratch_ld, x_local, ld_x, p->d.dinv_own, a.gcn, a.self_w, out, a.out_bf16, ld_out, fix_vec_ok, a.phase, bias, a.relu, a.no_self);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return hip_fail(e, "fix-up kernel launch");
        }
    }
    return MGG_OK;
}

}  // namespace mgg
