// Device code of the neighbour aggregation for gfx950 (section 1 "GNN" equation; section 4.1 LR / LL /
// AC stages; section 5.1 warp-per-partition mapping with local and remote work interleaved; section 5.2
// asynchronous remote access staged through shared memory).  Included by the translation units that
// instantiate the kernels for one element type each.
//
// Mapping, per 64-lane wavefront:
//   - a row of an embedding table is spread over LPR lanes (LPR = 4..64, a power of two), each lane
//     owning VEC contiguous elements per chunk (16-byte loads when the layout allows), so one load
//     instruction fetches NPW = 64/LPR neighbour rows;
//   - a work item is a run of neighbour partitions (<= ps neighbours each) of ONE owned row, local and
//     remote partitions taken alternately, so every wavefront mixes both kinds;
//   - the ids of a partition are loaded one per lane; the lane that holds an id turns it into the byte
//     offset of its table row once, and the offsets (and GCN factors) reach the lanes that gather
//     through cross-lane reads.  A gather is then one add and one load with a 32-bit offset from a
//     wave-uniform base, and the inner loop of full batches carries no predicate at all;
//   - the NPW sub-wave accumulators are combined with cross-lane shuffles at the end;
//   - short rows are handled one per sub-wave (several rows per wavefront);
//   - rows cut into several items leave raw partial sums in scratch rows, and a second small kernel
//     adds them in a fixed order (results do not depend on scheduling).
// Bound by the memory hierarchy (about 0.5 flop per byte): no MFMA here.
#pragma once

#include <hip/hip_runtime.h>

#include <type_traits>

#include "mgg_internal.h"

namespace mgg {

#ifndef MGG_AGG_INFLIGHT
#define MGG_AGG_INFLIGHT 8          // loads a lane keeps in flight per batch
#endif
constexpr int kWave = 64;
constexpr int kMaxWpb = 16;         // wavefronts per workgroup of the aggregation kernel
constexpr int kStageSlots = 8;      // LDS-staged variant: load instructions (1 KB each) per wavefront stage
constexpr int kStageWpb = 8;        // LDS-staged variant: most wavefronts per workgroup (a wavefront owns 2 stages of 8 KB)

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
    int32_t items_per_wave;  // work items a wavefront takes one after the other (M)
    int32_t short_per_wave;  // groups of 64/LPR short rows a wavefront takes one after the other
    const int4 *short_desc;  // per short row: row, start in local_col, start in remote_col, local count | remote count << 16
    int32_t ps;
    int32_t wide;            // a table reaches beyond 4 GB: row offsets are 64-bit
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
    // Wavefronts per SIMD the register allocation must allow.  The workgroup limit (16 wavefronts) gives 4;
    // the 256-byte fp32 variant sits one register above the budget of 5 and loses nothing when held to it
    // (2 % faster on the 602-column workload); the others would spill.
    static constexpr int MIN_WAVES = (!BF16_ && VEC_ == 4 && LPR_ == 16 && CH_ == 1) ? 5 : 4;
    using elem = typename std::conditional<BF16, uint16_t, float>::type;
    using raw = typename Raw<BF16, VEC>::type;
    static constexpr int VEC_BYTES = static_cast<int>(sizeof(raw));
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
    __device__ __forceinline__ void add(int c, const typename K::raw &r, float w)
    {
        float f[K::VEC];
        unpack<K::BF16, K::VEC>(r, f);
#pragma unroll
        for (int e = 0; e < K::VEC; ++e) v[c][e] = fmaf(w, f[e], v[c][e]);
    }
    __device__ __forceinline__ void add(int c, const typename K::raw &r)      // weight 1
    {
        float f[K::VEC];
        unpack<K::BF16, K::VEC>(r, f);
#pragma unroll
        for (int e = 0; e < K::VEC; ++e) v[c][e] += f[e];
    }
};

// Where the lanes of a wavefront sit in a table row: the byte offset of each chunk this lane gathers.
// A lane whose columns lie beyond the end of the slab gathers the slab's last vector instead (valid
// memory, never written back), so that no load of the inner loop needs a predicate.
template <class K>
struct Lanes {
    int sub;                    // which neighbour row of a load instruction
    int lis;                    // first vector of the row this lane owns
    int vend;                   // end of the column slab (in vectors)
    uint32_t col_off[K::CH];
    __device__ __forceinline__ void init(const AggArgs &a, int lane)
    {
        sub = lane / K::LPR;
        lis = lane % K::LPR + static_cast<int>(blockIdx.y) * a.slab_vecs;
        vend = min(a.nvec, (static_cast<int>(blockIdx.y) + 1) * a.slab_vecs);
#pragma unroll
        for (int c = 0; c < K::CH; ++c) col_off[c] = static_cast<uint32_t>(min(c * K::LPR + lis, vend - 1)) * K::VEC_BYTES;
    }
};

// value of lane j of the wavefront; j is wave-uniform when one row takes the whole wavefront
template <class K>
__device__ __forceinline__ uint32_t lane_read(uint32_t v, int j)
{
    if constexpr (K::NPW == 1) return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), j));
    else return static_cast<uint32_t>(__shfl(static_cast<int>(v), j));
}

template <class K, bool WIDE>
__device__ __forceinline__ typename K::raw load_row_chunk(const char *table, uint32_t off_lo, uint32_t off_hi, uint32_t col)
{
    if constexpr (WIDE) {
        const uint64_t off = (static_cast<uint64_t>(off_hi) << 32 | off_lo) + col;
        return *reinterpret_cast<const typename K::raw *>(table + off);
    } else if constexpr (K::NPW == 1) {
        return *reinterpret_cast<const typename K::raw *>((table + off_lo) + col);   // the row's address is wave-uniform
    } else {
        return *reinterpret_cast<const typename K::raw *>(table + (off_lo + col));   // 32-bit offset from a uniform base
    }
}

// Accumulate one neighbour partition.  `len` (<= 64) neighbours: lane i holds the byte offset of the
// table row of neighbour i (off_lo / off_hi) and, for GCN, its factor; sub-wave `sub` takes neighbours
// sub, sub + NPW, ...  Batches of U load steps; the batches in which every sub-wave has a neighbour run
// without predicates, at most one last batch clamps the neighbour index and drops what it must not add.
template <class K, bool GCN, bool WIDE>
__device__ __forceinline__ void accumulate_partition(Acc<K> &acc, const char *table, uint32_t off_lo, uint32_t off_hi,
                                                     float my_w, int len, const Lanes<K> &ln)
{
    const int full_steps = len / K::NPW, steps = (len + K::NPW - 1) / K::NPW;
    int t0 = 0;
    for (; t0 + K::U <= full_steps; t0 += K::U) {
        typename K::raw r[K::U][K::CH];
        float w[K::U];
#pragma unroll
        for (int u = 0; u < K::U; ++u) {
            const int j = (t0 + u) * K::NPW + ln.sub;
            const uint32_t lo = lane_read<K>(off_lo, j);
            const uint32_t hi = WIDE ? lane_read<K>(off_hi, j) : 0u;
            if constexpr (GCN) w[u] = __uint_as_float(lane_read<K>(__float_as_uint(my_w), j));
#pragma unroll
            for (int c = 0; c < K::CH; ++c) r[u][c] = load_row_chunk<K, WIDE>(table, lo, hi, ln.col_off[c]);
        }
#pragma unroll
        for (int u = 0; u < K::U; ++u)
#pragma unroll
            for (int c = 0; c < K::CH; ++c) {
                if constexpr (GCN) acc.add(c, r[u][c], w[u]);
                else acc.add(c, r[u][c]);
            }
    }
    if (t0 < steps) {                       // at most U steps are left
        typename K::raw r[K::U][K::CH];
        float w[K::U];
        bool ok[K::U];
#pragma unroll
        for (int u = 0; u < K::U; ++u) {
            const int j = (t0 + u) * K::NPW + ln.sub;
            ok[u] = j < len;
            const int jj = ok[u] ? j : 0;   // neighbour 0 exists: its row is valid memory
            const uint32_t lo = lane_read<K>(off_lo, jj);
            const uint32_t hi = WIDE ? lane_read<K>(off_hi, jj) : 0u;
            w[u] = GCN ? __uint_as_float(lane_read<K>(__float_as_uint(my_w), jj)) : 1.f;
            if ((t0 + u) * K::NPW < len) {  // wave-uniform
#pragma unroll
                for (int c = 0; c < K::CH; ++c) r[u][c] = load_row_chunk<K, WIDE>(table, lo, hi, ln.col_off[c]);
            } else {
#pragma unroll
                for (int c = 0; c < K::CH; ++c) __builtin_memset(&r[u][c], 0, sizeof r[u][c]);
                ok[u] = false;
            }
        }
#pragma unroll
        for (int u = 0; u < K::U; ++u)
#pragma unroll
            for (int c = 0; c < K::CH; ++c) {
                float f[K::VEC];
                unpack<K::BF16, K::VEC>(r[u][c], f);
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) acc.v[c][e] = fmaf(w[u], ok[u] ? f[e] : 0.f, acc.v[c][e]);   // a dropped row adds exactly nothing
            }
    }
}

// Ids (and GCN factors) of the partition starting at `pos`, one per lane; both arrays are read as
// coalesced streams (the factors are stored per edge, in the order of the column array).
template <bool GCN>
__device__ __forceinline__ void load_partition_ids(const int32_t *col, const float *wts, int pos, int len, int lane, int &idx, float &w)
{
    idx = 0; w = 0.f;
    if (lane < len) {
        idx = col[pos + lane];
        if constexpr (GCN) w = wts[pos + lane];
    }
}

template <bool WIDE>
__device__ __forceinline__ void row_offset(int idx, uint64_t ldb, uint32_t &lo, uint32_t &hi)
{
    if constexpr (WIDE) {
        const uint64_t o = static_cast<uint64_t>(static_cast<uint32_t>(idx)) * ldb;
        lo = static_cast<uint32_t>(o); hi = static_cast<uint32_t>(o >> 32);
    } else {
        lo = static_cast<uint32_t>(idx) * static_cast<uint32_t>(ldb); hi = 0u;
    }
}

// Final value of an owned row from its neighbour sum: adds the self term and the row factor.
template <class K>
__device__ __forceinline__ void write_final(const AggArgs &a, bool gcn, const Acc<K> &acc, const typename K::raw (&xs)[K::CH], int32_t row, int lis,
                                            int vend)
{
    float *o = static_cast<float *>(a.out) + static_cast<int64_t>(row) * a.ld_out;             // fp32 output
    uint16_t *ob = static_cast<uint16_t *>(a.out) + static_cast<int64_t>(row) * a.ld_out;     // bf16 output
    const float dv = gcn ? a.dinv_own[row] : 1.f;
    const float ws = gcn ? dv : a.self_w;     // GCN: dv * (sum + dv * x_v) = sum_u x_u/sqrt(du dv) + x_v/dv^2
#pragma unroll
    for (int c = 0; c < K::CH; ++c) {
        const int vi = c * K::LPR + lis;
        if (vi < vend) {
            float xv[K::VEC], r[K::VEC];
            if (a.no_self || a.phase == 2) {
#pragma unroll
                for (int e = 0; e < K::VEC; ++e) xv[e] = 0.f;
            } else {
                unpack<K::BF16, K::VEC>(xs[c], xv);         // requested when the item began
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

// ---- LDS staging of halo rows (section 5.2, "pipelined memory operation") -----------------------
// A wavefront owns two LDS stages of kStageSlots load instructions (1 KB each: NPW rows).  The rows of
// a remote partition are requested with global_load_lds -- memory to LDS, holding no registers while in
// flight -- one batch ahead: while batch k is being added from its stage, batch k + 1 is already on its
// way into the other stage, and the local partition of the pair is accumulated through registers in
// between.  Waits count outstanding loads (vmcnt(N)), so only the batch about to be consumed is waited
// for.  Only for 16-byte vectors and one chunk per lane.
typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

template <int N> __device__ __forceinline__ void wait_vmcnt()
{
    if constexpr (N <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else if constexpr (N == 1) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
    else if constexpr (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    else if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    else if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    else if constexpr (N == 16) asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// requests (up to) kStageSlots load steps of a remote partition, starting at step t0, into `stage`;
// always issues exactly kStageSlots instructions so that outstanding loads can be counted
template <class K>
__device__ __forceinline__ void stage_halo_batch(uint4 (*stage)[kWave], const char *table, uint32_t off_lo, int len, int t0,
                                                 const Lanes<K> &ln)
{
#pragma unroll
    for (int u = 0; u < kStageSlots; ++u) {
        const int j = (t0 + u) * K::NPW + ln.sub;
        const int jj = j < len ? j : 0;                       // neighbour 0 exists whenever a batch is staged
        const uint32_t lo = lane_read<K>(off_lo, jj);
        const char *src = table + (lo + ln.col_off[0]);
        __builtin_amdgcn_global_load_lds((gptr_t)(const void *)src, (lptr_t)(void *)&stage[u][0], 16, 0, 0);
    }
}

template <class K, bool GCN>
__device__ __forceinline__ void consume_stage(Acc<K> &acc, uint4 (*stage)[kWave], float my_w, int len, int t0, const Lanes<K> &ln, int lane)
{
#pragma unroll
    for (int u = 0; u < kStageSlots; ++u) {
        const int j = (t0 + u) * K::NPW + ln.sub;
        const bool ok = j < len;
        const float wj = GCN ? __uint_as_float(lane_read<K>(__float_as_uint(my_w), ok ? j : 0)) : 1.f;
        const uint4 q = stage[u][lane];
        typename K::raw r;
        __builtin_memcpy(&r, &q, sizeof r);
        float f[K::VEC];
        unpack<K::BF16, K::VEC>(r, f);
#pragma unroll
        for (int e = 0; e < K::VEC; ++e) acc.v[0][e] = fmaf(wj, ok ? f[e] : 0.f, acc.v[0][e]);
    }
}

// ---- the kernel -----------------------------------------------------------------------------------
// One work item after the other, M (a.items_per_wave) per wavefront, as a software pipeline: while the
// rows of one pair of partitions are gathered, the ids of the next pair -- of the same item or of the
// wavefront's next item -- are already on their way, the descriptor of the item after next has been
// requested, and the owned row's own embedding (needed only when the item is written out) was
// requested when the item began.  Nothing a wavefront needs next is first asked for when it is needed.
//
// Item descriptors travel as one dword per lane (lane f mod 8 holds field f of the 32-byte record)
// through the vector memory path, whose loads return in order behind the gathers already in flight.
struct ItemFields {
    int row, lbeg, lend, rbeg, rend, slot;
};
__device__ __forceinline__ ItemFields item_fields(int d)
{
    ItemFields f;
    f.row = __builtin_amdgcn_readlane(d, 0); f.lbeg = __builtin_amdgcn_readlane(d, 1); f.lend = __builtin_amdgcn_readlane(d, 2);
    f.rbeg = __builtin_amdgcn_readlane(d, 3); f.rend = __builtin_amdgcn_readlane(d, 4); f.slot = __builtin_amdgcn_readlane(d, 5);
    return f;
}

// the owned row's own embedding, requested ahead of its use in write_final
template <class K>
__device__ __forceinline__ void load_self_row(const AggArgs &a, int32_t row, const Lanes<K> &ln, typename K::raw (&xs)[K::CH])
{
    const char *base = static_cast<const char *>(a.x_local) + static_cast<int64_t>(row) * a.ld_x * static_cast<int64_t>(sizeof(typename K::elem));
#pragma unroll
    for (int c = 0; c < K::CH; ++c) xs[c] = *reinterpret_cast<const typename K::raw *>(base + ln.col_off[c]);
}

template <class K, bool GCN, bool WIDE>
__device__ __forceinline__ void gather_pair(Acc<K> &acc, const char *xl, const char *xh, uint64_t ldb, int idx_l, float w_l, int len_l,
                                            int idx_r, float w_r, int len_r, const Lanes<K> &ln)
{
    uint32_t lo, hi;
    if (len_l > 0) { row_offset<WIDE>(idx_l, ldb, lo, hi); accumulate_partition<K, GCN, WIDE>(acc, xl, lo, hi, w_l, len_l, ln); }
    if (len_r > 0) { row_offset<WIDE>(idx_r, ldb, lo, hi); accumulate_partition<K, GCN, WIDE>(acc, xh, lo, hi, w_r, len_r, ln); }
}

template <class K, bool GCN, bool LDSH>
__global__ __launch_bounds__(kWave * kMaxWpb) __attribute__((amdgpu_waves_per_eu(K::MIN_WAVES))) void aggregate_kernel(const AggArgs a)
{
    extern __shared__ uint4 stage_all[];        // LDS-staged variant: two stages of kStageSlots load instructions per wavefront
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / kWave);
    const int wpb = static_cast<int>(blockDim.x) / kWave;   // wavefronts per workgroup
    Lanes<K> ln;
    ln.init(a, lane);
    const char *xl = static_cast<const char *>(a.x_local);
    const char *xh = static_cast<const char *>(a.x_halo);
    const uint64_t ldb = static_cast<uint64_t>(a.ld_x) * sizeof(typename K::elem);
    const int ps = a.ps;
    Acc<K> acc;
    typename K::raw xs[K::CH];

    if (static_cast<int>(blockIdx.x) < a.n_item_blocks) {
        // ---- work items: M per wavefront.  Workgroup b runs on XCD b mod 8 and takes M consecutive
        // groups (of wpb items) of that XCD's queue; groups are interleaved XCD by XCD in `items`.
        const int M = a.items_per_wave;
        const int qb = static_cast<int>(blockIdx.x) / kXcd, xc = static_cast<int>(blockIdx.x) % kXcd;
        const int32_t *items32 = reinterpret_cast<const int32_t *>(a.items);
        auto load_desc = [&](int k) -> int {
            const int id = ((qb * M + k) * kXcd + xc) * wpb + wave;        // wave-uniform
            if (k < M && id < a.n_items) return items32[static_cast<int64_t>(id) * 8 + (lane & 7)];
            return -1;                                                      // nothing there: reads as a padding item
        };
        int d_cur = load_desc(0), d_nxt = load_desc(1);
        bool ids_ready = false;
        int idx_l = 0, idx_r = 0;
        float w_l = 0.f, w_r = 0.f;
        for (int k = 0; k < M; ++k) {
            const int d_nn = load_desc(k + 2);
            const ItemFields it = item_fields(d_cur);
            if (it.row >= 0) {
                const int n_l = a.phase == 2 ? 0 : it.lend - it.lbeg, n_r = a.phase == 1 ? 0 : it.rend - it.rbeg;
                const int g_l = (n_l + ps - 1) / ps, g_r = (n_r + ps - 1) / ps;
                const int g_n = g_l > g_r ? g_l : g_r;
                if (!ids_ready) {
                    load_partition_ids<GCN>(a.local_col, a.w_local, it.lbeg, min(ps, n_l), lane, idx_l, w_l);
                    load_partition_ids<GCN>(a.remote_col, a.w_remote, it.rbeg, min(ps, n_r), lane, idx_r, w_r);
                }
                const ItemFields nx = item_fields(d_nxt);
                const int nn_l = a.phase == 2 ? 0 : nx.lend - nx.lbeg, nn_r = a.phase == 1 ? 0 : nx.rend - nx.rbeg;
                const bool wants_self = it.slot < 0 && !a.no_self && a.phase != 2;
                if (wants_self) load_self_row<K>(a, it.row, ln, xs);
                acc.clear();
                for (int g = 0; g < g_n; ++g) {
                    // ids of the next pair -- of this item, or the first pair of the next one
                    int nidx_l = 0, nidx_r = 0;
                    float nw_l = 0.f, nw_r = 0.f;
                    if (g + 1 < g_n) {
                        const int off = (g + 1) * ps;
                        load_partition_ids<GCN>(a.local_col, a.w_local, it.lbeg + off, min(ps, n_l - off), lane, nidx_l, nw_l);
                        load_partition_ids<GCN>(a.remote_col, a.w_remote, it.rbeg + off, min(ps, n_r - off), lane, nidx_r, nw_r);
                    } else if (nx.row >= 0) {
                        load_partition_ids<GCN>(a.local_col, a.w_local, nx.lbeg, min(ps, nn_l), lane, nidx_l, nw_l);
                        load_partition_ids<GCN>(a.remote_col, a.w_remote, nx.rbeg, min(ps, nn_r), lane, nidx_r, nw_r);
                    }
                    const int len_l = min(ps, n_l - g * ps), len_r = min(ps, n_r - g * ps);
                    if (a.wide) {
                        gather_pair<K, GCN, true>(acc, xl, xh, ldb, idx_l, w_l, len_l, idx_r, w_r, len_r, ln);
                    } else if constexpr (LDSH) {
                        // remote rows travel into LDS one batch ahead of their accumulation; the local partition
                        // of the pair is gathered through registers while the first batch is in flight
                        uint4 (*stage)[kStageSlots][kWave] = reinterpret_cast<uint4 (*)[kStageSlots][kWave]>(stage_all + static_cast<size_t>(wave) * 2 * kStageSlots * kWave);
                        uint32_t lo_l, lo_r, hi;
                        row_offset<false>(idx_l, ldb, lo_l, hi);
                        row_offset<false>(idx_r, ldb, lo_r, hi);
                        const int steps_r = len_r > 0 ? (len_r + K::NPW - 1) / K::NPW : 0;
                        if (steps_r > 0) stage_halo_batch<K>(stage[0], xh, lo_r, len_r, 0, ln);
                        if (len_l > 0) accumulate_partition<K, GCN, false>(acc, xl, lo_l, 0u, w_l, len_l, ln);
                        int buf = 0;
                        for (int t0 = 0; t0 < steps_r; t0 += kStageSlots, buf ^= 1) {
                            if (t0 + kStageSlots < steps_r) {
                                stage_halo_batch<K>(stage[buf ^ 1], xh, lo_r, len_r, t0 + kStageSlots, ln);
                                wait_vmcnt<kStageSlots>();          // everything but the batch just requested has landed
                            } else {
                                wait_vmcnt<0>();
                            }
                            consume_stage<K, GCN>(acc, stage[buf], w_r, len_r, t0, ln, lane);
                            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this stage is free again
                        }
                    } else {
                        gather_pair<K, GCN, false>(acc, xl, xh, ldb, idx_l, w_l, len_l, idx_r, w_r, len_r, ln);
                    }
                    idx_l = nidx_l; w_l = nw_l; idx_r = nidx_r; w_r = nw_r;
                }
                ids_ready = g_n > 0 && nx.row >= 0;
                // combine the sub-wave accumulators: lanes with equal `lis` hold the same columns
#pragma unroll
                for (int off = K::LPR; off < kWave; off <<= 1)
#pragma unroll
                    for (int c = 0; c < K::CH; ++c)
#pragma unroll
                        for (int e = 0; e < K::VEC; ++e) acc.v[c][e] += __shfl_xor(acc.v[c][e], off);
                if (ln.sub == 0) {
                    if (it.slot < 0) write_final<K>(a, GCN, acc, xs, it.row, ln.lis, ln.vend);
                    else write_partial<K>(a, acc, it.slot, ln.lis, ln.vend);
                }
            } else {
                ids_ready = false;
            }
            d_cur = d_nxt; d_nxt = d_nn;
        }
    } else {
        // ---- short rows: one per sub-wave, a.short_per_wave groups of NPW rows per wavefront --------
        // A 16-byte record per short row (row, start of its two lists, their lengths) is requested two
        // groups ahead, the first ids of both lists one group ahead.  The sub-wave's lanes fetch ids LPR
        // at a time, turn them into row offsets and hand them round inside the sub-wave.
        const int Ms = a.short_per_wave;
        const int sw = (static_cast<int>(blockIdx.x) - a.n_item_blocks) * wpb + wave;
        const int lane_in_sub = lane % K::LPR, sub_base = lane - lane_in_sub;
        auto load_sd = [&](int k) -> int4 {
            const int64_t s_id = (static_cast<int64_t>(sw) * Ms + k) * K::NPW + ln.sub;
            if (k < Ms && s_id < a.n_short) return a.short_desc[s_id];
            return make_int4(-1, 0, 0, 0);
        };
        // first block of ids of both lists of the row described by sd
        auto load_first_ids = [&](const int4 &sd, int &il, float &wl, int &ir, float &wr) {
            il = 0; ir = 0; wl = 0.f; wr = 0.f;
            if (sd.x < 0) return;
            const int nl = a.phase == 2 ? 0 : (sd.w & 0xffff), nr = a.phase == 1 ? 0 : static_cast<int>(static_cast<uint32_t>(sd.w) >> 16);
            if (lane_in_sub < nl) { il = a.local_col[sd.y + lane_in_sub]; if constexpr (GCN) wl = a.w_local[sd.y + lane_in_sub]; }
            if (lane_in_sub < nr) { ir = a.remote_col[sd.z + lane_in_sub]; if constexpr (GCN) wr = a.w_remote[sd.z + lane_in_sub]; }
        };
        int4 sd_cur = load_sd(0), sd_nxt = load_sd(1);
        int fi_l, fi_r;
        float fw_l, fw_r;
        load_first_ids(sd_cur, fi_l, fw_l, fi_r, fw_r);
        for (int k = 0; k < Ms; ++k) {
            if ((static_cast<int64_t>(sw) * Ms + k) * K::NPW >= a.n_short) break;       // wave-uniform: nothing left
            const int4 sd_nn = load_sd(k + 2);
            int ni_l, ni_r;
            float nw_l, nw_r;
            load_first_ids(sd_nxt, ni_l, nw_l, ni_r, nw_r);
            const bool have = sd_cur.x >= 0;
            const int32_t row = have ? sd_cur.x : 0;
            if (have && !a.no_self && a.phase != 2) load_self_row<K>(a, row, ln, xs);
            acc.clear();
            for (int side = 0; side < 2; ++side) {
                if (side == 0 ? a.phase == 2 : a.phase == 1) continue;
                const int32_t *col = side == 0 ? a.local_col : a.remote_col;
                const float *wts = side == 0 ? a.w_local : a.w_remote;
                const char *table = side == 0 ? xl : xh;
                const int beg = side == 0 ? sd_cur.y : sd_cur.z;
                const int n = have ? (side == 0 ? (sd_cur.w & 0xffff) : static_cast<int>(static_cast<uint32_t>(sd_cur.w) >> 16)) : 0;
                // longest list among the sub-waves of this wavefront (wave-uniform loop bound)
                int n_max = n;
#pragma unroll
                for (int off = K::LPR; off < kWave; off <<= 1) n_max = max(n_max, __shfl_xor(n_max, off));
                n_max = __builtin_amdgcn_readfirstlane(n_max);
                for (int b0 = 0; b0 < n_max; b0 += K::LPR) {
                    int idx = side == 0 ? fi_l : fi_r;
                    float w = side == 0 ? fw_l : fw_r;
                    if (b0 > 0) {                                     // lists longer than a sub-wave: fetched as they come
                        idx = 0; w = 0.f;
                        if (b0 + lane_in_sub < n) {
                            idx = col[beg + b0 + lane_in_sub];
                            if constexpr (GCN) w = wts[beg + b0 + lane_in_sub];
                        }
                    }
                    uint32_t lo, hi;
                    if (a.wide) row_offset<true>(idx, ldb, lo, hi); else row_offset<false>(idx, ldb, lo, hi);
                    const int cnt = min(K::LPR, n - b0);                     // this sub-wave's neighbours in the block (may be <= 0)
                    const int cnt_max = min(K::LPR, n_max - b0);             // wave-uniform
                    for (int j0 = 0; j0 < cnt_max; j0 += K::U) {
                        typename K::raw r[K::U][K::CH];
                        float wv[K::U];
                        bool ok[K::U];
#pragma unroll
                        for (int u = 0; u < K::U; ++u) {
                            ok[u] = j0 + u < cnt;
                            const int src = sub_base + (ok[u] ? j0 + u : 0);
                            const uint32_t l = static_cast<uint32_t>(__shfl(static_cast<int>(lo), src));
                            const uint32_t h = a.wide ? static_cast<uint32_t>(__shfl(static_cast<int>(hi), src)) : 0u;
                            wv[u] = GCN ? __shfl(w, src) : 1.f;
                            if (j0 + u < cnt_max) {     // wave-uniform; a sub-wave with nothing left re-reads a row it has and drops it
#pragma unroll
                                for (int c = 0; c < K::CH; ++c)
                                    r[u][c] = a.wide ? load_row_chunk<K, true>(table, l, h, ln.col_off[c]) : load_row_chunk<K, false>(table, l, 0u, ln.col_off[c]);
                            } else {
#pragma unroll
                                for (int c = 0; c < K::CH; ++c) __builtin_memset(&r[u][c], 0, sizeof r[u][c]);
                                ok[u] = false;
                            }
                        }
#pragma unroll
                        for (int u = 0; u < K::U; ++u)
#pragma unroll
                            for (int c = 0; c < K::CH; ++c) {
                                float f[K::VEC];
                                unpack<K::BF16, K::VEC>(r[u][c], f);
#pragma unroll
                                for (int e = 0; e < K::VEC; ++e) acc.v[c][e] = fmaf(wv[u], ok[u] ? f[e] : 0.f, acc.v[c][e]);
                            }
                    }
                }
            }
            if (have) write_final<K>(a, GCN, acc, xs, row, ln.lis, ln.vend);
            sd_cur = sd_nxt; sd_nxt = sd_nn;
            fi_l = ni_l; fw_l = nw_l; fi_r = ni_r; fw_r = nw_r;
        }
    }
}

template <class K>
hipError_t launch_cfg(const AggArgs &a, bool gcn, dim3 grid, int wpb, hipStream_t stream, bool lds_halo)
{
    if constexpr (K::CH == 1 && sizeof(typename K::raw) == 16) {
        if (lds_halo && wpb <= kStageWpb && !a.wide) {
            const size_t lds = static_cast<size_t>(wpb) * 2 * kStageSlots * kWave * sizeof(uint4);     // 16 KB per wavefront
            if (gcn) hipLaunchKernelGGL((aggregate_kernel<K, true, true>), grid, dim3(kWave * wpb), lds, stream, a);
            else hipLaunchKernelGGL((aggregate_kernel<K, false, true>), grid, dim3(kWave * wpb), lds, stream, a);
            return hipGetLastError();
        }
    }
    if (gcn) hipLaunchKernelGGL((aggregate_kernel<K, true, false>), grid, dim3(kWave * wpb), 0, stream, a);
    else hipLaunchKernelGGL((aggregate_kernel<K, false, false>), grid, dim3(kWave * wpb), 0, stream, a);
    return hipGetLastError();
}

// LPR = smallest power of two >= the vectors of a slab (at least 4, at most 64); CH = chunks per lane.
template <bool BF16, int VEC>
hipError_t dispatch_shape(const AggArgs &a, bool gcn, dim3 grid, int wpb, hipStream_t stream, int lpr, int ch, bool lds)
{
    if (lpr == 4) return launch_cfg<Cfg<BF16, VEC, 4, 1>>(a, gcn, grid, wpb, stream, lds);
    if (lpr == 8) return launch_cfg<Cfg<BF16, VEC, 8, 1>>(a, gcn, grid, wpb, stream, lds);
    if (lpr == 16) return launch_cfg<Cfg<BF16, VEC, 16, 1>>(a, gcn, grid, wpb, stream, lds);
    if (lpr == 32) return launch_cfg<Cfg<BF16, VEC, 32, 1>>(a, gcn, grid, wpb, stream, lds);
    if (ch == 1) return launch_cfg<Cfg<BF16, VEC, 64, 1>>(a, gcn, grid, wpb, stream, lds);
    if (ch == 2) return launch_cfg<Cfg<BF16, VEC, 64, 2>>(a, gcn, grid, wpb, stream, lds);
    return launch_cfg<Cfg<BF16, VEC, 64, 4>>(a, gcn, grid, wpb, stream, lds);      // ch <= 4: the host cuts wider rows into slabs
}

// one translation unit per element type (aggregate_f32.hip, aggregate_bf16.hip)
hipError_t launch_aggregate_f32(const AggArgs &a, bool gcn, int vec, dim3 grid, int wpb, hipStream_t stream, int lpr, int ch, bool lds);
hipError_t launch_aggregate_bf16(const AggArgs &a, bool gcn, int vec, dim3 grid, int wpb, hipStream_t stream, int lpr, int ch, bool lds);

}  // namespace mgg
