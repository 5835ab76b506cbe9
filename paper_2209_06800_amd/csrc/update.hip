// Dense Update for gfx950 (section 1: Update is a fully-connected layer; section 7: X W with
// ReLU, and GIN's MLP): out = act(A . W + bias) on the matrix cores.
//
// Shape of the problem: A is tall (10^5..10^6 rows) and both d_in and d_out are small
// (16..602).  A workgroup of four wavefronts covers a tile of (32*WM) rows x (NT*32*WN)
// columns, WM*WN = 4; each wavefront owns 32 rows x NT*32 columns (NT <= 4, so that three
// wavefronts fit a SIMD and the load phase of one overlaps the MFMA phase of another; NT = 8 with
// two wavefronts per SIMD in the two-slab fp32 kernel, where a row of A is then read only once):
//   - A goes straight from HBM into registers in the MFMA operand layout, the fragment of the
//     next K slab being requested before the current slab is multiplied (no LDS round trip);
//   - W is staged slab by slab in LDS and shared by the workgroup;
//   - fp32 weights use v_mfma_f32_32x32x2_f32, bf16 weights v_mfma_f32_32x32x16_bf16,
//     both with fp32 accumulators; bias, ReLU and the output rounding are fused.
// MFMA sums over k in any order, so a lane takes whichever k values are contiguous for it in
// memory as long as the A and W operands agree; that makes the direct loads of A full-width.
//
// launch_update picks per shape: the whole-line kernels of update_stream.hip where they apply
// (HBM-bound shapes with whole K slabs), the kernels of this file otherwise -- weights resident in
// LDS with a grid sized to the chip, or staged slab by slab (two slabs in LDS for the fp32 MFMA,
// filled by loads that go from global memory straight into LDS).
// Row softmax runs as a second pass over the output.
#include <hip/hip_runtime.h>

#include "update_common.h"

namespace mgg {

namespace {

using namespace upd;

// ---- fp32 weights: v_mfma_f32_32x32x2_f32 ---------------------------------------------------
// K slab of 32: lane (i, h) holds A[m0+i][k0 + 16h .. k0 + 16h + 15]; MFMA number c contracts
// the k pair {k0 + c, k0 + 16 + c}.  W slab in LDS as [32][NC] floats.
// arow always points at a valid row (rows past the end are clamped to the last one and never
// stored), so the only predicate is the wave-uniform "this slab is complete and aligned".
__device__ __forceinline__ void load_a_f32(const UpdArgs &p, const float *arow, int kb, int k_slab_end, float (&af)[16])
{
    if (p.a_vec_ok && k_slab_end <= p.d_in) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 v = *reinterpret_cast<const float4 *>(arow + kb + 4 * q);
            af[4 * q] = v.x; af[4 * q + 1] = v.y; af[4 * q + 2] = v.z; af[4 * q + 3] = v.w;
        }
    } else if (p.a_vec_ok) {
        // the last, incomplete slab of aligned rows: whole 16-byte pieces as long as they start inside the
        // row (the leading dimension is a multiple of 4, so such a piece ends inside it too), then the
        // elements past d_in -- padding of the row -- are cleared
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = kb + 4 * q;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k < p.d_in) v = *reinterpret_cast<const float4 *>(arow + k);
            af[4 * q] = v.x;
            af[4 * q + 1] = k + 1 < p.d_in ? v.y : 0.f;
            af[4 * q + 2] = k + 2 < p.d_in ? v.z : 0.f;
            af[4 * q + 3] = k + 3 < p.d_in ? v.w : 0.f;
        }
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) af[e] = (kb + e < p.d_in) ? arow[kb + e] : 0.f;
    }
}

template <int NT, int WN>
__global__ __launch_bounds__(kThreads) void update_f32_kernel(const UpdArgs p)
{
    constexpr int BK = 32, NC = NT * 32 * WN, WM = kWaves / WN;
    __shared__ __attribute__((aligned(16))) float w_lds[BK * NC];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = (static_cast<int64_t>(blockIdx.x) * WM + wm) * 32;
    const int nb = blockIdx.y * NC;                 // first column of the workgroup
    const int n0 = nb + wn * NT * 32;               // first column of this wavefront
    const float *W = static_cast<const float *>(p.w);
    const int64_t row = m0 + i < p.n_rows ? m0 + i : p.n_rows - 1;
    const float *arow = static_cast<const float *>(p.a) + row * p.ld_a;

    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    float af[16], an[16];
    load_a_f32(p, arow, 16 * h, BK, af);
#pragma unroll 1
    for (int k0 = 0; k0 < p.d_in; k0 += BK) {
        if (k0 + BK < p.d_in) load_a_f32(p, arow, k0 + BK + 16 * h, k0 + 2 * BK, an);   // next slab's fragment
        __syncthreads();
        fill_w_f32<NC>(w_lds, W, k0, BK, nb, p);
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const float *wrow = w_lds + (16 * h + c) * NC + wn * NT * 32 + i;
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(wrow[t * 32], af[c], acc[t], 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 16; ++c) af[c] = an[c];
    }
    store_tiles<NT>(p, acc, m0, n0, lane);
}

// The same tile with two W slabs in LDS and workgroups that stay: the grid is sized to the chip and a
// workgroup walks over row tiles.  (tile, K slab) pairs form one sequence; while one pair is multiplied
// the next pair's W slab travels from global memory straight into the other LDS buffer and its A
// fragment into registers -- also across the end of a tile, so the stores of a finished tile and the
// first loads of the next one overlap with MFMAs instead of ending and starting a workgroup.  A slab
// costs one barrier.  For weight matrices whose rows allow 16-byte loads and whose width is a whole
// number of workgroup tiles.
extern __shared__ __attribute__((aligned(16))) unsigned char w_db[];
typedef const __attribute__((address_space(1))) void *gptr_t;
typedef __attribute__((address_space(3))) void *lptr_t;

template <int NT, int WN>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void update_f32_db_kernel(const UpdArgs p, int64_t n_tiles)
{
    constexpr int BK = 32, NC = NT * 32 * WN, WM = kWaves / WN;
    constexpr int UNITS = BK * NC / 4 / kThreads;          // 16-byte pieces of a W slab per thread
    float *w_lds = reinterpret_cast<float *>(w_db);         // [2][BK * NC]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    const int nb = blockIdx.y * NC;
    const int n0 = nb + wn * NT * 32;
    const float *W = static_cast<const float *>(p.w);
    const int n_slabs = (p.d_in + BK - 1) / BK;
    auto tile_rows = [&](int64_t tile, int64_t &m0) -> const float * {
        m0 = (tile * WM + wm) * 32;
        const int64_t row = m0 + i < p.n_rows ? m0 + i : p.n_rows - 1;     // rows past the end: a valid row, never stored
        return static_cast<const float *>(p.a) + row * p.ld_a;
    };

    // A W slab travels from global memory straight into LDS (global_load_lds, 16 bytes per lane): piece
    // id = u * kThreads + thread sits at float4 index id of the buffer, which is where lane `lane` of a
    // wave-wide load based at the wavefront's first piece lands.  Rows of the slab past d_in are written
    // as zeros by the lanes that would have loaded them.
    auto stage_w = [&](int k_begin, float *buf) {
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const int id0 = u * kThreads + wave * kWave;                 // first piece of this wavefront
            const int id = id0 + lane, kk = id / (NC / 4), n4 = id % (NC / 4);
            if (k_begin + kk < p.d_in) {
                const float *src = W + static_cast<int64_t>(k_begin + kk) * p.d_out + nb + 4 * n4;
                __builtin_amdgcn_global_load_lds((gptr_t)(const void *)src, (lptr_t)(void *)(reinterpret_cast<float4 *>(buf) + id0), 16, 0, 0);
            } else {
                reinterpret_cast<float4 *>(buf)[id] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        }
    };

    int64_t tile = blockIdx.x, m0;                           // the host launches at most n_tiles workgroups
    const float *arow = tile_rows(tile, m0);
    float af[16], an[16];
    stage_w(0, w_lds);
    load_a_f32(p, arow, 16 * h, BK, af);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // the slab has landed in LDS
    __syncthreads();
    int cur = 0;
#pragma unroll 1
    for (;;) {
        f32x16 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[t][q] = 0.f;
        const int64_t ntile = tile + gridDim.x;
        int64_t nm0 = m0;
        const float *narow = arow;
#pragma unroll 1
        for (int ks = 0; ks < n_slabs; ++ks) {
            // the pair after this one (all of this is uniform over the workgroup)
            const bool last_slab = ks + 1 == n_slabs;
            const bool more = !last_slab || ntile < n_tiles;
            const int nks = last_slab ? 0 : ks + 1;
            if (more) {
                if (last_slab) narow = tile_rows(ntile, nm0);
                stage_w(nks * BK, w_lds + (cur ^ 1) * (BK * NC));   // the other buffer: nobody reads it before the barrier below
                load_a_f32(p, narow, nks * BK + 16 * h, (nks + 1) * BK, an);
            }
            // W fragments are read from LDS one MFMA group ahead, so that the matrix pipe never waits for them.
            // MFMA number c contracts k0 + c and k0 + 16 + c: in the last slab the steps whose first k is
            // past d_in add nothing and are left out, four at a time.
            const int n_c = p.d_in - ks * BK;
            const float *wbuf = w_lds + cur * (BK * NC) + (16 * h) * NC + wn * NT * 32 + i;
            float wf[2][NT];
#pragma unroll
            for (int t = 0; t < NT; ++t) wf[0][t] = wbuf[t * 32];
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                if (c + 1 < 16) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) wf[(c + 1) & 1][t] = wbuf[(c + 1) * NC + t * 32];
                }
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[c & 1][t], af[c], acc[t], 0, 0, 0);
                if ((c & 3) == 3 && c + 1 < 16 && c + 1 >= n_c) break;
            }
            if (more) {
#pragma unroll
                for (int c = 0; c < 16; ++c) af[c] = an[c];
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");    // the next slab has landed in LDS
            __syncthreads();
            cur ^= 1;
        }
        // the stores leave while the next tile's first slab is multiplied; the wait one slab later is the
        // first that includes them
        // the output and bias pointers are made opaque per tile: what depends only on them and on the lane
        // (an address per output vector, the bias values) would otherwise be computed once ahead of all
        // loops and held in registers the accumulators need
        UpdArgs ps = p;
        asm volatile("" : "+s"(ps.out), "+s"(ps.bias), "+s"(ps.d_out));       // (d_out: a lane mask per column test)
        store_tiles<NT>(ps, acc, m0, n0, lane);
        if (ntile >= n_tiles) break;
        tile = ntile; m0 = nm0; arow = narow;
    }
}

// ---- bf16 weights: v_mfma_f32_32x32x16_bf16 -------------------------------------------------
// K slab of 64: lane (i, h) holds A[m0+i][k0 + 32h .. k0 + 32h + 31] as four 8-element
// operands; MFMA number c contracts k0 + 32h + 8c .. + 7 (both halves h at once).
// W slab in LDS transposed, [NC][64 + 8] bf16, so a lane's 8 k-values are contiguous.
union Frag8 { uint32_t u[4]; bf16x8 v; };

template <bool A_BF16>
__device__ __forceinline__ void load_a_bf16(const UpdArgs &p, const void *arow_v, int kb, int k_slab_end, Frag8 (&af)[4])
{
    const bool full = p.a_vec_ok && k_slab_end <= p.d_in;      // wave-uniform
    if constexpr (A_BF16) {
        const uint16_t *arow = static_cast<const uint16_t *>(arow_v);
        if (full) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const uint4 v = *reinterpret_cast<const uint4 *>(arow + kb + 8 * c);
                af[c].u[0] = v.x; af[c].u[1] = v.y; af[c].u[2] = v.z; af[c].u[3] = v.w;
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = kb + 8 * c + 2 * e;
                    const uint32_t lo = k < p.d_in ? arow[k] : 0u;
                    const uint32_t hi = k + 1 < p.d_in ? arow[k + 1] : 0u;
                    af[c].u[e] = lo | (hi << 16);
                }
        }
    } else {
        const float *arow = static_cast<const float *>(arow_v);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int k = kb + 8 * c;
            float f[8];
            if (full) {
                const float4 v0 = *reinterpret_cast<const float4 *>(arow + k);
                const float4 v1 = *reinterpret_cast<const float4 *>(arow + k + 4);
                f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) f[e] = k + e < p.d_in ? arow[k + e] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) af[c].u[e] = f32_to_bf16_bits(f[2 * e]) | (f32_to_bf16_bits(f[2 * e + 1]) << 16);
        }
    }
}

template <int NT, int WN, bool A_BF16>
__global__ __launch_bounds__(kThreads) void update_bf16_kernel(const UpdArgs p)
{
    constexpr int BK = 64, NC = NT * 32 * WN, LDW = BK + 8, WM = kWaves / WN;
    __shared__ __attribute__((aligned(16))) uint16_t w_lds[NC * LDW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    const int64_t m0 = (static_cast<int64_t>(blockIdx.x) * WM + wm) * 32;
    const int nb = blockIdx.y * NC;
    const int n0 = nb + wn * NT * 32;
    const uint16_t *W = static_cast<const uint16_t *>(p.w);
    const int64_t row = m0 + i < p.n_rows ? m0 + i : p.n_rows - 1;
    const void *arow = A_BF16 ? static_cast<const void *>(static_cast<const uint16_t *>(p.a) + row * p.ld_a)
                              : static_cast<const void *>(static_cast<const float *>(p.a) + row * p.ld_a);

    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    Frag8 af[4], an[4];
    load_a_bf16<A_BF16>(p, arow, 32 * h, BK, af);
#pragma unroll 1
    for (int k0 = 0; k0 < p.d_in; k0 += BK) {
        if (k0 + BK < p.d_in) load_a_bf16<A_BF16>(p, arow, k0 + BK + 32 * h, k0 + 2 * BK, an);
        __syncthreads();
        fill_w_bf16_t<NC>(w_lds, LDW, W, k0, BK, nb, p);
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                union { uint4 q; bf16x8 v; } bw;
                bw.q = *reinterpret_cast<const uint4 *>(&w_lds[(wn * NT * 32 + t * 32 + i) * LDW + 32 * h + 8 * c]);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw.v, af[c].v, acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) af[c] = an[c];
    }
    store_tiles<NT>(p, acc, m0, n0, lane);
}


// ---- W resident in LDS (small d_in * d_out) ---------------------------------------------------
// When the whole weight matrix fits 64 KB of LDS it is staged once per workgroup, and every
// wavefront then walks over many 32-row tiles of A on its own: no barrier in the main loop.
// These shapes are bound by HBM, and what a wavefront can keep in flight is what its registers
// hold, so the raw K slabs of A are requested D slabs ahead -- across tile boundaries -- and a
// slab is turned into MFMA operands only when its turn comes.  Loads that are waited for are
// always older than the stores of the tile finished last, so (memory operations of a wavefront
// retire in order) no wait ever includes a store.  The grid is sized to the chip, not to the matrix.
extern __shared__ __attribute__((aligned(16))) unsigned char w_res[];

// fp32 path: raw slab = the lane's 16 consecutive k values
struct RawF32 { float4 v[4]; };
__device__ __forceinline__ void load_raw_f32(const UpdArgs &p, const float *arow, int kb, int k_slab_end, RawF32 &r)
{
    if (p.a_vec_ok && k_slab_end <= p.d_in) {
#pragma unroll
        for (int q = 0; q < 4; ++q) r.v[q] = *reinterpret_cast<const float4 *>(arow + kb + 4 * q);
    } else {
        float f[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) f[e] = (kb + e < p.d_in) ? arow[kb + e] : 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) r.v[q] = make_float4(f[4 * q], f[4 * q + 1], f[4 * q + 2], f[4 * q + 3]);
    }
}

// Register budget: without a bound the compiler spends over 250 registers on the widest variant
// and one wavefront per SIMD is left; three (four for the narrow variants) run 1.2-1.3x faster.
#define MGG_UPD_WAVES(NT) ((NT) == 4 ? 3 : 4)
template <int NT, int D>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(MGG_UPD_WAVES(NT), MGG_UPD_WAVES(NT))))
void update_f32_resident_kernel(const UpdArgs p)
{
    constexpr int BK = 32, NC = NT * 32;
    float *w_lds = reinterpret_cast<float *>(w_res);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int n_slabs = (p.d_in + BK - 1) / BK;
    const float *W = static_cast<const float *>(p.w);
    fill_w_f32<NC>(w_lds, W, 0, n_slabs * BK, 0, p);
    __syncthreads();

    const int64_t n_tiles = (p.n_rows + 31) / 32, stride = static_cast<int64_t>(gridDim.x) * kWaves;
    int64_t tile = static_cast<int64_t>(blockIdx.x) * kWaves + wave;
    if (tile >= n_tiles) return;
    auto row_ptr_of = [&](int64_t t) {
        const int64_t r = t * 32 + i < p.n_rows ? t * 32 + i : p.n_rows - 1;
        return static_cast<const float *>(p.a) + r * p.ld_a;
    };
    // issue cursor: the slab requested next
    int64_t itile = tile;
    int is = 0;
    const float *irow = row_ptr_of(itile);
    RawF32 q[D];
    auto issue = [&](RawF32 &dst) {
        if (itile < n_tiles) {
            load_raw_f32(p, irow, is * BK + 16 * h, (is + 1) * BK, dst);
            if (++is == n_slabs) { is = 0; itile += stride; if (itile < n_tiles) irow = row_ptr_of(itile); }
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d) issue(q[d]);

    while (tile < n_tiles) {
        f32x16 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll 1
        for (int s = 0; s < n_slabs; ++s) {
            float af[16];
#pragma unroll
            for (int qq = 0; qq < 4; ++qq) { af[4 * qq] = q[0].v[qq].x; af[4 * qq + 1] = q[0].v[qq].y; af[4 * qq + 2] = q[0].v[qq].z; af[4 * qq + 3] = q[0].v[qq].w; }
#pragma unroll
            for (int d = 0; d + 1 < D; ++d) q[d] = q[d + 1];
            issue(q[D - 1]);
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                const float *wrow = w_lds + (s * BK + 16 * h + c) * NC + i;
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(wrow[t * 32], af[c], acc[t], 0, 0, 0);
            }
        }
        store_tiles<NT>(p, acc, tile * 32, 0, lane);
        tile += stride;
    }
}

// bf16 path: raw slab = the lane's 32 consecutive k values, fp32 (8 x 16 bytes) or bf16 (4 x 16 bytes)
template <bool A_BF16> struct RawB16 { uint4 v[A_BF16 ? 4 : 8]; };

template <bool A_BF16>
__device__ __forceinline__ void load_raw_b16(const UpdArgs &p, const void *arow_v, int kb, int k_slab_end, RawB16<A_BF16> &r)
{
    const bool full = p.a_vec_ok && k_slab_end <= p.d_in;      // wave-uniform
    if constexpr (A_BF16) {
        const uint16_t *arow = static_cast<const uint16_t *>(arow_v);
        if (full) {
#pragma unroll
            for (int c = 0; c < 4; ++c) r.v[c] = *reinterpret_cast<const uint4 *>(arow + kb + 8 * c);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint32_t u[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int k = kb + 8 * c + 2 * e;
                    const uint32_t lo = k < p.d_in ? arow[k] : 0u;
                    const uint32_t hi = k + 1 < p.d_in ? arow[k + 1] : 0u;
                    u[e] = lo | (hi << 16);
                }
                r.v[c] = make_uint4(u[0], u[1], u[2], u[3]);
            }
        }
    } else {
        const float *arow = static_cast<const float *>(arow_v);
        if (full) {
#pragma unroll
            for (int c = 0; c < 8; ++c) r.v[c] = *reinterpret_cast<const uint4 *>(arow + kb + 4 * c);
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                uint32_t u[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) u[e] = kb + 4 * c + e < p.d_in ? __float_as_uint(arow[kb + 4 * c + e]) : 0u;
                r.v[c] = make_uint4(u[0], u[1], u[2], u[3]);
            }
        }
    }
}

template <bool A_BF16>
__device__ __forceinline__ void raw_to_frags(const RawB16<A_BF16> &r, Frag8 (&af)[4])
{
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if constexpr (A_BF16) {
            af[c].u[0] = r.v[c].x; af[c].u[1] = r.v[c].y; af[c].u[2] = r.v[c].z; af[c].u[3] = r.v[c].w;
        } else {
            const uint4 lo = r.v[2 * c], hi = r.v[2 * c + 1];
            af[c].u[0] = f32_to_bf16_bits(__uint_as_float(lo.x)) | (f32_to_bf16_bits(__uint_as_float(lo.y)) << 16);
            af[c].u[1] = f32_to_bf16_bits(__uint_as_float(lo.z)) | (f32_to_bf16_bits(__uint_as_float(lo.w)) << 16);
            af[c].u[2] = f32_to_bf16_bits(__uint_as_float(hi.x)) | (f32_to_bf16_bits(__uint_as_float(hi.y)) << 16);
            af[c].u[3] = f32_to_bf16_bits(__uint_as_float(hi.z)) | (f32_to_bf16_bits(__uint_as_float(hi.w)) << 16);
        }
    }
}

template <int NT, bool A_BF16, int D>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(MGG_UPD_WAVES(NT), MGG_UPD_WAVES(NT))))
void update_bf16_resident_kernel(const UpdArgs p)
{
    constexpr int BK = 64, NC = NT * 32;
    uint16_t *w_lds = reinterpret_cast<uint16_t *>(w_res);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int n_slabs = (p.d_in + BK - 1) / BK;
    const int ldw = n_slabs * BK + 8;                       // padded row of the transposed copy
    const uint16_t *W = static_cast<const uint16_t *>(p.w);
    fill_w_bf16_t<NC>(w_lds, ldw, W, 0, n_slabs * BK, 0, p);
    __syncthreads();

    const int64_t n_tiles = (p.n_rows + 31) / 32, stride = static_cast<int64_t>(gridDim.x) * kWaves;
    int64_t tile = static_cast<int64_t>(blockIdx.x) * kWaves + wave;
    if (tile >= n_tiles) return;
    auto row_ptr_of = [&](int64_t t) -> const void * {
        const int64_t r = t * 32 + i < p.n_rows ? t * 32 + i : p.n_rows - 1;
        if constexpr (A_BF16) return static_cast<const uint16_t *>(p.a) + r * p.ld_a;
        else return static_cast<const float *>(p.a) + r * p.ld_a;
    };
    int64_t itile = tile;
    int is = 0;
    const void *irow = row_ptr_of(itile);
    RawB16<A_BF16> q[D];
    auto issue = [&](RawB16<A_BF16> &dst) {
        if (itile < n_tiles) {
            load_raw_b16<A_BF16>(p, irow, is * BK + 32 * h, (is + 1) * BK, dst);
            if (++is == n_slabs) { is = 0; itile += stride; if (itile < n_tiles) irow = row_ptr_of(itile); }
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d) issue(q[d]);

    while (tile < n_tiles) {
        f32x16 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll 1
        for (int s = 0; s < n_slabs; ++s) {
            Frag8 af[4];
            raw_to_frags<A_BF16>(q[0], af);
#pragma unroll
            for (int d = 0; d + 1 < D; ++d) q[d] = q[d + 1];
            issue(q[D - 1]);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    union { uint4 q4; bf16x8 v; } bw;
                    bw.q4 = *reinterpret_cast<const uint4 *>(&w_lds[(t * 32 + i) * ldw + s * BK + 32 * h + 8 * c]);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw.v, af[c].v, acc[t], 0, 0, 0);
                }
            }
        }
        store_tiles<NT>(p, acc, tile * 32, 0, lane);
        tile += stride;
    }
}

// slabs requested ahead (the raw fp32 slab of the bf16 path is twice the size of the others)
#ifndef MGG_UPD_DEPTH_F32
#define MGG_UPD_DEPTH_F32 2
#endif
#ifndef MGG_UPD_DEPTH_B16
#define MGG_UPD_DEPTH_B16 1
#endif

// ---- row softmax (section 7: the last step of the 2-layer GCN) ---------------------------------
// One wavefront per row, in place: the row is held in registers (lanes stride over the columns),
// maximum and sum are combined with cross-lane shuffles.  Bound by HBM: one read and one write.
template <bool BF16, int CPL>      // CPL: columns per lane
__global__ __launch_bounds__(kThreads) void row_softmax_kernel(void *x, int64_t n_rows, int32_t d, int64_t ld)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = static_cast<int64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6);
    if (row >= n_rows) return;
    float v[CPL];
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int col = c * kWave + lane;
        v[c] = -INFINITY;
        if (col < d) {
            if constexpr (BF16) v[c] = __uint_as_float(static_cast<uint32_t>(static_cast<const uint16_t *>(x)[row * ld + col]) << 16);
            else v[c] = static_cast<const float *>(x)[row * ld + col];
        }
        m = fmaxf(m, v[c]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        v[c] = c * kWave + lane < d ? expf(v[c] - m) : 0.f;
        sum += v[c];
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    const float inv = 1.f / sum;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int col = c * kWave + lane;
        if (col < d) {
            if constexpr (BF16) static_cast<uint16_t *>(x)[row * ld + col] = static_cast<uint16_t>(f32_to_bf16_bits(v[c] * inv));
            else static_cast<float *>(x)[row * ld + col] = v[c] * inv;
        }
    }
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <int NT>
hipError_t launch_resident(const UpdArgs &p, bool w_bf16, bool a_bf16, int blocks, size_t lds_bytes, hipStream_t s)
{
    if (!w_bf16) hipLaunchKernelGGL((update_f32_resident_kernel<NT, MGG_UPD_DEPTH_F32>), dim3(blocks), dim3(kThreads), lds_bytes, s, p);
    else if (a_bf16) hipLaunchKernelGGL((update_bf16_resident_kernel<NT, true, 2 * MGG_UPD_DEPTH_B16>), dim3(blocks), dim3(kThreads), lds_bytes, s, p);
    else hipLaunchKernelGGL((update_bf16_resident_kernel<NT, false, MGG_UPD_DEPTH_B16>), dim3(blocks), dim3(kThreads), lds_bytes, s, p);
    return hipGetLastError();
}

template <int NT, int WN>
hipError_t launch_shape(const UpdArgs &p, bool w_bf16, bool a_bf16, dim3 grid, int cus, hipStream_t s)
{
    if (!w_bf16 && p.w_vec_ok && p.d_out % (NT * 32 * WN) == 0 && option_update_stream() != 0) {
        constexpr int lds_bytes = 2 * 32 * NT * 32 * WN * 4;
        // Short contractions (d_in <= 256: at most 8 slabs): as many workgroups as the chip holds at once (two
        // per CU: 64 KB of LDS each, two wavefronts per SIMD), each walking over row tiles, so that a tile's
        // stores and the next tile's first loads hide behind MFMAs (100 -> 256: 227 -> 202 us).  Long ones:
        // a workgroup per tile, handed out by the dispatcher as CUs free up (602 -> 256: 693 us, 706 us when
        // the tiles are dealt out ahead of time).
        const int64_t slots = p.d_in <= 256 ? 2 * static_cast<int64_t>(cus) : INT64_MAX;
        if constexpr (NT == 4 && WN == 2) {
            // 256 columns: one wavefront per 32 rows x 256 columns, so that every row of A is read by one
            // wavefront only (two side by side, each reading the rows, measured 6 % slower on 602 -> 256)
            const int64_t n_tiles = (p.n_rows + 32 * kWaves - 1) / (32 * kWaves);
            grid.x = static_cast<unsigned>(n_tiles < slots ? n_tiles : slots);
            (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&update_f32_db_kernel<8, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            hipLaunchKernelGGL((update_f32_db_kernel<8, 1>), grid, dim3(kThreads), lds_bytes, s, p, n_tiles);
        } else {
            const int64_t n_tiles = (p.n_rows + 32 * (kWaves / WN) - 1) / (32 * (kWaves / WN));
            grid.x = static_cast<unsigned>(n_tiles < slots ? n_tiles : slots);
            // up to 64 KB of dynamic LDS: ask for it (cheap, so done at every launch rather than remembered)
            if (lds_bytes > 48 * 1024)
                (void)hipFuncSetAttribute(reinterpret_cast<const void *>(&update_f32_db_kernel<NT, WN>), hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
            hipLaunchKernelGGL((update_f32_db_kernel<NT, WN>), grid, dim3(kThreads), lds_bytes, s, p, n_tiles);
        }
    }
    else if (!w_bf16) hipLaunchKernelGGL((update_f32_kernel<NT, WN>), grid, dim3(kThreads), 0, s, p);
    else if (a_bf16) hipLaunchKernelGGL((update_bf16_kernel<NT, WN, true>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((update_bf16_kernel<NT, WN, false>), grid, dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace

mgg_status_t launch_row_softmax(int64_t n_rows, int32_t d, mgg_dtype_t dtype, void *x, int64_t ld, hipStream_t stream)
{
    if (n_rows == 0) return MGG_OK;
    if (d > 8 * kWave) return fail(MGG_ERR_UNSUPPORTED, "softmax over %d columns (at most %d)", d, 8 * kWave);
    const int64_t blocks = (n_rows + kWaves - 1) / kWaves;
    if (blocks > INT32_MAX) return fail(MGG_ERR_UNSUPPORTED, "too many rows for one launch");
    const dim3 grid(static_cast<unsigned>(blocks)), block(kThreads);
    const bool bf = dtype == MGG_BF16;
    const int cpl = (d + kWave - 1) / kWave;
#define MGG_SOFTMAX(C) do { if (bf) hipLaunchKernelGGL((row_softmax_kernel<true, C>), grid, block, 0, stream, x, n_rows, d, ld); \
                            else hipLaunchKernelGGL((row_softmax_kernel<false, C>), grid, block, 0, stream, x, n_rows, d, ld); } while (0)
    if (cpl <= 1) MGG_SOFTMAX(1);
    else if (cpl <= 2) MGG_SOFTMAX(2);
    else if (cpl <= 4) MGG_SOFTMAX(4);
    else MGG_SOFTMAX(8);
#undef MGG_SOFTMAX
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "softmax kernel launch");
    return MGG_OK;
}

static mgg_status_t launch_update_gemm(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
                                       mgg_dtype_t w_dtype, const void *w, const float *bias, int32_t d_out, mgg_act_t act,
                                       mgg_dtype_t out_dtype, void *out, int64_t ld_out, hipStream_t stream);

mgg_status_t launch_update(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
                           mgg_dtype_t w_dtype, const void *w, const float *bias, int32_t d_out, mgg_act_t act,
                           mgg_dtype_t out_dtype, void *out, int64_t ld_out, hipStream_t stream)
{
    // softmax couples the columns of a row: the product is written first, the rows are normalised in place
    const bool softmax = act == MGG_ACT_SOFTMAX;
    if (softmax && d_out > 8 * kWave) return fail(MGG_ERR_UNSUPPORTED, "softmax over %d columns (at most %d)", d_out, 8 * kWave);
    mgg_status_t s = launch_update_gemm(n_rows, a_dtype, a, ld_a, d_in, w_dtype, w, bias, d_out, softmax ? MGG_ACT_NONE : act,
                                        out_dtype, out, ld_out, stream);
    if (s != MGG_OK || !softmax) return s;
    return launch_row_softmax(n_rows, d_out, out_dtype, out, ld_out, stream);
}

mgg_status_t launch_update_mlp(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, const int32_t dims[3],
                               mgg_dtype_t w_dtype, const void *w1, const float *b1, mgg_act_t act1, const void *w2, const float *b2,
                               mgg_act_t act2, void *hidden, int64_t ld_hidden, mgg_dtype_t out_dtype, void *out, int64_t ld_out,
                               hipStream_t stream)
{
    if (n_rows == 0) return MGG_OK;
    if (w_dtype == MGG_BF16 && option_update_stream() != 0) {
        int dev = 0, cus = 256;
        if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        hipError_t e = hipSuccess;
        if (launch_mlp_stream(n_rows, a_dtype, a, ld_a, dims[0], w1, b1, act1, dims[1], w2, b2, act2, dims[2], out_dtype, out, ld_out, cus,
                              stream, &e)) {
            if (e != hipSuccess) return hip_fail(e, "MLP kernel launch");
            return MGG_OK;
        }
    }
    if (!hidden) return fail(MGG_ERR_INVALID_ARG, "hidden buffer is NULL and the shape is not covered by the one-kernel MLP");
    const mgg_dtype_t hid_dtype = w_dtype == MGG_BF16 ? MGG_BF16 : MGG_F32;
    mgg_status_t s = launch_update(n_rows, a_dtype, a, ld_a, dims[0], w_dtype, w1, b1, dims[1], act1, hid_dtype, hidden, ld_hidden, stream);
    if (s != MGG_OK) return s;
    return launch_update(n_rows, hid_dtype, hidden, ld_hidden, dims[1], w_dtype, w2, b2, dims[2], act2, out_dtype, out, ld_out, stream);
}

static mgg_status_t launch_update_gemm(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
                                       mgg_dtype_t w_dtype, const void *w, const float *bias, int32_t d_out, mgg_act_t act,
                                       mgg_dtype_t out_dtype, void *out, int64_t ld_out, hipStream_t stream)
{
    if (n_rows == 0) return MGG_OK;
    const bool w_bf16 = w_dtype == MGG_BF16, a_bf16 = a_dtype == MGG_BF16;
    UpdArgs p{};
    p.a = a; p.w = w; p.bias = bias; p.out = out;
    p.n_rows = n_rows; p.ld_a = ld_a; p.ld_out = ld_out;
    p.d_in = d_in; p.d_out = d_out;
    p.relu = act == MGG_ACT_RELU;
    p.out_bf16 = out_dtype == MGG_BF16;
    p.a_vec_ok = aligned16(a) && (ld_a % (a_bf16 ? 8 : 4) == 0);
    p.out_vec_ok = (ld_out % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % (out_dtype == MGG_BF16 ? 8 : 16) == 0);
    p.w_vec_ok = aligned16(w) && (d_out % (w_bf16 ? 8 : 4) == 0);

    // tiles of 32 columns per wavefront (1, 2 or 4) and wavefronts side by side (1 or 2);
    // outputs wider than 256 columns tile over grid.y
    int nt = 1, wn = 1;
    if (d_out > 128) { nt = 4; wn = 2; }
    else if (d_out > 64) nt = 4;
    else if (d_out > 32) nt = 2;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    // HBM-bound shapes with whole K slabs: the whole-line variant
    if (option_update_stream() != 0) {
        hipError_t e = hipSuccess;
        if (launch_update_stream(p, w_bf16, a_bf16, cus, stream, &e)) {
            if (e != hipSuccess) return hip_fail(e, "update kernel launch");
            return MGG_OK;
        }
    }
    // small weight matrices stay resident in LDS and the grid is sized to the chip
    if (wn == 1) {
        const size_t k_pad = w_bf16 ? (static_cast<size_t>(d_in) + 63) / 64 * 64 : (static_cast<size_t>(d_in) + 31) / 32 * 32;
        const size_t lds_bytes = w_bf16 ? static_cast<size_t>(nt) * 32 * (k_pad + 8) * 2 : k_pad * nt * 32 * 4;
        if (lds_bytes <= 64 * 1024) {
            int per_cu = static_cast<int>((160 * 1024) / (lds_bytes + 512));
            per_cu = per_cu < 1 ? 1 : (per_cu > (nt == 4 ? 3 : 4) ? (nt == 4 ? 3 : 4) : per_cu);
            const int64_t n_tiles = (n_rows + 31) / 32;
            const int64_t want = (n_tiles + kWaves - 1) / kWaves;
            const int blocks = static_cast<int>(want < static_cast<int64_t>(cus) * per_cu ? want : static_cast<int64_t>(cus) * per_cu);
            hipError_t e;
            if (nt == 1) e = launch_resident<1>(p, w_bf16, a_bf16, blocks, lds_bytes, stream);
            else if (nt == 2) e = launch_resident<2>(p, w_bf16, a_bf16, blocks, lds_bytes, stream);
            else e = launch_resident<4>(p, w_bf16, a_bf16, blocks, lds_bytes, stream);
            if (e != hipSuccess) return hip_fail(e, "update kernel launch");
            return MGG_OK;
        }
    }
    const int nc = nt * 32 * wn, rows_per_block = 32 * (kWaves / wn);
    const int64_t gx = (n_rows + rows_per_block - 1) / rows_per_block;
    if (gx > INT32_MAX) return fail(MGG_ERR_UNSUPPORTED, "too many rows for one launch");
    dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>((d_out + nc - 1) / nc));
    hipError_t e;
    if (wn == 2) e = launch_shape<4, 2>(p, w_bf16, a_bf16, grid, cus, stream);
    else if (nt == 1) e = launch_shape<1, 1>(p, w_bf16, a_bf16, grid, cus, stream);
    else if (nt == 2) e = launch_shape<2, 1>(p, w_bf16, a_bf16, grid, cus, stream);
    else e = launch_shape<4, 1>(p, w_bf16, a_bf16, grid, cus, stream);
    if (e != hipSuccess) return hip_fail(e, "update kernel launch");
    return MGG_OK;
}

}  // namespace mgg
