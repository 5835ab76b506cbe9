// Dense Update for gfx950 (section 1: Update is a fully-connected layer; section 7: X W with
// ReLU, and GIN's MLP): out = act(A . W + bias) on the matrix cores.
//
// Shape of the problem: A is tall (10^5..10^6 rows) and both d_in and d_out are small
// (16..602), so each wavefront owns 32 rows of A and ALL output columns of its block:
//   - A is read once, straight from HBM into registers in the MFMA operand layout
//     (no LDS round trip: nobody else needs those rows);
//   - W is staged slab by slab in LDS and shared by the block's four wavefronts;
//   - fp32 weights use v_mfma_f32_32x32x2_f32, bf16 weights v_mfma_f32_32x32x16_bf16,
//     both with fp32 accumulators; bias, ReLU and the output rounding are fused.
// MFMA sums over k in any order, so a lane may take whichever k values are contiguous for
// it in memory as long as the A and W operands agree; that is what makes the direct loads
// of A full-width.
#include <hip/hip_runtime.h>

#include "mgg_internal.h"

namespace mgg {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;
constexpr int kWaves = 4;
constexpr int kThreads = kWave * kWaves;
constexpr int kRowsPerWave = 32;
constexpr int kRowsPerBlock = kRowsPerWave * kWaves;

struct UpdArgs {
    const void *a;
    const void *w;
    const float *bias;
    void *out;
    int64_t n_rows, ld_a, ld_out;
    int32_t d_in, d_out;
    int32_t relu;
    int32_t out_bf16;
    int32_t a_vec_ok;   // rows of A allow 16-byte loads
};

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);       // round to nearest, ties to even
    return u >> 16;
}

// Epilogue shared by both paths.  In the 32x32 accumulator layout register r of lane
// (j = lane % 32, h = lane / 32) is element (row 8*(r/4) + 4*h + r%4, column j).
template <int NT>
__device__ __forceinline__ void store_tiles(const UpdArgs &p, const f32x16 (&acc)[NT], int64_t m0, int n0, int lane)
{
    const int j = lane & 31, h = lane >> 5;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int col = n0 + t * 32 + j;
        if (col >= p.d_out) continue;
        const float b = p.bias ? p.bias[col] : 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int64_t row = m0 + 8 * (r / 4) + 4 * h + (r % 4);
            if (row >= p.n_rows) continue;
            float v = acc[t][r] + b;
            if (p.relu) v = v > 0.f ? v : 0.f;
            if (p.out_bf16)
                static_cast<uint16_t *>(p.out)[row * p.ld_out + col] = static_cast<uint16_t>(f32_to_bf16_bits(v));
            else
                static_cast<float *>(p.out)[row * p.ld_out + col] = v;
        }
    }
}

// ---- fp32 weights: v_mfma_f32_32x32x2_f32 ---------------------------------------------------
// K slab of 32: lane (i, h) holds A[m0+i][k0 + 16h .. k0 + 16h + 15]; MFMA number c contracts
// the k pair {k0 + c, k0 + 16 + c}.  W slab in LDS as [32][NT*32] floats.
template <int NT>
__global__ __launch_bounds__(kThreads) void update_f32_kernel(const UpdArgs p)
{
    constexpr int BK = 32, NC = NT * 32;
    __shared__ float w_lds[BK * NC];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock + wave * kRowsPerWave;
    const int n0 = blockIdx.y * NC;
    const float *A = static_cast<const float *>(p.a);
    const float *W = static_cast<const float *>(p.w);
    const int64_t row = m0 + i;
    const bool row_ok = row < p.n_rows;
    const float *arow = A + (row_ok ? row : 0) * p.ld_a;

    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    for (int k0 = 0; k0 < p.d_in; k0 += BK) {
        // A fragment: 16 consecutive k of this lane's row
        float af[16];
        const int kb = k0 + 16 * h;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = kb + 4 * q;
            if (row_ok && p.a_vec_ok && k + 3 < p.d_in) {
                const float4 v = *reinterpret_cast<const float4 *>(arow + k);
                af[4 * q] = v.x; af[4 * q + 1] = v.y; af[4 * q + 2] = v.z; af[4 * q + 3] = v.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) af[4 * q + e] = (row_ok && k + e < p.d_in) ? arow[k + e] : 0.f;
            }
        }
        // W slab -> LDS (zeros outside the matrix)
        __syncthreads();
        for (int idx = threadIdx.x; idx < BK * NC; idx += kThreads) {
            const int kk = idx / NC, nn = idx % NC;
            const int k = k0 + kk, n = n0 + nn;
            w_lds[idx] = (k < p.d_in && n < p.d_out) ? W[static_cast<int64_t>(k) * p.d_out + n] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const float *wrow = w_lds + (16 * h + c) * NC + i;
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[c], wrow[t * 32], acc[t], 0, 0, 0);
        }
    }
    store_tiles<NT>(p, acc, m0, n0, lane);
}

// ---- bf16 weights: v_mfma_f32_32x32x16_bf16 -------------------------------------------------
// K slab of 64: lane (i, h) holds A[m0+i][k0 + 32h .. k0 + 32h + 31] as four 8-element
// operands; MFMA number c contracts k0 + 32h + 8c .. + 7 (both halves h at once).
// W slab in LDS transposed, [NT*32][64 + 8] bf16, so a lane's 8 k-values are contiguous.
template <int NT, bool A_BF16>
__global__ __launch_bounds__(kThreads) void update_bf16_kernel(const UpdArgs p)
{
    constexpr int BK = 64, NC = NT * 32, LDW = BK + 8;
    __shared__ __attribute__((aligned(16))) uint16_t w_lds[NC * LDW];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    const int64_t m0 = static_cast<int64_t>(blockIdx.x) * kRowsPerBlock + wave * kRowsPerWave;
    const int n0 = blockIdx.y * NC;
    const uint16_t *W = static_cast<const uint16_t *>(p.w);
    const int64_t row = m0 + i;
    const bool row_ok = row < p.n_rows;

    f32x16 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    for (int k0 = 0; k0 < p.d_in; k0 += BK) {
        union { uint32_t u[4]; bf16x8 v; } af[4];
        const int kb = k0 + 32 * h;
        if constexpr (A_BF16) {
            const uint16_t *arow = static_cast<const uint16_t *>(p.a) + (row_ok ? row : 0) * p.ld_a;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int k = kb + 8 * c;
                if (row_ok && p.a_vec_ok && k + 7 < p.d_in) {
                    const uint4 v = *reinterpret_cast<const uint4 *>(arow + k);
                    af[c].u[0] = v.x; af[c].u[1] = v.y; af[c].u[2] = v.z; af[c].u[3] = v.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t lo = (row_ok && k + 2 * e < p.d_in) ? arow[k + 2 * e] : 0u;
                        const uint32_t hi = (row_ok && k + 2 * e + 1 < p.d_in) ? arow[k + 2 * e + 1] : 0u;
                        af[c].u[e] = lo | (hi << 16);
                    }
                }
            }
        } else {
            const float *arow = static_cast<const float *>(p.a) + (row_ok ? row : 0) * p.ld_a;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int k = kb + 8 * c;
                float f[8];
                if (row_ok && p.a_vec_ok && k + 7 < p.d_in) {
                    const float4 v0 = *reinterpret_cast<const float4 *>(arow + k);
                    const float4 v1 = *reinterpret_cast<const float4 *>(arow + k + 4);
                    f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] = (row_ok && k + e < p.d_in) ? arow[k + e] : 0.f;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) af[c].u[e] = f32_to_bf16_bits(f[2 * e]) | (f32_to_bf16_bits(f[2 * e + 1]) << 16);
            }
        }
        // W slab -> LDS, transposed: thread takes a k pair of one column, writes one dword
        __syncthreads();
        for (int idx = threadIdx.x; idx < (BK / 2) * NC; idx += kThreads) {
            const int kp = idx / NC, nn = idx % NC;
            const int k = k0 + 2 * kp, n = n0 + nn;
            const uint32_t lo = (k < p.d_in && n < p.d_out) ? W[static_cast<int64_t>(k) * p.d_out + n] : 0u;
            const uint32_t hi = (k + 1 < p.d_in && n < p.d_out) ? W[static_cast<int64_t>(k + 1) * p.d_out + n] : 0u;
            *reinterpret_cast<uint32_t *>(&w_lds[nn * LDW + 2 * kp]) = lo | (hi << 16);
        }
        __syncthreads();
#pragma unroll
        for (int c = 0; c < 4; ++c) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                union { uint4 q; bf16x8 v; } bw;
                bw.q = *reinterpret_cast<const uint4 *>(&w_lds[(t * 32 + i) * LDW + 32 * h + 8 * c]);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[c].v, bw.v, acc[t], 0, 0, 0);
            }
        }
    }
    store_tiles<NT>(p, acc, m0, n0, lane);
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <int NT>
hipError_t launch_nt(const UpdArgs &p, bool w_bf16, bool a_bf16, dim3 grid, hipStream_t s)
{
    if (!w_bf16) hipLaunchKernelGGL(update_f32_kernel<NT>, grid, dim3(kThreads), 0, s, p);
    else if (a_bf16) hipLaunchKernelGGL((update_bf16_kernel<NT, true>), grid, dim3(kThreads), 0, s, p);
    else hipLaunchKernelGGL((update_bf16_kernel<NT, false>), grid, dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace

mgg_status_t launch_update(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in,
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

    // columns per block: all of them up to 256 (fp32) / 256 (bf16); wider outputs tile over grid.y
    int nt = 1;
    while (nt * 32 < d_out && nt < 8) nt <<= 1;
    const int nc = nt * 32;
    const int64_t gx = (n_rows + kRowsPerBlock - 1) / kRowsPerBlock;
    if (gx > INT32_MAX) return fail(MGG_ERR_UNSUPPORTED, "too many rows for one launch");
    dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>((d_out + nc - 1) / nc));
    hipError_t e;
    switch (nt) {
        case 1: e = launch_nt<1>(p, w_bf16, a_bf16, grid, stream); break;
        case 2: e = launch_nt<2>(p, w_bf16, a_bf16, grid, stream); break;
        case 4: e = launch_nt<4>(p, w_bf16, a_bf16, grid, stream); break;
        default: e = launch_nt<8>(p, w_bf16, a_bf16, grid, stream); break;
    }
    if (e != hipSuccess) return hip_fail(e, "update kernel launch");
    return MGG_OK;
}

}  // namespace mgg
