// Pieces shared by the Update kernels (update.hip, update_stream.hip): argument block, bf16
// rounding, the epilogue of the register-resident tiles and the staging of W in LDS.
#pragma once

#include <hip/hip_runtime.h>

#include "mgg_internal.h"

namespace mgg {
namespace upd {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kWave = 64;
constexpr int kWaves = 4;
constexpr int kThreads = kWave * kWaves;

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
    int32_t w_vec_ok;   // rows of W allow 16-byte loads
    int32_t out_vec_ok; // rows of out allow 16-byte (fp32) / 8-byte (bf16) stores
};

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);       // round to nearest, ties to even
    return u >> 16;
}

// Epilogue shared by both paths.  The kernels feed the W fragment as the first MFMA operand and
// the A fragment as the second, so the 32x32 accumulator holds the TRANSPOSED tile: register r
// of lane (m = lane % 32, h = lane / 32) is output row m, column 8*(r/4) + 4*h + r%4.  A lane
// therefore owns four consecutive columns of one row per group of four registers and writes
// them with one 16-byte (fp32) or 8-byte (bf16) store.
template <int NT>
__device__ __forceinline__ void store_tiles(const UpdArgs &p, const f32x16 (&acc)[NT], int64_t m0, int n0, int lane)
{
    const int m = lane & 31, h = lane >> 5;
    const int64_t row = m0 + m;
    if (row >= p.n_rows) return;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int col = n0 + t * 32 + 8 * q + 4 * h;
            if (col >= p.d_out) continue;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = acc[t][4 * q + e] + ((p.bias && col + e < p.d_out) ? p.bias[col + e] : 0.f);
                if (p.relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
            }
            const bool full = p.out_vec_ok && col + 3 < p.d_out;
            if (p.out_bf16) {
                uint16_t *o = static_cast<uint16_t *>(p.out) + row * p.ld_out + col;
                if (full) {
                    uint2 pk;
                    pk.x = f32_to_bf16_bits(v[0]) | (f32_to_bf16_bits(v[1]) << 16);
                    pk.y = f32_to_bf16_bits(v[2]) | (f32_to_bf16_bits(v[3]) << 16);
                    *reinterpret_cast<uint2 *>(o) = pk;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < p.d_out) o[e] = static_cast<uint16_t>(f32_to_bf16_bits(v[e]));
                }
            } else {
                float *o = static_cast<float *>(p.out) + row * p.ld_out + col;
                if (full) {
                    *reinterpret_cast<float4 *>(o) = make_float4(v[0], v[1], v[2], v[3]);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (col + e < p.d_out) o[e] = v[e];
                }
            }
        }
    }
}

// ---- staging W in LDS ---------------------------------------------------------------------------
// Loads are issued in batches before any LDS store so that several are in flight per thread.
// fp32: rows [k_begin, k_begin + n_k) and columns [nb, nb + NC) of W -> lds[n_k][NC], zeros
// outside the matrix.
template <int NC>
__device__ __forceinline__ void fill_w_f32(float *lds, const float *W, int k_begin, int n_k, int nb, const UpdArgs &p)
{
    constexpr int B = 4;
    if (p.w_vec_ok && nb + NC <= p.d_out) {
        const int units = n_k * (NC / 4);
        for (int base = threadIdx.x; base < units; base += kThreads * B) {
            float4 v[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                v[b] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (id < units) {
                    const int kk = id / (NC / 4), n4 = id % (NC / 4);
                    if (k_begin + kk < p.d_in)
                        v[b] = *reinterpret_cast<const float4 *>(W + static_cast<int64_t>(k_begin + kk) * p.d_out + nb + 4 * n4);
                }
            }
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                if (id < units) reinterpret_cast<float4 *>(lds)[id] = v[b];
            }
        }
    } else {
        const int units = n_k * NC;
        for (int base = threadIdx.x; base < units; base += kThreads * B) {
            float v[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                v[b] = 0.f;
                if (id < units) {
                    const int k = k_begin + id / NC, n = nb + id % NC;
                    if (k < p.d_in && n < p.d_out) v[b] = W[static_cast<int64_t>(k) * p.d_out + n];
                }
            }
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                if (id < units) lds[id] = v[b];
            }
        }
    }
}

// bf16: the same block of W, transposed -> lds[NC][ldw] (ldw even), element (n, k - k_begin).
template <int NC>
__device__ __forceinline__ void fill_w_bf16_t(uint16_t *lds, int ldw, const uint16_t *W, int k_begin, int n_k, int nb,
                                              const UpdArgs &p)
{
    uint32_t *lds32 = reinterpret_cast<uint32_t *>(lds);
    const int ldw2 = ldw / 2;
    if (p.w_vec_ok && nb + NC <= p.d_out) {
        // unit = a pair of k rows x 8 columns: two 16-byte loads, eight dword stores
        constexpr int B = 2;
        const int units = (n_k / 2) * (NC / 8);
        for (int base = threadIdx.x; base < units; base += kThreads * B) {
            uint4 lo[B], hi[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                lo[b] = make_uint4(0u, 0u, 0u, 0u);
                hi[b] = make_uint4(0u, 0u, 0u, 0u);
                if (id < units) {
                    const int kp = id / (NC / 8), n8 = id % (NC / 8);
                    const int k = k_begin + 2 * kp;
                    const uint16_t *src = W + static_cast<int64_t>(k) * p.d_out + nb + 8 * n8;
                    if (k < p.d_in) lo[b] = *reinterpret_cast<const uint4 *>(src);
                    if (k + 1 < p.d_in) hi[b] = *reinterpret_cast<const uint4 *>(src + p.d_out);
                }
            }
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                if (id < units) {
                    const int kp = id / (NC / 8), n8 = id % (NC / 8);
                    const uint32_t l[4] = {lo[b].x, lo[b].y, lo[b].z, lo[b].w}, u[4] = {hi[b].x, hi[b].y, hi[b].z, hi[b].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        lds32[(8 * n8 + 2 * e) * ldw2 + kp] = (l[e] & 0xffffu) | (u[e] << 16);
                        lds32[(8 * n8 + 2 * e + 1) * ldw2 + kp] = (l[e] >> 16) | (u[e] & 0xffff0000u);
                    }
                }
            }
        }
    } else {
        constexpr int B = 4;
        const int units = (n_k / 2) * NC;
        for (int base = threadIdx.x; base < units; base += kThreads * B) {
            uint32_t v[B];
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                v[b] = 0u;
                if (id < units) {
                    const int k = k_begin + 2 * (id / NC), n = nb + id % NC;
                    const uint32_t l = (k < p.d_in && n < p.d_out) ? W[static_cast<int64_t>(k) * p.d_out + n] : 0u;
                    const uint32_t u = (k + 1 < p.d_in && n < p.d_out) ? W[static_cast<int64_t>(k + 1) * p.d_out + n] : 0u;
                    v[b] = l | (u << 16);
                }
            }
#pragma unroll
            for (int b = 0; b < B; ++b) {
                const int id = base + b * kThreads;
                if (id < units) lds32[(id % NC) * ldw2 + id / NC] = v[b];
            }
        }
    }
}

}  // namespace upd

// Whole-line variant for shapes it covers (update_stream.hip); returns false when the shape is
// not covered and nothing was launched.
bool launch_update_stream(const upd::UpdArgs &p, bool w_bf16, bool a_bf16, int cus, hipStream_t stream, hipError_t *err);

// Two linears with bf16 weights in one kernel, hidden tile kept in registers (update_stream.hip);
// returns false when the shape is not covered and nothing was launched.
bool launch_mlp_stream(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in, const void *w1, const float *b1,
                       mgg_act_t act1, int32_t d_hid, const void *w2, const float *b2, mgg_act_t act2, int32_t d_out,
                       mgg_dtype_t out_dtype, void *out, int64_t ld_out, int cus, hipStream_t stream, hipError_t *err);

}  // namespace mgg
