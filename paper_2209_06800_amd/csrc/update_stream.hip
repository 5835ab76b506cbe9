// Dense Update for gfx950, whole-line variant (section 1: Update is a fully-connected layer;
// section 7: X W with ReLU, GIN's MLP) for the shapes that are bound by HBM: a tall A, a weight
// matrix small enough to stay in LDS.
//
// What the memory system rewards, measured with copy kernels of the same tile shape: every global
// instruction should consume whole 128-byte lines (a tile copy with 2 lanes per row moves 2.7 TB/s,
// with 8 or more lanes per row 4.2 TB/s), and no line should be visited by several instructions
// spread over time.  The MFMA operand layouts give a row to a lane, i.e. 2 lanes per row.  So here
//   - a K slab of A is read with 8 or 16 lanes per row (one or two whole lines per row and
//     instruction), held raw in registers D slabs ahead, then written -- converted to bf16 on the
//     bf16 path -- into a per-wavefront LDS buffer from which the MFMA operands are read;
//   - the output tile goes back through the same LDS buffer and leaves as whole lines too;
//   - everything a wavefront waits for is older than its last stores, and the loop over K slabs is
//     unrolled with the first tile peeled, so that the compiler's wait counts are exact and no wait
//     includes a store.
// W is staged once per workgroup (four wavefronts, each walking over its own 32-row tiles; the
// grid is sized to the chip).  Arithmetic and rounding are those of update.hip.
#include "update_common.h"

namespace mgg {

namespace {

using namespace upd;

// wavefronts per SIMD the register budget is cut for (the widest variant needs about 160 registers)
#ifndef MGG_UPD_STREAM_WAVES
#define MGG_UPD_STREAM_WAVES(NT) ((NT) == 4 ? 3 : 4)
#endif
// Slabs requested ahead.  Measured on MI355X: deeper queues (4, or 6 with two wavefronts per SIMD)
// cost registers or spills and are slower than these.
#ifndef MGG_SD_B16      // bf16 A (16 registers a slab); fp32 A on the bf16 path takes half as many
#define MGG_SD_B16 2
#endif
#ifndef MGG_SD_F32      // fp32 path (16 registers a slab)
#define MGG_SD_F32 2
#endif

extern __shared__ __attribute__((aligned(16))) unsigned char lds_all[];

__device__ __forceinline__ void wave_sync_lds()
{
    // LDS traffic of one wavefront is executed in order; this only keeps the compiler from moving
    // LDS reads of other lanes' data across the writes that produce them
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Output tile: acc holds the transposed 32x32 tiles (register r of lane (m, h): row m, column
// 8*(r/4) + 4*h + r%4).  Blocks of CW columns are written to the wavefront's LDS buffer as
// fp32 [32][CW + 4] and read back with CW/4 (fp32 out) or CW/8 (bf16 out) lanes per row.
template <int NT, bool OUT_BF16>
__device__ __forceinline__ void store_tile_lines(const UpdArgs &p, const f32x16 (&acc)[NT], float *cbuf, int64_t m0, int lane)
{
    constexpr int TPB = OUT_BF16 && NT >= 2 ? 2 : 1;      // 32-column tiles per block
    constexpr int CW = 32 * TPB, LDC = CW + 4;
    constexpr int EPL = OUT_BF16 ? 8 : 4;                  // output elements per lane and store (16 bytes)
    constexpr int LPR = CW / EPL;                          // lanes per row
    constexpr int RPI = kWave / LPR;                       // rows per store instruction
    const int m = lane & 31, h = lane >> 5;
#pragma unroll
    for (int b = 0; b < NT / TPB; ++b) {
#pragma unroll
        for (int tt = 0; tt < TPB; ++tt) {
            const int t = b * TPB + tt;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = t * 32 + 8 * q + 4 * h;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[e] = acc[t][4 * q + e] + ((p.bias && col + e < p.d_out) ? p.bias[col + e] : 0.f);
                    if (p.relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
                *reinterpret_cast<float4 *>(cbuf + m * LDC + tt * 32 + 8 * q + 4 * h) = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
        wave_sync_lds();
#pragma unroll
        for (int j = 0; j < 32 / RPI; ++j) {
            const int r = j * RPI + lane / LPR, c = (lane % LPR) * EPL;
            const int64_t row = m0 + r;
            const int col = b * CW + c;
            float v[EPL];
#pragma unroll
            for (int e4 = 0; e4 < EPL / 4; ++e4) {
                const float4 x = *reinterpret_cast<const float4 *>(cbuf + r * LDC + c + 4 * e4);
                v[4 * e4] = x.x; v[4 * e4 + 1] = x.y; v[4 * e4 + 2] = x.z; v[4 * e4 + 3] = x.w;
            }
            if (row < p.n_rows && col < p.d_out) {
                const bool full = p.out_vec_ok && col + EPL <= p.d_out;
                if constexpr (OUT_BF16) {
                    uint16_t *o = static_cast<uint16_t *>(p.out) + row * p.ld_out + col;
                    if (full && p.ld_out % 8 == 0 && (reinterpret_cast<uintptr_t>(p.out) & 15u) == 0) {
                        uint4 pk;
                        pk.x = f32_to_bf16_bits(v[0]) | (f32_to_bf16_bits(v[1]) << 16);
                        pk.y = f32_to_bf16_bits(v[2]) | (f32_to_bf16_bits(v[3]) << 16);
                        pk.z = f32_to_bf16_bits(v[4]) | (f32_to_bf16_bits(v[5]) << 16);
                        pk.w = f32_to_bf16_bits(v[6]) | (f32_to_bf16_bits(v[7]) << 16);
                        *reinterpret_cast<uint4 *>(o) = pk;
                    } else {
#pragma unroll
                        for (int e = 0; e < EPL; ++e)
                            if (col + e < p.d_out) o[e] = static_cast<uint16_t>(f32_to_bf16_bits(v[e]));
                    }
                } else {
                    float *o = static_cast<float *>(p.out) + row * p.ld_out + col;
                    if (full) {
                        *reinterpret_cast<float4 *>(o) = make_float4(v[0], v[1], v[2], v[3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < EPL; ++e)
                            if (col + e < p.d_out) o[e] = v[e];
                    }
                }
            }
        }
        wave_sync_lds();
    }
}

template <int NT, bool OUT_BF16>
constexpr int wave_lds_bytes(int a_bytes)
{
    constexpr int TPB = OUT_BF16 && NT >= 2 ? 2 : 1;
    constexpr int c_bytes = 32 * (32 * TPB + 4) * 4;
    return a_bytes > c_bytes ? a_bytes : c_bytes;
}

// ---- bf16 weights: v_mfma_f32_32x32x16_bf16, K slabs of 64 --------------------------------------
union Frag8 { uint32_t u[4]; uint4 q; bf16x8 v; };

template <bool A_BF16> struct Raw { uint4 v[A_BF16 ? 4 : 8]; };

// Slab `is` of tile `t`: 64 k values of 32 rows.  fp32: 256 bytes per row, 16 lanes per row, 4 rows
// per instruction; bf16: 128 bytes per row, 8 lanes per row, 8 rows per instruction.  Rows past
// the end of A are clamped to the last row (loaded, never stored).
template <bool A_BF16>
__device__ __forceinline__ void load_slab(const UpdArgs &p, int64_t t, int is, int lane, Raw<A_BF16> &r)
{
    constexpr int LPR = A_BF16 ? 8 : 16, RPI = kWave / LPR, NI = 32 / RPI;
    const int sub = lane / LPR, chunk = lane % LPR;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        int64_t row = t * 32 + j * RPI + sub;
        row = row < p.n_rows ? row : p.n_rows - 1;
        if constexpr (A_BF16)
            r.v[j] = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(p.a) + row * p.ld_a + is * 64 + chunk * 8);
        else
            r.v[j] = *reinterpret_cast<const uint4 *>(static_cast<const float *>(p.a) + row * p.ld_a + is * 64 + chunk * 4);
    }
}

// raw slab -> the wavefront's LDS buffer, bf16 [32][LDA]
template <bool A_BF16, int LDA>
__device__ __forceinline__ void stage_slab(const Raw<A_BF16> &r, uint16_t *abuf, int lane)
{
    constexpr int LPR = A_BF16 ? 8 : 16, RPI = kWave / LPR, NI = 32 / RPI;
    const int sub = lane / LPR, chunk = lane % LPR;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
        const int row = j * RPI + sub;
        if constexpr (A_BF16) {
            *reinterpret_cast<uint4 *>(abuf + row * LDA + chunk * 8) = r.v[j];
        } else {
            uint2 pk;
            pk.x = f32_to_bf16_bits(__uint_as_float(r.v[j].x)) | (f32_to_bf16_bits(__uint_as_float(r.v[j].y)) << 16);
            pk.y = f32_to_bf16_bits(__uint_as_float(r.v[j].z)) | (f32_to_bf16_bits(__uint_as_float(r.v[j].w)) << 16);
            *reinterpret_cast<uint2 *>(abuf + row * LDA + chunk * 4) = pk;
        }
    }
}

template <int NT, int NS, bool A_BF16, bool OUT_BF16, int D>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(MGG_UPD_STREAM_WAVES(NT), MGG_UPD_STREAM_WAVES(NT))))
void update_bf16_stream_kernel(const UpdArgs p)
{
    constexpr int BK = 64, NC = NT * 32, LDA = BK + 8, LDW = NS * BK + 8;
    constexpr int W_BYTES = (NC * LDW * 2 + 15) / 16 * 16;
    constexpr int WAVE_BYTES = wave_lds_bytes<NT, OUT_BF16>(32 * LDA * 2);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    uint16_t *w_lds = reinterpret_cast<uint16_t *>(lds_all);
    uint16_t *abuf = reinterpret_cast<uint16_t *>(lds_all + W_BYTES + wave * WAVE_BYTES);
    fill_w_bf16_t<NC>(w_lds, LDW, static_cast<const uint16_t *>(p.w), 0, NS * BK, 0, p);
    __syncthreads();

    const int64_t n_tiles = (p.n_rows + 31) / 32, stride = static_cast<int64_t>(gridDim.x) * kWaves;
    int64_t tile = static_cast<int64_t>(blockIdx.x) * kWaves + wave;
    if (tile >= n_tiles) return;
    // issue cursor: the slab requested next; it runs past the last tile (rows are clamped then)
    int64_t itile = tile;
    int is = 0;
    Raw<A_BF16> q[D];
    auto issue = [&]() {
        Raw<A_BF16> r;
        load_slab<A_BF16>(p, itile, is, lane, r);
        if (++is == NS) { is = 0; itile += stride; }
        return r;
    };
#pragma unroll
    for (int d = 0; d < D; ++d) q[d] = issue();

    auto do_tile = [&]() {
        f32x16 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            stage_slab<A_BF16, LDA>(q[0], abuf, lane);
#pragma unroll
            for (int d = 0; d + 1 < D; ++d) q[d] = q[d + 1];
            q[D - 1] = issue();
            wave_sync_lds();
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                Frag8 af;
                af.q = *reinterpret_cast<const uint4 *>(abuf + i * LDA + 32 * h + 8 * c);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    Frag8 bw;
                    bw.q = *reinterpret_cast<const uint4 *>(&w_lds[(t * 32 + i) * LDW + s * BK + 32 * h + 8 * c]);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw.v, af.v, acc[t], 0, 0, 0);
                }
            }
            wave_sync_lds();
        }
        store_tile_lines<NT, OUT_BF16>(p, acc, reinterpret_cast<float *>(abuf), tile * 32, lane);
        tile += stride;
    };
    do_tile();                      // peeled: the loop below then meets the same pattern of pending
    while (tile < n_tiles) do_tile();   // memory operations on entry and on its back edge
}

// ---- fp32 weights: v_mfma_f32_32x32x2_f32, K slabs of 32 ----------------------------------------
// Slab: 128 bytes per row, 8 lanes per row, 8 rows per instruction; staged as fp32 [32][36].
struct RawF { float4 v[4]; };

__device__ __forceinline__ void load_slab_f32(const UpdArgs &p, int64_t t, int is, int lane, RawF &r)
{
    const int sub = lane / 8, chunk = lane % 8;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int64_t row = t * 32 + j * 8 + sub;
        row = row < p.n_rows ? row : p.n_rows - 1;
        r.v[j] = *reinterpret_cast<const float4 *>(static_cast<const float *>(p.a) + row * p.ld_a + is * 32 + chunk * 4);
    }
}

template <int NT, int NS, int D>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(MGG_UPD_STREAM_WAVES(NT), MGG_UPD_STREAM_WAVES(NT))))
void update_f32_stream_kernel(const UpdArgs p)
{
    constexpr int BK = 32, NC = NT * 32, LDA = BK + 4;
    constexpr int W_BYTES = NS * BK * NC * 4;
    constexpr int WAVE_BYTES = wave_lds_bytes<NT, false>(32 * LDA * 4);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    float *w_lds = reinterpret_cast<float *>(lds_all);
    float *abuf = reinterpret_cast<float *>(lds_all + W_BYTES + wave * WAVE_BYTES);
    fill_w_f32<NC>(w_lds, static_cast<const float *>(p.w), 0, NS * BK, 0, p);
    __syncthreads();

    const int64_t n_tiles = (p.n_rows + 31) / 32, stride = static_cast<int64_t>(gridDim.x) * kWaves;
    int64_t tile = static_cast<int64_t>(blockIdx.x) * kWaves + wave;
    if (tile >= n_tiles) return;
    int64_t itile = tile;
    int is = 0;
    RawF q[D];
    auto issue = [&]() {
        RawF r;
        load_slab_f32(p, itile, is, lane, r);
        if (++is == NS) { is = 0; itile += stride; }
        return r;
    };
#pragma unroll
    for (int d = 0; d < D; ++d) q[d] = issue();

    auto do_tile = [&]() {
        f32x16 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            {
                const int sub = lane / 8, chunk = lane % 8;
#pragma unroll
                for (int j = 0; j < 4; ++j) *reinterpret_cast<float4 *>(abuf + (j * 8 + sub) * LDA + chunk * 4) = q[0].v[j];
            }
#pragma unroll
            for (int d = 0; d + 1 < D; ++d) q[d] = q[d + 1];
            q[D - 1] = issue();
            wave_sync_lds();
            // lane (i, h) takes k = 16h .. 16h + 15 of the slab, MFMA number c contracts {c, 16 + c}
            float af[16];
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                const float4 x = *reinterpret_cast<const float4 *>(abuf + i * LDA + 16 * h + 4 * c4);
                af[4 * c4] = x.x; af[4 * c4 + 1] = x.y; af[4 * c4 + 2] = x.z; af[4 * c4 + 3] = x.w;
            }
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                const float *wrow = w_lds + (s * BK + 16 * h + c) * NC + i;
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(wrow[t * 32], af[c], acc[t], 0, 0, 0);
            }
            wave_sync_lds();
        }
        store_tile_lines<NT, false>(p, acc, abuf, tile * 32, lane);
        tile += stride;
    };
    do_tile();
    while (tile < n_tiles) do_tile();
}

// ---- two linears in one kernel (GIN's MLP, section 7) ------------------------------------------
// out = act2(act1(A W1 + b1) W2 + b2) with bf16 weights, A the aggregation result (fp32 or bf16), a hidden
// width of at most 128.  The hidden tile never leaves the registers: the accumulators of the first
// product (register r of lane (m, h), tile t: row m, hidden column 32 t + 8 (r/4) + 4 h + r%4) get bias
// and ReLU, are rounded to bf16 -- as the hidden activations of the two-launch path are -- and eight
// consecutive registers packed together are, as they stand, the A operand of one MFMA of the second
// product.  MFMA sums over k in any order, so W2 is staged in LDS with its k index permuted to
// match: within every group of 16, hidden column 8 a + 4 h + e sits at position 8 h + 4 a + e.
constexpr int kMlpWaves = 8;
constexpr int kMlpThreads = kWave * kMlpWaves;

struct MlpArgs {
    const void *a;           // fp32 or bf16
    const uint16_t *w1, *w2;
    const float *b1, *b2;
    void *out;
    int64_t n_rows, ld_a, ld_out;
    int32_t d_in, d_hid, d_out;
    int32_t relu1, relu2, out_vec_ok;
};

template <int NS1, int NT2, bool A_BF16, bool OUT_BF16>
__global__ __launch_bounds__(kMlpThreads) __attribute__((amdgpu_waves_per_eu(2, 2)))
void mlp_bf16_stream_kernel(const MlpArgs m)
{
    constexpr int BK = 64, NT1 = 4, H = NT1 * 32, LDA = BK + 8, LDW1 = NS1 * BK + 8, LDW2 = H + 8, NC2 = NT2 * 32;
    constexpr int W1_BYTES = (H * LDW1 * 2 + 15) / 16 * 16, W2_BYTES = (NC2 * LDW2 * 2 + 15) / 16 * 16;
    constexpr int WAVE_BYTES = wave_lds_bytes<NT2, OUT_BF16>(32 * LDA * 2);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = lane & 31, h = lane >> 5;
    uint16_t *w1_lds = reinterpret_cast<uint16_t *>(lds_all);
    uint16_t *w2_lds = reinterpret_cast<uint16_t *>(lds_all + W1_BYTES);
    uint16_t *abuf = reinterpret_cast<uint16_t *>(lds_all + W1_BYTES + W2_BYTES + wave * WAVE_BYTES);
    {
        // W1^T [H][LDW1] and W2^T [NC2][LDW2] (k permuted), zero outside the matrices; pairs of k per dword
        uint32_t *l1 = reinterpret_cast<uint32_t *>(w1_lds), *l2 = reinterpret_cast<uint32_t *>(w2_lds);
        for (int id = threadIdx.x; id < (NS1 * BK / 2) * H; id += kMlpThreads) {
            const int k = 2 * (id / H), n = id % H;
            const uint32_t lo = (k < m.d_in && n < m.d_hid) ? m.w1[static_cast<int64_t>(k) * m.d_hid + n] : 0u;
            const uint32_t hi = (k + 1 < m.d_in && n < m.d_hid) ? m.w1[static_cast<int64_t>(k + 1) * m.d_hid + n] : 0u;
            l1[n * (LDW1 / 2) + k / 2] = lo | (hi << 16);
        }
        for (int id = threadIdx.x; id < (H / 2) * NC2; id += kMlpThreads) {
            const int k = 2 * (id / NC2), n = id % NC2;
            const uint32_t lo = (k < m.d_hid && n < m.d_out) ? m.w2[static_cast<int64_t>(k) * m.d_out + n] : 0u;
            const uint32_t hi = (k + 1 < m.d_hid && n < m.d_out) ? m.w2[static_cast<int64_t>(k + 1) * m.d_out + n] : 0u;
            const int o = k & 15, kp = (k & ~15) + 8 * ((o >> 2) & 1) + 4 * (o >> 3) + (o & 3);
            l2[n * (LDW2 / 2) + kp / 2] = lo | (hi << 16);
        }
    }
    __syncthreads();

    UpdArgs pa{};           // what the slab loads and the epilogue read
    pa.a = m.a; pa.n_rows = m.n_rows; pa.ld_a = m.ld_a;
    pa.out = m.out; pa.ld_out = m.ld_out; pa.d_out = m.d_out; pa.bias = m.b2; pa.relu = m.relu2; pa.out_vec_ok = m.out_vec_ok;

    const int64_t n_tiles = (m.n_rows + 31) / 32, stride = static_cast<int64_t>(gridDim.x) * kMlpWaves;
    int64_t tile = static_cast<int64_t>(blockIdx.x) * kMlpWaves + wave;
    if (tile >= n_tiles) return;
    int64_t itile = tile;
    int is = 0;
    Raw<A_BF16> q;
    auto issue = [&]() {
        Raw<A_BF16> r;
        load_slab<A_BF16>(pa, itile, is, lane, r);
        if (++is == NS1) { is = 0; itile += stride; }
        return r;
    };
    q = issue();

    auto do_tile = [&]() {
        f32x16 acc[NT1];
#pragma unroll
        for (int t = 0; t < NT1; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int s = 0; s < NS1; ++s) {
            stage_slab<A_BF16, LDA>(q, abuf, lane);
            q = issue();
            wave_sync_lds();
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                Frag8 af;
                af.q = *reinterpret_cast<const uint4 *>(abuf + i * LDA + 32 * h + 8 * c);
#pragma unroll
                for (int t = 0; t < NT1; ++t) {
                    Frag8 bw;
                    bw.q = *reinterpret_cast<const uint4 *>(&w1_lds[(t * 32 + i) * LDW1 + s * BK + 32 * h + 8 * c]);
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw.v, af.v, acc[t], 0, 0, 0);
                }
            }
            wave_sync_lds();
        }
        // hidden tile -> operands of the second product
        Frag8 hf[NT1 * 2];
#pragma unroll
        for (int t = 0; t < NT1; ++t)
#pragma unroll
            for (int qp = 0; qp < 2; ++qp) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int col = t * 32 + 16 * qp + 8 * (e / 4) + 4 * h + e % 4;
                    v[e] = acc[t][8 * qp + e] + ((m.b1 && col < m.d_hid) ? m.b1[col] : 0.f);
                    if (m.relu1) v[e] = v[e] > 0.f ? v[e] : 0.f;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) hf[t * 2 + qp].u[e] = f32_to_bf16_bits(v[2 * e]) | (f32_to_bf16_bits(v[2 * e + 1]) << 16);
            }
        f32x16 acc2[NT2];
#pragma unroll
        for (int t = 0; t < NT2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc2[t][r] = 0.f;
#pragma unroll
        for (int g = 0; g < NT1 * 2; ++g)
#pragma unroll
            for (int t = 0; t < NT2; ++t) {
                Frag8 bw;
                bw.q = *reinterpret_cast<const uint4 *>(&w2_lds[(t * 32 + i) * LDW2 + 16 * g + 8 * h]);
                acc2[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw.v, hf[g].v, acc2[t], 0, 0, 0);
            }
        store_tile_lines<NT2, OUT_BF16>(pa, acc2, reinterpret_cast<float *>(abuf), tile * 32, lane);
        tile += stride;
    };
    do_tile();
    while (tile < n_tiles) do_tile();
}

template <int NS1, int NT2>
hipError_t launch_mlp(const MlpArgs &m, bool a_bf16, bool out_bf16, int cus, hipStream_t s)
{
    constexpr int W1_BYTES = (128 * (NS1 * 64 + 8) * 2 + 15) / 16 * 16, W2_BYTES = (NT2 * 32 * 136 * 2 + 15) / 16 * 16;
    const int wave_bytes = out_bf16 ? wave_lds_bytes<NT2, true>(32 * 72 * 2) : wave_lds_bytes<NT2, false>(32 * 72 * 2);
    const size_t lds = static_cast<size_t>(W1_BYTES) + W2_BYTES + kMlpWaves * static_cast<size_t>(wave_bytes);
    const int64_t want = ((m.n_rows + 31) / 32 + kMlpWaves - 1) / kMlpWaves;
    const int blocks = static_cast<int>(want < cus ? want : cus);      // the LDS of a CU holds one workgroup
    auto go = [&](auto kernel) {
        // more than 64 KB of dynamic LDS: ask for it (cheap, so done at every launch rather than remembered)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kMlpThreads), lds, s, m);
        return hipGetLastError();
    };
    if (a_bf16) return out_bf16 ? go(mlp_bf16_stream_kernel<NS1, NT2, true, true>) : go(mlp_bf16_stream_kernel<NS1, NT2, true, false>);
    return out_bf16 ? go(mlp_bf16_stream_kernel<NS1, NT2, false, true>) : go(mlp_bf16_stream_kernel<NS1, NT2, false, false>);
}

template <int NT, int NS>
hipError_t launch_bf16(const UpdArgs &p, bool a_bf16, int cus, hipStream_t s)
{
    constexpr int LDW = NS * 64 + 8, W_BYTES = (NT * 32 * LDW * 2 + 15) / 16 * 16;
    auto go = [&](auto kernel, int wave_bytes) {
        const size_t lds = static_cast<size_t>(W_BYTES) + kWaves * static_cast<size_t>(wave_bytes);
        int per_cu = static_cast<int>((160 * 1024) / (lds + 512));
        { const int cap = MGG_UPD_STREAM_WAVES(NT); per_cu = per_cu < 1 ? 1 : (per_cu > cap ? cap : per_cu); }
        const int64_t want = ((p.n_rows + 31) / 32 + kWaves - 1) / kWaves;
        const int blocks = static_cast<int>(want < static_cast<int64_t>(cus) * per_cu ? want : static_cast<int64_t>(cus) * per_cu);
        hipLaunchKernelGGL(kernel, dim3(blocks), dim3(kThreads), lds, s, p);
        return hipGetLastError();
    };
    constexpr int A_BYTES = 32 * 72 * 2;
    if (p.out_bf16) {
        const int wb = wave_lds_bytes<NT, true>(A_BYTES);
        return a_bf16 ? go(update_bf16_stream_kernel<NT, NS, true, true, MGG_SD_B16>, wb) : go(update_bf16_stream_kernel<NT, NS, false, true, MGG_SD_B16 / 2>, wb);
    }
    const int wb = wave_lds_bytes<NT, false>(A_BYTES);
    return a_bf16 ? go(update_bf16_stream_kernel<NT, NS, true, false, MGG_SD_B16>, wb) : go(update_bf16_stream_kernel<NT, NS, false, false, MGG_SD_B16 / 2>, wb);
}

template <int NT, int NS>
hipError_t launch_f32(const UpdArgs &p, int cus, hipStream_t s)
{
    constexpr int W_BYTES = NS * 32 * NT * 32 * 4;
    const int wave_bytes = wave_lds_bytes<NT, false>(32 * 36 * 4);
    const size_t lds = static_cast<size_t>(W_BYTES) + kWaves * static_cast<size_t>(wave_bytes);
    int per_cu = static_cast<int>((160 * 1024) / (lds + 512));
    const int cap = MGG_UPD_STREAM_WAVES(NT);
    per_cu = per_cu < 1 ? 1 : (per_cu > cap ? cap : per_cu);
    const int64_t want = ((p.n_rows + 31) / 32 + kWaves - 1) / kWaves;
    const int blocks = static_cast<int>(want < static_cast<int64_t>(cus) * per_cu ? want : static_cast<int64_t>(cus) * per_cu);
    hipLaunchKernelGGL((update_f32_stream_kernel<NT, NS, MGG_SD_F32>), dim3(blocks), dim3(kThreads), lds, s, p);
    return hipGetLastError();
}

}  // namespace

bool launch_mlp_stream(int64_t n_rows, mgg_dtype_t a_dtype, const void *a, int64_t ld_a, int32_t d_in, const void *w1, const float *b1,
                       mgg_act_t act1, int32_t d_hid, const void *w2, const float *b2, mgg_act_t act2, int32_t d_out,
                       mgg_dtype_t out_dtype, void *out, int64_t ld_out, int cus, hipStream_t stream, hipError_t *err)
{
    // covered: A (fp32 or bf16) whose rows allow 16-byte loads, d_in = 64 or 128, 33..128 hidden and output
    // columns, elementwise activations
    const bool ab = a_dtype == MGG_BF16;
    if ((reinterpret_cast<uintptr_t>(a) & 15u) || ld_a % (ab ? 8 : 4) || (d_in != 64 && d_in != 128)) return false;
    if (d_hid <= 32 || d_hid > 128 || d_out <= 32 || d_out > 128) return false;
    if ((act1 != MGG_ACT_NONE && act1 != MGG_ACT_RELU) || (act2 != MGG_ACT_NONE && act2 != MGG_ACT_RELU)) return false;
    MlpArgs m{};
    m.a = a; m.w1 = static_cast<const uint16_t *>(w1); m.w2 = static_cast<const uint16_t *>(w2); m.b1 = b1; m.b2 = b2; m.out = out;
    m.n_rows = n_rows; m.ld_a = ld_a; m.ld_out = ld_out; m.d_in = d_in; m.d_hid = d_hid; m.d_out = d_out;
    m.relu1 = act1 == MGG_ACT_RELU; m.relu2 = act2 == MGG_ACT_RELU;
    const bool ob = out_dtype == MGG_BF16;
    m.out_vec_ok = (ld_out % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % (ob ? 8 : 16) == 0);
    const int nt2 = d_out > 64 ? 4 : 2;
    if (d_in == 64) *err = nt2 == 4 ? launch_mlp<1, 4>(m, ab, ob, cus, stream) : launch_mlp<1, 2>(m, ab, ob, cus, stream);
    else *err = nt2 == 4 ? launch_mlp<2, 4>(m, ab, ob, cus, stream) : launch_mlp<2, 2>(m, ab, ob, cus, stream);
    return true;
}

bool launch_update_stream(const upd::UpdArgs &p, bool w_bf16, bool a_bf16, int cus, hipStream_t stream, hipError_t *err)
{
    // covered: rows of A that allow 16-byte loads, d_in a whole number of K slabs (1, 2 or 4 of 64 for
    // bf16 weights; 1, 2, 4 or 8 of 32 for fp32 weights), 33..128 output columns
    if (!p.a_vec_ok || p.d_out <= 32 || p.d_out > 128) return false;
    const int nt = p.d_out > 64 ? 4 : 2;
    *err = hipSuccess;
    if (w_bf16) {
        if (p.d_in % 64) return false;
        const int ns = p.d_in / 64;
        if (nt == 2) {
            if (ns == 1) *err = launch_bf16<2, 1>(p, a_bf16, cus, stream);
            else if (ns == 2) *err = launch_bf16<2, 2>(p, a_bf16, cus, stream);
            else if (ns == 4) *err = launch_bf16<2, 4>(p, a_bf16, cus, stream);
            else return false;
        } else {
            if (ns == 1) *err = launch_bf16<4, 1>(p, a_bf16, cus, stream);
            else if (ns == 2) *err = launch_bf16<4, 2>(p, a_bf16, cus, stream);
            else if (ns == 4) *err = launch_bf16<4, 4>(p, a_bf16, cus, stream);
            else return false;
        }
        return true;
    }
    if (a_bf16 || p.d_in % 32) return false;
    const int ns = p.d_in / 32;
    if (nt == 2) {
        if (ns == 1) *err = launch_f32<2, 1>(p, cus, stream);
        else if (ns == 2) *err = launch_f32<2, 2>(p, cus, stream);
        else if (ns == 4) *err = launch_f32<2, 4>(p, cus, stream);
        else if (ns == 8) *err = launch_f32<2, 8>(p, cus, stream);
        else return false;
    } else {
        if (ns == 1) *err = launch_f32<4, 1>(p, cus, stream);
        else if (ns == 2) *err = launch_f32<4, 2>(p, cus, stream);
        else if (ns == 4) *err = launch_f32<4, 4>(p, cus, stream);
        else return false;          // 8 slabs of a 128-column matrix do not fit LDS next to the buffers
    }
    return true;
}

}  // namespace mgg
