// Decode path (few rows, HBM-bound): bf16, up to 64 rows.
//
// Two launches per call:
//
//  1. contract_kernel -- every contraction over d_in, streamed once from HBM:
//       * base:   partial[s][t][n] = sum_{k in slice s} W[n,k] x[t,k]        (Sec. 3.4: W x [x_0 .. x_n],
//                 shared by the whole batch).  A workgroup owns `kWaves*16` rows of W and one K-slice;
//                 each wave streams 16 rows of W straight from global memory into the A-operand of
//                 v_mfma_f32_16x16x32_bf16 (row = lane % 16, 8 consecutive k per lane), the rows of x
//                 are the B-operand, read from an LDS copy of the current 256-wide K-chunk.
//       * shrink: vpart[c][t][j] = sum_{k in slice c} A_i[j,k] x[t,k]        (A_i x_t of the row's own
//                 adapter, Sec. 3.4).  One (row, K-slice) unit per workgroup, done with plain FMAs and
//                 a wavefront reduction before the workgroup starts on its W tile.
//  2. finish_kernel -- per row t and output column n:
//       y[t,n] = bf16( sum_s partial[s][t][n] + s_i * sum_j B_i[n,j] * (sum_c vpart[c][t][j]) )
//     i.e. the K-split reduction, the expand B_i (A_i x_t), the combine and the store at the row's
//     own position (Sec. 3.4: results are combined and land at their original locations).
//
// Summation order is fixed (no float atomics): results are bit-identical from run to run.
#include "common.h"

using namespace elora;

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;        // waves per workgroup
constexpr int kRowsPerWave = 16; // W rows per wave (one MFMA row block)
constexpr int kTileRows = kWaves * kRowsPerWave;
constexpr int kChunk = 256;      // K elements per LDS stage
constexpr int kLdsStride = kChunk + 8;  // bf16 elements; +16 bytes so 16 rows hit 16 different bank groups
constexpr int kStepsPerChunk = kChunk / 32;

struct DecodeShape {
    int T, K, N;
    int split;        // K-slices of the base contraction
    int chunks_per_split;
    int vsplit;       // K-slices of the shrink
    int n_tiles;
};

template <int TT>
__global__ __launch_bounds__(kWaves * 64) void contract_kernel(DecodeShape sh, const uint16_t *__restrict__ x,
                                                               const uint16_t *__restrict__ W, PoolView pool,
                                                               RouteView route, int has_pool,
                                                               float *__restrict__ partial,
                                                               float *__restrict__ vpart)
{
    __shared__ __attribute__((aligned(16))) uint16_t xs[2][TT * 16][kLdsStride];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = sh.T, K = sh.K, N = sh.N;
    const int tile = blockIdx.x % sh.n_tiles, ks = blockIdx.x / sh.n_tiles;

    // ---- shrink unit of this workgroup (if any) --------------------------------------------
    if (has_pool) {
        for (int unit = blockIdx.x; unit < T * sh.vsplit; unit += gridDim.x) {
            int t = unit % T, c = unit / T;
            RowRoute rr = resolve_row(t, route, pool, false);
            if (rr.slot >= 0) {
                const int kv = K / sh.vsplit;  // multiple of 8 by construction
                const uint16_t *A = reinterpret_cast<const uint16_t *>(slot_A(pool, rr.slot)) + (size_t)c * kv;
                const uint16_t *xt = x + (size_t)t * K + (size_t)c * kv;
                for (int j = wave; j < rr.rank; j += kWaves) {
                    float s = 0.0f;
                    for (int k = lane * 8; k < kv; k += 64 * 8) {
                        uint4 av = *reinterpret_cast<const uint4 *>(A + (size_t)j * K + k);
                        uint4 xv = *reinterpret_cast<const uint4 *>(xt + k);
                        const uint32_t aw[4] = {av.x, av.y, av.z, av.w};
                        const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            s = fmaf(__uint_as_float(aw[q] << 16), __uint_as_float(xw[q] << 16), s);
                            s = fmaf(__uint_as_float(aw[q] & 0xffff0000u), __uint_as_float(xw[q] & 0xffff0000u), s);
                        }
                    }
                    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
                    if (lane == 0) vpart[((size_t)c * T + t) * pool.max_rank + j] = s;
                }
            }
        }
    }

    // ---- base tile ----------------------------------------------------------------------------
    const int m = lane & 15, g = lane >> 4;
    const int row = tile * kTileRows + wave * kRowsPerWave + m;  // W row this lane feeds
    const bool wave_active = (tile * kTileRows + wave * kRowsPerWave) < N;  // N % 16 == 0: whole block in or out
    const int k_begin = ks * sh.chunks_per_split * kChunk;
    const uint16_t *wrow = W + (size_t)(wave_active ? row : 0) * K + k_begin + g * 8;

    floatx4 acc[TT];
#pragma unroll
    for (int i = 0; i < TT; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    u32x4 wcur[kStepsPerChunk], wnext[kStepsPerChunk];
    // x staging: TT*16 rows x 256 k = TT*16*32 pieces of 16 bytes, TT*2 per thread
    constexpr int kXPieces = TT * 2;
    u32x4 xreg[kXPieces];

    auto load_w = [&](u32x4 *dst, int chunk) {
        const uint16_t *p = wrow + (size_t)chunk * kChunk;
#pragma unroll
        for (int j = 0; j < kStepsPerChunk; ++j)
            dst[j] = wave_active ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + j * 32)) : u32x4{0, 0, 0, 0};
    };
    auto load_x = [&](int chunk) {
#pragma unroll
        for (int i = 0; i < kXPieces; ++i) {
            int piece = tid + i * (kWaves * 64);
            int r = piece >> 5, c16 = piece & 31;
            xreg[i] = (r < T) ? *reinterpret_cast<const u32x4 *>(x + (size_t)r * K + k_begin + (size_t)chunk * kChunk + c16 * 8)
                              : u32x4{0, 0, 0, 0};
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kXPieces; ++i) {
            int piece = tid + i * (kWaves * 64);
            int r = piece >> 5, c16 = piece & 31;
            *reinterpret_cast<u32x4 *>(&xs[buf][r][c16 * 8]) = xreg[i];
        }
    };

    load_w(wcur, 0);
    load_x(0);
    store_x(0);
    __syncthreads();

    const int nchunks = sh.chunks_per_split;
    for (int c = 0; c < nchunks; ++c) {
        const bool more = (c + 1) < nchunks;
        if (more) {
            load_w(wnext, c + 1);
            load_x(c + 1);
        }
        const int buf = c & 1;
#pragma unroll
        for (int j = 0; j < kStepsPerChunk; ++j) {
            bf16x8 a = __builtin_bit_cast(bf16x8, wcur[j]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                bf16x8 b = *reinterpret_cast<const bf16x8 *>(&xs[buf][tt * 16 + m][j * 32 + g * 8]);
                acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[tt], 0, 0, 0);
            }
        }
        if (more) {
            store_x(buf ^ 1);
#pragma unroll
            for (int j = 0; j < kStepsPerChunk; ++j) wcur[j] = wnext[j];
        }
        __syncthreads();
    }

    // C layout of 16x16 MFMA: lane holds column (lane % 16) = token, rows (lane / 16) * 4 + 0..3 = W rows
    if (wave_active) {
        const int n_base = tile * kTileRows + wave * kRowsPerWave + g * 4;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            int t = tt * 16 + m;
            if (t < T) *reinterpret_cast<floatx4 *>(partial + ((size_t)ks * T + t) * N + n_base) = acc[tt];
        }
    }
}

constexpr int kFinishThreads = 256;
constexpr int kFinishCols = 2;  // output columns per thread

__global__ __launch_bounds__(kFinishThreads) void finish_kernel(DecodeShape sh, PoolView pool, RouteView route,
                                                                int has_pool, const float *__restrict__ partial,
                                                                const float *__restrict__ vpart,
                                                                uint16_t *__restrict__ y)
{
    __shared__ float v[kMaxRank];
    const int t = blockIdx.y;
    const int T = sh.T, N = sh.N;
    RowRoute rr{-1, 0, 0.0f};
    if (has_pool) rr = resolve_row(t, route, pool, blockIdx.x == 0 && threadIdx.x == 0);
    if (rr.slot >= 0) {
        for (int j = threadIdx.x; j < rr.rank; j += kFinishThreads) {
            float s = 0.0f;
            for (int c = 0; c < sh.vsplit; ++c) s += vpart[((size_t)c * T + t) * pool.max_rank + j];
            v[j] = s;
        }
    }
    __syncthreads();
    const int n = (blockIdx.x * kFinishThreads + threadIdx.x) * kFinishCols;
    if (n >= N) return;  // N is even
    float acc0 = 0.0f, acc1 = 0.0f;
    for (int s = 0; s < sh.split; ++s) {
        float2 p = *reinterpret_cast<const float2 *>(partial + ((size_t)s * T + t) * N + n);
        acc0 += p.x;
        acc1 += p.y;
    }
    if (rr.slot >= 0) {
        const uint16_t *B = reinterpret_cast<const uint16_t *>(slot_B(pool, rr.slot)) + (size_t)n * rr.rank;
        float d0 = 0.0f, d1 = 0.0f;
        const int r = rr.rank;
        if ((r & 7) == 0) {
            for (int j = 0; j < r; j += 8) {
                uint4 b0 = *reinterpret_cast<const uint4 *>(B + j);
                uint4 b1 = *reinterpret_cast<const uint4 *>(B + r + j);
                const uint32_t w0[4] = {b0.x, b0.y, b0.z, b0.w};
                const uint32_t w1[4] = {b1.x, b1.y, b1.z, b1.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    d0 = fmaf(__uint_as_float(w0[q] << 16), v[j + 2 * q], d0);
                    d0 = fmaf(__uint_as_float(w0[q] & 0xffff0000u), v[j + 2 * q + 1], d0);
                    d1 = fmaf(__uint_as_float(w1[q] << 16), v[j + 2 * q], d1);
                    d1 = fmaf(__uint_as_float(w1[q] & 0xffff0000u), v[j + 2 * q + 1], d1);
                }
            }
        } else {
            for (int j = 0; j < r; ++j) {
                d0 = fmaf(bf16_to_f32(B[j]), v[j], d0);
                d1 = fmaf(bf16_to_f32(B[r + j]), v[j], d1);
            }
        }
        acc0 += rr.scale * d0;
        acc1 += rr.scale * d1;
    }
    uint32_t packed = (uint32_t)f32_to_bf16(acc0) | ((uint32_t)f32_to_bf16(acc1) << 16);
    *reinterpret_cast<uint32_t *>(y + (size_t)t * N + n) = packed;
}

int pick_split(int K, int n_tiles)
{
    // aim at about two workgroups per compute unit (512), K-slices of whole 256-wide chunks
    int chunks = K / kChunk;
    int best = 1;
    for (int s = 1; s <= kDecodeMaxSplit; ++s) {
        if (chunks % s) continue;
        if (n_tiles * s <= 640) best = s;
    }
    return best;
}

int pick_vsplit(int K, int T, int grid)
{
    int vs = 1;
    while (vs * 2 <= kDecodeMaxVSplit && T * vs * 2 <= grid && (K / (vs * 2)) % 8 == 0 && K % (vs * 2) == 0 &&
           K / (vs * 2) >= 512)
        vs *= 2;
    return vs;
}

DecodeShape make_shape(int T, int K, int N)
{
    DecodeShape sh;
    sh.T = T;
    sh.K = K;
    sh.N = N;
    sh.n_tiles = (N + kTileRows - 1) / kTileRows;
    sh.split = pick_split(K, sh.n_tiles);
    sh.chunks_per_split = K / kChunk / sh.split;
    sh.vsplit = pick_vsplit(K, T, sh.n_tiles * sh.split);
    return sh;
}

}  // namespace

bool elora::decode_eligible(const elora_linear_desc_t &d, int max_rank)
{
    (void)max_rank;
    return d.dtype == ELORA_BF16 && d.wfmt == ELORA_W_SAME && d.n_tokens >= 1 && d.n_tokens <= kDecodeMaxTokens &&
           d.d_in % kChunk == 0 && d.d_out % 16 == 0;
}

void elora::decode_plan(const elora_linear_desc_t &d, elora_plan_t *plan)
{
    DecodeShape sh = make_shape(d.n_tokens, d.d_in, d.d_out);
    plan->n_launches = 2;
    plan->split_k = sh.split;
    plan->tile_rows = kTileRows;
    plan->tile_cols = 0;
    plan->grid = sh.n_tiles * sh.split;
}

int elora::launch_decode(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream)
{
    (void)plan;
    DecodeShape sh = make_shape(a.T, a.K, a.N);
    float *partial = reinterpret_cast<float *>(a.ws + a.wsl.partial);
    float *vpart = reinterpret_cast<float *>(a.ws + a.wsl.v);
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *W = static_cast<const uint16_t *>(a.W);
    int has_pool = a.has_pool ? 1 : 0;
    dim3 grid(sh.n_tiles * sh.split), block(kWaves * 64);
    int tt = (a.T + 15) / 16;
    switch (tt) {
    case 1: hipLaunchKernelGGL((contract_kernel<1>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, vpart); break;
    case 2: hipLaunchKernelGGL((contract_kernel<2>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, vpart); break;
    case 3: hipLaunchKernelGGL((contract_kernel<3>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, vpart); break;
    default: hipLaunchKernelGGL((contract_kernel<4>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, vpart); break;
    }
    ELORA_HIP_TRY(hipGetLastError());
    dim3 fgrid((a.N / kFinishCols + kFinishThreads - 1) / kFinishThreads, a.T);
    hipLaunchKernelGGL(finish_kernel, fgrid, dim3(kFinishThreads), 0, stream, sh, a.pool, a.route, has_pool, partial,
                       vpart, static_cast<uint16_t *>(a.y));
    ELORA_HIP_TRY(hipGetLastError());
    return ELORA_OK;
}
