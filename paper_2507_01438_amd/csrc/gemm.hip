// Prefill / mixed path (many rows, MFMA-bound): bf16 activations, bf16 or 4-bit base weights.
//
// Three launches per call:
//   route   per row: validated pool slot and scale (Sec. 3.4: each request names its adapter)
//   shrink  V[t, :] = bf16(s_t * A_i x_t) for every row, with the rows grouped by adapter inside each
//           32-row tile ("u-batches", Sec. 3.4 / 4.3: rows that share an adapter are computed together):
//           one masked MFMA pass per run of equal adapters
//   gemm    Y = X W^T (Sec. 3.4: the base product, shared by the whole batch) on 256 x 256 tiles with
//           LDS-staged 64-wide K blocks and v_mfma_f32_32x32x16_bf16; the expand B_i v_t is appended to
//           the K loop as extra K blocks (one per run of rows that share an adapter: A-operand = the
//           run's rows of V, B-operand = B_i), or, for runs too short to be worth a K block, added
//           per row in the epilogue with plain FMAs.  The epilogue rounds once to bf16 and stores each
//           row at its own position.
#include "common.h"

using namespace elora;

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// ------------------------------------------------------------------------------------------------
// route
// ------------------------------------------------------------------------------------------------
__global__ void gemm_route_kernel(int T, RouteView route, PoolView pool, int has_pool, int32_t *row_slot,
                                  float *row_scale)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    RowRoute r{-1, 0, 0.0f};
    if (has_pool) r = resolve_row(t, route, pool, true);
    row_slot[t] = r.slot;
    row_scale[t] = r.scale;
}

// ------------------------------------------------------------------------------------------------
// shrink: 32-row tiles, 4 waves split K, one masked pass per run of equal adapters
// ------------------------------------------------------------------------------------------------
constexpr int kShrinkRows = 32;
constexpr int kShrinkThreads = 256;
constexpr int kShrinkColsPerPass = 64;  // rank columns per pass (4 MFMA column blocks of 16)

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

__global__ __launch_bounds__(kShrinkThreads) void sgmv_shrink_kernel(int T, int K, const uint16_t *__restrict__ x,
                                                                     PoolView pool,
                                                                     const int32_t *__restrict__ row_slot,
                                                                     const float *__restrict__ row_scale,
                                                                     uint16_t *__restrict__ V, int Rpad)
{
    __shared__ int s_slot[kShrinkRows];
    __shared__ float s_red[4][kShrinkRows][kShrinkColsPerPass + 1];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = blockIdx.x * kShrinkRows;
    if (tid < kShrinkRows) s_slot[tid] = (r0 + tid < T) ? row_slot[r0 + tid] : -1;
    // rows without adapter and columns beyond the rank read as zero in the GEMM's K-extension
    for (int e = tid; e < kShrinkRows * Rpad; e += kShrinkThreads) {
        int r = e / Rpad;
        if (r0 + r < T) V[(size_t)(r0 + r) * Rpad + (e - r * Rpad)] = 0;
    }
    __syncthreads();

    const int m = lane & 15, g = lane >> 4;
    const int kq = K / 4;  // K % 64 == 0, so each wave's quarter is a multiple of 16; steps of 32 with a guard
    const int kbeg = wave * kq, kend = kbeg + kq;

    int run_start = 0;
    while (run_start < kShrinkRows) {
        const int slot = s_slot[run_start];
        int run_end = run_start + 1;
        while (run_end < kShrinkRows && s_slot[run_end] == slot) ++run_end;
        if (slot >= 0) {
            const int rank = pool.meta[slot].rank;
            const uint16_t *A = reinterpret_cast<const uint16_t *>(slot_A(pool, slot));
            for (int j0 = 0; j0 < rank; j0 += kShrinkColsPerPass) {
                floatx4 acc[2][4];
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
                const int ncb = min(4, (rank - j0 + 15) / 16);  // 16-column blocks in this pass
                for (int k = kbeg; k < kend; k += 32) {
                    const int kk = k + g * 8;
                    const bool kin = kk < kend;  // the last step of a quarter may be half empty
                    bf16x8 xa[2], ab[4];
#pragma unroll
                    for (int a = 0; a < 2; ++a) {
                        const int row = r0 + a * 16 + m;
                        u32x4 v = (kin && row < T) ? *reinterpret_cast<const u32x4 *>(x + (size_t)row * K + kk) : u32x4{0, 0, 0, 0};
                        xa[a] = __builtin_bit_cast(bf16x8, v);
                    }
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int j = j0 + b * 16 + m;
                        u32x4 v = (kin && b < ncb && j < rank) ? *reinterpret_cast<const u32x4 *>(A + (size_t)j * K + kk) : u32x4{0, 0, 0, 0};
                        ab[b] = __builtin_bit_cast(bf16x8, v);
                    }
#pragma unroll
                    for (int a = 0; a < 2; ++a)
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            if (b < ncb) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab[b], xa[a], acc[a][b], 0, 0, 0);
                }
                // MFMA rows = rank rows j (A-operand), columns = batch rows (B-operand):
                // lane holds batch row (lane % 16), rank rows (lane / 16) * 4 + 0..3
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b)
#pragma unroll
                        for (int i = 0; i < 4; ++i) s_red[wave][a * 16 + m][b * 16 + g * 4 + i] = acc[a][b][i];
                __syncthreads();
                for (int e = tid; e < kShrinkRows * kShrinkColsPerPass; e += kShrinkThreads) {
                    const int r = e / kShrinkColsPerPass, c = e - r * kShrinkColsPerPass;
                    const int j = j0 + c;
                    if (r >= run_start && r < run_end && j < rank && r0 + r < T) {
                        float s = s_red[0][r][c] + s_red[1][r][c] + s_red[2][r][c] + s_red[3][r][c];
                        V[(size_t)(r0 + r) * Rpad + j] = f32_to_bf16(row_scale[r0 + r] * s);
                    }
                }
                __syncthreads();
            }
        }
        run_start = run_end;
    }
}

// ------------------------------------------------------------------------------------------------
// gemm
// ------------------------------------------------------------------------------------------------
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kGemmThreads = 512;        // 8 waves: 2 along M x 4 along N, 128 x 64 outputs per wave
constexpr int kLdsRow = BK + 8;          // bf16 elements per staged row (+16 bytes: conflict-free 16-byte reads)
constexpr int kStageElems = (BM + BN) * kLdsRow;
constexpr int kMinRunForMfma = 16;       // shorter runs of equal adapters are expanded per row in the epilogue
constexpr int kMaxRuns = BM;

struct GemmArgs {
    int T, K, N;
    const uint16_t *x;
    const void *W;
    const uint16_t *w_scales;
    const int32_t *row_slot;
    const uint16_t *V;
    int Rpad;
    uint16_t *y;
    int tiles_m, tiles_n;
};

struct Run {
    int start, end, slot, rank;
};

template <int WFMT>
__global__ __launch_bounds__(kGemmThreads) void lora_gemm_kernel(GemmArgs ga, PoolView pool, int has_pool)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t *stage0 = reinterpret_cast<uint16_t *>(smem_raw);
    __shared__ int s_slot[BM];
    __shared__ unsigned long long s_mask[BM / 64];
    __shared__ Run s_runs[kMaxRuns];
    __shared__ int s_nruns;
    __shared__ unsigned char s_valu_row[BM];  // 1: this row's expand is added in the epilogue

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = ga.T, K = ga.K, N = ga.N;
    // consecutive workgroups walk down a column of row tiles so that they share the W tile in L2
    const int tm = blockIdx.x % ga.tiles_m, tn = blockIdx.x / ga.tiles_m;
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- runs of equal adapters among the tile's rows ---------------------------------------------
    if (tid == 0) s_nruns = 0;
    if (tid < BM) {
        int slot = -1;
        if (has_pool && m0 + tid < T) slot = ga.row_slot[m0 + tid];
        s_slot[tid] = slot;
        s_valu_row[tid] = 0;
    }
    __syncthreads();
    if (tid < BM) {
        const bool is_start = tid == 0 || s_slot[tid] != s_slot[tid - 1];
        const unsigned long long mk = __ballot(is_start);
        if (lane == 0) s_mask[wave] = mk;
    }
    __syncthreads();
    if (tid < BM && s_slot[tid] >= 0 && (tid == 0 || s_slot[tid] != s_slot[tid - 1])) {
        int end = BM;
        for (int w = wave; w < BM / 64; ++w) {
            unsigned long long mk = s_mask[w];
            if (w == wave) mk &= (lane == 63) ? 0ull : (~0ull << (lane + 1));
            if (mk) {
                end = w * 64 + __builtin_ctzll(mk);
                break;
            }
        }
        const int k = atomicAdd(&s_nruns, 1);
        s_runs[k] = Run{tid, end, s_slot[tid], pool.meta[s_slot[tid]].rank};
    }
    __syncthreads();
    const int nruns = s_nruns;
    // which runs go through the K-extension (MFMA), which are added per row in the epilogue
    if (tid < nruns) {
        const Run r = s_runs[tid];
        const bool mfma = (r.end - r.start) >= kMinRunForMfma && (r.rank & 7) == 0;
        if (!mfma) {
            for (int q = r.start; q < r.end; ++q) s_valu_row[q] = 1;
            s_runs[tid].rank = 0;  // no K blocks for this run
        }
    }
    __syncthreads();

    // ---- main loop ---------------------------------------------------------------------------------
    const int wm = wave >> 2, wn = wave & 3;  // wave's 128 x 64 block inside the tile
    floatx16 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // staging: 256 rows x 8 pieces of 16 bytes for each operand, 4 + 4 pieces per thread
    u32x4 ra[4], rb[4];
    const int base_blocks = K / BK;

    // K blocks: [0, base_blocks) are the base product; then, per run, ceil(rank / BK) blocks of the expand
    auto load_block = [&](int blk) {
        if (blk < base_blocks) {
            const int k0 = blk * BK;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int p = tid + i * kGemmThreads, r = p >> 3, c = p & 7;
                ra[i] = (m0 + r < T) ? *reinterpret_cast<const u32x4 *>(ga.x + (size_t)(m0 + r) * K + k0 + c * 8) : u32x4{0, 0, 0, 0};
            }
            if (WFMT == ELORA_W_SAME) {
                const uint16_t *W = static_cast<const uint16_t *>(ga.W);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int p = tid + i * kGemmThreads, r = p >> 3, c = p & 7;
                    rb[i] = (n0 + r < N) ? *reinterpret_cast<const u32x4 *>(W + (size_t)(n0 + r) * K + k0 + c * 8) : u32x4{0, 0, 0, 0};
                }
            } else {
                // 4-bit groups of 32: 8 consecutive weights = 4 bytes; w = scale * (code - 8)
                const uint8_t *W = static_cast<const uint8_t *>(ga.W);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int p = tid + i * kGemmThreads, r = p >> 3, c = p & 7;
                    u32x4 out{0, 0, 0, 0};
                    if (n0 + r < N) {
                        const int k = k0 + c * 8;
                        const uint32_t packed = *reinterpret_cast<const uint32_t *>(W + (size_t)(n0 + r) * (K >> 1) + (k >> 1));
                        const float sc = fp16_to_f32(ga.w_scales[(size_t)(n0 + r) * (K >> 5) + (k >> 5)]);
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int lo = (packed >> (8 * q)) & 15, hi = (packed >> (8 * q + 4)) & 15;
                            // scale * (code - 8) is exact in fp32 (fp16 scale times a 4-bit integer) and is
                            // then rounded once to bf16
                            out[q] = (uint32_t)f32_to_bf16(sc * (float)(lo - 8)) | ((uint32_t)f32_to_bf16(sc * (float)(hi - 8)) << 16);
                        }
                    }
                    rb[i] = out;
                }
            }
            return;
        }
        // expand blocks: find the run and the rank offset this block belongs to
        int e = blk - base_blocks;
        int ri = 0, j0 = 0;
        for (; ri < nruns; ++ri) {
            const int nb = (s_runs[ri].rank + BK - 1) / BK;
            if (e < nb) {
                j0 = e * BK;
                break;
            }
            e -= nb;
        }
        const Run run = s_runs[ri];
        const uint16_t *Bm = reinterpret_cast<const uint16_t *>(slot_B(pool, run.slot));
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = tid + i * kGemmThreads, r = p >> 3, c = p & 7;
            const int j = j0 + c * 8;
            // rows of V outside the run belong to other adapters: they contribute nothing here.
            // V holds zeros beyond the row's rank up to Rpad.
            ra[i] = (r >= run.start && r < run.end && j < ga.Rpad)
                        ? *reinterpret_cast<const u32x4 *>(ga.V + (size_t)(m0 + r) * ga.Rpad + j)
                        : u32x4{0, 0, 0, 0};
            rb[i] = (n0 + r < N && j < run.rank) ? *reinterpret_cast<const u32x4 *>(Bm + (size_t)(n0 + r) * run.rank + j)
                                                  : u32x4{0, 0, 0, 0};
        }
    };
    auto store_block = [&](int buf) {
        uint16_t *sa = stage0 + buf * kStageElems;
        uint16_t *sb = sa + BM * kLdsRow;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = tid + i * kGemmThreads, r = p >> 3, c = p & 7;
            *reinterpret_cast<u32x4 *>(sa + r * kLdsRow + c * 8) = ra[i];
            *reinterpret_cast<u32x4 *>(sb + r * kLdsRow + c * 8) = rb[i];
        }
    };
    auto compute_block = [&](int buf) {
        const uint16_t *sa = stage0 + buf * kStageElems + (wm * 128 + (lane & 31)) * kLdsRow + (lane >> 5) * 8;
        const uint16_t *sb = stage0 + buf * kStageElems + BM * kLdsRow + (wn * 64 + (lane & 31)) * kLdsRow + (lane >> 5) * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[4], fb[2];
#pragma unroll
            for (int a = 0; a < 4; ++a) fa[a] = *reinterpret_cast<const bf16x8 *>(sa + a * 32 * kLdsRow + ks * 16);
#pragma unroll
            for (int b = 0; b < 2; ++b) fb[b] = *reinterpret_cast<const bf16x8 *>(sb + b * 32 * kLdsRow + ks * 16);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[a], fb[b], acc[a][b], 0, 0, 0);
        }
    };

    int total_blocks = base_blocks;
    for (int ri = 0; ri < nruns; ++ri) total_blocks += (s_runs[ri].rank + BK - 1) / BK;

    load_block(0);
    store_block(0);
    __syncthreads();
    for (int blk = 0; blk < total_blocks; ++blk) {
        const int buf = blk & 1;
        const bool more = (blk + 1) < total_blocks;
        if (more) load_block(blk + 1);
        compute_block(buf);
        if (more) store_block(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue -----------------------------------------------------------------------------------
    // C layout of the 32x32 MFMA: lane holds column (lane % 32); value i sits in row (i / 4) * 8 + (lane / 32) * 4 + i % 4
#pragma unroll
    for (int a = 0; a < 4; ++a) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int rl = wm * 128 + a * 32 + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);  // row inside the tile
            const int row = m0 + rl;
            if (row >= T) continue;
            float o[2] = {acc[a][0][i], acc[a][1][i]};
            if (s_valu_row[rl]) {
                const int slot = s_slot[rl];
                const int rank = pool.meta[slot].rank;
                const uint16_t *Bm = reinterpret_cast<const uint16_t *>(slot_B(pool, slot));
                const uint16_t *v = ga.V + (size_t)row * ga.Rpad;
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    const int col = n0 + wn * 64 + b * 32 + (lane & 31);
                    if (col < N) {
                        float d = 0.0f;
                        for (int j = 0; j < rank; ++j) d = fmaf(bf16_to_f32(v[j]), bf16_to_f32(Bm[(size_t)col * rank + j]), d);
                        o[b] += d;
                    }
                }
            }
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int col = n0 + wn * 64 + b * 32 + (lane & 31);
                if (col < N) ga.y[(size_t)row * N + col] = f32_to_bf16(o[b]);
            }
        }
    }
}

int round_up(int v, int m) { return (v + m - 1) / m * m; }

}  // namespace

bool elora::gemm_eligible(const elora_linear_desc_t &d, int max_rank)
{
    (void)max_rank;
    return d.dtype == ELORA_BF16 && d.n_tokens >= 1 && d.d_in % BK == 0 && d.d_out % 8 == 0;
}

void elora::gemm_plan(const elora_linear_desc_t &d, elora_plan_t *plan)
{
    plan->n_launches = d.pool ? 3 : 2;
    plan->tile_rows = BM;
    plan->tile_cols = BN;
    plan->grid = ((d.n_tokens + BM - 1) / BM) * ((d.d_out + BN - 1) / BN);
}

size_t elora::gemm_v_bytes(int n_tokens, int max_rank) { return (size_t)n_tokens * round_up(max_rank, BK) * sizeof(uint16_t); }

int elora::launch_gemm(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream)
{
    (void)plan;
    int32_t *row_slot = reinterpret_cast<int32_t *>(a.ws + a.wsl.row_slot);
    float *row_scale = reinterpret_cast<float *>(a.ws + a.wsl.row_scale);
    uint16_t *V = reinterpret_cast<uint16_t *>(a.ws + a.wsl.v);
    const int Rpad = round_up(a.pool.max_rank, BK);
    const int has_pool = a.has_pool ? 1 : 0;
    hipLaunchKernelGGL(gemm_route_kernel, dim3((a.T + 255) / 256), dim3(256), 0, stream, a.T, a.route, a.pool, has_pool,
                       row_slot, row_scale);
    ELORA_HIP_TRY(hipGetLastError());
    if (a.has_pool) {
        hipLaunchKernelGGL(sgmv_shrink_kernel, dim3((a.T + kShrinkRows - 1) / kShrinkRows), dim3(kShrinkThreads), 0, stream,
                           a.T, a.K, static_cast<const uint16_t *>(a.x), a.pool, row_slot, row_scale, V, Rpad);
        ELORA_HIP_TRY(hipGetLastError());
    }
    GemmArgs ga;
    ga.T = a.T;
    ga.K = a.K;
    ga.N = a.N;
    ga.x = static_cast<const uint16_t *>(a.x);
    ga.W = a.W;
    ga.w_scales = static_cast<const uint16_t *>(a.w_scales);
    ga.row_slot = row_slot;
    ga.V = V;
    ga.Rpad = Rpad;
    ga.y = static_cast<uint16_t *>(a.y);
    ga.tiles_m = (a.T + BM - 1) / BM;
    ga.tiles_n = (a.N + BN - 1) / BN;
    const size_t lds = (size_t)2 * kStageElems * sizeof(uint16_t);
    dim3 grid(ga.tiles_m * ga.tiles_n), block(kGemmThreads);
    profile_mark_begin(stream);
    if (a.wfmt == ELORA_W_SAME) {
        static bool attr_done = false;
        if (!attr_done) {
            ELORA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&lora_gemm_kernel<ELORA_W_SAME>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            attr_done = true;
        }
        hipLaunchKernelGGL((lora_gemm_kernel<ELORA_W_SAME>), grid, block, lds, stream, ga, a.pool, has_pool);
    } else {
        static bool attr_done = false;
        if (!attr_done) {
            ELORA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&lora_gemm_kernel<ELORA_W_INT4_G32>),
                                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            attr_done = true;
        }
        hipLaunchKernelGGL((lora_gemm_kernel<ELORA_W_INT4_G32>), grid, block, lds, stream, ga, a.pool, has_pool);
    }
    ELORA_HIP_TRY(hipGetLastError());
    profile_mark_end(stream);
    return ELORA_OK;
}
