// Prefill / mixed path (many rows, MFMA-bound): bf16 activations; bf16, 4-bit or 8-bit base weights.
//
// Three launches per call (a 4-bit W with 768 rows or more and an 8-bit W are converted to bf16 once per call, into
// the workspace, in the shrink's launch, and the bf16 kernel runs on the copy; below that the 4-bit W is converted
// tile by tile inside the gemm):
//   route   per row: validated pool slot and scale (Sec. 3.4: each request names its adapter)
//   shrink  V[t, :] = bf16(s_t * A_i x_t) for every row, with the rows grouped by adapter inside each
//           32-row tile ("u-batches", Sec. 3.4 / 4.3: rows that share an adapter are computed together):
//           one masked MFMA pass per run of equal adapters
//   gemm    Y = X W^T (Sec. 3.4: the base product, shared by the whole batch) on 256 x 256 tiles with
//           LDS-staged 64-wide K blocks and v_mfma_f32_32x32x16_bf16; the expand B_i v_t is appended to
//           the K loop as extra K blocks: a run of rows that share an adapter takes rank (rounded up to
//           8) of a block's 64 K columns, with the run's rows of V as A-operand (zero in all other rows)
//           and B_i as B-operand in the same columns, so one block serves several short runs at once
//           (runs of at most 32 rows, such as the decode rows of a mixed batch, are added after the K loop
//           instead).  While the next two blocks are base blocks the loop is straight-line code in which the
//           LDS reads and the direct loads are dealt out by hand over the matrix instructions' slots.  The
//           epilogue rounds once to bf16 and stores each row at its own position.
#include <type_traits>

#include "common.h"

using namespace elora;

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// two floats -> packed bf16 pair, round-to-nearest-even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    bf16x2_t v = __builtin_convertvector(float2_t{lo, hi}, bf16x2_t);
    return __builtin_bit_cast(uint32_t, v);
}

// Eight consecutive values of an adapter kept in 8-bit blocks (they lie in one block: ranks and d_in are multiples of
// 8 there) as matrix-core operands: scale * code, exact in fp32, rounded once to bf16.  (The decode and generic
// kernels multiply the exact products; here the adapter passes through the matrix cores like every other operand.)
__device__ __forceinline__ u32x4 q8_to_bf16x8(u32x2 codes, float sc)
{
    u32x4 o;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const uint32_t w = codes[b >> 1] >> (16 * (b & 1));
        o[b] = pack_bf16x2(sc * (float)(int8_t)(w & 0xffu), sc * (float)(int8_t)((w >> 8) & 0xffu));
    }
    return o;
}

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
// shrink.  Workgroups [0, n_tiles): one 32-row tile each, 4 waves split K, one masked MFMA pass per run
// of >= kShortRun equal adapters.  Workgroups [n_tiles, n_tiles + T): one row each; a row that sits in a
// shorter run (a decode row of a mixed batch, or the few rows a run leaves in a neighbouring tile) is
// computed there with plain FMAs, straight from its own adapter, and all other row workgroups exit at once.
// Either way V[t, :] = bf16(s_t * A_i x_t), with zeros beyond the rank up to Rpad and in rows without adapter.
// ------------------------------------------------------------------------------------------------
constexpr int kShrinkRows = 32;
constexpr int kShrinkThreads = 256;
constexpr int kShrinkColsPerPass = 64;  // rank columns per pass (4 MFMA column blocks of 16)
constexpr int kShortRun = 8;
constexpr int kShrinkUnroll = 4;        // K steps of 32 whose loads are issued together

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;

template <bool kQ8>
__device__ __forceinline__ void shrink_block_t(int block, int T, int K, int n_tiles, const uint16_t *__restrict__ x,
                                             const PoolView &pool, const int32_t *__restrict__ row_slot,
                                             const float *__restrict__ row_scale, uint16_t *__restrict__ V, int Rpad,
                                             int (&s_slot)[kShrinkRows], float (&s_red)[4][kShrinkRows][kShrinkColsPerPass + 1])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    if (block >= n_tiles) {
        // ---- one row of a short run ---------------------------------------------------------------
        // (most rows of a batch of prompts sit in long runs and their workgroups end here: one load of the tile's slots
        // and a vote, not a walk along the rows with a dependent load per step)
        const int t = block - n_tiles;
        const int r0 = t / kShrinkRows * kShrinkRows, r1 = min(r0 + kShrinkRows, T);
        static_assert(kShrinkRows == 32, "one lane of a half-wave per row of the tile");
        const int l = lane & 31;
        const int mine = r0 + l < r1 ? row_slot[r0 + l] : INT32_MIN;
        const int slot = __builtin_amdgcn_readlane(mine, t - r0);
        const uint32_t same = (uint32_t)__ballot(mine == slot);       // (both halves of the wave vote alike)
        const int p = t - r0;
        const uint32_t below = ~same & ((1u << p) - 1u), above = ~same & ~((2u << p) - 1u);  // (2u << 31 == 0: nothing above)
        const int lo = below ? 32 - __builtin_clz(below) : 0, hi = above ? __builtin_ctz(above) : 32;  // the run's piece inside this tile
        if (hi - lo >= kShortRun) return;
        float *vrow = &s_red[0][0][0];  // Rpad <= 256 floats
        int rank = 0;
        if (slot >= 0) {
            rank = pool.meta[slot].rank;
            const uint16_t *A = reinterpret_cast<const uint16_t *>(slot_A(pool, slot));
            for (int j0 = 2 * wave; j0 < rank; j0 += 2 * 4) {
                const bool two = (j0 + 1) < rank;
                const int j1 = two ? j0 + 1 : j0;
                float a0, a1;
                if constexpr (kQ8) {
                    const char *Ac = reinterpret_cast<const char *>(A);
                    const uint16_t *As = slot_A_scales(pool, slot);
                    shrink_pair_q8(Ac + (size_t)j0 * K, Ac + (size_t)j1 * K, As + (((size_t)j0 * K) >> 5), As + (((size_t)j1 * K) >> 5),
                                   x + (size_t)t * K, K, lane, a0, a1);
                } else
                shrink_pair(A + (size_t)j0 * K, A + (size_t)j1 * K, x + (size_t)t * K, K, lane, a0, a1);
                if (lane == 0) {
                    vrow[j0] = a0;
                    if (two) vrow[j0 + 1] = a1;
                }
            }
        }
        __syncthreads();
        const float sc = slot >= 0 ? row_scale[t] : 0.0f;
        for (int j = tid; j < Rpad; j += kShrinkThreads) V[(size_t)t * Rpad + j] = (j < rank) ? f32_to_bf16(sc * vrow[j]) : (uint16_t)0;
        return;
    }

    // ---- 32-row tile ------------------------------------------------------------------------------
    const int r0 = block * kShrinkRows;
    if (tid < kShrinkRows) s_slot[tid] = (r0 + tid < T) ? row_slot[r0 + tid] : -1;
    __syncthreads();
    // rows of long runs: zero now, the passes below fill in the rank columns (short-run rows belong to
    // their own workgroups)
    for (int r = 0; r < kShrinkRows && r0 + r < T;) {
        int e = r + 1;
        while (e < kShrinkRows && s_slot[e] == s_slot[r]) ++e;
        if (e - r >= kShortRun)
            for (int q = tid; q < (e - r) * Rpad; q += kShrinkThreads) {
                const int rr = r + q / Rpad;
                if (r0 + rr < T) V[(size_t)(r0 + rr) * Rpad + q % Rpad] = 0;
            }
        r = e;
    }
    __syncthreads();

    const int m = lane & 15, g = lane >> 4;
    const int kq = K / 4;  // K % 64 == 0: each wave's quarter of K is a multiple of 16
    const int kbeg = wave * kq, kend = kbeg + kq;

    int run_start = 0;
    while (run_start < kShrinkRows) {
        const int slot = s_slot[run_start];
        int run_end = run_start + 1;
        while (run_end < kShrinkRows && s_slot[run_end] == slot) ++run_end;
        if (slot >= 0 && run_end - run_start >= kShortRun) {
            const int rank = pool.meta[slot].rank;
            const uint16_t *A = reinterpret_cast<const uint16_t *>(slot_A(pool, slot));
            const char *Ac = reinterpret_cast<const char *>(A);       // (8-bit blocks: codes, and their scales)
            const uint16_t *As = kQ8 ? slot_A_scales(pool, slot) : nullptr;
            for (int j0 = 0; j0 < rank; j0 += kShrinkColsPerPass) {
                floatx4 acc[2][4];
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) acc[a][b] = floatx4{0.f, 0.f, 0.f, 0.f};
                const int ncb = min(4, (rank - j0 + 15) / 16);  // 16-column blocks in this pass
                for (int k = kbeg; k < kend; k += 32 * kShrinkUnroll) {
                    bf16x8 xa[kShrinkUnroll][2], ab[kShrinkUnroll][4];
#pragma unroll
                    for (int u = 0; u < kShrinkUnroll; ++u) {
                        const int kk = k + u * 32 + g * 8;
                        const bool kin = kk < kend;  // the tail of a quarter may be partly empty
#pragma unroll
                        for (int a = 0; a < 2; ++a) {
                            const int row = min(r0 + a * 16 + m, T - 1);
                            u32x4 v = *reinterpret_cast<const u32x4 *>(x + (size_t)row * K + (kin ? kk : kbeg));
                            if (!kin) v = u32x4{0, 0, 0, 0};
                            xa[u][a] = __builtin_bit_cast(bf16x8, v);
                        }
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const int j = j0 + b * 16 + m;
                            u32x4 v{0, 0, 0, 0};
                            if constexpr (kQ8) {
                                if (b < ncb) {
                                    const size_t e = (size_t)min(j, rank - 1) * K + (kin ? kk : kbeg);
                                    v = q8_to_bf16x8(*reinterpret_cast<const u32x2 *>(Ac + e), fp16_to_f32(As[e >> 5]));
                                }
                            } else {
                                if (b < ncb) v = *reinterpret_cast<const u32x4 *>(A + (size_t)min(j, rank - 1) * K + (kin ? kk : kbeg));
                            }
                            if (j >= rank) v = u32x4{0, 0, 0, 0};
                            ab[u][b] = __builtin_bit_cast(bf16x8, v);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kShrinkUnroll; ++u)
#pragma unroll
                        for (int a = 0; a < 2; ++a)
#pragma unroll
                            for (int b = 0; b < 4; ++b)
                                if (b < ncb) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab[u][b], xa[u][a], acc[a][b], 0, 0, 0);
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

// (the pool's storage format is a property of the launch: decided at run time inside the kernel, the bf16 shrink of two
// projections in one launch took 114 instead of 83 us)
template <bool kQ8>
__device__ __forceinline__ void shrink_block(int block, int T, int K, int n_tiles, const uint16_t *__restrict__ x,
                                             const PoolView &pool, const int32_t *__restrict__ row_slot,
                                             const float *__restrict__ row_scale, uint16_t *__restrict__ V, int Rpad)
{
    __shared__ int s_slot[kShrinkRows];
    __shared__ float s_red[4][kShrinkRows][kShrinkColsPerPass + 1];
    shrink_block_t<kQ8>(block, T, K, n_tiles, x, pool, row_slot, row_scale, V, Rpad, s_slot, s_red);
}

template <bool kQ8>
__global__ __launch_bounds__(kShrinkThreads) void sgmv_shrink_kernel(int T, int K, int n_tiles,
                                                                     const uint16_t *__restrict__ x, PoolView pool,
                                                                     const int32_t *__restrict__ row_slot,
                                                                     const float *__restrict__ row_scale,
                                                                     uint16_t *__restrict__ V, int Rpad)
{
    shrink_block<kQ8>((int)blockIdx.x, T, K, n_tiles, x, pool, row_slot, row_scale, V, Rpad);
}

// The shrink of several projections that read the same x (q / k / v, gate / up: Sec. 4.3 builds base model and adapters
// of a batch into one graph; Sec. 5.3: the adapters target Q, K, V, Up, Down) in one launch: block `blk` of projection p
// is workgroup ((blk / 8) * n + p) * 8 + blk % 8, so the workgroups that read the same rows of x run next to each other
// on one XCD (workgroup b runs on XCD b % 8) and all but the first find those rows in its L2.
constexpr int kShrinkMulti = 3;
struct ShrinkMulti {
    int n;
    PoolView pool[kShrinkMulti];
    int32_t *row_slot[kShrinkMulti];
    float *row_scale[kShrinkMulti];
    uint16_t *V[kShrinkMulti];
    int Rpad[kShrinkMulti];
};
// route of several projections with the same routing tables (each against its own pool) in one launch
__global__ void gemm_route_multi_kernel(int T, RouteView route, ShrinkMulti sm)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    for (int p = 0; p < sm.n; ++p) {
        const RowRoute r = resolve_row(t, route, sm.pool[p], true);
        sm.row_slot[p][t] = r.slot;
        sm.row_scale[p][t] = r.scale;
    }
}
template <bool kQ8>
__global__ __launch_bounds__(kShrinkThreads) void sgmv_shrink_multi_kernel(int T, int K, int n_tiles, const uint16_t *__restrict__ x,
                                                                           ShrinkMulti sm)
{
    const int xcd = blockIdx.x % 8, j = blockIdx.x / 8;
    const int p = j % sm.n, blk = (j / sm.n) * 8 + xcd;
    if (blk >= n_tiles + T) return;
    shrink_block<kQ8>(blk, T, K, n_tiles, x, sm.pool[p], sm.row_slot[p], sm.row_scale[p], sm.V[p], sm.Rpad[p]);
}

// ------------------------------------------------------------------------------------------------
// gemm
// ------------------------------------------------------------------------------------------------
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kGemmThreads = 256;        // 4 waves, one per SIMD: 2 along M x 2 along N, 128 x 128 outputs per wave
constexpr int kStageElems = (BM + BN) * BK;            // one LDS stage: 256 rows of X and 256 rows of W, 64 KiB
constexpr int kPieces = BM * (BK / 8) / kGemmThreads;  // 16-byte pieces per operand and thread (8)

// A staged row is 8 chunks of 16 bytes.  Chunk c of tile row r lives in slot c ^ ((r >> 1) & 7) of that row,
// which spreads the 16-byte fragment reads of 16 consecutive rows over all LDS banks without padding
// (the direct global->LDS loads can only fill LDS contiguously, 1 KiB per wave and instruction).
__device__ __forceinline__ int lds_pos(int r, int c) { return r * BK + ((c ^ ((r >> 1) & 7)) << 3); }
constexpr int kMaxRuns = BM;
constexpr int kXcds = 8, kSuperM = 4, kSuperN = 8;  // tile block per XCD (32 compute units each)

int gemm_grid(int tiles_m, int tiles_n) { return (tiles_m * tiles_n + kXcds - 1) / kXcds * kXcds; }

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

// A piece of the expand: rank entries [j0, j0 + width) of run `run`, placed at K columns [kcol, kcol + width)
// of an expand block (width and kcol are multiples of 8).
struct Item {
    uint16_t run, j0;
    uint8_t kcol, width;
    uint16_t pad;
};
constexpr int kMaxItems = kMaxRuns * (kMaxRank / BK);

template <int V> using ic = std::integral_constant<int, V>;

// Short runs (decode rows of a mixed batch, short prompts).  As columns of an expand block a run costs its rank's
// share of a whole 256 x 256 x 64 block whatever its length; a run of at most 32 rows is instead added after the K
// loop, to the one or two 32-row accumulator blocks it lies in: per block and 16 rank entries one fragment of V and
// four of B_i straight from memory and four matrix instructions in each of the two waves that own the rows.
constexpr int kEpiRows = 32;
__device__ __forceinline__ bool run_is_short(int start, int end, int rank, int N, int q8)
{
    // (a lane's offset into B_i fits 32 bits; adapters kept in 8-bit blocks always travel as expand blocks)
    return end - start <= kEpiRows && (rank & 7) == 0 && N < (1 << 22) && !q8;
}
constexpr int kEpiAhead = 8;  // (run, block, 16 rank entries) steps whose loads are in flight per wave
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(ic<I>{});
        static_for<I + 1, N>(f);
    }
}


template <int WFMT>
__global__ __launch_bounds__(kGemmThreads) void lora_gemm_kernel(GemmArgs ga, PoolView pool, int has_pool)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    uint16_t *stage0 = reinterpret_cast<uint16_t *>(smem_raw);
    __shared__ int s_slot[BM];
    __shared__ unsigned long long s_mask[BM / 64];
    __shared__ Run s_runs[kMaxRuns];
    __shared__ int s_nruns;
    __shared__ Item s_items[kMaxItems];
    __shared__ uint16_t s_blk_first[kMaxItems + 1];  // expand block b holds items [s_blk_first[b], s_blk_first[b + 1])
    __shared__ int s_nblk;
    __shared__ uint8_t s_pairs[BM / 32][32];  // short runs that have rows in 32-row block g of the tile
    __shared__ int s_npairs[BM / 32], s_nsteps[BM / 32];
    __shared__ int s_nlong, s_nshort, s_short_cols, s_use_ring;  // runs that go into expand blocks / that may be added afterwards

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = ga.T, K = ga.K, N = ga.N;
    // Workgroup b runs on XCD b % 8 (round-robin dispatch) and every XCD has its own L2.  The tiles are
    // listed block by block (blocks of 4 x 8 tiles; the blocks column by column through the grid, the tiles
    // column-major inside a block) and each XCD takes one contiguous eighth of that list.  So the 32
    // workgroups it runs side by side sit in one or two blocks, walk through K together and share the staged
    // slabs of X and W in its L2; every XCD gets the same number of tiles; and every XCD's share runs through
    // all rows of the batch, so that rows with many expand blocks (decode rows of a mixed batch) are spread
    // over all XCDs.
    const int n_valid = ga.tiles_m * ga.tiles_n, per_xcd = (n_valid + kXcds - 1) / kXcds;
    const int xcd = blockIdx.x % kXcds, seq = blockIdx.x / kXcds;
    int pos = xcd * per_xcd + seq;
    if (seq >= per_xcd || pos >= n_valid) return;
    const int sc = pos / (ga.tiles_m * kSuperN);            // only the last column of blocks can be narrower than 8
    const int sw = min(kSuperN, ga.tiles_n - sc * kSuperN);
    pos -= sc * ga.tiles_m * kSuperN;
    const int sr = pos / (kSuperM * sw);                    // only the last block of a column can be lower than 4
    const int sh = min(kSuperM, ga.tiles_m - sr * kSuperM);
    pos -= sr * kSuperM * sw;
    const int tm = sr * kSuperM + pos % sh, tn = sc * kSuperN + pos / sh;
    const int m0 = tm * BM, n0 = tn * BN;

    // ---- runs of equal adapters among the tile's rows (one thread per row) ------------------------
    static_assert(kGemmThreads == BM, "one thread per tile row");
    if (tid == 0) {
        s_nruns = 0;
        s_nblk = 0;
        s_nlong = 0;
        s_nshort = 0;
        s_short_cols = 0;
        s_use_ring = 0;
    }
    if (tid < BM / 32) {
        s_npairs[tid] = 0;
        s_nsteps[tid] = 0;
    }
    {
        int slot = -1;
        if (has_pool && m0 + tid < T) slot = ga.row_slot[m0 + tid];
        s_slot[tid] = slot;
    }
    __syncthreads();
    {
        const bool is_start = tid == 0 || s_slot[tid] != s_slot[tid - 1];
        const unsigned long long mk = __ballot(is_start);
        if (lane == 0) s_mask[wave] = mk;
    }
    __syncthreads();
    if (s_slot[tid] >= 0 && (tid == 0 || s_slot[tid] != s_slot[tid - 1])) {
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
        const int rank = pool.meta[s_slot[tid]].rank;
        s_runs[k] = Run{tid, end, s_slot[tid], rank};
        if (rank > 0 && run_is_short(tid, end, rank, N, pool.q8)) {
            atomicAdd(&s_nshort, 1);
            atomicAdd(&s_short_cols, (rank + 7) & ~7);
            for (int g = tid >> 5; g <= (end - 1) >> 5; ++g) {  // a 32-row block has rows of at most 32 runs
                s_pairs[g][atomicAdd(&s_npairs[g], 1)] = (uint8_t)k;
                atomicAdd(&s_nsteps[g], (rank + 15) >> 4);
            }
        } else if (rank > 0) {
            atomicAdd(&s_nlong, 1);
        }
    }
    __syncthreads();
    const int nruns = s_nruns;
    // Pack the rank columns of the long runs into expand blocks of 64 K columns.  Short runs whose columns all fit
    // into what the last of these blocks has left travel with them for nothing (the tail of a prompt next to the
    // head of the next one); otherwise they are added after the K loop.
    if (tid == 0 && nruns > 0) {
        int nitems = 0, nblk = 0, used = BK;
        auto pack = [&](int ri) {
            const int rank = s_runs[ri].rank;
            for (int j0 = 0; j0 < rank; j0 += BK) {
                const int w = (min(BK, rank - j0) + 7) & ~7;
                if (used + w > BK) {
                    s_blk_first[nblk++] = (uint16_t)nitems;
                    used = 0;
                }
                s_items[nitems++] = Item{(uint16_t)ri, (uint16_t)j0, (uint8_t)used, (uint8_t)w, 0};
                used += w;
            }
        };
        const int nshort = s_nshort;
        if (s_nlong > 0)
            for (int ri = 0; ri < nruns; ++ri)
                if (!run_is_short(s_runs[ri].start, s_runs[ri].end, s_runs[ri].rank, N, pool.q8)) pack(ri);
        if (nshort > 0 && nblk > 0 && s_short_cols <= BK - used) {
            for (int ri = 0; ri < nruns; ++ri)
                if (run_is_short(s_runs[ri].start, s_runs[ri].end, s_runs[ri].rank, N, pool.q8)) pack(ri);
        } else if (nshort > 0) {
            s_use_ring = 1;
        }
        s_blk_first[nblk] = (uint16_t)nitems;
        s_nblk = nblk;
    }
    __syncthreads();
    const int base_blocks = K / BK;
    const int total_blocks = base_blocks + s_nblk;

    // ---- main loop -----------------------------------------------------------------------------------
    const int wm = wave >> 1, wn = wave & 1;  // wave's 128 x 128 block inside the tile
    floatx16 acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.0f;

    // Staging of the next K block.  Base blocks: X rows (and bf16 W rows) travel global -> LDS directly
    // (global_load_lds_dwordx4: no registers, no LDS store instructions); 4-bit W rows are fetched as
    // codes + scale and converted when they are parked in LDS.  Expand blocks (few) go through registers
    // because rows outside the run have to be zeroed.  Rows past the end of X / W are clamped to the last
    // row: what they produce is never stored.
    u32x4 rr[kPieces];     // register staging (expand blocks)
    uint32_t rq[2][kPieces];  // 4-bit W: packed codes of 8 weights and their group scale; set 0 = the block that is
    float rs[2][kPieces];     // being parked in LDS during this iteration, set 1 = the block after it (in flight)
    const int prow = tid >> 3, pchunk = tid & 7;  // register path: piece i = row prow + 32 i, chunk pchunk
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;

    // issue the loads of K block `blk` into stage `buf`
    auto issue_block = [&](int blk, int buf) {
        uint16_t *sa = stage0 + buf * kStageElems;
        uint16_t *sb = sa + BM * BK;
        if (blk < base_blocks) {
            const int k0 = blk * BK;
            // instruction q of a wave fills rows 8q .. 8q+7 of the stage: lane -> (row 8q + lane / 8, slot lane % 8)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int q = wave * 8 + i, row = 8 * q + (lane >> 3);
                const int chunk = (lane & 7) ^ ((row >> 1) & 7);
                const int gr = min(m0 + row, T - 1);
                __builtin_amdgcn_global_load_lds((gptr_t)(ga.x + (size_t)gr * K + k0 + chunk * 8), (lptr_t)(sa + q * 512), 16, 0, 0);
            }
            if (WFMT == ELORA_W_SAME) {
                const uint16_t *W = static_cast<const uint16_t *>(ga.W);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int q = wave * 8 + i, row = 8 * q + (lane >> 3);
                    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
                    const int gr = min(n0 + row, N - 1);
                    __builtin_amdgcn_global_load_lds((gptr_t)(W + (size_t)gr * K + k0 + chunk * 8), (lptr_t)(sb + q * 512), 16, 0, 0);
                }
            }
        }
    };
    // 4-bit W: fetch codes and scales of K block `blk` (groups of 32 along K: 8 consecutive weights = 4 bytes,
    // one fp16 scale per group) into register set `set`
    auto fetch_codes = [&](int blk, int set) {
        if (WFMT == ELORA_W_SAME || blk >= base_blocks) return;
        const uint8_t *W = static_cast<const uint8_t *>(ga.W);
        const int k = blk * BK + pchunk * 8;
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int r = min(n0 + prow + 32 * i, N - 1);
            rq[set][i] = *reinterpret_cast<const uint32_t *>(W + (size_t)r * (K >> 1) + (k >> 1));
            rs[set][i] = fp16_to_f32(ga.w_scales[(size_t)r * (K >> 5) + (k >> 5)]);
        }
    };
    // 4-bit W: convert pieces [i0, i1) of register set `set` to bf16 and park them in stage `buf`.
    // w = scale * (code - 8) = fma(code, scale, -8 scale): exact in fp32 (fp16 scale times a small integer),
    // then rounded once to bf16.
    auto park_codes = [&](int blk, int buf, int set, int i0, int i1) {
        if (WFMT == ELORA_W_SAME || blk >= base_blocks) return;
        uint16_t *sb = stage0 + buf * kStageElems + BM * BK;
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            if (i < i0 || i >= i1) continue;
            const float sc = rs[set][i], c8 = -8.0f * sc;
            const uint32_t lo = rq[set][i] & 0x0f0f0f0fu, hi = (rq[set][i] >> 4) & 0x0f0f0f0fu;
            u32x4 out;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                out[q] = pack_bf16x2(fmaf((float)((lo >> (8 * q)) & 0xffu), sc, c8), fmaf((float)((hi >> (8 * q)) & 0xffu), sc, c8));
            *reinterpret_cast<u32x4 *>(sb + lds_pos(prow + 32 * i, pchunk)) = out;
        }
    };
    // make stage `buf` hold K block `blk` (everything that is not a direct load happens here)
    auto commit_block = [&](int blk, int buf) {
        uint16_t *sa = stage0 + buf * kStageElems;
        uint16_t *sb = sa + BM * BK;
        if (blk < base_blocks) return;
        // expand block: K columns 8 * pchunk .. + 7 of this thread's pieces belong to exactly one item (or none)
        const int e = blk - base_blocks;
        const int kc = pchunk * 8;
        int run_start = 0, run_end = 0, run_rank = 0, j = 0;
        const uint16_t *Bm = nullptr, *Bs = nullptr;  // (Bs: block scales of an adapter kept in 8-bit blocks)
        for (int it = s_blk_first[e]; it < s_blk_first[e + 1]; ++it) {
            const Item item = s_items[it];
            if (kc >= item.kcol && kc < item.kcol + item.width) {
                const Run run = s_runs[item.run];
                run_start = run.start;
                run_end = run.end;
                run_rank = run.rank;
                j = item.j0 + (kc - item.kcol);
                Bm = reinterpret_cast<const uint16_t *>(slot_B(pool, run.slot));
                if (pool.q8) Bs = slot_B_scales(pool, run.slot);
            }
        }
        // A-operand: the run's rows of V (zero beyond the rank up to Rpad); every other row contributes nothing
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int r = prow + 32 * i;
            rr[i] = (r >= run_start && r < run_end) ? *reinterpret_cast<const u32x4 *>(ga.V + (size_t)(m0 + r) * ga.Rpad + j)
                                                    : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int i = 0; i < kPieces; ++i) *reinterpret_cast<u32x4 *>(sa + lds_pos(prow + 32 * i, pchunk)) = rr[i];
        // B-operand: B_i[n, j .. j + 7] (row stride = rank; zero at and beyond the rank)
        const bool vec = Bm != nullptr && (run_rank & 7) == 0;
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            const int n = n0 + prow + 32 * i;
            u32x4 v{0, 0, 0, 0};
            if (Bs != nullptr && n < N) {
                // (8-bit blocks: ranks are multiples of 8, the eight values lie in one block)
                const size_t e = (size_t)n * run_rank + j;
                if (j < run_rank) v = q8_to_bf16x8(*reinterpret_cast<const u32x2 *>(reinterpret_cast<const char *>(Bm) + e), fp16_to_f32(Bs[e >> 5]));
            } else if (Bm != nullptr && n < N) {
                const uint16_t *src = Bm + (size_t)n * run_rank + j;
                if (vec) {
                    if (j < run_rank) v = *reinterpret_cast<const u32x4 *>(src);
                } else {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t lo = (j + 2 * q < run_rank) ? src[2 * q] : 0u;
                        const uint32_t hi = (j + 2 * q + 1 < run_rank) ? src[2 * q + 1] : 0u;
                        v[q] = lo | (hi << 16);
                    }
                }
            }
            rr[i] = v;
        }
#pragma unroll
        for (int i = 0; i < kPieces; ++i) *reinterpret_cast<u32x4 *>(sb + lds_pos(prow + 32 * i, pchunk)) = rr[i];
    };
    bf16x8 fr[2][8];  // fragments of one 16-wide K step: [0..3] rows of X, [4..7] rows of W; double-buffered
    // fragment row = block base (multiple of 32) + lane % 32, so the swizzle term only depends on the lane
    const int fsw = ((lane & 31) >> 1) & 7, fhalf = lane >> 5;
    auto read_frags = [&](bf16x8 *dst, int buf, int ks) {
        const int slot = ((ks * 2 + fhalf) ^ fsw) << 3;
        const uint16_t *sa = stage0 + buf * kStageElems + (wm * 128 + (lane & 31)) * BK + slot;
        const uint16_t *sb = stage0 + buf * kStageElems + BM * BK + (wn * 128 + (lane & 31)) * BK + slot;
#pragma unroll
        for (int a = 0; a < 4; ++a) dst[a] = *reinterpret_cast<const bf16x8 *>(sa + a * 32 * BK);
#pragma unroll
        for (int b = 0; b < 4; ++b) dst[4 + b] = *reinterpret_cast<const bf16x8 *>(sb + b * 32 * BK);
    };
    auto mfma_step = [&](const bf16x8 *f) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[a], f[4 + b], acc[a][b], 0, 0, 0);
    };

    issue_block(0, 0);
    fetch_codes(0, 0);
    park_codes(0, 0, 0, 0, kPieces);
    fetch_codes(1, 0);
    commit_block(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the direct loads have landed in LDS
    __syncthreads();
    read_frags(fr[0], 0, 0);
    // One K block per iteration, four K steps of 16.  While the matrix cores work on step s the LDS
    // reads of step s + 1 are already under way; the loads of the next block are issued at the top and
    // land in the other stage on their own (4-bit W: its codes were fetched one iteration earlier and are
    // converted and parked between the steps); the one barrier of the iteration sits before the last
    // step, so that the matrix cores drain step 2 while the waves meet.
    int blk0 = 0;
    if (WFMT == ELORA_W_SAME && base_blocks > 2) {
        // While the two blocks after this one are base blocks, nothing in an iteration is conditional: straight-line
        // code in which every matrix instruction has its slot, and what else the wave has to issue is dealt out over
        // the slots by hand (a matrix instruction keeps its pipe busy for 32 cycles, during which the wave can issue
        // a handful of other instructions: two or three per slot go unnoticed).
        //  - LDS reads: the eight fragments of the next K step, one behind each of the first eight matrix
        //    instructions of this one.  (Left alone, the compiler moves them to the end of the step, to save
        //    registers, and the wave then waits for them.)
        //  - Direct loads: the sixteen of a block in two halves of eight, one load per slot: the first half behind the
        //    last K step of iteration b (block b + 2; the barrier just before has shown that everybody is done reading
        //    the stage it fills, the one block b sat in), the second half behind the first K step of iteration b + 1;
        //    they are waited for at that iteration's barrier.  Sixteen loads in eight consecutive slots were 5 % slower
        //    (4 waves x 16 KiB at once are more than the CU's path to the L2 takes in that time, and a load that is
        //    not accepted holds up the matrix instruction behind it); thinner spreads, over three or four K steps,
        //    were slower as well: their last loads have too little time to land.
        // Addresses: one base per matrix that is the same for the whole wave (the tile's first row at the block's first
        // column; it lives in scalar registers) plus a 32-bit byte offset per lane and load that never changes (row
        // inside the tile, clamped to the matrix, and 16-byte chunk), and wave-uniform LDS destinations: a load costs
        // two scalar instructions besides itself.  (Written as instructions: the compiler's own form of the load takes
        // a 64-bit address per lane, i.e. a 64-bit vector addition per load, and reads the LDS address out of a vector
        // register; M0 holds the LDS address of the wave's 1 KiB and needs a cycle to settle.  No other code of this
        // kernel keeps a value in M0 across statements.)
        const int swave = __builtin_amdgcn_readfirstlane(wave);
        uint32_t xoff[8], woff[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = 8 * (swave * 8 + i) + (lane >> 3);
            const int chunk = (lane & 7) ^ ((row >> 1) & 7);
            xoff[i] = (uint32_t)(((size_t)(min(m0 + row, T - 1) - m0) * K + chunk * 8) * 2);
            woff[i] = (uint32_t)(((size_t)(min(n0 + row, N - 1) - n0) * K + chunk * 8) * 2);
        }
        const char *const xbase = reinterpret_cast<const char *>(ga.x + (size_t)m0 * K);
        const char *const wbase = reinterpret_cast<const char *>(static_cast<const uint16_t *>(ga.W) + (size_t)n0 * K);
        const uint32_t lds0 = (uint32_t)(uintptr_t)(lptr_t)(stage0 + swave * 8 * 512);
        // load k of a block's sixteen: rows 8 (k / 2) .. + 7 of the wave's 64, of X (k even) or of W (k odd)
        auto issue_one = [&](int blk, int buf, int k) __attribute__((always_inline)) {
            const int i = k >> 1;
            const uint32_t off = (k & 1) ? woff[i] : xoff[i];
            const char *base = ((k & 1) ? wbase : xbase) + (size_t)blk * BK * 2;
            const uint32_t lds = lds0 + (uint32_t)(buf * kStageElems + ((k & 1) ? BM * BK : 0) + i * 512) * 2;
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds) : "memory");
        };
        auto read_frag = [&](bf16x8 *dst, int buf, int ks, int f) __attribute__((always_inline)) {
            const int slot = ((ks * 2 + fhalf) ^ fsw) << 3;
            const uint16_t *src = stage0 + buf * kStageElems + (f < 4 ? 0 : BM * BK) + ((f < 4 ? wm : wn) * 128 + (lane & 31) + (f & 3) * 32) * BK + slot;
            dst[f] = *reinterpret_cast<const bf16x8 *>(src);
        };
        // One K step: sixteen matrix instructions on the fragments `cur`; behind each of the first eight a fragment
        // of the step after it is read into `nxt`, behind each of the last eight (kLoads) load kFirst + 0 .. 7 of block
        // lblk.  Nothing may move across the slots: the order below is the order of the instructions.
        auto k_step = [&](auto first_c, auto loads_c, const bf16x8 *cur, bf16x8 *nxt, int rbuf, int rks, int lblk, int lbuf) __attribute__((always_inline)) {
            constexpr int kFirst = decltype(first_c)::value;
            constexpr bool kLoads = decltype(loads_c)::value;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                acc[e >> 2][e & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur[e >> 2], cur[4 + (e & 3)], acc[e >> 2][e & 3], 0, 0, 0);
                if (e < 8) read_frag(nxt, rbuf, rks, e);
                else if (kLoads) issue_one(lblk, lbuf, kFirst + e - 8);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        using std::integral_constant;
        const integral_constant<bool, true> with_loads;
        const integral_constant<bool, false> no_loads;
#pragma unroll
        for (int k = 0; k < 8; ++k) issue_one(1, 1, k);  // (the loop's first turn asks for the second half of block 1)
        for (; blk0 + 2 < base_blocks; ++blk0) {
            const int buf = blk0 & 1;
            k_step(integral_constant<int, 8>{}, with_loads, fr[0], fr[1], buf, 1, blk0 + 1, buf ^ 1);
            k_step(integral_constant<int, 0>{}, no_loads, fr[1], fr[0], buf, 2, 0, 0);
            k_step(integral_constant<int, 0>{}, no_loads, fr[0], fr[1], buf, 3, 0, 0);
            __builtin_amdgcn_s_waitcnt(0x0F70);  // block blk0 + 1 has landed
            __syncthreads();
            k_step(integral_constant<int, 0>{}, with_loads, fr[1], fr[0], buf ^ 1, 0, blk0 + 2, buf);
        }
        // (the first half of block blk0 + 1 is on its way; the loop below asks for the whole block, which is harmless:
        // same bytes, same place)
    }
    for (int blk = blk0; blk < total_blocks; ++blk) {
        const int buf = blk & 1;
        const bool more = (blk + 1) < total_blocks;
        if (more) {
            issue_block(blk + 1, buf ^ 1);
            fetch_codes(blk + 2, 1);
        }
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fr[1], buf, 1);
        mfma_step(fr[0]);
        if (more) park_codes(blk + 1, buf ^ 1, 0, 0, 3);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fr[0], buf, 2);
        mfma_step(fr[1]);
        if (more) park_codes(blk + 1, buf ^ 1, 0, 3, 6);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(fr[1], buf, 3);
        mfma_step(fr[0]);
        if (more) park_codes(blk + 1, buf ^ 1, 0, 6, kPieces);
        __builtin_amdgcn_sched_barrier(0);
        if (more) {
            commit_block(blk + 1, buf ^ 1);
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
            read_frags(fr[0], buf ^ 1, 0);
            if (WFMT != ELORA_W_SAME) {
#pragma unroll
                for (int i = 0; i < kPieces; ++i) {
                    rq[0][i] = rq[1][i];
                    rs[0][i] = rs[1][i];
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(fr[1]);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- short runs: v B_i^T added block by block ----------------------------------------------------------
    // A step is (32-row block, run, 16 rank entries): the A-operand is the block's rows of V with every row outside
    // the run zero (lane -> row lane % 32, entries 8 (lane / 32) .. + 7 of the 16), the B-operands are the same
    // entries of B_i for the wave's 4 x 32 columns.  The steps of a (block, run) pair follow each other in rank
    // order and no two pairs of a block share a row, so the sums do not depend on the order the pairs were listed in.
    // The steps of the upper and of the lower four blocks are first written out as a table each (one thread per
    // block, into the stages, which are free now), every block filled up to a multiple of the ring's length with
    // empty steps, so that ring slot and accumulator block of every multiplication are compile-time constants and
    // the loop that walks the table has no branch in it: with one wave per SIMD, what bounds this part is the
    // number of instructions per step (a cursor kept in scalar registers took 2.5 times as long as the table).
    // The loads of kEpiAhead steps are in flight while one is multiplied; a step issues its five loads whatever
    // the lane's row and whether it is empty (addresses inside some run's own data, the fragment of V masked when it
    // is used), and every multiplication waits for exactly the loads issued after its own (the loads are written as
    // instructions and counted by hand: left to the compiler, the loop waits for all loads once per turn).
    // Entries at and beyond the rank are zero in V, so B_i's fragment there only has to be finite: it re-reads
    // entry 0; an empty step re-reads the step before it.
    {
        constexpr int kTabBlock = kEpiRows * (kMaxRank / 16);             // steps of a block: 32 runs of 16 steps
        constexpr int kTabHalf = 4 * kTabBlock + kEpiAhead + 1;           // + the steps issued past the end
        static_assert(2 * kTabHalf * 16 <= 2 * kStageElems * 2, "the tables fit into the stages");
        static_assert(kTabBlock % kEpiAhead == 0 && (kEpiAhead & (kEpiAhead - 1)) == 0 && 5 * (kEpiAhead - 1) < 64, "a power of two; the load counter has six bits");
        auto up = [](int n) { return (n + kEpiAhead - 1) & ~(kEpiAhead - 1); };
        int nst[BM / 32];
        int any = 0;
#pragma unroll
        for (int g = 0; g < BM / 32; ++g) {
            nst[g] = __builtin_amdgcn_readfirstlane(s_nsteps[g]);
            any += nst[g];
        }
        if (!s_use_ring) any = 0;
        if (any > 0) {
            u32x4 *tab = reinterpret_cast<u32x4 *>(smem_raw);
            // step record: x = first row | (end row << 9) | (block << 18) (rows counted in the tile), y = first entry |
            // (rank << 16), z / w = byte offset of B_i from the pool's first slot
            auto record = [&](const Run &run, int g, int j0) {
                const unsigned long long off = (unsigned long long)run.slot * pool.slot_bytes + pool.b_offset;
                return u32x4{(uint32_t)(run.start | (run.end << 9) | (g << 18)), (uint32_t)(j0 | (run.rank << 16)), (uint32_t)off, (uint32_t)(off >> 32)};
            };
            __syncthreads();  // every wave is done with the stages
            if (tid < BM / 32) {
                const int g = tid;
                int off = 0;
                for (int h = g & ~3; h < g; ++h) off += up(s_nsteps[h]);
                u32x4 *out = tab + (g >> 2) * kTabHalf + off;
                int n = 0;
                for (int i = 0; i < s_npairs[g]; ++i) {
                    const Run run = s_runs[s_pairs[g][i]];
                    for (int j0 = 0; j0 < run.rank; j0 += 16) out[n++] = record(run, g, j0);
                }
                for (; (n & (kEpiAhead - 1)) != 0; ++n) out[n] = u32x4{0, out[n - 1][1], out[n - 1][2], out[n - 1][3]};
            } else if (tid < BM / 32 + 2) {
                // past the end of a half's table: empty steps that re-read the half's first run
                const int half = tid - BM / 32;
                int total = 0, first = -1;
                for (int h = 4 * half; h < 4 * half + 4; ++h) {
                    if (first < 0 && s_npairs[h] > 0) first = h;
                    total += up(s_nsteps[h]);
                }
                if (first >= 0) {
                    u32x4 r = record(s_runs[s_pairs[first][0]], first, 0);
                    r[0] = 0;
                    for (int i = 0; i <= kEpiAhead; ++i) tab[half * kTabHalf + total + i] = r;
                }
            }
            __syncthreads();
            const int g0 = wm * 4;
            if (nst[g0] + nst[g0 + 1] + nst[g0 + 2] + nst[g0 + 3] > 0) {
                u32x4 va[kEpiAhead], vb[kEpiAhead][4];
                bool in_run[kEpiAhead];
                const u32x4 *next = tab + wm * kTabHalf;
                u32x4 rec = *next;
                auto load16 = [](const void *p) {
                    u32x4 v;
                    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(p) : "memory");
                    return v;
                };
                uint32_t ncol[4];
#pragma unroll
                for (int b = 0; b < 4; ++b) ncol[b] = (uint32_t)min(n0 + wn * 128 + b * 32 + (lane & 31), N - 1);
                auto issue = [&](auto dc) {
                    constexpr int d = decltype(dc)::value;
                    const u32x4 r = rec;
                    rec = *++next;  // (read now, used by the next step)
                    const int row = (int)(r[0] >> 18) * 32 + (lane & 31);
                    in_run[d] = row >= (int)(r[0] & 511u) && row < (int)((r[0] >> 9) & 511u);
                    const uint32_t rank = r[1] >> 16, j = (r[1] & 0xffffu) + (lane >> 5) * 8;
                    va[d] = load16(ga.V + (size_t)min(m0 + row, T - 1) * ga.Rpad + j);
                    const uint32_t jb = j < rank ? j : 0;
                    const char *Bb = pool.slots + (((unsigned long long)r[3] << 32) | r[2]);
#pragma unroll
                    for (int b = 0; b < 4; ++b) vb[d][b] = load16(Bb + (size_t)((ncol[b] * rank + jb) * 2u));
                };
                static_for<0, kEpiAhead>(issue);
                auto block_steps = [&](auto ac) {
                    constexpr int a = decltype(ac)::value;
                    const int n_up = up(nst[g0 + a]);
                    auto consume = [&](auto dc) {
                        constexpr int d = decltype(dc)::value;
                        // five loads per step, kEpiAhead - 1 younger steps in flight; the operands tie what follows to the wait
                        asm volatile("s_waitcnt vmcnt(%5)" : "+v"(va[d]), "+v"(vb[d][0]), "+v"(vb[d][1]), "+v"(vb[d][2]), "+v"(vb[d][3]) : "n"(5 * (kEpiAhead - 1)) : "memory");
                        const bf16x8 fa = __builtin_bit_cast(bf16x8, in_run[d] ? va[d] : u32x4{0, 0, 0, 0});
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, __builtin_bit_cast(bf16x8, vb[d][b]), acc[a][b], 0, 0, 0);
                    };
                    for (int i = 0; i < n_up; i += kEpiAhead)
                        static_for<0, kEpiAhead>([&](auto dc) {
                            consume(dc);
                            issue(dc);
                        });
                };
                block_steps(ic<0>{});
                block_steps(ic<1>{});
                block_steps(ic<2>{});
                block_steps(ic<3>{});
                // the empty steps issued last are still on their way into registers the compiler takes to be free
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        }
    }

    // ---- epilogue -------------------------------------------------------------------------------------
    // C layout of the 32x32 MFMA: lane holds column (lane % 32); value i sits in row (i / 4) * 8 + (lane / 32) * 4 + i % 4.
    // A lane rounds its two values of a row pair into one register (low half: row i0, high half: row i1), neighbouring
    // lanes exchange that register (one cross-lane move inside the quad, no LDS), and a byte permute picks the two
    // halves that belong to the lane's row: the even lane stores row i0, the odd lane row i1, two adjacent columns
    // (4 bytes) each.  A tile that lies wholly inside y, the usual case, stores without any test: 128 stores per lane,
    // each of which would otherwise sit in a branch of its own.  The stores are marked as streaming: y is tens to
    // hundreds of MB that nobody reads again before the kernel ends, and kept in the caches it pushes out slabs of X and
    // W that the next tiles, and the launches that follow, would find there (config 5: 0.307 -> 0.300 ms per step).
    const bool odd = lane & 1;
    const uint32_t pick = odd ? 0x03020706u : 0x05040100u;  // bytes of {neighbour's register : own register}
    char *const ycorner = reinterpret_cast<char *>(ga.y + (size_t)m0 * N + n0 + wn * 128);
    auto store_tile = [&](auto checked) {
#pragma unroll
        for (int a = 0; a < 4; ++a) {
#pragma unroll
            for (int ip = 0; ip < 8; ++ip) {
                const int i_mine = 2 * ip + (odd ? 1 : 0);
                const int rl = wm * 128 + a * 32 + (i_mine >> 2) * 8 + (lane >> 5) * 4 + (i_mine & 3);
                const int row = m0 + rl;
                // (the wave's corner of y is the same for all lanes; a lane's place relative to it fits 32 bits)
                char *yrow = ycorner + (uint32_t)(((uint32_t)rl * (uint32_t)N + (uint32_t)(lane & 30)) * 2u);  // even column of the pair
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const uint32_t own = pack_bf16x2(acc[a][b][2 * ip], acc[a][b][2 * ip + 1]);
                    const uint32_t other = (uint32_t)__builtin_amdgcn_mov_dpp((int)own, 0xB1, 0xF, 0xF, true);  // quad_perm [1, 0, 3, 2]
                    const uint32_t packed = __builtin_amdgcn_perm(other, own, pick);
                    if (!decltype(checked)::value || (row < T && n0 + wn * 128 + b * 32 + (lane & 30) < N))
                        __builtin_nontemporal_store(packed, reinterpret_cast<uint32_t *>(yrow + b * 64));
                }
            }
        }
    };
    if (m0 + BM <= T && n0 + BN <= N) store_tile(std::false_type{});
    else store_tile(std::true_type{});
}

int round_up(int v, int m) { return (v + m - 1) / m * m; }

// ------------------------------------------------------------------------------------------------
// 4-bit W, many rows: W is converted to bf16 once per call, into the workspace, and the bf16 kernel runs on the copy.
// Converted tile by tile inside the GEMM (WFMT = ELORA_W_INT4_G32 above) every row tile of the batch repeats the
// conversion of the W tiles it meets, on the same vector units that feed the matrix cores, and the kernel runs at half
// the bf16 rate; the copy costs one pass over W at memory speed (d_out x d_in x 2.6 bytes), which that saving repays
// from a few hundred rows on.  Same arithmetic as park_codes: w = fma(code, scale, -8 scale) in fp32, rounded once.
// One thread per 8 weights (4 bytes of codes in, 16 bytes out; four threads share a group's fp16 scale): a wave
// reads 256 and writes 1024 consecutive bytes.
// ------------------------------------------------------------------------------------------------
int g_dequant_first_rows = 768;  // (elora_debug_w4_copy_rows)

// 8-bit W (groups of 32 along d_in, w = scale * code: exact in fp32, rounded once to bf16): the same copy, one thread
// per 8 weights (8 bytes of codes in, 16 bytes out).
__device__ __forceinline__ void w8_dequant_piece(size_t i, size_t n_pieces, const uint32_t *__restrict__ codes,
                                                 const uint16_t *__restrict__ scales, u32x4 *__restrict__ out)
{
    if (i >= n_pieces) return;
    const u32x2 q = reinterpret_cast<const u32x2 *>(codes)[i];
    const float sc = fp16_to_f32(scales[i >> 2]);
    u32x4 o;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const uint32_t w = q[b >> 1] >> (16 * (b & 1));
        o[b] = pack_bf16x2(sc * (float)(int8_t)(w & 0xffu), sc * (float)(int8_t)((w >> 8) & 0xffu));
    }
    out[i] = o;
}

__device__ __forceinline__ void w4_dequant_piece(size_t i, size_t n_pieces, const uint32_t *__restrict__ codes,
                                                 const uint16_t *__restrict__ scales, u32x4 *__restrict__ out)
{
    if (i >= n_pieces) return;
    const uint32_t q = codes[i];
    const float sc = fp16_to_f32(scales[i >> 2]), c8 = -8.0f * sc;
    const uint32_t lo = q & 0x0f0f0f0fu, hi = (q >> 4) & 0x0f0f0f0fu;
    u32x4 o;
#pragma unroll
    for (int b = 0; b < 4; ++b)
        o[b] = pack_bf16x2(fmaf((float)((lo >> (8 * b)) & 0xffu), sc, c8), fmaf((float)((hi >> (8 * b)) & 0xffu), sc, c8));
    out[i] = o;
}

template <int WFMT>
__device__ __forceinline__ void w_dequant_piece(size_t i, size_t n_pieces, const uint32_t *__restrict__ codes,
                                                const uint16_t *__restrict__ scales, u32x4 *__restrict__ out)
{
    if (WFMT == ELORA_W_INT8_G32) w8_dequant_piece(i, n_pieces, codes, scales, out);
    else w4_dequant_piece(i, n_pieces, codes, scales, out);
}

template <int WFMT>
__global__ __launch_bounds__(256) void w_dequant_kernel(size_t n_pieces, const uint32_t *__restrict__ codes,
                                                        const uint16_t *__restrict__ scales, u32x4 *__restrict__ out)
{
    w_dequant_piece<WFMT>((size_t)blockIdx.x * 256 + threadIdx.x, n_pieces, codes, scales, out);
}

// The shrink and the copy of W do not depend on each other, and the shrink of a few hundred rows is a few dozen
// workgroups that wait for memory most of the time: in one launch (the shrink's workgroups first, so that they start
// at once) the copy fills the rest of the device meanwhile and the call is one launch and one kernel's time shorter.
static_assert(kShrinkThreads == 256, "one block shape for both halves");
constexpr int kCopyPerThread = 8;
template <int WFMT, bool kQ8>
__global__ __launch_bounds__(kShrinkThreads) void sgmv_shrink_w_dequant_kernel(int n_shrink, int T, int K, int n_tiles,
                                                                                const uint16_t *__restrict__ x, PoolView pool,
                                                                                const int32_t *__restrict__ row_slot,
                                                                                const float *__restrict__ row_scale,
                                                                                uint16_t *__restrict__ V, int Rpad, size_t n_pieces,
                                                                                const uint32_t *__restrict__ codes,
                                                                                const uint16_t *__restrict__ scales,
                                                                                u32x4 *__restrict__ out)
{
    if ((int)blockIdx.x < n_shrink) {
        shrink_block<kQ8>((int)blockIdx.x, T, K, n_tiles, x, pool, row_slot, row_scale, V, Rpad);
        return;
    }
    // (the shrink's LDS counts for these workgroups too and halves how many of them a compute unit holds: each takes
    // kCopyPerThread pieces per thread, their loads under way together)
    const size_t base = (size_t)(blockIdx.x - n_shrink) * (256 * kCopyPerThread) + threadIdx.x;
#pragma unroll
    for (int u = 0; u < kCopyPerThread; ++u) w_dequant_piece<WFMT>(base + (size_t)u * 256, n_pieces, codes, scales, out);
}

}  // namespace

bool elora::gemm_eligible(const elora_linear_desc_t &d, int max_rank)
{
    (void)max_rank;
    if (!(d.dtype == ELORA_BF16 && d.n_tokens >= 1 && d.d_in % BK == 0 && d.d_out % 8 == 0)) return false;
    // a lane's byte offset inside a tile (up to 255 rows of d_in or d_out bf16) is kept in 32 bits
    if (d.d_in > (1 << 22) || d.d_out > (1 << 22)) return false;
    // an 8-bit W is always multiplied from its bf16 copy here (batches too small for one belong to the decode kernel)
    return d.wfmt != ELORA_W_INT8_G32 || gemm_wcopy_bytes(d.wfmt, d.n_tokens, d.d_in, d.d_out) != 0;
}

void elora::gemm_plan(const elora_linear_desc_t &d, elora_plan_t *plan)
{
    const bool copy_first = gemm_wcopy_bytes(d.wfmt, d.n_tokens, d.d_in, d.d_out) != 0;
    plan->n_launches = (d.pool ? 3 : 2) + (copy_first && !d.pool ? 1 : 0);  // (with a pool the copy shares the shrink's launch)
    plan->tile_rows = BM;
    plan->tile_cols = BN;
    plan->grid = gemm_grid((d.n_tokens + BM - 1) / BM, (d.d_out + BN - 1) / BN);
}

void elora::gemm_set_w4_copy_rows(int rows) { g_dequant_first_rows = rows; }

size_t elora::gemm_w4_bytes(int n_tokens, int d_in, int d_out)
{
    return n_tokens >= g_dequant_first_rows ? (size_t)d_in * (size_t)d_out * sizeof(uint16_t) : 0;
}

// room for the call's bf16 copy of a group-wise W: 4-bit from 768 rows on (below that it is converted tile by tile),
// 8-bit for every batch that has more rows than the decode kernel takes
size_t elora::gemm_wcopy_bytes(int wfmt, int n_tokens, int d_in, int d_out)
{
    if (wfmt == ELORA_W_INT4_G32) return gemm_w4_bytes(n_tokens, d_in, d_out);
    if (wfmt == ELORA_W_INT8_G32) return n_tokens > kDecodeMaxTokens * kDecodeMaxPasses ? (size_t)d_in * (size_t)d_out * sizeof(uint16_t) : 0;
    return 0;
}

size_t elora::gemm_v_bytes(int n_tokens, int max_rank) { return (size_t)n_tokens * round_up(max_rank, BK) * sizeof(uint16_t); }

namespace {
// what follows route and shrink: (the copy of a 4-bit W and) the GEMM with the expand in its K loop
int launch_gemm_back(const LinearArgs &a, hipStream_t stream, bool copy_done = false)
{
    int32_t *row_slot = reinterpret_cast<int32_t *>(a.ws + a.wsl.row_slot);
    uint16_t *V = reinterpret_cast<uint16_t *>(a.ws + a.wsl.v);
    const int Rpad = round_up(a.pool.max_rank, BK);
    const int has_pool = a.has_pool ? 1 : 0;
    // 4-bit W and enough rows: the bf16 kernel on a copy made now
    const bool copy_first = a.wfmt != ELORA_W_SAME && a.wsl.wdeq_bytes != 0;
    if (copy_first && !copy_done) {
        const size_t n_pieces = (size_t)a.N * (size_t)(a.K / 8);
        const dim3 cgrid((unsigned)((n_pieces + 255) / 256));
        if (a.wfmt == ELORA_W_INT8_G32)
            hipLaunchKernelGGL(w_dequant_kernel<ELORA_W_INT8_G32>, cgrid, dim3(256), 0, stream, n_pieces, static_cast<const uint32_t *>(a.W),
                               static_cast<const uint16_t *>(a.w_scales), reinterpret_cast<u32x4 *>(a.ws + a.wsl.wdeq));
        else
            hipLaunchKernelGGL(w_dequant_kernel<ELORA_W_INT4_G32>, cgrid, dim3(256), 0, stream, n_pieces, static_cast<const uint32_t *>(a.W),
                               static_cast<const uint16_t *>(a.w_scales), reinterpret_cast<u32x4 *>(a.ws + a.wsl.wdeq));
        ELORA_HIP_TRY(hipGetLastError());
    }
    if (a.wfmt == ELORA_W_INT8_G32 && !copy_first) return ELORA_E_DTYPE;  // (no tile-by-tile conversion for 8-bit W)
    GemmArgs ga;
    ga.T = a.T;
    ga.K = a.K;
    ga.N = a.N;
    ga.x = static_cast<const uint16_t *>(a.x);
    ga.W = copy_first ? static_cast<const void *>(a.ws + a.wsl.wdeq) : a.W;
    ga.w_scales = static_cast<const uint16_t *>(a.w_scales);
    ga.row_slot = row_slot;
    ga.V = V;
    ga.Rpad = Rpad;
    ga.y = static_cast<uint16_t *>(a.y);
    ga.tiles_m = (a.T + BM - 1) / BM;
    ga.tiles_n = (a.N + BN - 1) / BN;
    const size_t lds = (size_t)2 * kStageElems * sizeof(uint16_t);
    dim3 grid(gemm_grid(ga.tiles_m, ga.tiles_n)), block(kGemmThreads);
    profile_mark_begin(stream);
    if (a.wfmt == ELORA_W_SAME || copy_first) {
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
}  // namespace

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
    bool copy_done = false;
    if (a.has_pool) {
        const int n_tiles = (a.T + kShrinkRows - 1) / kShrinkRows;
        const size_t n_pieces = (size_t)a.N * (size_t)(a.K / 8), n_copy = (n_pieces + 256 * kCopyPerThread - 1) / (256 * kCopyPerThread);
        if (a.wfmt != ELORA_W_SAME && a.wsl.wdeq_bytes != 0 && n_copy + (size_t)(n_tiles + a.T) < (size_t)1 << 31) {
            const dim3 mgrid((unsigned)(n_tiles + a.T + n_copy));
            auto go = [&](auto kern) {
                hipLaunchKernelGGL(kern, mgrid, dim3(kShrinkThreads), 0, stream, n_tiles + a.T, a.T, a.K, n_tiles,
                                   static_cast<const uint16_t *>(a.x), a.pool, row_slot, row_scale, V, Rpad, n_pieces,
                                   static_cast<const uint32_t *>(a.W), static_cast<const uint16_t *>(a.w_scales),
                                   reinterpret_cast<u32x4 *>(a.ws + a.wsl.wdeq));
            };
            if (a.wfmt == ELORA_W_INT8_G32) {
                if (a.pool.q8) go(sgmv_shrink_w_dequant_kernel<ELORA_W_INT8_G32, true>);
                else go(sgmv_shrink_w_dequant_kernel<ELORA_W_INT8_G32, false>);
            } else {
                if (a.pool.q8) go(sgmv_shrink_w_dequant_kernel<ELORA_W_INT4_G32, true>);
                else go(sgmv_shrink_w_dequant_kernel<ELORA_W_INT4_G32, false>);
            }
            copy_done = true;
        } else if (a.pool.q8) {
            hipLaunchKernelGGL(sgmv_shrink_kernel<true>, dim3(n_tiles + a.T), dim3(kShrinkThreads), 0, stream, a.T, a.K, n_tiles,
                               static_cast<const uint16_t *>(a.x), a.pool, row_slot, row_scale, V, Rpad);
        } else {
            hipLaunchKernelGGL(sgmv_shrink_kernel<false>, dim3(n_tiles + a.T), dim3(kShrinkThreads), 0, stream, a.T, a.K, n_tiles,
                               static_cast<const uint16_t *>(a.x), a.pool, row_slot, row_scale, V, Rpad);
        }
        ELORA_HIP_TRY(hipGetLastError());
    }
    return launch_gemm_back(a, stream, copy_done);
}

// Two or three calls of this path that read the same x with the same routing tables (each with a pool of its own):
// one route launch, ONE shrink launch over the adapters of all of them, then each call's GEMM.
bool elora::gemm_group_shares_shrink(const LinearArgs *a, int n)
{
    if (n < 2 || n > kShrinkMulti) return false;
    for (int i = 0; i < n; ++i) {
        if (!a[i].has_pool || a[i].x != a[0].x || a[i].T != a[0].T || a[i].K != a[0].K) return false;
        if ((a[i].pool.q8 != 0) != (a[0].pool.q8 != 0)) return false;  // (one storage format of the pools per shrink launch)
        const RouteView &r = a[i].route, &r0 = a[0].route;
        if (r.adapter_idx != r0.adapter_idx || r.seg_offsets != r0.seg_offsets || r.seg_adapter != r0.seg_adapter ||
            r.n_segments != r0.n_segments || r.scales != r0.scales)
            return false;
    }
    return true;
}

int elora::launch_gemm_group(const LinearArgs *a, int n, hipStream_t stream)
{
    ShrinkMulti sm;
    sm.n = n;
    for (int i = 0; i < n; ++i) {
        sm.pool[i] = a[i].pool;
        sm.row_slot[i] = reinterpret_cast<int32_t *>(a[i].ws + a[i].wsl.row_slot);
        sm.row_scale[i] = reinterpret_cast<float *>(a[i].ws + a[i].wsl.row_scale);
        sm.V[i] = reinterpret_cast<uint16_t *>(a[i].ws + a[i].wsl.v);
        sm.Rpad[i] = round_up(a[i].pool.max_rank, BK);
    }
    const int T = a[0].T, K = a[0].K;
    hipLaunchKernelGGL(gemm_route_multi_kernel, dim3((T + 255) / 256), dim3(256), 0, stream, T, a[0].route, sm);
    ELORA_HIP_TRY(hipGetLastError());
    const int n_tiles = (T + kShrinkRows - 1) / kShrinkRows;
    const int per = (n_tiles + T + 7) / 8 * 8;
    if (a[0].pool.q8)
        hipLaunchKernelGGL(sgmv_shrink_multi_kernel<true>, dim3(per * n), dim3(kShrinkThreads), 0, stream, T, K, n_tiles,
                           static_cast<const uint16_t *>(a[0].x), sm);
    else
        hipLaunchKernelGGL(sgmv_shrink_multi_kernel<false>, dim3(per * n), dim3(kShrinkThreads), 0, stream, T, K, n_tiles,
                           static_cast<const uint16_t *>(a[0].x), sm);
    ELORA_HIP_TRY(hipGetLastError());
    for (int i = 0; i < n; ++i) {
        const int rc = launch_gemm_back(a[i], stream);
        if (rc != ELORA_OK) return rc;
    }
    return ELORA_OK;
}
