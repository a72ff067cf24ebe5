// Decode path (few rows, HBM-bound): bf16, up to 64 rows, ONE launch per call.
//
// The grid holds two kinds of workgroups:
//
//   shrink workgroups (the first n_shrink_wgs): each wave takes (row t, two rank rows j) units and
//       computes  v[t][j] = sum_k A_i[j,k] x[t,k]  over the whole of d_in with plain FMAs and one
//       wavefront reduction (A_i x_t of the row's own adapter, Sec. 3.4).  When a workgroup has
//       stored its results it adds one to sync[kCntV].
//   base workgroups (tile, ks): 64 rows of W and one K-slice,
//       partial[ks][t][n] = sum_{k in slice ks} W[n,k] x[t,k]   (Sec. 3.4: W x [x_0..x_n], shared by
//       the whole batch).  Each wave streams 16 rows of W straight from global memory into the
//       A-operand of v_mfma_f32_16x16x32_bf16 (row = lane % 16, 8 consecutive k per lane); the rows of
//       x are the B-operand, read from an LDS copy of the current 256-wide K-chunk.  W loads are
//       issued two chunks ahead.  The LAST of a tile's `split` workgroups to arrive (atomic ticket,
//       nobody waits for a ticket) runs the tile epilogue: it sums the K-split partials in fixed
//       order and writes  y[t,n] = bf16(base + s_i * sum_j B_i[n,j] v[t][j])  at the row's own
//       position (Sec. 3.4: results are combined and land at their original locations).
//
// The only wait in the kernel is the epilogue's wait for the shrink workgroups (sync[kCntV]).  Those
// come first in the grid and wait for nothing, and at most n_tiles workgroups can be waiting, so the
// wait always ends; it is bounded all the same, and a workgroup whose bound runs out computes the
// v[t][:] it needs by itself.  Counters live in the first bytes of the caller's workspace and are back
// at zero when the kernel ends (so the call can be replayed from a HIP graph).
//
// Summation order is fixed (no float atomics): results are bit-identical from run to run.
#include "common.h"

using namespace elora;

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;         // waves per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kRowsPerWave = 16;  // W rows per wave (one MFMA row block)
constexpr int kTileRows = kWaves * kRowsPerWave;
constexpr int kChunk = 256;             // K elements per LDS stage
constexpr int kLdsStride = kChunk + 8;  // bf16 elements; +16 bytes so 16 rows hit 16 different bank groups
constexpr int kStepsPerChunk = kChunk / 32;

// sync area (ints) at the start of the workspace
constexpr int kCntV = 0;      // shrink units finished
constexpr int kCntDone = 1;   // tile epilogues finished
constexpr int kCntTile = 16;  // + tile: K-split workgroups of that tile that have arrived

int g_spin_limit = 1 << 22;

// tuning constants (overridable at compile time for experiments)
#ifndef ELORA_DEC_TARGET_WGS
#define ELORA_DEC_TARGET_WGS 640  // upper bound on base workgroups when choosing the K-split
#endif
#ifndef ELORA_DEC_PREFETCH
#define ELORA_DEC_PREFETCH 2      // W chunks requested ahead of the one being consumed (1 or 2)
#endif

// Optional phase timestamps for tuning (compiled in only with -DELORA_TRACE): slot i of workgroup b.
#ifdef ELORA_TRACE
__device__ long long elora_trace_buf[4096 * 16];
#define TRACE(i)                                                                                   \
    do {                                                                                           \
        if (threadIdx.x == 0 && blockIdx.x < 4096) elora_trace_buf[blockIdx.x * 16 + (i)] = wall_clock64(); \
    } while (0)
#else
#define TRACE(i) do {} while (0)
#endif

struct DecodeShape {
    int T, K, N;
    int split;  // K-slices of the base contraction
    int chunks_per_split;
    int n_tiles;
    int n_shrink_wgs;  // leading workgroups that compute v = A_i x_t
    int jgroups;       // pairs of rank rows per row of x: ceil(max_rank / 2)
    int spin_limit;
};

// Data that one workgroup writes and another reads inside the same launch (partial, v) goes
// through agent-scope accesses, which on gfx950 write through / read past the per-XCD L2, so the
// hand-over needs no cache-wide write-back or invalidate (those cost tens of microseconds here).
__device__ __forceinline__ void store_shared_f32(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void store_shared_f32x2(float *p, float a, float b)
{
    uint64_t u = (uint64_t)__float_as_uint(a) | ((uint64_t)__float_as_uint(b) << 32);
    __hip_atomic_store(reinterpret_cast<uint64_t *>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_shared_f32(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 load_shared_f32x2(const float *p)
{
    uint64_t u = __hip_atomic_load(reinterpret_cast<const uint64_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return float2{__uint_as_float((uint32_t)u), __uint_as_float((uint32_t)(u >> 32))};
}

template <int TT>
__global__ __launch_bounds__(kThreads) void decode_kernel(DecodeShape sh, const uint16_t *__restrict__ x,
                                                          const uint16_t *__restrict__ W, PoolView pool,
                                                          RouteView route, int has_pool, float *__restrict__ partial,
                                                          float *__restrict__ v, int *__restrict__ sync,
                                                          uint16_t *__restrict__ y)
{
    // x chunks (two stages) during the contraction; v of every row during the epilogue
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * TT * 16 * kLdsStride * 2];
    __shared__ int s_slot[TT * 16], s_rank[TT * 16];
    __shared__ float s_scale[TT * 16];
    __shared__ int s_last, s_vok;
    auto xs = reinterpret_cast<uint16_t(*)[TT * 16][kLdsStride]>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = sh.T, K = sh.K, N = sh.N;
    const int R = pool.max_rank;
    TRACE(0);

    // ---- shrink workgroups ---------------------------------------------------------------------
    if ((int)blockIdx.x < sh.n_shrink_wgs) {
        const int n_units = T * sh.jgroups;
        for (int wu = blockIdx.x * kWaves + wave; wu < n_units; wu += sh.n_shrink_wgs * kWaves) {
            const int t = wu / sh.jgroups, j0 = (wu - t * sh.jgroups) * 2;
            RowRoute rr = resolve_row(t, route, pool, j0 == 0 && lane == 0);
            if (rr.slot < 0 || j0 >= rr.rank) continue;
            const bool two = (j0 + 1) < rr.rank;
            const uint16_t *A0 = reinterpret_cast<const uint16_t *>(slot_A(pool, rr.slot)) + (size_t)j0 * K;
            const uint16_t *A1 = two ? A0 + K : A0;
            float r0, r1;
            shrink_pair(A0, A1, x + (size_t)t * K, K, lane, r0, r1);
            if (lane == 0) {
                store_shared_f32(&v[(size_t)t * R + j0], r0);
                if (two) store_shared_f32(&v[(size_t)t * R + j0 + 1], r1);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the write-through stores have been acknowledged
        __syncthreads();
        if (tid == 0) atomicAdd(&sync[kCntV], 1);
        TRACE(1);
        return;
    }

    // ---- base workgroups: issue the first W and x loads before anything else -------------------
    const int bid = blockIdx.x - sh.n_shrink_wgs;
    const int tile = bid % sh.n_tiles, ks = bid / sh.n_tiles;
    const int m = lane & 15, g = lane >> 4;
    const int row = tile * kTileRows + wave * kRowsPerWave + m;                // W row this lane feeds
    const bool wave_active = (tile * kTileRows + wave * kRowsPerWave) < N;     // N % 16 == 0: all 16 rows in or out
    const int k_begin = ks * sh.chunks_per_split * kChunk;
    const uint16_t *wrow = W + (size_t)(wave_active ? row : 0) * K + k_begin + g * 8;
    const int nchunks = sh.chunks_per_split;

    u32x4 wbuf[2][kStepsPerChunk];
    constexpr int kXPieces = TT * 2;  // TT*16 rows x 32 pieces of 16 bytes over 256 threads
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
            int piece = tid + i * kThreads;
            int r = piece >> 5, c16 = piece & 31;
            xreg[i] = (r < T) ? *reinterpret_cast<const u32x4 *>(x + (size_t)r * K + k_begin + (size_t)chunk * kChunk + c16 * 8)
                              : u32x4{0, 0, 0, 0};
        }
    };
    auto store_x = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kXPieces; ++i) {
            int piece = tid + i * kThreads;
            int r = piece >> 5, c16 = piece & 31;
            *reinterpret_cast<u32x4 *>(&xs[buf][r][c16 * 8]) = xreg[i];
        }
    };

    load_x(0);
    load_w(wbuf[0], 0);
    if (ELORA_DEC_PREFETCH > 1 && nchunks > 1) load_w(wbuf[1], 1);

    // ---- 2. base tile ----------------------------------------------------------------------------
    floatx4 acc[TT];
#pragma unroll
    for (int i = 0; i < TT; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    store_x(0);
    __syncthreads();
    TRACE(2);  // first x chunk staged

    auto compute = [&](const u32x4 *wc, int buf) {
#pragma unroll
        for (int j = 0; j < kStepsPerChunk; ++j) {
            bf16x8 a = __builtin_bit_cast(bf16x8, wc[j]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                bf16x8 b = *reinterpret_cast<const bf16x8 *>(&xs[buf][tt * 16 + m][j * 32 + g * 8]);
                acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[tt], 0, 0, 0);
            }
        }
    };
    // chunk c: x from LDS stage c & 1, W from register set c & 1; the next x chunk is fetched while
    // computing and W chunk c + 2 is requested as soon as set c & 1 has been consumed
    for (int c = 0; c < nchunks; c += 2) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int cc = c + h;
            if (cc < nchunks) {
                const bool more = (cc + 1) < nchunks;
                if (more) load_x(cc + 1);
                if (ELORA_DEC_PREFETCH == 1 && more) load_w(wbuf[h ^ 1], cc + 1);
                compute(wbuf[h], h);
                if (ELORA_DEC_PREFETCH > 1 && cc + 2 < nchunks) load_w(wbuf[h], cc + 2);
                if (more) store_x(h ^ 1);
                __syncthreads();
            }
        }
    }

    TRACE(3);  // contraction done
    // C layout of the 16x16 MFMA: lane holds column (lane % 16) = row t of x, rows (lane / 16) * 4 + 0..3 = W rows
    if (wave_active) {
        const int n_base = tile * kTileRows + wave * kRowsPerWave + g * 4;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            int t = tt * 16 + m;
            if (t < T) {
                float *p = partial + ((size_t)ks * T + t) * N + n_base;
                store_shared_f32x2(p, acc[tt][0], acc[tt][1]);
                store_shared_f32x2(p + 2, acc[tt][2], acc[tt][3]);
            }
        }
    }

    // ---- 3. ticket: is this the last K-slice of the tile? ------------------------------------
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the write-through stores have been acknowledged
    __syncthreads();
    TRACE(4);  // partial stores acknowledged
    if (tid == 0) s_last = (sh.split == 1 || atomicAdd(&sync[kCntTile + tile], 1) == sh.split - 1) ? 1 : 0;
    __syncthreads();
    TRACE(5);  // ticket drawn
    if (s_last == 0) return;

    // ---- tile epilogue ---------------------------------------------------------------------------
    if (tid < TT * 16) {
        RowRoute rr{-1, 0, 0.0f};
        if (has_pool && tid < T) rr = resolve_row(tid, route, pool, false);
        s_slot[tid] = rr.slot;
        s_rank[tid] = rr.rank;
        s_scale[tid] = rr.scale;
    }
    if (tid == 0) {
        int ok = 1;
        if (sh.n_shrink_wgs > 0) {
            ok = 0;
            for (int spin = 0; spin < sh.spin_limit; ++spin) {
                if (__hip_atomic_load(&sync[kCntV], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= sh.n_shrink_wgs) {
                    ok = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(4);
            }
        }
        s_vok = ok;
    }
    __syncthreads();
    // partial and v of the other workgroups are read past the L2 from here on
    TRACE(6);  // routes resolved, shrink results available
    float *vs = reinterpret_cast<float *>(smem);  // [T][R]; T*R*4 <= TT*16*256*4 < sizeof(smem)
    if (sh.n_shrink_wgs > 0) {
        if (s_vok) {
            for (int e0 = 0; e0 < T * R; e0 += kThreads * 8) {
                float tmp[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int e = e0 + i * kThreads + tid;
                    const int t = e / R, j = e - t * R;
                    tmp[i] = (e < T * R && j < s_rank[t]) ? load_shared_f32(&v[e]) : 0.0f;
                }
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int e = e0 + i * kThreads + tid;
                    if (e < T * R) vs[e] = tmp[i];
                }
            }
        } else {
            // the shrink workgroups did not report in time: compute v here
            for (int wu = wave; wu < T * sh.jgroups; wu += kWaves) {
                const int t = wu / sh.jgroups, j0 = (wu - t * sh.jgroups) * 2;
                const int slot = s_slot[t], rank = s_rank[t];
                float r0 = 0.0f, r1 = 0.0f;
                if (slot >= 0 && j0 < rank) {
                    const uint16_t *A0 = reinterpret_cast<const uint16_t *>(slot_A(pool, slot)) + (size_t)j0 * K;
                    shrink_pair(A0, (j0 + 1 < rank) ? A0 + K : A0, x + (size_t)t * K, K, lane, r0, r1);
                    if (j0 + 1 >= rank) r1 = 0.0f;
                }
                if (lane == 0) {
                    vs[t * R + j0] = r0;
                    if (j0 + 1 < R) vs[t * R + j0 + 1] = r1;
                }
            }
        }
    }
    __syncthreads();
    TRACE(7);  // v_t formed
    // 8 threads per row of x, 8 output columns each
    const int n0 = tile * kTileRows;
    for (int item = tid; item < T * 8; item += kThreads) {
        const int t = item >> 3, n = n0 + (item & 7) * 8;
        if (n >= N) continue;  // N % 8 == 0
        float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        {
            float2 pv[kDecodeMaxSplit][4];
#pragma unroll
            for (int s = 0; s < kDecodeMaxSplit; ++s)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    pv[s][q] = load_shared_f32x2(partial + ((size_t)(s < sh.split ? s : 0) * T + t) * N + n + 2 * q);
            __builtin_amdgcn_sched_barrier(0);  // all loads first (slices beyond `split` re-read slice 0 and are dropped)
#pragma unroll
            for (int s = 0; s < kDecodeMaxSplit; ++s)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    o[2 * q] += (s < sh.split) ? pv[s][q].x : 0.0f;
                    o[2 * q + 1] += (s < sh.split) ? pv[s][q].y : 0.0f;
                }
        }
        TRACE(9);  // partials summed
        const int slot = s_slot[t];
        if (slot >= 0) {
            const int r = s_rank[t];
            const float sc = s_scale[t];
            const uint16_t *B = reinterpret_cast<const uint16_t *>(slot_B(pool, slot)) + (size_t)n * r;
            const float *vt = vs + t * R;
            if ((r & 7) == 0) {
                float d[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                for (int j = 0; j < r; j += 16) {
                    // 8 output columns x 16 rank entries: 16 loads of 16 bytes in flight together
                    const bool second = (j + 8) < r;
                    u32x4 b[8][2];
#pragma unroll
                    for (int q = 0; q < 8; ++q) {
                        b[q][0] = *reinterpret_cast<const u32x4 *>(B + q * r + j);
                        b[q][1] = *reinterpret_cast<const u32x4 *>(B + q * r + (second ? j + 8 : j));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int q = 0; q < 8; ++q)
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            if (h == 1 && !second) continue;
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                d[q] = fmaf(__uint_as_float(b[q][h][u] << 16), vt[j + 8 * h + 2 * u], d[q]);
                                d[q] = fmaf(__uint_as_float(b[q][h][u] & 0xffff0000u), vt[j + 8 * h + 2 * u + 1], d[q]);
                            }
                        }
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) o[q] += sc * d[q];
            } else {
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    float d = 0.0f;
                    for (int j = 0; j < r; ++j) d = fmaf(bf16_to_f32(B[q * r + j]), vt[j], d);
                    o[q] += sc * d;
                }
            }
        }
        TRACE(10);  // expand done
        u32x4 packed;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            packed[q] = (uint32_t)f32_to_bf16(o[2 * q]) | ((uint32_t)f32_to_bf16(o[2 * q + 1]) << 16);
        *reinterpret_cast<u32x4 *>(y + (size_t)t * N + n) = packed;
    }

    TRACE(8);  // y written
    // ---- leave the counters at zero for the next call --------------------------------------------
    // The last epilogue has seen sync[kCntV] complete, so no shrink workgroup will touch it any more.
    if (tid == 0) {
        __hip_atomic_store(&sync[kCntTile + tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (atomicAdd(&sync[kCntDone], 1) == sh.n_tiles - 1) {
            __hip_atomic_store(&sync[kCntV], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&sync[kCntDone], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

int pick_split(int K, int n_tiles)
{
    // aim at about two workgroups per compute unit (512), K-slices of whole 256-wide chunks
    int chunks = K / kChunk;
    int best = 1;
    for (int s = 1; s <= kDecodeMaxSplit; ++s) {
        if (chunks % s) continue;
        if (n_tiles * s <= ELORA_DEC_TARGET_WGS) best = s;
    }
    return best;
}

DecodeShape make_shape(int T, int K, int N, int max_rank, bool has_pool)
{
    DecodeShape sh;
    sh.T = T;
    sh.K = K;
    sh.N = N;
    sh.n_tiles = (N + kTileRows - 1) / kTileRows;
    sh.split = pick_split(K, sh.n_tiles);
    sh.chunks_per_split = K / kChunk / sh.split;
    sh.jgroups = (max_rank + 1) / 2;
    sh.n_shrink_wgs = 0;
    if (has_pool) {
        int wgs = (T * sh.jgroups + kWaves - 1) / kWaves;  // one (row, rank-row pair) unit per wave
        sh.n_shrink_wgs = wgs < 512 ? wgs : 512;
    }
    sh.spin_limit = g_spin_limit;
    return sh;
}

}  // namespace

void elora::decode_set_spin_limit(int limit) { g_spin_limit = limit; }

#ifdef ELORA_TRACE
extern "C" int elora_trace_read(long long *host_out, int n_values)
{
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(elora_trace_buf), sizeof(long long) * n_values) == hipSuccess ? 0 : 10;
}
extern "C" int elora_trace_clear()
{
    static long long zeros[4096 * 16];
    return hipMemcpyToSymbol(HIP_SYMBOL(elora_trace_buf), zeros, sizeof zeros) == hipSuccess ? 0 : 10;
}
#endif

bool elora::decode_eligible(const elora_linear_desc_t &d, int max_rank)
{
    (void)max_rank;
    return d.dtype == ELORA_BF16 && d.wfmt == ELORA_W_SAME && d.n_tokens >= 1 && d.n_tokens <= kDecodeMaxTokens &&
           d.d_in % kChunk == 0 && d.d_out % 16 == 0 && (d.d_out + kTileRows - 1) / kTileRows <= kSyncInts - kCntTile;
}

void elora::decode_plan(const elora_linear_desc_t &d, elora_plan_t *plan)
{
    DecodeShape sh = make_shape(d.n_tokens, d.d_in, d.d_out, d.pool ? d.pool->max_rank : 1, d.pool != nullptr);
    plan->n_launches = 1;
    plan->split_k = sh.split;
    plan->tile_rows = kTileRows;
    plan->tile_cols = 0;
    plan->grid = sh.n_tiles * sh.split + sh.n_shrink_wgs;
}

int elora::launch_decode(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream)
{
    (void)plan;
    DecodeShape sh = make_shape(a.T, a.K, a.N, a.pool.max_rank, a.has_pool);
    float *partial = reinterpret_cast<float *>(a.ws + a.wsl.partial);
    float *v = reinterpret_cast<float *>(a.ws + a.wsl.v);
    int *sync = reinterpret_cast<int *>(a.ws + a.wsl.sync);
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *W = static_cast<const uint16_t *>(a.W);
    uint16_t *y = static_cast<uint16_t *>(a.y);
    int has_pool = a.has_pool ? 1 : 0;
    dim3 grid(sh.n_tiles * sh.split + sh.n_shrink_wgs), block(kThreads);
    int tt = (a.T + 15) / 16;
    profile_mark_begin(stream);
    switch (tt) {
    case 1: hipLaunchKernelGGL((decode_kernel<1>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, y); break;
    case 2: hipLaunchKernelGGL((decode_kernel<2>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, y); break;
    case 3: hipLaunchKernelGGL((decode_kernel<3>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, y); break;
    default: hipLaunchKernelGGL((decode_kernel<4>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, y); break;
    }
    ELORA_HIP_TRY(hipGetLastError());
    profile_mark_end(stream);
    return ELORA_OK;
}
