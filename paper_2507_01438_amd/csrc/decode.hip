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
constexpr int kChunk = 256;             // K elements per register set of W (8 MFMA K steps)
constexpr int kStepsPerChunk = kChunk / 32;
#ifndef ELORA_DEC_SPAN
#define ELORA_DEC_SPAN 1024        // elements of x per row parked in LDS at a time when at most 32 rows are in the batch
#endif
// x of the workgroup's K-slice is parked in LDS in spans of kSpan(TT) elements per row (row pitch +16 bytes so
// that 16 rows hit 16 different bank groups): 1024 for up to 32 rows of x, 512 for up to 64 (about 66 KiB)
__host__ __device__ constexpr int span_of(int tt) { return tt <= 2 ? ELORA_DEC_SPAN : 512; }

// sync area (ints) at the start of the workspace
constexpr int kCntV = 0;      // shrink units finished
constexpr int kCntDone = 1;   // tile epilogues finished
constexpr int kCntTile = 16;  // + tile: K-split workgroups of that tile that have arrived

int g_spin_limit = 1 << 22;

// tuning constants (overridable at compile time for experiments)
#ifndef ELORA_DEC_MAX_SHRINK_WGS
#define ELORA_DEC_MAX_SHRINK_WGS 512  // upper bound on shrink workgroups (each wave then loops over several units)
#endif
#ifndef ELORA_DEC_TARGET_WGS
#define ELORA_DEC_TARGET_WGS 640  // upper bound on base workgroups when choosing the K-split
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
                                                          int *__restrict__ row_slot, int *__restrict__ row_rank,
                                                          float *__restrict__ row_scale, uint16_t *__restrict__ y)
{
    // x span during the contraction; v of every row during the epilogue
    constexpr int kSpan = span_of(TT), kPitch = kSpan + 8, kChunksPerSpan = kSpan / kChunk;
    __shared__ __attribute__((aligned(16))) uint16_t xs[TT * 16][kPitch];
    __shared__ int s_slot[TT * 16], s_rank[TT * 16];
    __shared__ float s_scale[TT * 16];
    __shared__ int s_last, s_vok;

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
            if (j0 == 0 && lane == 0) {  // the row's route, for the tile epilogues
                __hip_atomic_store(&row_slot[t], rr.slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(&row_rank[t], rr.rank, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                store_shared_f32(&row_scale[t], rr.scale);
            }
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
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;

    auto load_w = [&](u32x4 *dst, int chunk) {
        const uint16_t *p = wrow + (size_t)chunk * kChunk;
#pragma unroll
        for (int j = 0; j < kStepsPerChunk; ++j)
            dst[j] = wave_active ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p + j * 32)) : u32x4{0, 0, 0, 0};
    };
    // Park x[:, chunks c0 .. c0 + nc) of the K-slice in LDS, global -> LDS directly.  One instruction moves 512
    // consecutive elements of one row (two chunks; the odd last chunk of a span moves with half the lanes).
    // Rows past the batch repeat the last row: what they produce is never stored.
    auto park_x = [&](int c0, int nc) {
        const int units = TT * 16 * ((nc + 1) >> 1);  // (row, pair of chunks)
        for (int u = wave; u < units; u += kWaves) {
            const int r = u % (TT * 16), pr = u / (TT * 16);
            const uint16_t *src = x + (size_t)min(r, T - 1) * K + k_begin + (size_t)(c0 + 2 * pr) * kChunk + lane * 8;
            uint16_t *dst = &xs[r][pr * 2 * kChunk];
            if (2 * pr + 1 < nc || lane < 32)
                __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)dst, 16, 0, 0);
        }
    };

    park_x(0, min(nchunks, kChunksPerSpan));
    load_w(wbuf[0], 0);
    if (nchunks > 1) load_w(wbuf[1], 1);

    // ---- base tile -------------------------------------------------------------------------------
    floatx4 acc[TT];
#pragma unroll
    for (int i = 0; i < TT; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    auto compute = [&](const u32x4 *wc, int cs) {  // cs = chunk inside the span
#pragma unroll
        for (int j = 0; j < kStepsPerChunk; ++j) {
            bf16x8 a = __builtin_bit_cast(bf16x8, wc[j]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                bf16x8 b = *reinterpret_cast<const bf16x8 *>(&xs[tt * 16 + m][cs * kChunk + j * 32 + g * 8]);
                acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[tt], 0, 0, 0);
            }
        }
    };
    // The waves only meet when a span of x is exchanged; inside a span each wave streams its 16 rows of W on
    // its own, two chunks (16 loads of 16 bytes per lane) ahead of the one it multiplies.
    for (int c0 = 0; c0 < nchunks; c0 += kChunksPerSpan) {
        const int nc = min(kChunksPerSpan, nchunks - c0);
        if (c0 > 0) {
            __syncthreads();  // everybody is done with the previous span
            park_x(c0, nc);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wave's share of the span has landed (so has its W prefetch)
        __syncthreads();
        if (c0 == 0) TRACE(2);  // first span of x parked
        for (int cs = 0; cs < nc; cs += 2) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int cc = c0 + cs + h;  // kChunksPerSpan is even, so chunk cc uses register set h
                if (cs + h < nc) {
                    compute(wbuf[h], cs + h);
                    if (cc + 2 < nchunks) load_w(wbuf[h], cc + 2);
                }
            }
        }
    }

    TRACE(3);  // contraction done

    // ---- expand share of this workgroup ------------------------------------------------------------
    // Rows t = ks, ks + split, ... of the batch get  s_t * B_i v_t  for this tile's 64 columns added to this
    // workgroup's K-slice partial, so the expand of a tile is spread over its `split` workgroups (and B_i is
    // read where the partial is still in registers).
    const int n0 = tile * kTileRows;
    const int nq = (sh.n_shrink_wgs > 0 && ks < T) ? (T - ks + sh.split - 1) / sh.split : 0;
    if (nq > 0) {
        __syncthreads();  // xs is reused below
        if (tid == 0) {
            int ok = 0;
            for (int spin = 0; spin < sh.spin_limit; ++spin) {
                if (__hip_atomic_load(&sync[kCntV], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= sh.n_shrink_wgs) {
                    ok = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(4);
            }
            s_vok = ok;
        }
        __syncthreads();
        // v and the rows' routes written by the shrink workgroups are read past the L2 from here on
        const bool vok = s_vok != 0;
        TRACE(4);  // shrink results available
        float *vs = reinterpret_cast<float *>(&xs[0][0]);  // [rows of this pass][R], then d [rows][64]
        const int qb_max = (int)(sizeof(xs) / ((R + kTileRows) * sizeof(float)));
        for (int q0 = 0; q0 < nq; q0 += qb_max) {
            const int qb = min(qb_max, nq - q0);
            float *dls = vs + qb * R;
            if (q0 > 0) __syncthreads();
            if (tid < qb) {
                const int t = ks + (q0 + tid) * sh.split;
                RowRoute rr;
                if (vok) {
                    rr.slot = __hip_atomic_load(&row_slot[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    rr.rank = __hip_atomic_load(&row_rank[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    rr.scale = load_shared_f32(&row_scale[t]);
                } else {
                    rr = resolve_row(t, route, pool, false);
                }
                s_slot[tid] = rr.slot;
                s_rank[tid] = rr.rank;
                s_scale[tid] = rr.scale;
            }
            __syncthreads();
            if (vok) {
                for (int e0 = 0; e0 < qb * R; e0 += kThreads * 8) {
                    float tmp[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int e = e0 + i * kThreads + tid;
                        const int q = e / R, j = e - q * R;
                        tmp[i] = (e < qb * R && j < s_rank[q]) ? load_shared_f32(&v[(size_t)(ks + (q0 + q) * sh.split) * R + j]) : 0.0f;
                    }
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int e = e0 + i * kThreads + tid;
                        if (e < qb * R) vs[e] = tmp[i];
                    }
                }
            } else {
                // the shrink workgroups did not report in time: compute v of these rows here
                for (int wu = wave; wu < qb * sh.jgroups; wu += kWaves) {
                    const int q = wu / sh.jgroups, j0 = (wu - q * sh.jgroups) * 2;
                    const int t = ks + (q0 + q) * sh.split;
                    const int slot = s_slot[q], rank = s_rank[q];
                    float r0 = 0.0f, r1 = 0.0f;
                    if (slot >= 0 && j0 < rank) {
                        const uint16_t *A0 = reinterpret_cast<const uint16_t *>(slot_A(pool, slot)) + (size_t)j0 * K;
                        shrink_pair(A0, (j0 + 1 < rank) ? A0 + K : A0, x + (size_t)t * K, K, lane, r0, r1);
                        if (j0 + 1 >= rank) r1 = 0.0f;
                    }
                    if (lane == 0) {
                        vs[q * R + j0] = r0;
                        if (j0 + 1 < R) vs[q * R + j0 + 1] = r1;
                    }
                }
            }
            __syncthreads();
            // d[q][c] = s * sum_j B_i[n0 + c][j] v[q][j]: one (row, column) item per thread, four items at a time
            // so that up to 32 loads of 16 bytes are in flight per thread
            constexpr int IB = 4;
            for (int it0 = tid; it0 < qb * kTileRows; it0 += kThreads * IB) {
                int iq[IB], ir[IB];
                const uint16_t *bp[IB];
                float d[IB];
                bool vec = true;
#pragma unroll
                for (int ii = 0; ii < IB; ++ii) {
                    const int item = it0 + ii * kThreads;
                    const bool in = item < qb * kTileRows;
                    const int q = in ? item / kTileRows : 0, c = in ? item - q * kTileRows : 0;
                    const int slot = s_slot[q];
                    iq[ii] = q;
                    ir[ii] = (in && slot >= 0 && n0 + c < N) ? s_rank[q] : 0;
                    bp[ii] = reinterpret_cast<const uint16_t *>(slot_B(pool, slot >= 0 ? slot : 0)) + (size_t)min(n0 + c, N - 1) * s_rank[q];
                    d[ii] = 0.0f;
                    vec = vec && ((ir[ii] & 7) == 0);
                }
                if (vec) {
                    int rmax = 0;
#pragma unroll
                    for (int ii = 0; ii < IB; ++ii) rmax = max(rmax, ir[ii]);
                    for (int j = 0; j < rmax; j += 64) {
                        u32x4 b[IB][8];
#pragma unroll
                        for (int ii = 0; ii < IB; ++ii)
#pragma unroll
                            for (int h = 0; h < 8; ++h)
                                b[ii][h] = (j + 8 * h < ir[ii]) ? *reinterpret_cast<const u32x4 *>(bp[ii] + j + 8 * h) : u32x4{0, 0, 0, 0};
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int ii = 0; ii < IB; ++ii) {
                            const float *vq = vs + iq[ii] * R + j;
#pragma unroll
                            for (int h = 0; h < 8; ++h) {
                                if (j + 8 * h >= ir[ii]) continue;
#pragma unroll
                                for (int u = 0; u < 4; ++u) {
                                    d[ii] = fmaf(__uint_as_float(b[ii][h][u] << 16), vq[8 * h + 2 * u], d[ii]);
                                    d[ii] = fmaf(__uint_as_float(b[ii][h][u] & 0xffff0000u), vq[8 * h + 2 * u + 1], d[ii]);
                                }
                            }
                        }
                    }
                } else {
#pragma unroll
                    for (int ii = 0; ii < IB; ++ii)
                        for (int j = 0; j < ir[ii]; ++j) d[ii] = fmaf(bf16_to_f32(bp[ii][j]), vs[iq[ii] * R + j], d[ii]);
                }
#pragma unroll
                for (int ii = 0; ii < IB; ++ii) {
                    const int item = it0 + ii * kThreads;
                    if (item < qb * kTileRows) dls[item] = d[ii] * s_scale[iq[ii]];
                }
            }
            __syncthreads();
            // add to the accumulators: lane holds row t = tt * 16 + m of the batch, columns wave * 16 + g * 4 + 0..3
#pragma unroll
            for (int tt = 0; tt < TT; ++tt) {
                const int t = tt * 16 + m;
                const int q = (t - ks) / sh.split - q0;
                if (t < T && t >= ks && (t - ks) % sh.split == 0 && q >= 0 && q < qb) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) acc[tt][i] += dls[q * kTileRows + wave * kRowsPerWave + g * 4 + i];
                }
            }
        }
    }

    // C layout of the 16x16 MFMA: lane holds column (lane % 16) = row t of x, rows (lane / 16) * 4 + 0..3 = W rows
    if (wave_active) {
        const int n_base = n0 + wave * kRowsPerWave + g * 4;
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

    // ---- ticket: is this the last K-slice of the tile? -----------------------------------------------
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the write-through stores have been acknowledged
    __syncthreads();
    if (tid == 0) s_last = (sh.split == 1 || atomicAdd(&sync[kCntTile + tile], 1) == sh.split - 1) ? 1 : 0;
    __syncthreads();
    TRACE(5);  // ticket drawn
    if (s_last == 0) return;

    // ---- tile epilogue: sum the K-slices in fixed order, round once, store each row at its own position ----
    // 8 threads per row of x, 8 output columns each
    for (int item = tid; item < T * 8; item += kThreads) {
        const int t = item >> 3, n = n0 + (item & 7) * 8;
        if (n >= N) continue;  // N % 8 == 0
        float2 pv[kDecodeMaxSplit][4];
#pragma unroll
        for (int s = 0; s < kDecodeMaxSplit; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                pv[s][q] = load_shared_f32x2(partial + ((size_t)(s < sh.split ? s : 0) * T + t) * N + n + 2 * q);
        __builtin_amdgcn_sched_barrier(0);  // all loads first (slices beyond `split` re-read slice 0 and are dropped)
        float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < kDecodeMaxSplit; ++s)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                o[2 * q] += (s < sh.split) ? pv[s][q].x : 0.0f;
                o[2 * q + 1] += (s < sh.split) ? pv[s][q].y : 0.0f;
            }
        u32x4 packed;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            packed[q] = (uint32_t)f32_to_bf16(o[2 * q]) | ((uint32_t)f32_to_bf16(o[2 * q + 1]) << 16);
        *reinterpret_cast<u32x4 *>(y + (size_t)t * N + n) = packed;
    }

    TRACE(8);  // y written
    // ---- leave the counters at zero for the next call --------------------------------------------
    // When the last epilogue gets here every base workgroup has drawn its ticket, which it does after
    // its wait for the shrink workgroups, so nobody looks at sync[kCntV] any more.
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
        sh.n_shrink_wgs = wgs < ELORA_DEC_MAX_SHRINK_WGS ? wgs : ELORA_DEC_MAX_SHRINK_WGS;
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
    int *row_slot = reinterpret_cast<int *>(a.ws + a.wsl.row_slot);
    int *row_rank = reinterpret_cast<int *>(a.ws + a.wsl.row_rank);
    float *row_scale = reinterpret_cast<float *>(a.ws + a.wsl.row_scale);
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *W = static_cast<const uint16_t *>(a.W);
    uint16_t *y = static_cast<uint16_t *>(a.y);
    int has_pool = a.has_pool ? 1 : 0;
    dim3 grid(sh.n_tiles * sh.split + sh.n_shrink_wgs), block(kThreads);
    int tt = (a.T + 15) / 16;
    profile_mark_begin(stream);
    switch (tt) {
    case 1: hipLaunchKernelGGL((decode_kernel<1>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, row_slot, row_rank, row_scale, y); break;
    case 2: hipLaunchKernelGGL((decode_kernel<2>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, row_slot, row_rank, row_scale, y); break;
    case 3: hipLaunchKernelGGL((decode_kernel<3>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, row_slot, row_rank, row_scale, y); break;
    default: hipLaunchKernelGGL((decode_kernel<4>), grid, block, 0, stream, sh, x, W, a.pool, a.route, has_pool, partial, v, sync, row_slot, row_rank, row_scale, y); break;
    }
    ELORA_HIP_TRY(hipGetLastError());
    profile_mark_end(stream);
    return ELORA_OK;
}
