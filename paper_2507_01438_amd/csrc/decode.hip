// Decode path (few rows, HBM-bound): bf16, up to 64 rows, ONE launch per call.
//
// Every workgroup is a (tile, ks) pair: 64 rows of W (= 64 output columns) and one K-slice.  It runs
// three phases:
//
//   1. shrink share.  The (row t, two rank rows j) units of  v[t][j] = sum_k A_i[j,k] x[t,k]  (A_i x_t of
//      the row's own adapter, Sec. 3.4) are dealt out over the workgroups: bf16 dot products over the whole of
//      d_in and one wavefront reduction.  Results go into the v mailbox.
//   2. base contraction.  partial[ks][t][n] = sum_{k in slice ks} W[n,k] x[t,k]  (Sec. 3.4: W x [x_0..x_n],
//      shared by the whole batch) with v_mfma_f32_16x16x32_bf16: 16 rows of W per wave as A-operand, the rows
//      of x as B-operand.  The K-slice goes by in sub-spans of 128 elements through a ring in LDS that
//      direct-to-LDS loads keep filled: always the rows of x, and the tile's rows of W as well (whole cache
//      lines per load instruction) unless the shape wants two workgroups per compute unit with more than 32
//      rows of x; W then goes straight into the A-operand registers.
//   3. exchange and expand.  Workgroup ks OWNS 64 / split of the tile's columns.  Every workgroup posts the
//      pieces of its partial to their owners' mailboxes; each owner takes v, forms
//          d[t][n] = s_t * sum_j B_i[n,j] v[t][j]      for its own columns,
//      adds the pieces in fixed order (slice 0, 1, ...) and d, rounds once and writes
//          y[t,n] = bf16(W x_t + s_i B_i A_i x_t)   at the row's own position (Sec. 3.4: results are
//      combined and land at their original locations).
//
// Mailboxes hold the bit pattern 0xFFFFFFFF ("empty") between calls.  A reader polls the data itself
// until no word is empty, so a hand-over costs one store and one load, with no flags, counters or
// fences on the way.  Piece mailboxes have one reader, who puts the empty pattern back; the v mailbox
// is emptied by the last workgroup of the call to finish.  Arithmetic cannot produce the pattern: it is
// a NaN whose low mantissa bits are set, while every NaN here descends from a bf16 (low 16 bits zero)
// or is the default NaN.  The v mailbox is accessed at agent scope (past the per-XCD L2); the pieces of
// a tile travel between workgroups of one XCD and meet in that XCD's L2.
//
// Every wait is bounded.  A reader whose bound runs out computes what it needs from the inputs on its
// own (v of the rows it is working on, or its columns of y from scratch) and, for pieces, raises the
// call's dirty flag: the last workgroup to finish then empties all piece mailboxes, because pieces
// posted to a reader that gave up are still lying there.  Nobody waits before its own shrink share is
// posted, and owners only wait for the workgroups of their own tile, which sit next to each other in
// the grid and on the same XCD.  Counters and flags are zero again when the kernel ends, so a call can
// be replayed from a HIP graph.
//
// Summation order is fixed (no float atomics): results are bit-identical from run to run.
#include "common.h"

#include <type_traits>

using namespace elora;

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWaves = 4;         // waves per workgroup
constexpr int kThreads = kWaves * 64;
constexpr int kRowsPerWave = 16;  // W rows per wave (one MFMA row block)
constexpr int kTileRows = kWaves * kRowsPerWave;
constexpr int kGranules = kTileRows / 4;  // a granule = 4 adjacent columns = what one lane holds of one row of x
constexpr int kChunk = 256;               // K elements per register set of W (8 MFMA K steps)
// The ring of sub-spans in LDS (dynamic LDS: the only such array of the kernel; the staging after the contraction reuses
// it).  A sub-span is 128 elements of K.  Up to 32 rows of x: 5 slots, more rows: 3.  A slot holds the rows of x and,
// where W travels through the ring as well (see the kernel), the tile's 64 rows of W.
constexpr int kSubSpan = 128;
__host__ __device__ constexpr int ring_slots(int tt) { return tt <= 2 ? 5 : 3; }
__host__ __device__ constexpr int slot_rows(int tt, bool wlds) { return tt * 16 + (wlds ? kTileRows : 0); }
__host__ __device__ constexpr int ring_bytes(int tt, bool wlds) { return ring_slots(tt) * slot_rows(tt, wlds) * kSubSpan * 2; }
constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr int kMetaLds = 512;  // slot tables up to this many entries are copied to LDS whole

constexpr int kXcds = 8;                  // workgroup b runs on XCD b % 8

// sync area (ints) at the start of the workspace
constexpr int kCntAll = 0;        // XCDs all of whose workgroups have finished
constexpr int kCntXcd = 32;       // + 32 x (a cache line of its own): workgroups of XCD x that have finished, plus
constexpr int kGaveUp = 1 << 16;  // this much for every owner on XCD x that gave up (its piece mailboxes may hold pieces nobody took)

int g_spin_limit = 1 << 22;
int g_local_override = -1;
constexpr int kMaxDevices = 64;
int g_local[kMaxDevices];  // per device: is workgroup b placed on XCD b % 8?  0 not probed yet (treated as no), 1 yes, -1 no

// tuning constants (overridable at compile time for experiments)
#ifndef ELORA_DEC_AHEAD
#define ELORA_DEC_AHEAD 4  // sub-spans of K (128 elements) a workgroup keeps in flight with up to 32 rows of x: 2 or 4
#endif
#ifndef ELORA_DEC_TARGET_WGS
#define ELORA_DEC_TARGET_WGS 512  // workgroups aimed at: two per compute unit, if that many fit
#endif

// Optional phase timestamps for tuning (compiled in only with -DELORA_TRACE): slot i of workgroup b.  The stamps are
// kept in registers and written out when the workgroup is done, so that taking them adds no memory operations.
#ifdef ELORA_TRACE
__device__ long long elora_trace_buf[4096 * 16];
#define TRACE_DECL long long trace_t[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}
#define TRACE(i) trace_t[i] = wall_clock64()
#define TRACE_DUMP                                                                                   \
    do {                                                                                             \
        if (threadIdx.x == 0 && blockIdx.x < 4096)                                                   \
            for (int i_ = 0; i_ < 16; ++i_) elora_trace_buf[blockIdx.x * 16 + i_] = trace_t[i_];     \
    } while (0)
#else
#define TRACE_DECL do {} while (0)
#define TRACE(i) do {} while (0)
#define TRACE_DUMP do {} while (0)
#endif

struct DecodeShape {
    int T, K, N;
    int split;      // K-slices of the base contraction = owners per tile: 1, 2, 4 or 8
    int lgS;        // log2 split
    int chunks;     // K / 256; slice ks covers chunks [ks * chunks / split, (ks + 1) * chunks / split)
    int n_tiles;
    int total;      // n_tiles * split (tile, ks) pairs
    int grid;       // workgroups launched, a multiple of 8 * split, at least `total`: the surplus only shares in the shrink
    int real_per_xcd;  // workgroups per XCD that have a (tile, ks) pair: total / 8 rounded up to a multiple of split
    int n_pub;      // the first n_pub workgroups of the grid share the shrink units
    int jgroups;    // pairs of rank rows per row of x: ceil(max_rank / 2)
    unsigned jg_inv;  // floor(2^32 / jgroups) + 1: u / jgroups == (u * jg_inv) >> 32 for every u below 2^24 (jgroups <= 128)
    int G;          // granules per owner: 16 / split
    int lgG;        // log2 G
    int lgRp;       // log2 of max_rank rounded up to a power of two
    int spin_limit;
    int zero;       // 0
    int local;      // 1: workgroup b runs on XCD b % 8 (checked once per device), so a tile's workgroups share an L2
};

// ---- mailbox accesses (agent scope: past the per-XCD L2) -----------------------------------------
__device__ __forceinline__ void mb_store_f32(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ uint32_t mb_load_u32(const float *p)
{
    return __hip_atomic_load(reinterpret_cast<const uint32_t *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// immediate of s_waitcnt for "at most n vector-memory operations outstanding" (other counters: no wait)
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 15) | 0x0F70 | ((n >> 4) << 14); }

// Piece mailboxes are written and read by workgroups of one tile, which share an XCD, so the XCD's L2 is where they
// meet.  Stores are write-through all the way to memory (agent scope: nothing is left for the cache write-back at
// the end of the kernel) and leave the line in the L2; reads are plain loads the first time (nothing of these lines
// can be in the first-level cache yet) and atomic read-modify-writes (OR with zero) when they have to be repeated:
// those always execute in the L2, so they can neither see a stale first-level line nor have to go out to memory.
// (one 16-byte store per lane, so that a wave writes whole cache lines: written through in 8-byte halves the same data
// costs four times the memory traffic)
// The wait states after the store are part of the statement: the hardware reads the data registers of a store of more
// than 8 bytes a little after it is issued, the compiler inserts the idle cycles this needs only for stores it knows
// of, and what follows an assembly statement may well overwrite its operands at once.
__device__ __forceinline__ void piece_store(float *p, float a, float b, float c, float d)
{
    const u32x4 v = {__float_as_uint(a), __float_as_uint(b), __float_as_uint(c), __float_as_uint(d)};
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void piece_clear(float *p)
{
    const u32x4 v = {kEmpty, kEmpty, kEmpty, kEmpty};
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2" ::"v"(p), "v"(v) : "memory");
}
// `zero` is 0, but only the host knows (the compiler would turn an OR with a literal zero into a plain load).
// Without the one-XCD guarantee the read-modify-write is done at agent scope (past the L2, in memory).
__device__ __forceinline__ u32x4 piece_load(const float *p, uint64_t zero, bool local)
{
    uint64_t *q = reinterpret_cast<uint64_t *>(const_cast<float *>(p));
    uint64_t lo, hi;
    if (local) {
        lo = __hip_atomic_fetch_or(q, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        hi = __hip_atomic_fetch_or(q + 1, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    } else {
        lo = __hip_atomic_fetch_or(q, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        hi = __hip_atomic_fetch_or(q + 1, zero, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return u32x4{(uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32)};
}

// LDS reads the compiler does not see as such.  While direct-to-LDS loads are in flight it holds EVERY LDS read back
// until all of them have landed (it cannot tell what they overwrite), which would stall whatever reads LDS between the
// first requests of the stream and the stream's own loop.  These reads wait for nothing but themselves.
__device__ __forceinline__ int lds_read_i32(const int *p)
{
    int v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p) : "memory");
    return v;
}
__device__ __forceinline__ float lds_read_f32(const float *p)
{
    float v;
    asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p) : "memory");
    return v;
}

// LDS writes the compiler does not see as such, for the same reason (it holds a write back, too)
__device__ __forceinline__ void lds_write_b32(void *p, uint32_t v)
{
    asm volatile("ds_write_b32 %0, %1" ::"v"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)p), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_write_b128(void *p, u32x4 v)
{
    asm volatile("ds_write_b128 %0, %1\n\ts_nop 2" ::"v"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)p), "v"(v) : "memory");
}
__device__ __forceinline__ u32x4 lds_read_b128(const void *p)
{
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void *)p) : "memory");
    return v;
}

// piece (tile, owner, sender): [T][G][4] floats
__device__ __forceinline__ size_t piece_floats(const DecodeShape &sh) { return (size_t)sh.T * sh.G * 4; }
__device__ __forceinline__ float *piece_ptr(float *mail, const DecodeShape &sh, int tile, int owner, int sender)
{
    return mail + ((size_t)(tile * sh.split + owner) * sh.split + sender) * piece_floats(sh);
}

// Columns [nc0, nc0 + ncols) of y for all rows, from the inputs alone (after a wait ran out): slow, exact.
__device__ void recompute_columns(const DecodeShape &sh, const uint16_t *__restrict__ x, const uint16_t *__restrict__ W,
                                  const PoolView &pool, const RouteView &route, int has_pool, uint16_t *__restrict__ y,
                                  int nc0, int ncols, int wave, int lane)
{
    const int T = sh.T, K = sh.K, N = sh.N;
    for (int t = wave; t < T; t += kWaves) {
        RowRoute rr{-1, 0, 0.0f};
        if (has_pool) rr = resolve_row(t, route, pool, false);
        const uint16_t *xt = x + (size_t)t * K;
        float d = 0.0f;  // lane c: adapter term of column nc0 + c
        if (rr.slot >= 0) {
            const uint16_t *A = reinterpret_cast<const uint16_t *>(slot_A(pool, rr.slot));
            const uint16_t *B = reinterpret_cast<const uint16_t *>(slot_B(pool, rr.slot));
            for (int j0 = 0; j0 < rr.rank; j0 += 2) {
                const bool two = (j0 + 1) < rr.rank;
                float r0, r1;
                shrink_pair(A + (size_t)j0 * K, A + (size_t)(two ? j0 + 1 : j0) * K, xt, K, lane, r0, r1);
                if (lane < ncols && nc0 + lane < N) {
                    const uint16_t *Bn = B + (size_t)(nc0 + lane) * rr.rank;
                    d = fmaf(bf16_to_f32(Bn[j0]), r0, d);
                    if (two) d = fmaf(bf16_to_f32(Bn[j0 + 1]), r1, d);
                }
            }
        }
        for (int c = 0; c < ncols && nc0 + c < N; ++c) {
            const uint16_t *wn = W + (size_t)(nc0 + c) * K;
            float s = 0.0f;
            for (int k = lane * 8; k < K; k += 64 * 8) {
                const u32x4 wv = *reinterpret_cast<const u32x4 *>(wn + k), xv = *reinterpret_cast<const u32x4 *>(xt + k);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    s = fmaf(__uint_as_float(wv[q] << 16), __uint_as_float(xv[q] << 16), s);
                    s = fmaf(__uint_as_float(wv[q] & 0xffff0000u), __uint_as_float(xv[q] & 0xffff0000u), s);
                }
            }
            for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
            const float dc = __shfl(d, c);
            if (lane == 0) y[(size_t)t * N + nc0 + c] = f32_to_bf16(s + rr.scale * dc);
        }
    }
}

template <int TT, bool kWLds>
__global__ __launch_bounds__(kThreads, 2) void decode_kernel(DecodeShape sh, const uint16_t *__restrict__ x,
                                                                           const uint16_t *__restrict__ W, PoolView pool,
                                                                           RouteView route, int has_pool, float *__restrict__ mail,
                                                                           float *__restrict__ vmail, int *__restrict__ sync,
                                                                           uint16_t *__restrict__ y)
{
    // x ring during the contraction; staging of pieces, v and d afterwards
    extern __shared__ __attribute__((aligned(16))) uint16_t xs[];  // ring_bytes(TT, kWLds)
    __shared__ int s_slot[kDecodeMaxTokens], s_rank[kDecodeMaxTokens];
    __shared__ float s_scale[kDecodeMaxTokens];
    __shared__ int s_flag, s_fail, s_vfail, s_odd;
    __shared__ float s_red[2][kWaves][2];
    __shared__ __attribute__((aligned(16))) SlotMeta s_meta[kMetaLds];  // the pool's slot table, if it is small enough

    // Every argument is wanted within the first few hundred instructions.  Left alone the compiler fetches each one
    // where it is first used, one round trip to the scalar cache after the other; named here, they are all asked for
    // at once.
    asm volatile("" ::"s"(sh.T), "s"(sh.K), "s"(sh.N), "s"(sh.split), "s"(sh.lgS), "s"(sh.chunks), "s"(sh.n_tiles), "s"(sh.total),
                 "s"(sh.grid), "s"(sh.real_per_xcd), "s"(sh.n_pub), "s"(sh.jgroups), "s"(sh.jg_inv), "s"(sh.G), "s"(sh.lgG), "s"(sh.lgRp), "s"(sh.spin_limit),
                 "s"(sh.zero), "s"(sh.local), "s"(x), "s"(W), "s"(y), "s"(mail), "s"(vmail), "s"(sync), "s"(has_pool));
    asm volatile("" ::"s"(pool.meta), "s"(pool.slots), "s"(pool.err), "s"(pool.slot_bytes), "s"(pool.b_offset), "s"(pool.capacity),
                 "s"(pool.max_rank), "s"(route.adapter_idx), "s"(route.seg_offsets), "s"(route.seg_adapter), "s"(route.n_segments),
                 "s"(route.scales));
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T = sh.T, K = sh.K, N = sh.N;
    const int R = pool.max_rank;
    float *const lds_f = reinterpret_cast<float *>(&xs[0]);
    constexpr int kLdsFloats = ring_bytes(TT, kWLds) / 4;  // the area counted in floats
    TRACE_DECL;
    TRACE(0);
    if (tid == 0) {
        s_fail = 0;
        s_vfail = 0;
        s_odd = 0;
    }

    // Workgroup b runs on XCD b % 8.  The (tile, ks) pairs are numbered tile-major and every XCD takes a contiguous
    // eighth of them (a multiple of `split`), so the workgroups that exchange pieces share an XCD: they start together.
    // (real_per_xcd of an XCD's workgroups, a multiple of `split`, have a pair; the others are surplus on every XCD alike)
    const int per_xcd = sh.grid / kXcds;
    const int pair = (int)(blockIdx.x % kXcds) * sh.real_per_xcd + (int)(blockIdx.x / kXcds);
    const bool idle = (int)(blockIdx.x / kXcds) >= sh.real_per_xcd || pair >= sh.total;  // surplus workgroup: only shares in the shrink
    const int tile = idle ? 0 : pair >> sh.lgS, ks = idle ? 0 : pair & (sh.split - 1);

    // Finishing is counted per XCD and then over the XCDs.  The last workgroup of an XCD empties, if some owner there
    // gave up, the piece mailboxes of the XCD's tiles (through the same L2 the pieces went through); the last
    // workgroup of the call empties the v mailbox (everybody has read what it needed).  Counters and flags go back
    // to zero.  Everything this workgroup posted has been acknowledged before it counts itself.
    auto finish_call = [&]() {
        const int xcd = blockIdx.x % kXcds;
        if (tid == 0) {
            int flag = 0;
            // (counted in the XCD's own L2 when every workgroup that touches this counter is known to run on this XCD)
            const int before = sh.local ? __hip_atomic_fetch_add(&sync[kCntXcd + 32 * xcd], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)
                                        : __hip_atomic_fetch_add(&sync[kCntXcd + 32 * xcd], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((before & (kGaveUp - 1)) == per_xcd - 1) {
                if (sh.local) __hip_atomic_store(&sync[kCntXcd + 32 * xcd], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                else __hip_atomic_store(&sync[kCntXcd + 32 * xcd], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (before >= kGaveUp) flag |= 2;
                if (atomicAdd(&sync[kCntAll], 1) == kXcds - 1) {
                    __hip_atomic_store(&sync[kCntAll], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    flag |= 1;
                }
            }
            s_flag = flag;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if ((s_flag & 1) && has_pool)
            for (int e = tid; e < T * R; e += kThreads) mb_store_f32(&vmail[e], __uint_as_float(kEmpty));
        if (s_flag & 2) {
            // pairs xcd * real_per_xcd .. + real_per_xcd - 1 (those below `total`): split pieces each
            const int p0 = xcd * sh.real_per_xcd, p1 = min(p0 + sh.real_per_xcd, sh.total);
            float *base = mail + (size_t)p0 * sh.split * piece_floats(sh);
            const size_t n = p1 > p0 ? (size_t)(p1 - p0) * sh.split * piece_floats(sh) : 0;
            for (size_t e = (size_t)tid * 4; e < n; e += (size_t)kThreads * 4) piece_clear(base + e);
        }
        TRACE(14);
        TRACE_DUMP;
    };

    // ---- set-up of the base contraction (its first loads go out in the middle of phase 1) ----------------------
    const int m = lane & 15, g = lane >> 4;
    const int n0 = tile * kTileRows;
    const int row = n0 + wave * kRowsPerWave + m;                    // W row this lane feeds
    const bool wave_active = !idle && (n0 + wave * kRowsPerWave) < N;  // N % 16 == 0: all 16 rows in or out
    const int c_begin = (ks * sh.chunks) >> sh.lgS;
    const int nchunks = (((ks + 1) * sh.chunks) >> sh.lgS) - c_begin;  // >= 1: split <= chunks
    const int k_begin = c_begin * kChunk;
    const uint16_t *wrow = W + (size_t)(wave_active ? row : 0) * K + k_begin + g * 8;

    // The K-slice goes by in sub-spans of 128 elements (4 MFMA K steps).  Per sub-span every wave moves its share of
    // the rows of x global -> LDS, and its own 16 rows of W either the same way (kWLds: four instructions of 4 rows x
    // 256 bytes, whole cache lines; fetched straight into the registers in the layout the matrix instruction wants,
    // an instruction touches 16 rows x 64 bytes, half a cache line each, and the same stream takes about 1.7 us longer
    // per 32 MiB) or as 4 register loads per thread (more than 32 rows of x and a shape that wants two workgroups per
    // compute unit, for which the ring with W in it leaves no room).  kAhead sub-spans are on their way at any time.
    constexpr int kSub = kSubSpan, kSubSteps = kSub / 32;
    constexpr int kBufs = ring_slots(TT);                  // the sub-spans in flight and the one being multiplied
    constexpr int kAhead = kBufs - 1;                      // sub-spans in flight while one is being multiplied
    constexpr int kSlotElems = slot_rows(TT, kWLds) * kSub;
    static_assert(ELORA_DEC_AHEAD == 4, "ring depth for up to 32 rows");
    constexpr int kRowsPerInstr = 512 / kSub;              // a direct-to-LDS instruction moves 1 KiB: 4 rows of 128 elements
    constexpr int kLanesPerRow = 64 / kRowsPerInstr;
    constexpr int kXInstr = TT * 16 / kRowsPerInstr / kWaves;  // such instructions per wave and sub-span
    constexpr int kOps = kXInstr + kSubSteps;                  // vector-memory operations per wave and sub-span
    static_assert(kAhead == 2 || kAhead == 4, "ring depth");
    static_assert(kAhead * kOps + 8 < 64, "vmcnt range");
    u32x4 wset[kAhead][kSubSteps];
    typedef const __attribute__((address_space(1))) void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;
    uint16_t *const xring = &xs[0];  // [kBufs][rows of x, then rows of W][kSub / 8 places of 8 elements]; place = chunk ^ (row % 16)
    const int nsub = nchunks * (kChunk / kSub);  // even, at least 2

    // x first, then W: when the wave's W loads of a sub-span are back, so is its share of x (in-order counter).
    // Rows past the batch repeat the last row, and waves whose 16 rows of W lie past d_out load row 0: what they
    // produce is never posted, but every wave issues the same number of operations.
    // (W through LDS) instruction i of a wave moves rows wave * 16 + 4 i .. + 3 of the tile: lane = (row, place)
    const uint16_t *wdma[kSubSteps];
#pragma unroll
    for (int i = 0; i < kSubSteps; ++i) {
        const int r = i * kRowsPerInstr + lane / kLanesPerRow;  // row among the wave's 16
        const int chunk = (lane % kLanesPerRow) ^ r;
        wdma[i] = W + (size_t)min(n0 + wave * kRowsPerWave + r, N - 1) * K + k_begin + chunk * 8;
    }
    auto issue = [&](int p, u32x4 *dst) {
        uint16_t *buf = xring + (size_t)(p % kBufs) * kSlotElems;
#pragma unroll
        for (int i = 0; i < kXInstr; ++i) {
            const int r = (wave * kXInstr + i) * kRowsPerInstr + lane / kLanesPerRow;
            const int chunk = (lane % kLanesPerRow) ^ (r & 15);
            const uint16_t *src = x + (size_t)min(r, T - 1) * K + k_begin + (size_t)p * kSub + chunk * 8;
            __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(buf + (wave * kXInstr + i) * 512), 16, 0, 0);
        }
        if constexpr (kWLds) {
#pragma unroll
            for (int i = 0; i < kSubSteps; ++i)
                __builtin_amdgcn_global_load_lds((gptr_t)(wdma[i] + (size_t)p * kSub),
                                                 (lptr_t)(buf + (TT * 16 + wave * kRowsPerWave + i * kRowsPerInstr) * kSub), 16, 0, 0);
        } else {
            const uint16_t *pw = wrow + (size_t)p * kSub;
#pragma unroll
            for (int j = 0; j < kSubSteps; ++j) dst[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(pw + j * 32));
        }
    };

    floatx4 acc[TT];
#pragma unroll
    for (int i = 0; i < TT; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};

    // wait until at most `later` sub-spans are still on their way, meet the other waves (their shares of x for
    // sub-span p are in LDS then, and everybody is done with sub-span p - 1), multiply
    // wait until at most `later` younger sub-spans are still on their way, then meet the other waves: their shares of x
    // for the oldest sub-span are in LDS then, and everybody is done with the one before it
    auto meet = [&]() {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    auto arrive = [&](int later) {
        if (later >= 3) __builtin_amdgcn_s_waitcnt(vmcnt_imm(3 * kOps));
        else if (later == 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * kOps));
        else if (later == 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(1 * kOps));
        else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        meet();
    };
    auto multiply = [&](int p, const u32x4 *wc) {
        // The LDS reads are written as assembly: the compiler holds every LDS read back until ALL direct-to-LDS
        // loads in flight have landed (it cannot tell the ring's buffers apart), which would undo the prefetch.  All
        // reads of a sub-span and the wait for them sit in ONE statement: the compiler takes an output of an assembly
        // statement for valid as soon as the statement is over, and may copy or spill it right there.
        const uint32_t base = (uint32_t)(uintptr_t)(lptr_t)(xring + (size_t)(p % kBufs) * kSlotElems) + (uint32_t)m * (kSub * 2);
        static_assert(kSubSteps == 4 && kSub * 2 * 16 == 4096, "operand lists below");
        const uint32_t a0 = base + (uint32_t)(((0 * 4 + g) ^ m) << 4), a1 = base + (uint32_t)(((1 * 4 + g) ^ m) << 4);
        const uint32_t a2 = base + (uint32_t)(((2 * 4 + g) ^ m) << 4), a3 = base + (uint32_t)(((3 * 4 + g) ^ m) << 4);
        // (W through LDS) the wave's row m of W sits TT * 16 + wave * 16 rows below row m of x, in the same places
        const uint32_t wofs = (uint32_t)((TT * 16 + wave * kRowsPerWave) * kSub * 2);
        u32x4 b[kSubSteps][TT];
        u32x4 aw[kSubSteps];
        if constexpr (TT == 1) {
            asm volatile("ds_read_b128 %0, %12\n\tds_read_b128 %1, %13\n\tds_read_b128 %2, %14\n\tds_read_b128 %3, %15\n\t"
                         "ds_read_b128 %4, %8\n\tds_read_b128 %5, %9\n\tds_read_b128 %6, %10\n\tds_read_b128 %7, %11\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(aw[0]), "=&v"(aw[1]), "=&v"(aw[2]), "=&v"(aw[3]), "=&v"(b[0][0]), "=&v"(b[1][0]), "=&v"(b[2][0]), "=&v"(b[3][0])
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(a0 + wofs), "v"(a1 + wofs), "v"(a2 + wofs), "v"(a3 + wofs)
                         : "memory");
        } else if constexpr (TT == 2) {
            asm volatile("ds_read_b128 %0, %16\n\tds_read_b128 %1, %17\n\tds_read_b128 %2, %18\n\tds_read_b128 %3, %19\n\t"
                         "ds_read_b128 %4, %12\n\tds_read_b128 %5, %12 offset:4096\n\t"
                         "ds_read_b128 %6, %13\n\tds_read_b128 %7, %13 offset:4096\n\t"
                         "ds_read_b128 %8, %14\n\tds_read_b128 %9, %14 offset:4096\n\t"
                         "ds_read_b128 %10, %15\n\tds_read_b128 %11, %15 offset:4096\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(aw[0]), "=&v"(aw[1]), "=&v"(aw[2]), "=&v"(aw[3]), "=&v"(b[0][0]), "=&v"(b[0][1]), "=&v"(b[1][0]), "=&v"(b[1][1]),
                           "=&v"(b[2][0]), "=&v"(b[2][1]), "=&v"(b[3][0]), "=&v"(b[3][1])
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(a0 + wofs), "v"(a1 + wofs), "v"(a2 + wofs), "v"(a3 + wofs)
                         : "memory");
        } else if constexpr (TT == 3 && kWLds) {
            asm volatile("ds_read_b128 %0, %20\n\tds_read_b128 %1, %21\n\tds_read_b128 %2, %22\n\tds_read_b128 %3, %23\n\t"
                         "ds_read_b128 %4, %16\n\tds_read_b128 %5, %16 offset:4096\n\tds_read_b128 %6, %16 offset:8192\n\t"
                         "ds_read_b128 %7, %17\n\tds_read_b128 %8, %17 offset:4096\n\tds_read_b128 %9, %17 offset:8192\n\t"
                         "ds_read_b128 %10, %18\n\tds_read_b128 %11, %18 offset:4096\n\tds_read_b128 %12, %18 offset:8192\n\t"
                         "ds_read_b128 %13, %19\n\tds_read_b128 %14, %19 offset:4096\n\tds_read_b128 %15, %19 offset:8192\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(aw[0]), "=&v"(aw[1]), "=&v"(aw[2]), "=&v"(aw[3]), "=&v"(b[0][0]), "=&v"(b[0][1]), "=&v"(b[0][2]), "=&v"(b[1][0]),
                           "=&v"(b[1][1]), "=&v"(b[1][2]), "=&v"(b[2][0]), "=&v"(b[2][1]), "=&v"(b[2][2]), "=&v"(b[3][0]), "=&v"(b[3][1]),
                           "=&v"(b[3][2])
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(a0 + wofs), "v"(a1 + wofs), "v"(a2 + wofs), "v"(a3 + wofs)
                         : "memory");
        } else if constexpr (TT == 4 && kWLds) {
            asm volatile("ds_read_b128 %0, %24\n\tds_read_b128 %1, %25\n\tds_read_b128 %2, %26\n\tds_read_b128 %3, %27\n\t"
                         "ds_read_b128 %4, %20\n\tds_read_b128 %5, %20 offset:4096\n\tds_read_b128 %6, %20 offset:8192\n\tds_read_b128 %7, %20 offset:12288\n\t"
                         "ds_read_b128 %8, %21\n\tds_read_b128 %9, %21 offset:4096\n\tds_read_b128 %10, %21 offset:8192\n\tds_read_b128 %11, %21 offset:12288\n\t"
                         "ds_read_b128 %12, %22\n\tds_read_b128 %13, %22 offset:4096\n\tds_read_b128 %14, %22 offset:8192\n\tds_read_b128 %15, %22 offset:12288\n\t"
                         "ds_read_b128 %16, %23\n\tds_read_b128 %17, %23 offset:4096\n\tds_read_b128 %18, %23 offset:8192\n\tds_read_b128 %19, %23 offset:12288\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(aw[0]), "=&v"(aw[1]), "=&v"(aw[2]), "=&v"(aw[3]), "=&v"(b[0][0]), "=&v"(b[0][1]), "=&v"(b[0][2]), "=&v"(b[0][3]),
                           "=&v"(b[1][0]), "=&v"(b[1][1]), "=&v"(b[1][2]), "=&v"(b[1][3]), "=&v"(b[2][0]), "=&v"(b[2][1]), "=&v"(b[2][2]),
                           "=&v"(b[2][3]), "=&v"(b[3][0]), "=&v"(b[3][1]), "=&v"(b[3][2]), "=&v"(b[3][3])
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "v"(a0 + wofs), "v"(a1 + wofs), "v"(a2 + wofs), "v"(a3 + wofs)
                         : "memory");
        } else if constexpr (TT == 3) {
            asm volatile("ds_read_b128 %0, %12\n\tds_read_b128 %1, %12 offset:4096\n\tds_read_b128 %2, %12 offset:8192\n\t"
                         "ds_read_b128 %3, %13\n\tds_read_b128 %4, %13 offset:4096\n\tds_read_b128 %5, %13 offset:8192\n\t"
                         "ds_read_b128 %6, %14\n\tds_read_b128 %7, %14 offset:4096\n\tds_read_b128 %8, %14 offset:8192\n\t"
                         "ds_read_b128 %9, %15\n\tds_read_b128 %10, %15 offset:4096\n\tds_read_b128 %11, %15 offset:8192\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(b[0][0]), "=&v"(b[0][1]), "=&v"(b[0][2]), "=&v"(b[1][0]), "=&v"(b[1][1]), "=&v"(b[1][2]), "=&v"(b[2][0]),
                           "=&v"(b[2][1]), "=&v"(b[2][2]), "=&v"(b[3][0]), "=&v"(b[3][1]), "=&v"(b[3][2])
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
                         : "memory");
        } else {
            static_assert(TT == 4, "operand lists");
            asm volatile("ds_read_b128 %0, %16\n\tds_read_b128 %1, %16 offset:4096\n\tds_read_b128 %2, %16 offset:8192\n\tds_read_b128 %3, %16 offset:12288\n\t"
                         "ds_read_b128 %4, %17\n\tds_read_b128 %5, %17 offset:4096\n\tds_read_b128 %6, %17 offset:8192\n\tds_read_b128 %7, %17 offset:12288\n\t"
                         "ds_read_b128 %8, %18\n\tds_read_b128 %9, %18 offset:4096\n\tds_read_b128 %10, %18 offset:8192\n\tds_read_b128 %11, %18 offset:12288\n\t"
                         "ds_read_b128 %12, %19\n\tds_read_b128 %13, %19 offset:4096\n\tds_read_b128 %14, %19 offset:8192\n\tds_read_b128 %15, %19 offset:12288\n\t"
                         "s_waitcnt lgkmcnt(0)"
                         : "=&v"(b[0][0]), "=&v"(b[0][1]), "=&v"(b[0][2]), "=&v"(b[0][3]), "=&v"(b[1][0]), "=&v"(b[1][1]), "=&v"(b[1][2]),
                           "=&v"(b[1][3]), "=&v"(b[2][0]), "=&v"(b[2][1]), "=&v"(b[2][2]), "=&v"(b[2][3]), "=&v"(b[3][0]), "=&v"(b[3][1]),
                           "=&v"(b[3][2]), "=&v"(b[3][3])
                         : "v"(a0), "v"(a1), "v"(a2), "v"(a3)
                         : "memory");
        }
#pragma unroll
        for (int j = 0; j < kSubSteps; ++j) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, kWLds ? aw[j] : wc[j]);
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
                acc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, b[j][tt]), acc[tt], 0, 0, 0);
        }
    };

    // ---- phase 1: routes of all rows, and this workgroup's share of the shrink ---------------------------
    // A unit = (row t, rank rows j0 and j0 + 1) is worked on by the whole workgroup: thread = 16-byte pieces tid,
    // tid + 256, ... of the three rows involved (x_t and two rows of A_i), 1024 pieces (K = 4096 elements) a round.
    constexpr int UL = 2;  // pieces per thread and round (3 * UL = 6 loads: see first_issue_then_wait)
    const int pieces = K >> 3;
    auto unit_load = [&](const uint16_t *A0, const uint16_t *A1, const uint16_t *xt, int pb, u32x4 *xv, u32x4 *a0, u32x4 *a1) {
#pragma unroll
        for (int i = 0; i < UL; ++i) {
            const int pc = pb + i * kThreads + tid;
            const size_t off = (size_t)(pc < pieces ? pc : 0) * 8;  // past the row: some piece of it, dropped below
            xv[i] = *reinterpret_cast<const u32x4 *>(xt + off);
            a0[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(A0 + off));
            a1[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(A1 + off));
        }
    };
    auto unit_dot = [&](int pb, const u32x4 *xv, const u32x4 *a0, const u32x4 *a1, float &s0, float &s1) {
#pragma unroll
        for (int i = 0; i < UL; ++i) {
            const bool in = pb + i * kThreads + tid < pieces;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t xw = in ? xv[i][q] : 0u, aw0 = a0[i][q], aw1 = a1[i][q];
                s0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(elora_bf16x2, aw0), __builtin_bit_cast(elora_bf16x2, xw), s0, false);
                s1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(elora_bf16x2, aw1), __builtin_bit_cast(elora_bf16x2, xw), s1, false);
            }
        }
    };
    // the four waves' sums of one unit meet in LDS (two sets, used in turn: one barrier per unit); thread 0 posts v
    auto unit_finish = [&](int n, int t, int j0, bool valid, bool two, float s0, float s1) {
        s0 = wave_sum(s0);
        s1 = wave_sum(s1);
        if (lane == 0) {
            lds_write_b32(&s_red[n & 1][wave][0], __float_as_uint(s0));
            lds_write_b32(&s_red[n & 1][wave][1], __float_as_uint(s1));
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (tid == 0 && valid) {
            const float(*rd)[2] = s_red[n & 1];
            const float r0 = (lds_read_f32(&rd[0][0]) + lds_read_f32(&rd[1][0])) + (lds_read_f32(&rd[2][0]) + lds_read_f32(&rd[3][0]));
            const float r1 = (lds_read_f32(&rd[0][1]) + lds_read_f32(&rd[1][1])) + (lds_read_f32(&rd[2][1]) + lds_read_f32(&rd[3][1]));
            mb_store_f32(&vmail[(size_t)t * R + j0], r0);
            if (two) mb_store_f32(&vmail[(size_t)t * R + j0 + 1], r1);
        }
    };
    const int n_units = has_pool ? T * sh.jgroups : 0;
    // Units number n_first on of this workgroup (the routes are in LDS): one per wave at a time, 24 loads of 16 bytes per
    // lane in flight (a workgroup with many units has four of them under way instead of one after the other).
    auto units_from = [&](int n_first) {
        if ((int)blockIdx.x >= sh.n_pub) return;
        for (int n = n_first + wave;; n += kWaves) {
            const long long u = (long long)blockIdx.x + (long long)sh.n_pub * n;
            if (u >= n_units) break;
            const int t = sh.jgroups == 1 ? (int)u : (int)__umulhi((unsigned)u, sh.jg_inv), j0 = ((int)u - t * sh.jgroups) * 2;
            const int slot = lds_read_i32(&s_slot[t]), rank = lds_read_i32(&s_rank[t]);
            if (slot < 0 || j0 >= rank) continue;
            const bool two = (j0 + 1) < rank;
            const uint16_t *A0 = reinterpret_cast<const uint16_t *>(slot_A(pool, slot)) + (size_t)j0 * K;
            float r0, r1;
            shrink_pair(A0, two ? A0 + K : A0, x + (size_t)t * K, K, lane, r0, r1);
            if (lane == 0) {
                mb_store_f32(&vmail[(size_t)t * R + j0], r0);
                if (two) mb_store_f32(&vmail[(size_t)t * R + j0 + 1], r1);
            }
        }
    };
    if (idle) {
        if (has_pool) {
            if (tid < T) {
                const RowRoute rr = resolve_row(tid, route, pool, blockIdx.x == 0);
                s_slot[tid] = rr.slot;
                s_rank[tid] = rr.rank;
            }
            __syncthreads();
            units_from(0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // this workgroup's stores have been acknowledged
        __syncthreads();
        finish_call();
        return;
    }
    // A route takes two dependent loads: index, then the slot's table entry.  A small slot table is fetched whole
    // alongside the index, so that the second one is an LDS read.  (Left to itself that load comes back when most of the
    // stream's first requests have, and at very different times in different workgroups: those that have it start
    // streaming and are in the way of those that do not.)
    if (has_pool) {
        const int tr = min(tid, T - 1);  // threads past the batch repeat its last row and keep nothing
        const bool unit0 = (int)blockIdx.x < sh.n_pub && (int)blockIdx.x < n_units;
        const int t0 = !unit0 ? 0 : sh.jgroups == 1 ? (int)blockIdx.x : (int)__umulhi(blockIdx.x, sh.jg_inv), j00 = ((int)blockIdx.x - t0 * sh.jgroups) * 2;
        const bool table = pool.capacity <= kMetaLds;
        u32x4 tab[kMetaLds / kThreads];
        if (table) {
#pragma unroll
            for (int i = 0; i < kMetaLds / kThreads; ++i)
                if (tid + i * kThreads < pool.capacity) tab[i] = reinterpret_cast<const u32x4 *>(pool.meta)[tid + i * kThreads];
        }
        const RouteIndex ri = route_index(tr, route);
        const int idx_c = (ri.idx >= 0 && ri.idx < pool.capacity) ? ri.idx : 0;
        const float so = (route.scales != nullptr && ri.idx != -1) ? route.scales[ri.scale_at] : 0.0f;
        SlotMeta mt{0, 0.0f, 0, 0};
        if (!table) mt = pool.meta[idx_c];  // a big pool: the entry is fetched on its own, one more round trip
        // Index, scale and table (or entry) are here before the stream starts.  They are used below, after the stream's
        // first requests: without this the compiler would wait for them there, and for those requests with them; and
        // no load may sit in a branch from here on, or it waits for everything at the next join.
        asm volatile("" ::"v"(ri.idx), "v"(ri.scale_at), "v"(so), "v"(mt.rank), "v"(mt.scale), "v"(mt.loaded));
        if (table) {
#pragma unroll
            for (int i = 0; i < kMetaLds / kThreads; ++i) asm volatile("" ::"v"(tab[i]));
        }
        TRACE(11);  // index known
        // the first two sub-spans of the stream go out now; from here to the end of the contraction LDS is only read
        // through lds_read_* and the assembly in multiply()
        issue(0, wset[0]);
        issue(1, wset[1]);
        auto meet_lds = [&]() {  // LDS writes visible to the workgroup (no fence: that would wait for the stream, too)
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        };
        if (table) {
#pragma unroll
            for (int i = 0; i < kMetaLds / kThreads; ++i)
                if (tid + i * kThreads < pool.capacity) lds_write_b128(&s_meta[tid + i * kThreads], tab[i]);
            meet_lds();
            const u32x4 m4 = lds_read_b128(&s_meta[idx_c]);
            mt.rank = (int)m4[0];
            mt.scale = __uint_as_float(m4[1]);
            mt.loaded = (int)m4[2];
            mt.pad = 0;
        }
        const RowRoute rr = route_finish(tr, ri, mt, so, route, pool, blockIdx.x == 0 && tid < T);
        TRACE(12);  // table entry here
        if (tid < T) {
            lds_write_b32(&s_slot[tid], (uint32_t)rr.slot);
            lds_write_b32(&s_rank[tid], (uint32_t)rr.rank);
            lds_write_b32(&s_scale[tid], __float_as_uint(rr.scale));
            if (rr.rank & 7) lds_write_b32(&s_odd, 1u);  // rows of this B_i are not 16-byte aligned
        }
        meet_lds();
        TRACE(13);  // routes in LDS
        // The workgroup's first shrink unit and the next sub-spans of the stream go out together.  (One straight-line
        // copy of this per case: across a branch the compiler stops counting loads in flight and waits for all of them.)
        // (made uniform for the compiler: otherwise the cases below become predicated code one after the other, and each
        // waits for the loads the one before it might have issued)
        const int slot0 = __builtin_amdgcn_readfirstlane(lds_read_i32(&s_slot[t0])), rank0 = __builtin_amdgcn_readfirstlane(lds_read_i32(&s_rank[t0]));
        const bool valid0 = unit0 && slot0 >= 0 && j00 < rank0, two0 = (j00 + 1) < rank0;
        auto first_requests = [&](auto four, auto with_unit) {
            constexpr int n_first = decltype(four)::value ? 4 : 2;
            u32x4 uxv[UL], ua0[UL], ua1[UL];
            const uint16_t *uA0 = nullptr, *uA1 = nullptr;
            if constexpr (decltype(with_unit)::value) {
                uA0 = reinterpret_cast<const uint16_t *>(slot_A(pool, slot0)) + (size_t)j00 * K;
                uA1 = two0 ? uA0 + K : uA0;
                unit_load(uA0, uA1, x + (size_t)t0 * K, 0, uxv, ua0, ua1);
            }
#pragma unroll
            for (int p = 2; p < n_first; ++p) issue(p, wset[p % kAhead]);
            if constexpr (decltype(with_unit)::value) {
                float s0 = 0.0f, s1 = 0.0f;
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm((n_first - 2) * kOps));  // the unit's loads are back
                __builtin_amdgcn_sched_barrier(0);
                unit_dot(0, uxv, ua0, ua1, s0, s1);
                for (int pb = UL * kThreads; pb < pieces; pb += UL * kThreads) {  // K above 4096: the other rounds
                    u32x4 xv[UL], a0[UL], a1[UL];
                    unit_load(uA0, uA1, x + (size_t)t0 * K, pb, xv, a0, a1);
                    unit_dot(pb, xv, a0, a1, s0, s1);
                }
                unit_finish(0, t0, j00, true, two0, s0, s1);
            }
        };
        const bool four = kAhead == 4 && nsub >= 4;
        if (valid0) {
            if (four) first_requests(std::true_type{}, std::true_type{});
            else first_requests(std::false_type{}, std::true_type{});
        } else {
            if (four) first_requests(std::true_type{}, std::false_type{});
            else first_requests(std::false_type{}, std::false_type{});
        }
        if (unit0) units_from(1);
        TRACE(1);
    } else {
        issue(0, wset[0]);
        issue(1, wset[1]);
        if (kAhead == 4 && nsub >= 4) {
            issue(2, wset[2 % kAhead]);
            issue(3, wset[3 % kAhead]);
        }
    }

    // own columns: granules og0 .. og0 + G - 1 of the tile, columns nc0 .. nc0 + 4 G - 1 of y
    const int og0 = ks * sh.G, nc0 = n0 + og0 * 4, ncols = sh.G * 4;
    const int n_cells = T * sh.G;  // (row, granule) cells of the owned columns
    // What follows the contraction runs on four waves with nothing to overlap it, and a wave on its own issues an
    // instruction only every 8 to 10 clocks: the number of instructions on that path is what the tail of the kernel
    // costs.  The common case (every rank a multiple of 8, none above 64) therefore has a short path of its own.
    const bool lean = !has_pool || (__builtin_amdgcn_readfirstlane(lds_read_i32(&s_odd)) == 0 && R <= 64 && sh.lgRp >= 3);
    const int lgRp = sh.lgRp, Rp = 1 << lgRp;  // pitch of v in LDS: max_rank rounded up to a power of two, 8 .. 64
    float *const vs = lds_f;                                     // [T][Rp]
    constexpr int VV = kDecodeMaxTokens * 64 / 4 / kThreads;     // 16-byte vectors of v per thread, at most
    const int nch = has_pool ? R >> 3 : 0;                       // 16-byte pieces of a row of B_i at the largest rank
    const int n_bit = has_pool ? T << (sh.lgG + 2) : 0;          // (row, own column) items
    u32x4 vv[VV];
    bool vneed[VV];
    u32x4 b[2][8];
    const float *vrow[2];
    bool valid[2];
    // rows of B_i for two items (it0, it0 + 256); pieces of a row past its rank repeat its last piece (v is zero there)
    auto b_issue = [&](int it0) {
#pragma unroll
        for (int ii = 0; ii < 2; ++ii) {
            const int item = it0 + ii * kThreads;
            const int t = item < n_bit ? item >> (sh.lgG + 2) : 0, c = item & (ncols - 1);
            const int slot = s_slot[t], rank = s_rank[t];  // (plain LDS reads: nothing of the stream is in flight any more)
            valid[ii] = item < n_bit && slot >= 0 && nc0 + c < N;
            const uint16_t *bp = reinterpret_cast<const uint16_t *>(slot_B(pool, valid[ii] ? slot : 0)) +
                                 (valid[ii] ? (size_t)(nc0 + c) * rank : 0);
            const int last = valid[ii] ? rank - 8 : 0;
#pragma unroll
            for (int hh = 0; hh < 8; ++hh)
                if (hh < nch) b[ii][hh] = *reinterpret_cast<const u32x4 *>(bp + min(8 * hh, last));
            vrow[ii] = vs + (t << lgRp);
        }
    };
    // The adapter term's inputs.  v: through the L2 (the workgroups of an XCD all want the same values, and the L2 holds
    // nothing from before this launch); what is not there yet is asked for again, past the L2.  The rows of B_i for
    // this thread's first items go out with it: they only need the routes.  (Asking for all this before the last
    // sub-span of the stream is waited for, so that it travels meanwhile, was slower: the contraction then ends later.)
    auto tail_requests = [&]() {
#pragma unroll
        for (int i = 0; i < VV; ++i) {
            const int vi = tid + i * kThreads;
            const int t = vi >> (lgRp - 2), j = (vi & ((Rp >> 2) - 1)) * 4;
            vneed[i] = t < T && j < s_rank[min(t, T - 1)];
            vv[i] = u32x4{0, 0, 0, 0};
            if (vneed[i]) vv[i] = *reinterpret_cast<const u32x4 *>(vmail + (size_t)t * R + j);
        }
        b_issue(tid);
    };

    // ---- phase 2: base contraction -------------------------------------------------------------------------
    // kAhead sub-spans are in flight, no more: requests a compute unit has queued beyond what the memory system is
    // working on only delay whatever that unit asks for next, without adding bandwidth.  The steady-state loop is
    // straight-line code (the compiler then knows exactly which loads a register set is still waiting for).
    {
        int p = 0;
        if (nsub >= kAhead) {
            for (; p + 2 * kAhead <= nsub; p += kAhead) {
#pragma unroll
                for (int d = 0; d < kAhead; ++d) {
                    __builtin_amdgcn_s_waitcnt(vmcnt_imm((kAhead - 1) * kOps));
                    meet();
                    if (p == 0 && d == 0) TRACE(4);
                    multiply(p + d, wset[d]);
                    issue(p + d + kAhead, wset[d]);
                }
            }
        }
        // what is left: at most 2 kAhead - 1 sub-spans, the first kAhead of them (or all) already asked for
#pragma unroll
        for (int i = 0; i < 2 * kAhead - 1; ++i) {
            const int q = p + i;
            if (q < nsub) {
                arrive(min(kAhead - 1, nsub - 1 - q));
                multiply(q, wset[i % kAhead]);
                if (q + kAhead < nsub) issue(q + kAhead, wset[i % kAhead]);
            }
        }
    }
    TRACE(5);  // contraction done

    // ---- phase 3: post the pieces of this K-slice to their owners ---------------------------------------------
    // C layout of the 16x16 MFMA: lane holds column (lane % 16) = row t of x, rows (lane / 16) * 4 + 0..3 = W rows,
    // i.e. granule wave * 4 + g of the tile
    if (wave_active) {
        const int q16 = wave * 4 + g;
        float *dst0 = piece_ptr(mail, sh, tile, q16 >> sh.lgG, ks) + (size_t)(q16 & (sh.G - 1)) * 4;
        // (the stores below are assembly statements: the idle cycles a store needs between a matrix instruction writing a
        // register and the store reading it are not inserted for them)
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" ::: "memory");
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
            const int t = tt * 16 + m;
            if (t < T) piece_store(dst0 + (size_t)t * sh.G * 4, acc[tt][0], acc[tt][1], acc[tt][2], acc[tt][3]);
        }
    }

    bool acked = false;  // everything this thread posted to other workgroups has been acknowledged
    if (lean) {
        float *const dsum = lds_f + (has_pool ? (T << lgRp) : 0);    // [T][ncols]
        const size_t pstride = piece_floats(sh);
        u32x4 pv[kDecodeMaxSplit];
        // the pieces of one (row, granule) cell: plain loads
        auto p_issue = [&](int cell) {
            const float *src0 = piece_ptr(mail, sh, tile, ks, 0) + (size_t)cell * 4;
#pragma unroll
            for (int sd = 0; sd < kDecodeMaxSplit; ++sd)
                if (sd < sh.split) pv[sd] = *reinterpret_cast<const u32x4 *>(src0 + sd * pstride);
        };
        if (has_pool) tail_requests();
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();  // the x ring is reused below (no fence: the requests above stay in flight)
        asm volatile("" ::: "memory");
        TRACE(8);
        if (has_pool) {
            bool gave_up = sh.spin_limit == 0;
            for (int spin = 0; !gave_up; ++spin) {
                bool all = true;
#pragma unroll
                for (int i = 0; i < VV; ++i)
                    all = all && !(vneed[i] && (vv[i][0] == kEmpty || vv[i][1] == kEmpty || vv[i][2] == kEmpty || vv[i][3] == kEmpty));
                if (all) break;
                if (spin >= sh.spin_limit) {
                    gave_up = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(2);
#pragma unroll
                for (int i = 0; i < VV; ++i) {
                    const int vi = tid + i * kThreads;
                    const float *src = vmail + (size_t)(vi >> (lgRp - 2)) * R + (vi & ((Rp >> 2) - 1)) * 4;
                    if (vneed[i])
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (vv[i][u] == kEmpty) vv[i][u] = mb_load_u32(src + u);
                }
            }
#pragma unroll
            for (int i = 0; i < VV; ++i) {
                const int vi = tid + i * kThreads;
                if (vi < (T << (lgRp - 2))) *reinterpret_cast<u32x4 *>(vs + (size_t)vi * 4) = vv[i];  // zeros at and above the rank
            }
            if (gave_up) s_vfail = 1;
            TRACE(9);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (s_vfail) {
                // the shrink results did not arrive in time: compute v here
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
                        vs[(t << lgRp) + j0] = r0;
                        if (j0 + 1 < Rp) vs[(t << lgRp) + j0 + 1] = r1;
                    }
                }
                __syncthreads();
            }
            TRACE(10);
        }
        // With a pool: the pieces of this thread's first cell are asked for now (the other K-slices have had time to
        // arrive), and the loads are under way while the adapter term is formed.
        // Without one the other K-slices are mostly not done yet, and everybody polling every piece of its own with
        // read-modify-writes keeps the L2's atomic units busy for microseconds.  Then one lane per K-slice waits
        // (read-modify-writes in the L2) for the piece that slice posts last to this owner; once all are there, plain
        // loads find every piece in the L2.
        const bool use_probe = !has_pool;
        if (!use_probe) {
            if (tid < n_cells) p_issue(tid);
        } else {
            if (wave == 0 && lane < sh.split && nc0 < N) {
                const float *probe = piece_ptr(mail, sh, tile, ks, lane) + ((size_t)(T - 1) * sh.G + min(sh.G - 1, ((N - nc0) >> 2) - 1)) * 4;
                for (int spin = 0; spin < sh.spin_limit; ++spin) {
                    const u32x4 pr = piece_load(probe, (uint64_t)(uint32_t)sh.zero, sh.local != 0);
                    if (pr[0] != kEmpty && pr[1] != kEmpty && pr[2] != kEmpty && pr[3] != kEmpty) break;
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (tid < n_cells) p_issue(tid);
        }
        if (has_pool) {
            // d[t][c] = s_t * sum_j B_i[nc0 + c][j] v[t][j]: one (row, own column) item per thread, two items at a time
            for (int it0 = tid; it0 < n_bit; it0 += 2 * kThreads) {
                if (it0 != tid) b_issue(it0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ii = 0; ii < 2; ++ii) {
                    float d = 0.0f;
#pragma unroll
                    for (int hh = 0; hh < 8; ++hh) {
                        if (hh < nch) {
                            const floatx4 v0 = *reinterpret_cast<const floatx4 *>(vrow[ii] + 8 * hh);
                            const floatx4 v1 = *reinterpret_cast<const floatx4 *>(vrow[ii] + 8 * hh + 4);
                            d = fmaf(__uint_as_float(b[ii][hh][0] << 16), v0[0], d);
                            d = fmaf(__uint_as_float(b[ii][hh][0] & 0xffff0000u), v0[1], d);
                            d = fmaf(__uint_as_float(b[ii][hh][1] << 16), v0[2], d);
                            d = fmaf(__uint_as_float(b[ii][hh][1] & 0xffff0000u), v0[3], d);
                            d = fmaf(__uint_as_float(b[ii][hh][2] << 16), v1[0], d);
                            d = fmaf(__uint_as_float(b[ii][hh][2] & 0xffff0000u), v1[1], d);
                            d = fmaf(__uint_as_float(b[ii][hh][3] << 16), v1[2], d);
                            d = fmaf(__uint_as_float(b[ii][hh][3] & 0xffff0000u), v1[3], d);
                        }
                    }
                    const int item = it0 + ii * kThreads;
                    if (item < n_bit) dsum[item] = valid[ii] ? d * s_scale[item >> (sh.lgG + 2)] : 0.0f;
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        TRACE(2);  // adapter term formed
        // Everything this thread has posted so far (pieces, shrink results) is acknowledged once the piece loads that
        // are needed next are back; the workgroup can then count itself done right after its last stores, without
        // waiting for those.
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        acked = true;
        // every (row, granule) cell of the own columns: the piece of each K-slice (again through L2 atomics while one
        // is missing), added in fixed order, plus d, rounded once, stored at the row's own position
        for (int cell = tid; cell < n_cells; cell += kThreads) {
            const int t = cell >> sh.lgG, qo = cell & (sh.G - 1);
            const int n = nc0 + qo * 4;
            if (cell != tid) p_issue(cell);
            if (n >= N) continue;
            float *src0 = piece_ptr(mail, sh, tile, ks, 0) + (size_t)cell * 4;
            bool gave_up = sh.spin_limit == 0;
            for (int spin = 0; !gave_up; ++spin) {
                bool all = true;
#pragma unroll
                for (int sd = 0; sd < kDecodeMaxSplit; ++sd)
                    if (sd < sh.split) all = all && pv[sd][0] != kEmpty && pv[sd][1] != kEmpty && pv[sd][2] != kEmpty && pv[sd][3] != kEmpty;
                if (all) break;
                if (spin >= sh.spin_limit) {
                    gave_up = true;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
#pragma unroll
                for (int sd = 0; sd < kDecodeMaxSplit; ++sd)
                    if (sd < sh.split && (pv[sd][0] == kEmpty || pv[sd][1] == kEmpty || pv[sd][2] == kEmpty || pv[sd][3] == kEmpty)) {
                        pv[sd] = piece_load(src0 + sd * pstride, (uint64_t)(uint32_t)sh.zero, sh.local != 0);
                    }
            }
            if (gave_up) {
                s_fail = 1;
                continue;
            }
            floatx4 o = __builtin_bit_cast(floatx4, pv[0]);
#pragma unroll
            for (int sd = 1; sd < kDecodeMaxSplit; ++sd) {
                if (sd < sh.split) {
                    const floatx4 pc = __builtin_bit_cast(floatx4, pv[sd]);
                    o[0] += pc[0];
                    o[1] += pc[1];
                    o[2] += pc[2];
                    o[3] += pc[3];
                }
            }
            if (has_pool) {
                const floatx4 dd = *reinterpret_cast<const floatx4 *>(dsum + (size_t)cell * 4);
                o[0] += dd[0];
                o[1] += dd[1];
                o[2] += dd[2];
                o[3] += dd[3];
            }
            const uint64_t packed = (uint64_t)f32_to_bf16(o[0]) | ((uint64_t)f32_to_bf16(o[1]) << 16) |
                                    ((uint64_t)f32_to_bf16(o[2]) << 32) | ((uint64_t)f32_to_bf16(o[3]) << 48);
            *reinterpret_cast<uint64_t *>(y + (size_t)t * N + n) = packed;
#pragma unroll
            for (int sd = 0; sd < kDecodeMaxSplit; ++sd)
                if (sd < sh.split) piece_clear(src0 + sd * pstride);  // empty again for the next call
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        TRACE(6);
        if (s_fail) {
            // some piece did not arrive in time: this workgroup computes its columns from the inputs, and the pieces
            // that are still on their way are removed when the call ends
            if (tid == 0) {
            if (sh.local) __hip_atomic_fetch_add(&sync[kCntXcd + 32 * (blockIdx.x % kXcds)], kGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            else __hip_atomic_fetch_add(&sync[kCntXcd + 32 * (blockIdx.x % kXcds)], kGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
            recompute_columns(sh, x, W, pool, route, has_pool, y, nc0, ncols, wave, lane);
            acked = false;
        }
    } else {
    const int n_items = sh.split * n_cells;  // (sender, cell) = 16 T: at most four per thread
    // LDS: [pieces: n_items x 4][d: n_cells x 4][v of a block of rows: qb x R]
    float *const stage = lds_f, *const dsum = stage + (size_t)n_items * 4, *const vs = dsum + (size_t)n_cells * 4;
    const int qb_max = (kLdsFloats - (n_items + n_cells) * 4) / (has_pool ? R : 1);  // rows of v that fit: at least 8

    // Three hand-overs end here: the pieces of the other K-slices, v, and (plain loads) the rows of B_i.  All first
    // requests go out together, before anything is waited for.
    // (index spaces are laid out so that they come apart with shifts and divisions by constants: this part of the
    // kernel runs on four waves per workgroup with nothing to overlap it)
    constexpr int PB = TT, VB = 8, IB = 2;
    u32x4 pval[PB];
    bool pneed[PB];
    const float *psrc[PB];
    int pdst[PB];
#pragma unroll
    for (int u = 0; u < PB; ++u) {
        // item = (sender, row of the 16 TT, granule): TT * 256 items, TT per thread
        const int item = tid + u * kThreads;
        const int qo = item & (sh.G - 1), rs = item >> sh.lgG;
        const int sd = rs / (TT * 16), t = rs - sd * (TT * 16);
        const int cell = t * sh.G + qo;
        pneed[u] = t < T && nc0 + qo * 4 < N;
        psrc[u] = piece_ptr(mail, sh, tile, ks, sd) + (size_t)(pneed[u] ? cell : 0) * 4;
        pdst[u] = (sd * n_cells + cell) * 4;
    }
    auto p_load = [&]() {
#pragma unroll
        for (int u = 0; u < PB; ++u)
            if (pneed[u]) pval[u] = piece_load(psrc[u], (uint64_t)(uint32_t)sh.zero, sh.local != 0);
    };
    // v: element e of the block of rows q0 .. q0 + qb - 1 is (row q0 + (e >> lgRp), rank column e & (Rp - 1))
    const int Rp = 1 << sh.lgRp;
    auto v_load = [&](int q0, int qb, int e0, uint32_t *val, bool *need) {
#pragma unroll
        for (int i = 0; i < VB; ++i) {
            const int e = e0 + i * kThreads + tid;
            const int q = e >> sh.lgRp, j = e & (Rp - 1);
            need[i] = q < qb && j < s_rank[q0 + min(q, qb - 1)];
            // first through the L2 (the workgroups of an XCD all want the same values; the L2 holds nothing from before
            // this launch); a value that was not there yet is asked for again past the L2
            val[i] = need[i] ? reinterpret_cast<const uint32_t *>(vmail)[(size_t)(q0 + q) * R + j] : 0u;
        }
    };
    // B_i: item = (row q of the block, own column c); 16-byte pieces of the row, 8 at a time, from rank column j on
    struct BItem {
        const uint16_t *bp;  // row nc0 + c of B_i (or some valid address if the item has nothing to add)
        int q, rank;         // rank 0: nothing to add
        bool vec;            // rows of B_i are 16-byte aligned
    };
    auto b_item = [&](int q0, int qb, int item) {
        BItem it;
        const int q1 = item >> (sh.lgG + 2), c = item & (ncols - 1);
        const bool in = q1 < qb;
        const int q = in ? q1 : 0;
        const int slot = s_slot[q0 + q], rank = s_rank[q0 + q];
        const bool use = in && slot >= 0 && nc0 + c < N;
        it.q = q;
        it.rank = use ? rank : 0;
        it.vec = (rank & 7) == 0;
        it.bp = reinterpret_cast<const uint16_t *>(slot_B(pool, use ? slot : 0)) + (use ? (size_t)(nc0 + c) * rank : 0);
        return it;
    };
    auto b_load = [&](const BItem &it, int j, u32x4 *b) {
#pragma unroll
        for (int hh = 0; hh < 8; ++hh) {
            if (j + 8 * hh >= R) continue;  // nobody's rank reaches this far
            const bool in = it.vec && j + 8 * hh < it.rank;
            b[hh] = *reinterpret_cast<const u32x4 *>(in ? it.bp + j + 8 * hh : reinterpret_cast<const uint16_t *>(slot_B(pool, 0)));
        }
    };

    uint32_t vval[VB];
    bool vneed[VB];
    BItem bit[IB];
    u32x4 bpre[IB][8];
    if (has_pool) {
        const int qb = min(qb_max, T);
        v_load(0, qb, 0, vval, vneed);
#pragma unroll
        for (int ii = 0; ii < IB; ++ii) {
            bit[ii] = b_item(0, qb, tid + ii * kThreads);
            b_load(bit[ii], 0, bpre[ii]);
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();  // the x ring is reused below (no fence: the requests above stay in flight)
    asm volatile("" ::: "memory");
    TRACE(8);

    // ---- the adapter term of the own columns -------------------------------------------------------------------
    if (has_pool) {
        for (int q0 = 0; q0 < T; q0 += qb_max) {
            const int qb = min(qb_max, T - q0);
            if (q0 > 0) __syncthreads();
            // v of these rows out of the mailbox (entries below the row's rank; the others count as zero)
            bool gave_up = false;
            for (int e0 = 0; e0 < (qb << sh.lgRp) && !gave_up; e0 += kThreads * VB) {
                if (q0 > 0 || e0 > 0) v_load(q0, qb, e0, vval, vneed);
                for (int spin = 0;; ++spin) {
                    bool all = true;
#pragma unroll
                    for (int i = 0; i < VB; ++i) all = all && !(vneed[i] && vval[i] == kEmpty);
                    if (all) break;
                    if (spin >= sh.spin_limit) {
                        gave_up = true;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
#pragma unroll
                    for (int i = 0; i < VB; ++i) {
                        const int e = e0 + i * kThreads + tid;
                        if (vneed[i] && vval[i] == kEmpty) vval[i] = mb_load_u32(&vmail[(size_t)(q0 + (e >> sh.lgRp)) * R + (e & (Rp - 1))]);
                    }
                }
#pragma unroll
                for (int i = 0; i < VB; ++i) {
                    const int e = e0 + i * kThreads + tid;
                    const int q = e >> sh.lgRp, j = e & (Rp - 1);
                    if (q < qb && j < R) vs[q * R + j] = vneed[i] ? __uint_as_float(vval[i]) : 0.0f;
                }
            }
            if (gave_up || sh.spin_limit == 0) s_vfail = 1;
            TRACE(9);
            __syncthreads();
            TRACE(10);
            if (s_vfail) {
                // the shrink results did not arrive in time: compute v of these rows here
                for (int wu = wave; wu < qb * sh.jgroups; wu += kWaves) {
                    const int q = wu / sh.jgroups, j0 = (wu - q * sh.jgroups) * 2;
                    const int slot = s_slot[q0 + q], rank = s_rank[q0 + q];
                    float r0 = 0.0f, r1 = 0.0f;
                    if (slot >= 0 && j0 < rank) {
                        const uint16_t *A0 = reinterpret_cast<const uint16_t *>(slot_A(pool, slot)) + (size_t)j0 * K;
                        shrink_pair(A0, (j0 + 1 < rank) ? A0 + K : A0, x + (size_t)(q0 + q) * K, K, lane, r0, r1);
                        if (j0 + 1 >= rank) r1 = 0.0f;
                    }
                    if (lane == 0) {
                        vs[q * R + j0] = r0;
                        if (j0 + 1 < R) vs[q * R + j0 + 1] = r1;
                    }
                }
                __syncthreads();
            }
            // d[t][c] = s_t * sum_j B_i[nc0 + c][j] v[t][j]: one (row, column) item per thread, two items at a time
            for (int it0 = tid; it0 < qb * ncols; it0 += kThreads * IB) {
                const bool first = q0 == 0 && it0 == tid;
                float d[IB];
                int rmax = 0;
#pragma unroll
                for (int ii = 0; ii < IB; ++ii) {
                    if (!first) bit[ii] = b_item(q0, qb, it0 + ii * kThreads);
                    d[ii] = 0.0f;
                    rmax = max(rmax, bit[ii].vec ? bit[ii].rank : 0);
                }
                for (int j = 0; j < rmax; j += 64) {
                    if (!first || j > 0) {
#pragma unroll
                        for (int ii = 0; ii < IB; ++ii) b_load(bit[ii], j, bpre[ii]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int ii = 0; ii < IB; ++ii) {
                        const float *vq = vs + bit[ii].q * R + j;
#pragma unroll
                        for (int hh = 0; hh < 8; ++hh) {
                            if (!bit[ii].vec || j + 8 * hh >= bit[ii].rank) continue;
#pragma unroll
                            for (int u = 0; u < 4; ++u) {
                                d[ii] = fmaf(__uint_as_float(bpre[ii][hh][u] << 16), vq[8 * hh + 2 * u], d[ii]);
                                d[ii] = fmaf(__uint_as_float(bpre[ii][hh][u] & 0xffff0000u), vq[8 * hh + 2 * u + 1], d[ii]);
                            }
                        }
                    }
                }
#pragma unroll
                for (int ii = 0; ii < IB; ++ii) {
                    if (!bit[ii].vec)  // rows of B_i not 16-byte aligned: element by element
                        for (int j = 0; j < bit[ii].rank; ++j) d[ii] = fmaf(bf16_to_f32(bit[ii].bp[j]), vs[bit[ii].q * R + j], d[ii]);
                    const int item = it0 + ii * kThreads;
                    if (item < qb * ncols) dsum[(size_t)q0 * ncols + item] = d[ii] * s_scale[q0 + bit[ii].q];
                }
            }
        }
    }
    TRACE(2);  // adapter term formed

    // ---- take the pieces of every (row, granule) cell --------------------------------------------------------------
    {
        bool gave_up = sh.spin_limit == 0;
        for (int spin = 0; !gave_up; ++spin) {
            p_load();
            bool all = true;
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                if (pneed[u] && pval[u][0] != kEmpty && pval[u][1] != kEmpty && pval[u][2] != kEmpty && pval[u][3] != kEmpty) {
                    pneed[u] = false;
                    *reinterpret_cast<u32x4 *>(stage + pdst[u]) = pval[u];
                    piece_clear(const_cast<float *>(psrc[u]));  // empty again for the next call
                }
                all = all && !pneed[u];
            }
            if (all) break;
            if (spin >= sh.spin_limit) {
                gave_up = true;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (gave_up) s_fail = 1;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();  // staging complete (no fence: nobody has to wait for the mailbox stores here)
    asm volatile("" ::: "memory");
    TRACE(6);  // pieces in
    if (s_fail == 0) {
        // add in fixed order, round once, store each row at its own position
        for (int cell = tid; cell < n_cells; cell += kThreads) {
            const int t = cell >> sh.lgG, qo = cell & (sh.G - 1);
            const int n = nc0 + qo * 4;
            if (n >= N) continue;
            floatx4 o = *reinterpret_cast<const floatx4 *>(stage + (size_t)cell * 4);
            for (int sd = 1; sd < sh.split; ++sd) {
                const floatx4 pc = *reinterpret_cast<const floatx4 *>(stage + ((size_t)sd * n_cells + cell) * 4);
                o[0] += pc[0];
                o[1] += pc[1];
                o[2] += pc[2];
                o[3] += pc[3];
            }
            if (has_pool) {
                const floatx4 dd = *reinterpret_cast<const floatx4 *>(dsum + (size_t)cell * 4);
                o[0] += dd[0];
                o[1] += dd[1];
                o[2] += dd[2];
                o[3] += dd[3];
            }
            const uint64_t packed = (uint64_t)f32_to_bf16(o[0]) | ((uint64_t)f32_to_bf16(o[1]) << 16) |
                                    ((uint64_t)f32_to_bf16(o[2]) << 32) | ((uint64_t)f32_to_bf16(o[3]) << 48);
            *reinterpret_cast<uint64_t *>(y + (size_t)t * N + n) = packed;
        }
    } else {
        // some piece did not arrive in time: this workgroup computes its columns from the inputs, and the pieces that
        // are still on their way are removed when the call ends
        if (tid == 0) {
            if (sh.local) __hip_atomic_fetch_add(&sync[kCntXcd + 32 * (blockIdx.x % kXcds)], kGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            else __hip_atomic_fetch_add(&sync[kCntXcd + 32 * (blockIdx.x % kXcds)], kGaveUp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        recompute_columns(sh, x, W, pool, route, has_pool, y, nc0, ncols, wave, lane);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
    }
    }
    TRACE(7);  // y written
    if (!acked) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // what this workgroup posted has been acknowledged
        __syncthreads();
    }
    finish_call();
}

// workgroups of decode_kernel<tt, wlds> the device holds at once (registers and LDS decide; asked once per instance),
// and its number of compute units
template <int TT, bool WL>
hipError_t ask_occupancy(int *per_cu)
{
    // (the ring may be larger than the LDS a kernel gets without asking)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&decode_kernel<TT, WL>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       ring_bytes(TT, WL));
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(per_cu, decode_kernel<TT, WL>, kThreads, ring_bytes(TT, WL));
    return e;
}
int resident_workgroups(int tt, bool wlds, int *n_cus)
{
    static int cached[5][2] = {{0, 0}, {0, 0}, {0, 0}, {0, 0}, {0, 0}};
    static int cached_cus = 0;
    if (cached[tt][wlds] == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) {
            switch (tt) {
            case 1: e = ask_occupancy<1, true>(&per_cu); break;
            case 2: e = ask_occupancy<2, true>(&per_cu); break;
            case 3: e = wlds ? ask_occupancy<3, true>(&per_cu) : ask_occupancy<3, false>(&per_cu); break;
            default: e = wlds ? ask_occupancy<4, true>(&per_cu) : ask_occupancy<4, false>(&per_cu); break;
            }
        }
        if (e != hipSuccess) {
            (void)hipGetLastError();
            *n_cus = 64;
            return 64;  // not cached: a cautious figure for this call (e.g. no device in this process yet)
        }
        cached[tt][wlds] = per_cu * cus > 0 ? per_cu * cus : 64;
        cached_cus = cus > 0 ? cus : 64;
    }
    *n_cus = cached_cus;
    return cached[tt][wlds];
}

// K-slices = owners per tile: 1, 2, 4 or 8.  All workgroups of the call have to be resident at once, and there are
// never more than ELORA_DEC_TARGET_WGS of them.  If some split gives (nearly) exactly one workgroup per compute unit,
// that one is taken: the stream then ends at about the same time everywhere, with half the pieces to exchange
// (measured: 64 tiles as 4 x 64 workgroups 0.3 to 1.4 us per call ahead of 8 x 64).  Otherwise the largest that fits:
// two workgroups per unit hide more latency than one on seven eighths of the units (224 tiles: 2 x 224 ahead of 224).
int pick_split(int K, int n_tiles, int resident, int n_cus)
{
    const int chunks = K / kChunk;
    const int target = resident < ELORA_DEC_TARGET_WGS ? resident : ELORA_DEC_TARGET_WGS;
    int best = 1;
    for (int s = 2; s <= kDecodeMaxSplit; s *= 2)
        if (s <= chunks && n_tiles * s <= target) best = s;
    for (int s = 1; s <= best; s *= 2)
        if (n_tiles * s <= n_cus && n_tiles * s * 20 >= n_cus * 19) return s;
    return best;
}

// Up to 32 rows of x W always travels through LDS.  With more rows the ring with W in it leaves room for one workgroup
// per compute unit only: taken if that costs no workgroups, or if the call then has (nearly) one per unit; else W goes
// into registers and two workgroups share a unit (measured at 64 rows, 4096 x 4096: 27.4 against 28.9 us; 14336 x 4096:
// 53.9 against 60.8; 4096 x 14336, 224 tiles: 63.8 against 61.8).
DecodeShape make_shape(int T, int K, int N, int max_rank, bool *w_lds)
{
    DecodeShape sh;
    sh.T = T;
    sh.K = K;
    sh.N = N;
    sh.chunks = K / kChunk;
    sh.n_tiles = (N + kTileRows - 1) / kTileRows;
    sh.jgroups = (max_rank + 1) / 2;
    sh.jg_inv = (unsigned)((1ull << 32) / (unsigned)sh.jgroups) + 1u;
    const int tt = (T + 15) / 16;
    int n_cus = 0;
    bool wlds = true;
    int resident = resident_workgroups(tt, true, &n_cus);
    sh.split = pick_split(K, sh.n_tiles, resident, n_cus);
    if (tt > 2) {
        const int resident_r = resident_workgroups(tt, false, &n_cus);
        const int split_r = pick_split(K, sh.n_tiles, resident_r, n_cus);
        const int wgs = sh.n_tiles * sh.split;
        if (split_r != sh.split && !(wgs <= n_cus && wgs * 20 >= n_cus * 19)) {
            wlds = false;
            resident = resident_r;
            sh.split = split_r;
        }
    }
    *w_lds = wlds;
    sh.lgS = 0;
    while ((1 << sh.lgS) < sh.split) ++sh.lgS;
    sh.total = sh.n_tiles * sh.split;
    const int unit = kXcds * sh.split;
    sh.grid = (sh.total + unit - 1) / unit * unit;
    sh.real_per_xcd = sh.grid / kXcds;
    // A call that leaves compute units without a workgroup gets surplus ones for them: they only share in the shrink,
    // which for few output columns is most of the work (k_proj / v_proj at 64 rows: 2048 units of two rank rows on 128
    // workgroups).
#ifndef ELORA_NO_SURPLUS
    if (sh.jgroups > 1) {
        const int room = (resident < n_cus ? resident : n_cus) / unit * unit;
        if (room > sh.grid) sh.grid = room;
    }
#endif
    // the workgroups that share the shrink must all be running before anybody can wait for them
    sh.n_pub = sh.grid < resident ? sh.grid : resident;
    sh.G = kGranules / sh.split;
    sh.lgG = 0;
    while ((1 << sh.lgG) < sh.G) ++sh.lgG;
    sh.lgRp = 0;
    while ((1 << sh.lgRp) < max_rank) ++sh.lgRp;
    sh.spin_limit = g_spin_limit;
    sh.zero = 0;
    int dev = 0;
    sh.local = (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices && g_local[dev] == 1 && g_local_override != 0) ? 1 : 0;
    return sh;
}

// ---- is workgroup b of a launch placed on XCD b % 8? -----------------------------------------------
__global__ void xcc_probe_kernel(int *xcc_of_block) { xcc_of_block[blockIdx.x] = __builtin_amdgcn_s_getreg(20 | (31 << 11)) & 15; }  // HW_REG_XCC_ID

}  // namespace

// One small launch and a blocking copy: called from set-up code (workspace initialisation), never from a linear call.
int elora::decode_probe_device(hipStream_t stream)
{
    int dev = 0;
    ELORA_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices || g_local[dev] != 0) return ELORA_OK;
    constexpr int n = 256;
    int *d = nullptr;
    int h[n];
    ELORA_HIP_TRY(hipMalloc(&d, sizeof(h)));
    hipLaunchKernelGGL(xcc_probe_kernel, dim3(n), dim3(64), 0, stream, d);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(h, d, sizeof(h), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    (void)hipFree(d);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return ELORA_E_HIP;
    }
    // blocks with the same b % 8 must share an XCD (one XCD in all is the degenerate case of that)
    bool ok = true;
    for (int b = kXcds; b < n; ++b) ok = ok && h[b] == h[b % kXcds];
    g_local[dev] = ok ? 1 : -1;
    return ELORA_OK;
}

void elora::decode_set_spin_limit(int limit) { g_spin_limit = limit; }
void elora::decode_set_local_override(int mode) { g_local_override = mode; }

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
           d.d_in % kChunk == 0 && d.d_out % 16 == 0;
}

// bytes of the piece mailboxes for d_out output columns: up to 8 K-slices, up to 64 rows
size_t elora::decode_mail_bytes(int d_out)
{
    const size_t n_tiles = ((size_t)d_out + kTileRows - 1) / kTileRows;
    return n_tiles * kDecodeMaxSplit * kDecodeMaxTokens * kTileRows * sizeof(float);
}

void elora::decode_plan(const elora_linear_desc_t &d, elora_plan_t *plan)
{
    bool wlds = true;
    DecodeShape sh = make_shape(d.n_tokens, d.d_in, d.d_out, d.pool ? d.pool->max_rank : 1, &wlds);
    plan->n_launches = 1;
    plan->split_k = sh.split;
    plan->tile_rows = kTileRows;
    plan->tile_cols = 0;
    plan->grid = sh.grid;
}

int elora::launch_decode(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream)
{
    (void)plan;
    bool wlds = true;
    DecodeShape sh = make_shape(a.T, a.K, a.N, a.has_pool ? a.pool.max_rank : 1, &wlds);
    float *mail = reinterpret_cast<float *>(a.ws + a.wsl.mail);
    float *vmail = reinterpret_cast<float *>(a.ws + a.wsl.vmail);
    int *sync = reinterpret_cast<int *>(a.ws + a.wsl.sync);
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *W = static_cast<const uint16_t *>(a.W);
    uint16_t *y = static_cast<uint16_t *>(a.y);
    int has_pool = a.has_pool ? 1 : 0;
    dim3 grid(sh.grid), block(kThreads);
    int tt = (a.T + 15) / 16;
    profile_mark_begin(stream);
    switch (tt) {
    case 1: hipLaunchKernelGGL((decode_kernel<1, true>), grid, block, ring_bytes(1, true), stream, sh, x, W, a.pool, a.route, has_pool, mail, vmail, sync, y); break;
    case 2: hipLaunchKernelGGL((decode_kernel<2, true>), grid, block, ring_bytes(2, true), stream, sh, x, W, a.pool, a.route, has_pool, mail, vmail, sync, y); break;
    case 3:
        if (wlds) hipLaunchKernelGGL((decode_kernel<3, true>), grid, block, ring_bytes(3, true), stream, sh, x, W, a.pool, a.route, has_pool, mail, vmail, sync, y);
        else hipLaunchKernelGGL((decode_kernel<3, false>), grid, block, ring_bytes(3, false), stream, sh, x, W, a.pool, a.route, has_pool, mail, vmail, sync, y);
        break;
    default:
        if (wlds) hipLaunchKernelGGL((decode_kernel<4, true>), grid, block, ring_bytes(4, true), stream, sh, x, W, a.pool, a.route, has_pool, mail, vmail, sync, y);
        else hipLaunchKernelGGL((decode_kernel<4, false>), grid, block, ring_bytes(4, false), stream, sh, x, W, a.pool, a.route, has_pool, mail, vmail, sync, y);
        break;
    }
    ELORA_HIP_TRY(hipGetLastError());
    profile_mark_end(stream);
    return ELORA_OK;
}
