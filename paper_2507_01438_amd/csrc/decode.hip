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
//
// The kernel body lives in decode_body.inc and is included into two kernels: decode_kernel (one call per launch) and
// decode_group_kernel (two or three calls that are due together, each with a grid of its own inside the launch).
// A call with a pool that would leave compute units without a workgroup gets surplus workgroups that only share
// in the shrink.
#include "common.h"

#include <type_traits>

using namespace elora;

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRowsPerWave = 16;  // W rows per wave (one MFMA row block)
constexpr int kChunk = 256;               // K elements per register set of W (8 MFMA K steps)
// The ring of sub-spans in LDS (dynamic LDS: the only such array of the kernel; the staging after the contraction reuses
// it).  A sub-span is 128 elements of K.  Up to 32 rows of x: 5 slots, more rows: 4.  A slot holds the rows of x and,
// where W travels through the ring as well (see the kernel), the tile's 64 rows of W.
constexpr int kSubSpan = 128;
// (nw = waves per workgroup: 4, or 8 for the wide kernel whose tile is 128 rows of W: 3 slots of 48 KiB)
// (rows of 256 bytes: a row of x, a row of a bf16 W, or two rows of an 8-bit W; the wide kernel for an 8-bit W has 4
// slots of 32 KiB, and every wide kernel gets the LDS of the bf16 one, because what follows the contraction stages as
// much there)
__host__ __device__ constexpr int ring_slots(int tt, bool wlds, int nw, bool w8 = false) { return nw > 4 ? (w8 ? 4 : 3) : tt <= 2 ? 5 : 4; }
__host__ __device__ constexpr int slot_rows(int tt, bool wlds, int nw, bool w8 = false)
{
    return tt * 16 + (wlds ? nw * kRowsPerWave / (w8 ? 2 : 1) : 0);
}
__host__ __device__ constexpr int ring_bytes(int tt, bool wlds, int nw, bool w8 = false)
{
    return nw > 4 ? 3 * (tt * 16 + nw * kRowsPerWave) * kSubSpan * 2 : ring_slots(tt, wlds, nw, w8) * slot_rows(tt, wlds, nw, w8) * kSubSpan * 2;
}
static_assert(ring_slots(4, true, 8, true) * slot_rows(4, true, 8, true) <= 3 * (64 + 128), "the 8-bit wide ring fits");
constexpr uint32_t kEmpty = 0xFFFFFFFFu;
constexpr int kMetaLds = 512;  // slot tables up to this many entries are copied to LDS whole

constexpr int kXcds = 8;                  // workgroup b runs on XCD b % 8
template <int V> using ic = std::integral_constant<int, V>;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16_pair_t __attribute__((ext_vector_type(2)));
typedef float float_pair_t __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 pair (low half first), round-to-nearest-even
__device__ __forceinline__ uint32_t pack_bf16_pair(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(float_pair_t{lo, hi}, bf16_pair_t));
}

// sync area (ints) at the start of the workspace
constexpr int kCntAll = 0;        // XCDs all of whose workgroups have finished
constexpr int kCntXcd = 32;       // + 32 x (a cache line of its own): workgroups of XCD x that have finished, plus
constexpr int kGaveUp = 1 << 16;  // this much for every owner on XCD x that gave up (its piece mailboxes may hold pieces nobody took)

int g_spin_limit = 1 << 22;
int g_wait_us = 200;
int g_pass_mode = -1;  // calls of 65 to 256 rows as several launches: 0 never, otherwise always
int g_local_override = -1;
int g_k_rotate = 1;
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
    int wait_ticks; // a wait for another workgroup gives up after this many ticks of the 100 MHz clock
    int tile_rows;  // rows of W per tile: 64 (four waves) or 128 (the wide kernel, eight waves)
    int rot_mask;   // a workgroup starts its K-slice (tile number on its XCD & rot_mask) sub-spans in: 2^n - 1, below every slice's length
    const uint16_t *w_scales;  // 8-bit W: fp16 [d_out][d_in / 32] group scales; else nullptr
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
__device__ __forceinline__ void recompute_columns(const DecodeShape &sh, const uint16_t *__restrict__ x, const uint16_t *__restrict__ W,
                                  const PoolView &pool, const RouteView &route, int has_pool, uint16_t *__restrict__ y,
                                  int nc0, int ncols, int wave, int n_waves, int lane)
{
    const int T = sh.T, K = sh.K, N = sh.N;
    for (int t = wave; t < T; t += n_waves) {
        RowRoute rr{-1, 0, 0.0f};
        if (has_pool) rr = resolve_row(t, route, pool, false);
        const uint16_t *xt = x + (size_t)t * K;
        float d = 0.0f;  // lane c: adapter term of column nc0 + c
        if (rr.slot >= 0) {
            const uint16_t *A = reinterpret_cast<const uint16_t *>(slot_A(pool, rr.slot));
            const uint16_t *B = reinterpret_cast<const uint16_t *>(slot_B(pool, rr.slot));
            const uint16_t *As = slot_A_scales(pool, rr.slot), *Bs = slot_B_scales(pool, rr.slot);  // (8-bit blocks)
            for (int j0 = 0; j0 < rr.rank; j0 += 2) {
                const bool two = (j0 + 1) < rr.rank;
                const int j1 = two ? j0 + 1 : j0;
                float r0, r1;
                if (pool.q8) {
                    const char *Ac = reinterpret_cast<const char *>(A);
                    shrink_pair_q8(Ac + (size_t)j0 * K, Ac + (size_t)j1 * K, As + (((size_t)j0 * K) >> 5), As + (((size_t)j1 * K) >> 5), xt,
                                   K, lane, r0, r1);
                } else {
                    shrink_pair(A + (size_t)j0 * K, A + (size_t)j1 * K, xt, K, lane, r0, r1);
                }
                if (lane < ncols && nc0 + lane < N) {
                    const size_t e = (size_t)(nc0 + lane) * rr.rank;
                    const float b0 = pool.q8 ? q8_elem(reinterpret_cast<const char *>(B), Bs, e + j0) : bf16_to_f32(B[e + j0]);
                    d = fmaf(b0, r0, d);
                    if (two) d = fmaf(pool.q8 ? q8_elem(reinterpret_cast<const char *>(B), Bs, e + j0 + 1) : bf16_to_f32(B[e + j0 + 1]), r1, d);
                }
            }
        }
        for (int c = 0; c < ncols && nc0 + c < N; ++c) {
            const uint16_t *wn = W + (size_t)(nc0 + c) * K;
            float s = 0.0f;
            if (sh.w_scales != nullptr) {
                // 8-bit W: w = bf16(scale * code), the value the main path multiplies
                const int8_t *wc = reinterpret_cast<const int8_t *>(W) + (size_t)(nc0 + c) * K;
                const uint16_t *ws = sh.w_scales + (size_t)(nc0 + c) * (K >> 5);
                for (int k = lane * 8; k < K; k += 64 * 8) {
                    const u32x2 cv = *reinterpret_cast<const u32x2 *>(wc + k);
                    const u32x4 xv = *reinterpret_cast<const u32x4 *>(xt + k);
                    const float sc = fp16_to_f32(ws[k >> 5]);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const uint32_t cw = cv[q >> 1] >> (16 * (q & 1));
                        const uint32_t wp = pack_bf16_pair(sc * (float)(int8_t)(cw & 0xffu), sc * (float)(int8_t)((cw >> 8) & 0xffu));
                        s = fmaf(__uint_as_float(wp << 16), __uint_as_float(xv[q] << 16), s);
                        s = fmaf(__uint_as_float(wp & 0xffff0000u), __uint_as_float(xv[q] & 0xffff0000u), s);
                    }
                }
            } else
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

template <int TT, bool kWLds, int NW, bool kQ8, bool kW8, bool kLeanOnly>
__global__ __launch_bounds__(NW * 64, NW > 4 ? 1 : 2) void decode_kernel(DecodeShape sh, const uint16_t *__restrict__ x,
                                                                           const uint16_t *__restrict__ W, PoolView pool,
                                                                           RouteView route, int has_pool, float *__restrict__ mail,
                                                                           float *__restrict__ vmail, int *__restrict__ sync,
                                                                           uint16_t *__restrict__ y)
{
#define ELORA_WG blockIdx.x
#include "decode_body.inc"
#undef ELORA_WG
}

// Several calls in one launch (projections that are due at the same time: q/k/v, gate/up): call i owns workgroups
// first[i] .. first[i + 1) and every workgroup does exactly what it would do in a launch of its call alone.  The
// calls share nothing (each has its own workspace), so the body is the same text; what is saved is the start and
// the end of a launch, which for a small projection is most of its time.  All workgroups of the launch are resident.
// (The body is included rather than called: as a function of its own the single-call kernel came out 1 us slower.)
constexpr int kGroupMax = 3;
struct DecodeCall {
    DecodeShape sh;
    const uint16_t *x, *W;
    PoolView pool;
    RouteView route;
    int has_pool;
    float *mail, *vmail;
    int *sync;
    uint16_t *y;
};
struct DecodeGroup {
    int n;
    int first[kGroupMax + 1];  // multiples of 8: workgroup b of the launch and workgroup b - first[i] of its call share b % 8
    DecodeCall call[kGroupMax];
};

template <int TT, bool kWLds, int NW, bool kQ8, bool kW8, bool kLeanOnly>
__global__ __launch_bounds__(NW * 64, NW > 4 ? 1 : 2) void decode_group_kernel(DecodeGroup grp_)
{
    int call_i = 0;
    if (grp_.n > 1 && (int)blockIdx.x >= grp_.first[1]) call_i = 1;
    if (grp_.n > 2 && (int)blockIdx.x >= grp_.first[2]) call_i = 2;
    const DecodeCall &c_ = grp_.call[call_i];
    const DecodeShape sh = c_.sh;
    const uint16_t *__restrict__ x = c_.x, *__restrict__ W = c_.W;
    const PoolView pool = c_.pool;
    const RouteView route = c_.route;
    const int has_pool = c_.has_pool;
    float *__restrict__ mail = c_.mail, *__restrict__ vmail = c_.vmail;
    int *__restrict__ sync = c_.sync;
    uint16_t *__restrict__ y = c_.y;
    const unsigned wg_ = blockIdx.x - (unsigned)grp_.first[call_i];
#define ELORA_WG wg_
#include "decode_body.inc"
#undef ELORA_WG
}

// The kernel instances: 16-row blocks of x (1..4), W through the LDS ring or into registers, waves per workgroup.
// The wide kernel (8 waves, 128 rows of W per tile, x read once per 128 rows instead of once per 64) exists for more
// than 32 rows of x only, with four blocks of x and W through the ring.
struct Variant {
    int tt;
    bool wlds;
    int nw;
    bool q8 = false;  // the pool keeps its adapters in 8-bit blocks (W through the ring always)
    bool w8 = false;  // W is 8-bit (into registers on four waves, through the ring on eight)
    // the instances without the general tail (bf16 W through the ring, bf16 pool or none; eight waves, or four waves
    // with one or two blocks of x): for calls whose pool, as the host knows it, holds only ranks that are multiples of
    // 8, up to 64.  14 to 24 KB less code per instance; config 3: 178.0 -> 175.1 us per step, config 2: 15.45 -> 14.8.
    // (In the eight-wave instance the kernel also takes the short tail for granted; in the four-wave ones it still
    // looks, which is what the compiler made the faster code of: 14.8 against 15.9 us.)
    bool lean = false;
    int index() const
    {
        if (lean) return 33 + (nw > 4 ? 2 : tt - 1);
        return w8 ? (nw > 4 ? 26 : 21 + tt) + (q8 ? 6 : 0) : (nw > 4 ? 10 : tt * 2 + (wlds ? 1 : 0)) + (q8 ? 11 : 0);
    }
    void allow_lean(bool ok) { lean = ok && !q8 && !w8 && wlds && (nw > 4 || tt <= 2); }
    int threads() const { return nw * 64; }
    int tile_rows() const { return nw * kRowsPerWave; }
    int lds() const { return ring_bytes(tt, wlds, nw, w8); }
};
constexpr int kVariants = 36;
template <typename F>
auto with_variant_bf16(const Variant &v, F &&f)
{
    if (v.nw > 4) return f(ic<4>{}, std::true_type{}, ic<8>{});
    switch (v.tt) {
    case 1: return f(ic<1>{}, std::true_type{}, ic<4>{});
    case 2: return f(ic<2>{}, std::true_type{}, ic<4>{});
    case 3: return v.wlds ? f(ic<3>{}, std::true_type{}, ic<4>{}) : f(ic<3>{}, std::false_type{}, ic<4>{});
    default: return v.wlds ? f(ic<4>{}, std::true_type{}, ic<4>{}) : f(ic<4>{}, std::false_type{}, ic<4>{});
    }
}

template <typename F>
auto with_variant(const Variant &v, F &&f)  // f(blocks of x, W through the ring, waves, 8-bit pool, 8-bit W, no general tail)
{
    const std::true_type yes{};
    const std::false_type no{};
    if (v.lean) {
        if (v.nw > 4) return f(ic<4>{}, yes, ic<8>{}, no, no, yes);
        if (v.tt == 1) return f(ic<1>{}, yes, ic<4>{}, no, no, yes);
        return f(ic<2>{}, yes, ic<4>{}, no, no, yes);
    }
    if (v.w8 && v.q8) {
        if (v.nw > 4) return f(ic<4>{}, yes, ic<8>{}, yes, yes, no);
        switch (v.tt) {
        case 1: return f(ic<1>{}, no, ic<4>{}, yes, yes, no);
        case 2: return f(ic<2>{}, no, ic<4>{}, yes, yes, no);
        default: return f(ic<4>{}, no, ic<4>{}, yes, yes, no);
        }
    }
    if (v.w8) {
        if (v.nw > 4) return f(ic<4>{}, yes, ic<8>{}, no, yes, no);
        switch (v.tt) {
        case 1: return f(ic<1>{}, no, ic<4>{}, no, yes, no);
        case 2: return f(ic<2>{}, no, ic<4>{}, no, yes, no);
        default: return f(ic<4>{}, no, ic<4>{}, no, yes, no);
        }
    }
    if (v.q8) {
        if (v.nw > 4) return f(ic<4>{}, yes, ic<8>{}, yes, no, no);
        switch (v.tt) {
        case 1: return f(ic<1>{}, yes, ic<4>{}, yes, no, no);
        case 2: return f(ic<2>{}, yes, ic<4>{}, yes, no, no);
        case 3: return f(ic<3>{}, yes, ic<4>{}, yes, no, no);
        default: return f(ic<4>{}, yes, ic<4>{}, yes, no, no);
        }
    }
    return with_variant_bf16(v, [&](auto tt, auto wl, auto nw) { return f(tt, wl, nw, no, no, no); });
}
// workgroups of a kernel instance the device holds at once (registers and LDS decide; asked once per instance), and
// its number of compute units.  group: the kernel that carries several calls; 0 if it cannot be asked (then calls
// are launched one by one).
int resident_of(const Variant &v, bool group, int *n_cus)
{
    static int cached[2][kVariants];
    static int cached_cus = 0;
    int &slot = cached[group ? 1 : 0][v.index()];
    if (slot == 0) {
        int per_cu = 0, cus = 0, dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess)
            e = with_variant(v, [&](auto tt, auto wl, auto nw, auto q8, auto w8, auto ln) {
                constexpr int TT = decltype(tt)::value, NW = decltype(nw)::value;
                constexpr bool WL = decltype(wl)::value, Q8 = decltype(q8)::value, W8 = decltype(w8)::value, LN = decltype(ln)::value;
                // (the ring may be larger than the LDS a kernel gets without asking)
                if constexpr (W8) {
                    const void *fn8 = group ? reinterpret_cast<const void *>(&decode_group_kernel<TT, WL, NW, Q8, true, LN>)
                                            : reinterpret_cast<const void *>(&decode_kernel<TT, WL, NW, Q8, true, LN>);
                    hipError_t e8 = hipFuncSetAttribute(fn8, hipFuncAttributeMaxDynamicSharedMemorySize, ring_bytes(TT, WL, NW, true));
                    if (e8 != hipSuccess) return e8;
                    return group ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_group_kernel<TT, WL, NW, Q8, true, LN>, NW * 64, ring_bytes(TT, WL, NW, true))
                                 : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<TT, WL, NW, Q8, true, LN>, NW * 64, ring_bytes(TT, WL, NW, true));
                } else {
                const void *fn = group ? reinterpret_cast<const void *>(&decode_group_kernel<TT, WL, NW, Q8, false, LN>)
                                       : reinterpret_cast<const void *>(&decode_kernel<TT, WL, NW, Q8, false, LN>);
                hipError_t e2 = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, ring_bytes(TT, WL, NW));
                if (e2 != hipSuccess) return e2;
                return group ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_group_kernel<TT, WL, NW, Q8, false, LN>, NW * 64, ring_bytes(TT, WL, NW))
                             : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_kernel<TT, WL, NW, Q8, false, LN>, NW * 64, ring_bytes(TT, WL, NW));
                }
            });
        if (e != hipSuccess) {
            (void)hipGetLastError();
            if (n_cus) *n_cus = 64;
            return group ? 0 : 64;  // not cached: a cautious figure for this call (e.g. no device in this process yet)
        }
        slot = per_cu * cus > 0 ? per_cu * cus : (group ? 0 : 64);
        cached_cus = cus > 0 ? cus : 64;
        if (slot == 0) return 0;
    }
    if (n_cus) *n_cus = cached_cus;
    return slot;
}
int resident_group_workgroups(const Variant &v) { return resident_of(v, true, nullptr); }
int resident_workgroups(const Variant &v, int *n_cus) { return resident_of(v, false, n_cus); }

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
// With more than 32 rows the wide kernel (128 rows of W per workgroup) is taken where its grid covers at least seven
// eighths of the compute units: every workgroup re-reads its K-slice of x, and twice the rows of W per workgroup
// halve that share of what a compute unit has to take in.
void finish_shape(DecodeShape &sh, int max_rank, int resident, int n_cus, bool surplus);

int g_wide_mode = -1;  // -1: where it pays, 0: never, 1: wherever the shape allows it

bool wide_allowed(int T) { return g_wide_mode != 0 && T > 32; }

// what the kernel's short tail serves (its `lean`), as far as the host can tell: every loaded rank a multiple of 8, and
// max_rank from 5 to 64
bool ranks_fit_short_tail(int n_odd_ranks, int max_rank) { return n_odd_ranks == 0 && max_rank <= 64 && max_rank > 4; }

DecodeShape make_shape(int T, int K, int N, int max_rank, bool q8, Variant *var, const uint16_t *w_scales = nullptr, bool lean_ok = false)
{
    DecodeShape sh;
    sh.w_scales = w_scales;
    sh.T = T;
    sh.K = K;
    sh.N = N;
    sh.chunks = K / kChunk;
    sh.jgroups = (max_rank + 1) / 2;
    sh.jg_inv = (unsigned)((1ull << 32) / (unsigned)sh.jgroups) + 1u;
    const int tt = (T + 15) / 16;
    int n_cus = 0;
    if (w_scales != nullptr) {
        // 8-bit W: into registers on four waves; more than 32 rows: 128 rows of W per workgroup, through the ring, where
        // that grid covers the device
        if (wide_allowed(T)) {
            const Variant wide{4, true, 8, q8, true};
            const int resident = resident_workgroups(wide, &n_cus);
            const int n_tiles = (N + wide.tile_rows() - 1) / wide.tile_rows();
            const int split = pick_split(K, n_tiles, resident, n_cus);
            if (n_tiles * split <= resident && (g_wide_mode == 1 || n_tiles * split * 8 >= n_cus * 7)) {
                sh.tile_rows = wide.tile_rows();
                sh.n_tiles = n_tiles;
                sh.split = split;
                *var = wide;
                finish_shape(sh, max_rank, resident, n_cus, true);
                return sh;
            }
        }
        // (33 to 48 rows take the instance for four blocks of x: the one for three needs more registers than a wave has,
        // and what the compiler would move to scratch memory there may be the target of a load still on its way)
        Variant v8{tt == 3 ? 4 : tt, false, 4, q8, true};
        sh.tile_rows = v8.tile_rows();
        sh.n_tiles = (N + sh.tile_rows - 1) / sh.tile_rows;
        const int resident = resident_workgroups(v8, &n_cus);
        sh.split = pick_split(K, sh.n_tiles, resident, n_cus);
        *var = v8;
        finish_shape(sh, max_rank, resident, n_cus, true);
        return sh;
    }
    if (wide_allowed(T)) {
        Variant wide{4, true, 8, q8};
        wide.allow_lean(lean_ok);
        const int resident = resident_workgroups(wide, &n_cus);
        const int n_tiles = (N + wide.tile_rows() - 1) / wide.tile_rows();
        const int split = pick_split(K, n_tiles, resident, n_cus);
        if (n_tiles * split <= resident && (g_wide_mode == 1 || n_tiles * split * 8 >= n_cus * 7)) {
            sh.tile_rows = wide.tile_rows();
            sh.n_tiles = n_tiles;
            sh.split = split;
            *var = wide;
            finish_shape(sh, max_rank, resident, n_cus, true);
            return sh;
        }
    }
    Variant v{tt, true, 4, q8};
    v.allow_lean(lean_ok);
    sh.tile_rows = v.tile_rows();
    sh.n_tiles = (N + sh.tile_rows - 1) / sh.tile_rows;
    int resident = resident_workgroups(v, &n_cus);
    sh.split = pick_split(K, sh.n_tiles, resident, n_cus);
    if (tt > 2 && !q8) {
        const Variant r{tt, false, 4};
        const int resident_r = resident_workgroups(r, &n_cus);
        const int split_r = pick_split(K, sh.n_tiles, resident_r, n_cus);
        const int wgs = sh.n_tiles * sh.split;
        if (split_r != sh.split && !(wgs <= n_cus && wgs * 20 >= n_cus * 19)) {
            v = r;
            resident = resident_r;
            sh.split = split_r;
        }
    }
    *var = v;
    finish_shape(sh, max_rank, resident, n_cus, true);
    return sh;
}

// everything that follows from T, K, N, jgroups, tile_rows, n_tiles and split
void finish_shape(DecodeShape &sh, int max_rank, int resident, int n_cus, bool surplus)
{
    sh.lgS = 0;
    while ((1 << sh.lgS) < sh.split) ++sh.lgS;
    sh.total = sh.n_tiles * sh.split;
    const int unit = kXcds * sh.split;
    sh.grid = (sh.total + unit - 1) / unit * unit;
    sh.real_per_xcd = sh.grid / kXcds;
    // A call that leaves compute units without a workgroup gets surplus ones for them: they only share in the shrink,
    // which for few output columns is most of the work (k_proj / v_proj at 64 rows: 2048 units of two rank rows on 128
    // workgroups).
    if (surplus && sh.jgroups > 1) {
        const int room = (resident < n_cus ? resident : n_cus) / unit * unit;
        if (room > sh.grid) sh.grid = room;
    }
    // the workgroups that share the shrink must all be running before anybody can wait for them
    sh.n_pub = sh.grid < resident ? sh.grid : resident;
    sh.G = sh.tile_rows / 4 / sh.split;
    sh.lgG = 0;
    while ((1 << sh.lgG) < sh.G) ++sh.lgG;
    sh.lgRp = 0;
    while ((1 << sh.lgRp) < max_rank) ++sh.lgRp;
    sh.spin_limit = g_spin_limit;
    sh.wait_ticks = g_wait_us * 100;
    sh.zero = 0;
    // the shortest K-slice has 2 * (chunks / split) sub-spans (up to 32 rows the turn did not pay: 15.6 -> 15.8 us)
    sh.rot_mask = 0;
    if (g_k_rotate && sh.T > 32) {
        int pow2 = 1;
        while (pow2 * 2 <= 2 * (sh.chunks / sh.split)) pow2 *= 2;
        sh.rot_mask = pow2 - 1;
    }
    int dev = 0;
    sh.local = (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < kMaxDevices && g_local[dev] == 1 && g_local_override != 0) ? 1 : 0;
}

// ---- is workgroup b of a launch placed on XCD b % 8? -----------------------------------------------
__global__ void xcc_probe_kernel(int *xcc_of_block) { xcc_of_block[blockIdx.x] = __builtin_amdgcn_s_getreg(20 | (31 << 11)) & 15; }  // HW_REG_XCC_ID

}  // namespace

// One small launch and a blocking copy: called from set-up code (workspace initialisation), never from a linear call.
// `scratch`: device memory the probe may overwrite (a corner of the workspace that is being initialised); with less
// than 1 KiB of it the device stays unprobed (such a workspace is too small for the decode kernel anyway).
int elora::decode_probe_device(void *scratch, size_t scratch_bytes, hipStream_t stream)
{
    int dev = 0;
    ELORA_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices || g_local[dev] != 0) return ELORA_OK;
    constexpr int n = 256;
    int h[n];
    if (scratch == nullptr || scratch_bytes < sizeof(h)) return ELORA_OK;
    int *d = static_cast<int *>(scratch);
    hipLaunchKernelGGL(xcc_probe_kernel, dim3(n), dim3(64), 0, stream, d);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(h, d, sizeof(h), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
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

// Several decode calls with the same number of rows in one launch, if K-slice counts can be found with which all
// their workgroups are resident together: starting from what each call would take alone, the call whose workgroups
// have the least to stream gives up half of its K-slices until the sum fits.  More than 32 rows: the wide kernel is
// tried first if its workgroups then cover at least seven eighths of the compute units; then W through LDS (one
// workgroup per compute unit); then W into registers, which leaves room for two per unit.
namespace {
bool group_splits(int T, int n, const int *K, const int *N, int *split, Variant *var, bool w8 = false, bool q8 = false, bool lean_ok = false)
{
    if (n < 2 || n > kGroupMax || T < 1 || T > kDecodeMaxTokens) return false;
    const int tt = (T + 15) / 16;
    Variant cand[3];
    int n_cand = 0;
    if (w8) {  // (an 8-bit W: through the ring on eight waves, into registers on four)
        if (wide_allowed(T)) cand[n_cand++] = Variant{4, true, 8, q8, true};
        cand[n_cand++] = Variant{tt == 3 ? 4 : tt, false, 4, q8, true};
    } else if (q8) {  // (adapters in 8-bit blocks: W through the ring always)
        if (wide_allowed(T)) cand[n_cand++] = Variant{4, true, 8, true, false};
        cand[n_cand++] = Variant{tt, true, 4, true, false};
    } else {
        if (wide_allowed(T)) cand[n_cand++] = Variant{4, true, 8};
        cand[n_cand++] = Variant{tt, true, 4};
        if (tt > 2) cand[n_cand++] = Variant{tt, false, 4};
        for (int i = 0; i < n_cand; ++i) cand[i].allow_lean(lean_ok);
    }
    for (int attempt = 0; attempt < n_cand; ++attempt) {
        const Variant v = cand[attempt];
        int n_cus = 0;
        (void)resident_workgroups(v, &n_cus);
        const int resident = resident_group_workgroups(v);
        if (resident <= 0) return false;
        int tiles[kGroupMax];
        auto grid_of = [&](int i) { return (tiles[i] * split[i] + kXcds * split[i] - 1) / (kXcds * split[i]) * (kXcds * split[i]); };
        for (int i = 0; i < n; ++i) {
            tiles[i] = (N[i] + v.tile_rows() - 1) / v.tile_rows();
            split[i] = pick_split(K[i], tiles[i], resident, n_cus);
        }
        for (;;) {
            int total = 0;
            for (int i = 0; i < n; ++i) total += grid_of(i);
            if (total <= resident) {
                if (v.nw > 4 && g_wide_mode != 1 && total * 8 < n_cus * 7) break;  // too few workgroups: the next kind
                *var = v;
                return true;
            }
            int pick = -1;  // least K per workgroup; among equals the larger grid
            for (int i = 0; i < n; ++i) {
                if (split[i] == 1) continue;
                if (pick < 0 || (long long)K[i] * split[pick] < (long long)K[pick] * split[i] ||
                    ((long long)K[i] * split[pick] == (long long)K[pick] * split[i] && grid_of(i) > grid_of(pick)))
                    pick = i;
            }
            if (pick < 0) break;
            split[pick] /= 2;
        }
    }
    return false;
}
}  // namespace

bool elora::decode_group_splits(int T, int n, const int *K, const int *N, int *split, bool *w_lds, bool w8, bool q8)
{
    Variant v{1, true, 4};
    const bool ok = group_splits(T, n, K, N, split, &v, w8, q8);
    if (ok) *w_lds = v.wlds;
    return ok;
}

// Returns ELORA_OK after the launch, -1 if the calls do not fit together (nothing enqueued).
int elora::launch_decode_group(const LinearArgs *a, int n, hipStream_t stream)
{
    if (n < 2 || n > kGroupMax) return -1;
    // W in the dtype of x in every call, or 8-bit in every call; the pools all bf16, or all in 8-bit blocks
    const bool w8 = a[0].wfmt == ELORA_W_INT8_G32;
    bool q8 = false;
    for (int i = 0; i < n; ++i) q8 = q8 || (a[i].has_pool && a[i].pool.q8);
    for (int i = 0; i < n; ++i)
        if ((a[i].has_pool && (a[i].pool.q8 != 0) != q8) || a[i].wfmt != a[0].wfmt || (a[i].wfmt != ELORA_W_SAME && !w8)) return -1;
    const int T = a[0].T;
    int Ks[kGroupMax], Ns[kGroupMax], split[kGroupMax];
    for (int i = 0; i < n; ++i) {
        if (a[i].T != T) return -1;
        Ks[i] = a[i].K;
        Ns[i] = a[i].N;
    }
    Variant var{1, true, 4};
    bool lean_ok = true;
    for (int i = 0; i < n; ++i) lean_ok = lean_ok && (!a[i].has_pool || ranks_fit_short_tail(a[i].pool.n_odd_ranks, a[i].pool.max_rank));
    if (!group_splits(T, n, Ks, Ns, split, &var, w8, q8, lean_ok)) return -1;
    int n_cus = 0;
    (void)resident_workgroups(var, &n_cus);
    const int resident = resident_group_workgroups(var);
    DecodeGroup grp;
    grp.n = n;
    int first = 0;
    for (int i = 0; i < n; ++i) {
        DecodeCall &c = grp.call[i];
        const int max_rank = a[i].has_pool ? a[i].pool.max_rank : 1;
        c.sh.w_scales = w8 ? static_cast<const uint16_t *>(a[i].w_scales) : nullptr;
        c.sh.T = T;
        c.sh.K = a[i].K;
        c.sh.N = a[i].N;
        c.sh.chunks = a[i].K / kChunk;
        c.sh.tile_rows = var.tile_rows();
        c.sh.n_tiles = (a[i].N + c.sh.tile_rows - 1) / c.sh.tile_rows;
        c.sh.jgroups = (max_rank + 1) / 2;
        c.sh.jg_inv = (unsigned)((1ull << 32) / (unsigned)c.sh.jgroups) + 1u;
        c.sh.split = split[i];
        finish_shape(c.sh, max_rank, resident, n_cus, false);
        c.sh.n_pub = c.sh.grid;  // the whole launch is resident
        c.x = static_cast<const uint16_t *>(a[i].x);
        c.W = static_cast<const uint16_t *>(a[i].W);
        c.pool = a[i].pool;
        c.route = a[i].route;
        c.has_pool = a[i].has_pool ? 1 : 0;
        c.mail = reinterpret_cast<float *>(a[i].ws + a[i].wsl.mail);
        c.vmail = reinterpret_cast<float *>(a[i].ws + a[i].wsl.vmail);
        c.sync = reinterpret_cast<int *>(a[i].ws + a[i].wsl.sync);
        c.y = static_cast<uint16_t *>(a[i].y);
        grp.first[i] = first;
        first += c.sh.grid;
    }
    for (int i = n; i <= kGroupMax; ++i) grp.first[i] = first;
    dim3 grid(first), block(var.threads());
    profile_mark_begin(stream);
    with_variant(var, [&](auto tt, auto wl, auto nw, auto q8c, auto w8c, auto ln) {
        constexpr int TT = decltype(tt)::value, NW = decltype(nw)::value;
        constexpr bool WL = decltype(wl)::value, Q8 = decltype(q8c)::value, W8 = decltype(w8c)::value, LN = decltype(ln)::value;
        hipLaunchKernelGGL((decode_group_kernel<TT, WL, NW, Q8, W8, LN>), grid, block, ring_bytes(TT, WL, NW, W8), stream, grp);
        return 0;
    });
    ELORA_HIP_TRY(hipGetLastError());
    profile_mark_end(stream);
    return ELORA_OK;
}

void elora::decode_set_spin_limit(int limit) { g_spin_limit = limit; }
void elora::decode_set_wait_us(int us) { g_wait_us = us; }
void elora::decode_set_local_override(int mode) { g_local_override = mode; }
void elora::decode_set_k_rotate(int on) { g_k_rotate = on; }
void elora::decode_set_wide(int mode) { g_wide_mode = mode; }
void elora::decode_set_passes(int mode) { g_pass_mode = mode; }

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

// Batches of 65 to 256 rows: too many for one launch of this kernel, too few to fill the device with the 256 x 256
// tiles of the MFMA GEMM path (at 4096 output columns that path has 16 workgroups for up to 256 rows), and with a
// different adapter in every row that path's shrink and expand work row by row.  Such a call runs as 2 to 4 launches
// of the decode kernel over balanced row ranges, each streaming W once.  Measured with per-row adapters of mixed rank,
// 4096 x 4096 / 4096 x 14336 / 14336 x 4096: 128 rows 47 / 91 / 90 us against 384 / 388 / 657 us on the GEMM path,
// 256 rows 88 / 171 / 167 us against 574 / 587 / 868 us.
int elora::decode_passes(const elora_linear_desc_t &d)
{
    const bool w_ok = d.wfmt == ELORA_W_SAME || d.wfmt == ELORA_W_INT8_G32;
    if (!(d.dtype == ELORA_BF16 && w_ok && d.n_tokens >= 1 && d.d_in % kChunk == 0 && d.d_out % 16 == 0)) return 0;
    const int passes = (d.n_tokens + kDecodeMaxTokens - 1) / kDecodeMaxTokens;
    if (passes == 1) return 1;
    if (passes > kDecodeMaxPasses || g_pass_mode == 0) return 0;
    return passes;
}

bool elora::decode_eligible(const elora_linear_desc_t &d, int max_rank)
{
    (void)max_rank;
    return decode_passes(d) >= 1;
}

// bytes of the piece mailboxes for d_out output columns: up to 8 K-slices, up to 64 rows (columns rounded up to
// whole tiles of the widest kernel)
size_t elora::decode_mail_bytes(int d_out)
{
    constexpr size_t wide_rows = 8 * kRowsPerWave;
    const size_t n_tiles = ((size_t)d_out + wide_rows - 1) / wide_rows;
    return n_tiles * kDecodeMaxSplit * kDecodeMaxTokens * wide_rows * sizeof(float);
}

void elora::decode_plan(const elora_linear_desc_t &d, elora_plan_t *plan)
{
    Variant var{1, true, 4};
    const int passes = decode_passes(d);
    const int rows = (d.n_tokens + passes - 1) / passes;  // the longest row range
    DecodeShape sh = make_shape(rows, d.d_in, d.d_out, d.pool ? d.pool->max_rank : 1, d.pool && d.pool->q8, &var,
                                d.wfmt == ELORA_W_INT8_G32 ? static_cast<const uint16_t *>(d.w_scales) : nullptr,
                                !d.pool || ranks_fit_short_tail(d.pool->n_odd_ranks, d.pool->max_rank));
    plan->n_launches = passes;
    plan->split_k = sh.split;
    plan->tile_rows = sh.tile_rows;
    plan->tile_cols = 0;
    plan->grid = sh.grid;
}

int elora::launch_decode(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream)
{
    (void)plan;
    Variant var{1, true, 4};
    DecodeShape sh = make_shape(a.T, a.K, a.N, a.has_pool ? a.pool.max_rank : 1, a.has_pool && a.pool.q8 != 0, &var,
                                a.wfmt == ELORA_W_INT8_G32 ? static_cast<const uint16_t *>(a.w_scales) : nullptr,
                                !a.has_pool || ranks_fit_short_tail(a.pool.n_odd_ranks, a.pool.max_rank));
    float *mail = reinterpret_cast<float *>(a.ws + a.wsl.mail);
    float *vmail = reinterpret_cast<float *>(a.ws + a.wsl.vmail);
    int *sync = reinterpret_cast<int *>(a.ws + a.wsl.sync);
    const uint16_t *x = static_cast<const uint16_t *>(a.x);
    const uint16_t *W = static_cast<const uint16_t *>(a.W);
    uint16_t *y = static_cast<uint16_t *>(a.y);
    int has_pool = a.has_pool ? 1 : 0;
    dim3 grid(sh.grid), block(var.threads());
    profile_mark_begin(stream);
    with_variant(var, [&](auto tt, auto wl, auto nw, auto q8, auto w8, auto ln) {
        constexpr int TT = decltype(tt)::value, NW = decltype(nw)::value;
        constexpr bool WL = decltype(wl)::value, Q8 = decltype(q8)::value, W8 = decltype(w8)::value, LN = decltype(ln)::value;
        hipLaunchKernelGGL((decode_kernel<TT, WL, NW, Q8, W8, LN>), grid, block, ring_bytes(TT, WL, NW, W8), stream, sh, x, W, a.pool, a.route, has_pool,
                           mail, vmail, sync, y);
        return 0;
    });
    ELORA_HIP_TRY(hipGetLastError());
    profile_mark_end(stream);
    return ELORA_OK;
}
