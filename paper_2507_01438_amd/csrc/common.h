// Shared declarations of libelora's translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/elora.h"

namespace elora {

// ---- device-visible views (passed to kernels by value) ---------------------

struct SlotMeta {  // one entry of the pool's device-side slot table
    int rank;      // 0 while the slot is empty
    float scale;   // alpha / rank
    int loaded;    // 1 once A and B are in place
    int pad;
};

struct PoolView {
    const SlotMeta *meta;  // [capacity]
    const char *slots;     // block 0; block i at slots + i * slot_bytes
    int *err;              // [0] = rows with a bad index so far, [1] = smallest such row (INT_MAX if none)
    size_t slot_bytes;     // A region [max_rank, d_in] then B region [d_out, rank] (row stride = rank)
    size_t b_offset;       // byte offset of the B region inside a block
    int capacity;
    int max_rank;
    // Adapters kept in 8-bit blocks (q8 != 0): the A and B regions hold int8 codes in the same shapes, and each is
    // followed by its fp16 scales, one per block of 32 consecutive values in row-major order (value = scale * code).
    int q8;
    size_t a_scale_off;    // byte offset of A's scales inside a block
    size_t b_scale_off;    // byte offset of B's scales inside a block
    // (host knowledge, for the choice of a kernel instance) loaded adapters whose rank is no multiple of 8: the decode
    // kernel's short tail only serves ranks that are, and instances without the general tail exist for pools without others
    int n_odd_ranks;
};

struct RouteView {
    const int32_t *adapter_idx;  // decode form, or nullptr
    const int32_t *seg_offsets;  // prefill form
    const int32_t *seg_adapter;
    int n_segments;
    const float *scales;  // per row (decode form) / per segment (prefill form), or nullptr
    int row_base;         // the tables speak of the batch's rows; row t of this launch is row t + row_base of the batch
};

struct RowRoute {
    int slot;     // validated pool slot, -1 = base model only
    int rank;     // 0 if slot < 0
    float scale;  // 0 if slot < 0
};

// Workspace sections (byte offsets from the 256-byte aligned base).
// The first three sections belong to the decode kernel, sit at offsets that do not depend on the batch, and
// are in their idle state between calls (counters zero, mailboxes all-ones); nothing else writes there.
struct WsLayout {
    size_t sync;       // int [kSyncInts] counters of the decode kernel
    size_t vmail;      // float [kDecodeMaxTokens][kMaxRank] mailbox for the shrink results of the decode kernel
    size_t mail;       // float mailboxes for the K-slice pieces of the decode kernel (decode_mail_bytes(d_out))
    size_t row_slot;   // int32 [T]
    size_t row_scale;  // float [T]
    size_t row_rank;   // int32 [T]
    size_t v;          // float/bf16 shrink results of the generic and gemm kernels
    size_t wdeq;       // bf16 [d_out][d_in]: a call's dequantised copy of a 4-bit or 8-bit W (gemm_wcopy_bytes(); 0 bytes below
    size_t wdeq_bytes; //   the row count from which converting W once pays)
    size_t total;
};

constexpr int kDecodeMaxTokens = 64;  // rows the streaming (decode) kernels take per launch
constexpr int kDecodeMaxPasses = 4;   // a call with more rows may run as this many launches of that kernel at most
constexpr int kDecodeMaxSplit = 8;    // K-splits of the base contraction
constexpr int kMaxRank = 256;
constexpr int kSyncInts = 1024;       // ints in the workspace's counter area

WsLayout ws_layout(int n_tokens, int d_in, int d_out, int max_rank, int wfmt);

// ---- host-side pool object --------------------------------------------------

}  // namespace elora

struct elora_pool {
    int d_in, d_out, max_rank, capacity, dtype;
    int q8;  // 1: adapters stay in 8-bit blocks (dtype is then that of x and y: bf16)
    size_t a_scale_off, b_scale_off;
    char *storage;
    size_t storage_bytes;
    size_t meta_offset, slots_offset, slot_bytes, b_offset;
    bool device_cleared;
    elora::SlotMeta *host_meta;  // mirror of the device slot table (written through set_host_meta)
    int n_odd_ranks;             // loaded slots whose rank is no multiple of 8
    void set_host_meta(int slot, const elora::SlotMeta &m)
    {
        n_odd_ranks += (int)(m.loaded && (m.rank & 7) != 0) - (int)(host_meta[slot].loaded && (host_meta[slot].rank & 7) != 0);
        host_meta[slot] = m;
    }
    elora::PoolView view() const;
};

namespace elora {

// lazily clears the device slot table; enqueued on `stream`
int pool_ensure_cleared(elora_pool *pool, hipStream_t stream);

struct LinearArgs {
    int T, K, N;
    int dtype, wfmt;
    const void *x, *W, *w_scales;
    void *y;
    bool has_pool;
    PoolView pool;
    RouteView route;
    char *ws;
    WsLayout wsl;
};

int launch_generic(const LinearArgs &a, hipStream_t stream);
int launch_decode(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream);
int launch_gemm(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream);
bool gemm_group_shares_shrink(const LinearArgs *a, int n);  // same x and routing tables, a pool each: one shrink launch serves all
int launch_gemm_group(const LinearArgs *a, int n, hipStream_t stream);
int launch_decode_group(const LinearArgs *a, int n, hipStream_t stream);  // -1: the calls do not fit into one launch
bool decode_group_splits(int T, int n, const int *K, const int *N, int *split, bool *w_lds, bool w8 = false, bool q8 = false);  // K-slices per call if they fit

void decode_set_spin_limit(int limit);
void decode_set_wait_us(int us);
void gemm_set_w4_copy_rows(int rows);
void decode_set_passes(int mode);  // -1: several launches per call where they pay, 0: never, 1: whenever the row count allows
void decode_set_wide(int mode);    // -1: 128-row tiles where they pay, 0: never, 1: wherever the shape allows
void decode_set_k_rotate(int on);  // 0: every workgroup walks its K-slice from the start
void decode_set_local_override(int mode);  // 0: never assume XCD-local hand-overs, -1: as probed
int decode_probe_device(void *scratch, size_t scratch_bytes, hipStream_t stream);  // finds out, once per device, how workgroups are placed on the XCDs
bool decode_eligible(const elora_linear_desc_t &d, int max_rank);
int decode_passes(const elora_linear_desc_t &d);  // launches of the decode kernel this call is cut into (1 up to 64 rows), 0: not that path
void decode_plan(const elora_linear_desc_t &d, elora_plan_t *plan);
size_t decode_mail_bytes(int d_out);  // mailboxes of the decode kernel for d_out output columns
bool gemm_eligible(const elora_linear_desc_t &d, int max_rank);
void gemm_plan(const elora_linear_desc_t &d, elora_plan_t *plan);
size_t gemm_wcopy_bytes(int wfmt, int n_tokens, int d_in, int d_out);  // (see below)
size_t gemm_w4_bytes(int n_tokens, int d_in, int d_out);  // room for the bf16 copy of a 4-bit W; 0: converted tile by tile
size_t gemm_v_bytes(int n_tokens, int max_rank);  // bf16 shrink results, rank padded to the GEMM's K block

// benchmark hook: bracket the dominant kernel of a call with events when armed
void profile_mark_begin(hipStream_t stream);
void profile_mark_end(hipStream_t stream);

#define ELORA_HIP_TRY(expr)                  \
    do {                                     \
        if ((expr) != hipSuccess) {          \
            (void)hipGetLastError();         \
            return ELORA_E_HIP;              \
        }                                    \
    } while (0)

// ---- device helpers ----------------------------------------------------------

#if defined(__HIPCC__)

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even; NaN stays NaN (quiet)
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float fp16_to_f32(uint16_t h)
{
    _Float16 v;
    __builtin_memcpy(&v, &h, 2);
    return (float)v;
}

template <typename E> __device__ __forceinline__ float load_elem(const E *p, size_t i);
template <> __device__ __forceinline__ float load_elem<float>(const float *p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float load_elem<uint16_t>(const uint16_t *p, size_t i) { return bf16_to_f32(p[i]); }

template <typename E> __device__ __forceinline__ void store_elem(E *p, size_t i, float v);
template <> __device__ __forceinline__ void store_elem<float>(float *p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void store_elem<uint16_t>(uint16_t *p, size_t i, float v) { p[i] = f32_to_bf16(v); }

// Which adapter row t uses (Sec. 3.4: every request of the batch names its own adapter), in two steps so
// that a caller can put other work between the dependent loads.
// Step 1: the index the routing tables give for row t (-1 = none) and where its scale override sits.
struct RouteIndex {
    int idx;
    int scale_at;
};
__device__ __forceinline__ RouteIndex route_index(int t, const RouteView &r)
{
    t += r.row_base;
    RouteIndex out{-1, t};
    if (r.adapter_idx != nullptr) {
        out.idx = r.adapter_idx[t];
    } else {
        // last segment s with seg_offsets[s] <= t (empty segments have equal offsets and are skipped over)
        int lo = 0, hi = r.n_segments;  // invariant: seg_offsets[lo] <= t < seg_offsets[hi]
        while (hi - lo > 1) {
            int mid = (lo + hi) >> 1;
            if (r.seg_offsets[mid] <= t) lo = mid; else hi = mid;
        }
        out.idx = (r.n_segments > 0 && r.seg_offsets[lo] <= t && t < r.seg_offsets[lo + 1]) ? r.seg_adapter[lo] : -1;
        out.scale_at = lo;
    }
    return out;
}
// Step 2: validate against the slot's table entry `m` (read from p.meta[idx] by the caller when idx is inside the
// pool, anything otherwise) and pick the scale (`scale_override` = r.scales[ri.scale_at], read by the caller when
// r.scales is given and idx is not -1).  Index -1 means none.  Any other index outside the pool, or naming an
// empty slot, is turned into "none" and, if `record`, counted in the pool's sticky error record.
__device__ __forceinline__ RowRoute route_finish(int t, const RouteIndex &ri, const SlotMeta &m, float scale_override,
                                                 const RouteView &r, const PoolView &p, bool record)
{
    RowRoute out{-1, 0, 0.0f};
    if (ri.idx == -1) return out;
    const bool ok = ri.idx >= 0 && ri.idx < p.capacity && m.loaded == 1 && m.rank >= 1 && m.rank <= p.max_rank;
    if (!ok) {
        if (record) {
            atomicAdd(&p.err[0], 1);
            atomicMin(&p.err[1], t + r.row_base);
        }
        return out;
    }
    out.slot = ri.idx;
    out.rank = m.rank;
    out.scale = (r.scales != nullptr) ? scale_override : m.scale;
    return out;
}
__device__ __forceinline__ RowRoute resolve_row(int t, const RouteView &r, const PoolView &p, bool record)
{
    const RouteIndex ri = route_index(t, r);
    SlotMeta m{0, 0.0f, 0, 0};
    if (ri.idx >= 0 && ri.idx < p.capacity) m = p.meta[ri.idx];
    const float so = (r.scales != nullptr && ri.idx != -1) ? r.scales[ri.scale_at] : 0.0f;
    return route_finish(t, ri, m, so, r, p, record);
}

typedef uint32_t elora_u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 elora_bf16x2 __attribute__((ext_vector_type(2)));

// Sum over the 64 lanes of a wave, the same value in every lane, with cross-lane operations of the vector ALU only
// (quad permutes and row mirrors inside rows of 16 lanes, then one lane of each row).  Unlike a shuffle it is no
// LDS-pipeline instruction, so it does not wait for direct-to-LDS loads that happen to be in flight.
__device__ __forceinline__ float wave_sum(float v)
{
    int b = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, b, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
    b = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, b, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
    b = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, b, 0x141, 0xF, 0xF, false));  // row_half_mirror
    b = __float_as_int(v);
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, b, 0x140, 0xF, 0xF, false));  // row_mirror
    b = __float_as_int(v);
    return (__int_as_float(__builtin_amdgcn_readlane(b, 0)) + __int_as_float(__builtin_amdgcn_readlane(b, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(b, 32)) + __int_as_float(__builtin_amdgcn_readlane(b, 48)));
}

// One wave: v[t][j0], v[t][j0+1] = A_i[j0..j0+1, :] . x[t, :] over the whole of K (K % 256 == 0).
// NL: 16-byte pieces per row, lane and round trip to memory (3 NL loads in flight per lane).
template <int NL = 8>
__device__ __forceinline__ void shrink_pair(const uint16_t *__restrict__ A0, const uint16_t *__restrict__ A1,
                                            const uint16_t *__restrict__ xt, int K, int lane, float &r0, float &r1)
{
    float s0 = 0.0f, s1 = 0.0f;
    const int pieces = K >> 3;  // 16-byte pieces per row
    for (int pb = 0; pb < pieces; pb += 64 * NL) {
        elora_u32x4 xv[NL], a0[NL], a1[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int p = pb + i * 64 + lane;
            const bool in = p < pieces;
            const size_t off = (size_t)(in ? p : 0) * 8;
            xv[i] = *reinterpret_cast<const elora_u32x4 *>(xt + off);
            a0[i] = __builtin_nontemporal_load(reinterpret_cast<const elora_u32x4 *>(A0 + off));
            a1[i] = __builtin_nontemporal_load(reinterpret_cast<const elora_u32x4 *>(A1 + off));
        }
        __builtin_amdgcn_sched_barrier(0);  // keep all loads of a round in flight together: do not interleave the math
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            if (pb + i * 64 + lane >= pieces) xv[i] = elora_u32x4{0, 0, 0, 0};  // past the row: contributes nothing
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                // two bf16 products and the running sum in one instruction (products exact, fp32 accumulation)
                // (elements are copied to scalars first: a bit cast straight from a vector element picks element 0)
                const uint32_t xw = xv[i][q], aw0 = a0[i][q], aw1 = a1[i][q];
                s0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(elora_bf16x2, aw0), __builtin_bit_cast(elora_bf16x2, xw), s0, false);
                s1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(elora_bf16x2, aw1), __builtin_bit_cast(elora_bf16x2, xw), s1, false);
            }
        }
    }
    r0 = wave_sum(s0);
    r1 = wave_sum(s1);
}

__device__ __forceinline__ const uint16_t *slot_A_scales(const PoolView &p, int slot)
{
    return reinterpret_cast<const uint16_t *>(p.slots + (size_t)slot * p.slot_bytes + p.a_scale_off);
}
__device__ __forceinline__ const uint16_t *slot_B_scales(const PoolView &p, int slot)
{
    return reinterpret_cast<const uint16_t *>(p.slots + (size_t)slot * p.slot_bytes + p.b_scale_off);
}
// entry `idx` (row-major) of a matrix kept in 8-bit blocks: the block's scale times the code (exact in fp32)
__device__ __forceinline__ float q8_elem(const char *codes, const uint16_t *scales, size_t idx)
{
    return fp16_to_f32(scales[idx >> 5]) * (float)reinterpret_cast<const int8_t *>(codes)[idx];
}
// sum of code[j] * x[j] over 16 consecutive values: codes in c (4 per word, signed), x as 16 bf16 in xa, xb
__device__ __forceinline__ float q8_dot16(const elora_u32x4 &c, const elora_u32x4 &xa, const elora_u32x4 &xb)
{
    float s = 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t cw = c[q];
        const uint32_t x01 = q < 2 ? xa[2 * q] : xb[2 * q - 4], x23 = q < 2 ? xa[2 * q + 1] : xb[2 * q - 3];
        s = fmaf((float)(int8_t)(cw & 0xffu), __uint_as_float(x01 << 16), s);
        s = fmaf((float)(int8_t)((cw >> 8) & 0xffu), __uint_as_float(x01 & 0xffff0000u), s);
        s = fmaf((float)(int8_t)((cw >> 16) & 0xffu), __uint_as_float(x23 << 16), s);
        s = fmaf((float)(int8_t)(cw >> 24), __uint_as_float(x23 & 0xffff0000u), s);
    }
    return s;
}

// One wave: v[t][j0], v[t][j0+1] = A_i[j0..j0+1, :] . x[t, :] over the whole of K for an adapter kept in 8-bit blocks
// (K % 256 == 0): 16 codes per lane and load, every 16 inside one block of 32, so one scale per load.
__device__ __forceinline__ void shrink_pair_q8(const char *__restrict__ A0, const char *__restrict__ A1,
                                               const uint16_t *__restrict__ S0, const uint16_t *__restrict__ S1,
                                               const uint16_t *__restrict__ xt, int K, int lane, float &r0, float &r1)
{
    float s0 = 0.0f, s1 = 0.0f;
    const int pieces = K >> 4;  // 16-value pieces per row
    for (int pb = 0; pb < pieces; pb += 64 * 4) {
        elora_u32x4 xa[4], xb[4], c0[4], c1[4];
        uint16_t sc0[4], sc1[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int p = pb + i * 64 + lane;
            const size_t pc = (size_t)(p < pieces ? p : 0);
            xa[i] = *reinterpret_cast<const elora_u32x4 *>(xt + pc * 16);
            xb[i] = *reinterpret_cast<const elora_u32x4 *>(xt + pc * 16 + 8);
            c0[i] = __builtin_nontemporal_load(reinterpret_cast<const elora_u32x4 *>(A0 + pc * 16));
            c1[i] = __builtin_nontemporal_load(reinterpret_cast<const elora_u32x4 *>(A1 + pc * 16));
            sc0[i] = S0[pc >> 1];
            sc1[i] = S1[pc >> 1];
        }
        __builtin_amdgcn_sched_barrier(0);  // all loads of a round in flight together
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (pb + i * 64 + lane < pieces) {
                s0 = fmaf(fp16_to_f32(sc0[i]), q8_dot16(c0[i], xa[i], xb[i]), s0);
                s1 = fmaf(fp16_to_f32(sc1[i]), q8_dot16(c1[i], xa[i], xb[i]), s1);
            }
        }
    }
    r0 = wave_sum(s0);
    r1 = wave_sum(s1);
}

__device__ __forceinline__ const char *slot_A(const PoolView &p, int slot) { return p.slots + (size_t)slot * p.slot_bytes; }
__device__ __forceinline__ const char *slot_B(const PoolView &p, int slot) { return p.slots + (size_t)slot * p.slot_bytes + p.b_offset; }

#endif  // __HIPCC__

}  // namespace elora
