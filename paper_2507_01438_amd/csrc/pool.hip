// The resident adapter pool (Sec. 3.3 / 4.2 of the paper: fixed-size pre-allocated blocks, one
// per adapter, assigned and released at run time without allocating memory).
//
// Device layout inside the caller's storage (all sections 256-byte aligned):
//   [0, 256)            error record: int n_bad_rows, int first_bad_row
//   [meta_offset, ..)   SlotMeta[capacity]
//   [slots_offset, ..)  capacity blocks of slot_bytes:
//                         A region: [rank, d_in] row-major at the block start (room for max_rank rows)
//                         B region: [d_out, rank] row-major at b_offset, row stride = the adapter's
//                                   own rank (packed, so a low-rank adapter in a max_rank block is
//                                   read as one contiguous stream)
#include <limits.h>
#include <new>

#include "common.h"

using namespace elora;

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
size_t elem_bytes(int dtype) { return dtype == ELORA_F32 ? 4 : 2; }

bool pool_dims_ok(int d_in, int d_out, int max_rank, int capacity, int dtype)
{
    return d_in > 0 && d_out > 0 && capacity > 0 && max_rank >= 1 && max_rank <= kMaxRank &&
           (dtype == ELORA_F32 || dtype == ELORA_BF16);
}

__global__ void pool_clear_kernel(int *err, SlotMeta *meta, int capacity)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        err[0] = 0;
        err[1] = INT_MAX;
    }
    if (i < capacity) meta[i] = SlotMeta{0, 0.0f, 0, 0};
}

__global__ void pool_set_meta_kernel(SlotMeta *meta, int slot, int rank, float scale, int loaded)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) meta[slot] = SlotMeta{rank, scale, loaded, 0};
}

// Several adapters in one launch: the GPU reads the sources itself (device memory, or pinned host memory across the
// bus) and fills the blocks; entry blockIdx.y, 16 bytes per thread and step.  Nothing else may use these blocks
// meanwhile (the caller orders that), so the table entries can be written by the same launch.
constexpr int kLoadBatch = 16;
struct LoadBatch {
    int n;
    int slot[kLoadBatch], rank[kLoadBatch];
    float scale[kLoadBatch];
    const uint4 *A[kLoadBatch], *B[kLoadBatch];
    unsigned a_vecs[kLoadBatch], b_vecs[kLoadBatch];  // 16-byte pieces of A and of B
};

__global__ __launch_bounds__(256) void pool_load_batch_kernel(LoadBatch lb, char *slots, size_t slot_bytes, size_t b_offset,
                                                              SlotMeta *meta)
{
    const int e = blockIdx.y;
    uint4 *dst_a = reinterpret_cast<uint4 *>(slots + (size_t)lb.slot[e] * slot_bytes);
    uint4 *dst_b = reinterpret_cast<uint4 *>(slots + (size_t)lb.slot[e] * slot_bytes + b_offset);
    const unsigned na = lb.a_vecs[e], total = na + lb.b_vecs[e];
    for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        if (i < na) dst_a[i] = lb.A[e][i];
        else dst_b[i - na] = lb.B[e][i - na];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) meta[lb.slot[e]] = SlotMeta{lb.rank[e], lb.scale[e], 1, 0};
}

// The same for adapters kept in 8-bit blocks (32 consecutive values, one fp16 scale, value = scale * code): the
// blocks are turned into the pool's bf16 on the way in.  One thread per 8 values: 8 bytes of codes in, 16 bytes out,
// four threads share a scale.  scale * code is exact in fp32 (11-bit times 8-bit significand); one rounding to bf16.
struct LoadBatchQ8 {
    int n;
    int slot[kLoadBatch], rank[kLoadBatch];
    float scale[kLoadBatch];
    const uint2 *A[kLoadBatch], *B[kLoadBatch];
    const uint16_t *As[kLoadBatch], *Bs[kLoadBatch];
    unsigned a_vecs[kLoadBatch], b_vecs[kLoadBatch];  // groups of 8 values of A and of B
};

__device__ __forceinline__ uint4 q8_to_bf16x8(uint2 codes, uint16_t scale_bits)
{
    const float sc = fp16_to_f32(scale_bits);
    const uint32_t w[2] = {codes.x, codes.y};
    uint32_t out[4];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const float lo = sc * (float)(int8_t)((w[h] >> (16 * p)) & 0xffu), hi = sc * (float)(int8_t)((w[h] >> (16 * p + 8)) & 0xffu);
            out[h * 2 + p] = (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
        }
    return uint4{out[0], out[1], out[2], out[3]};
}

__global__ __launch_bounds__(256) void pool_load_q8_batch_kernel(LoadBatchQ8 lb, char *slots, size_t slot_bytes, size_t b_offset,
                                                                 SlotMeta *meta)
{
    const int e = blockIdx.y;
    uint4 *dst_a = reinterpret_cast<uint4 *>(slots + (size_t)lb.slot[e] * slot_bytes);
    uint4 *dst_b = reinterpret_cast<uint4 *>(slots + (size_t)lb.slot[e] * slot_bytes + b_offset);
    const unsigned na = lb.a_vecs[e], total = na + lb.b_vecs[e];
    for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        if (i < na) dst_a[i] = q8_to_bf16x8(lb.A[e][i], lb.As[e][i >> 2]);
        else dst_b[i - na] = q8_to_bf16x8(lb.B[e][i - na], lb.Bs[e][(i - na) >> 2]);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) meta[lb.slot[e]] = SlotMeta{lb.rank[e], lb.scale[e], 1, 0};
}

// Adapters that stay in their 8-bit blocks (a pool created by elora_pool_create_q8): codes and scales are copied as
// they are, 8 bytes of codes or 2 bytes of scales per thread and step.
struct LoadBatchQ8Keep {
    int n;
    int slot[kLoadBatch], rank[kLoadBatch];
    float scale[kLoadBatch];
    const uint2 *A[kLoadBatch], *B[kLoadBatch];
    const uint16_t *As[kLoadBatch], *Bs[kLoadBatch];
    unsigned a_vals[kLoadBatch], b_vals[kLoadBatch];  // values of A and of B
};
__global__ __launch_bounds__(256) void pool_keep_q8_batch_kernel(LoadBatchQ8Keep lb, char *slots, size_t slot_bytes, size_t a_scale_off,
                                                                 size_t b_offset, size_t b_scale_off, SlotMeta *meta)
{
    const int e = blockIdx.y;
    char *block = slots + (size_t)lb.slot[e] * slot_bytes;
    const unsigned na = lb.a_vals[e] / 8, nb = lb.b_vals[e] / 8, nas = lb.a_vals[e] / 32, nbs = lb.b_vals[e] / 32;
    const unsigned total = na + nb + nas + nbs;
    for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < total; i += gridDim.x * blockDim.x) {
        if (i < na) reinterpret_cast<uint2 *>(block)[i] = lb.A[e][i];
        else if (i < na + nb) reinterpret_cast<uint2 *>(block + b_offset)[i - na] = lb.B[e][i - na];
        else if (i < na + nb + nas) reinterpret_cast<uint16_t *>(block + a_scale_off)[i - na - nb] = lb.As[e][i - na - nb];
        else reinterpret_cast<uint16_t *>(block + b_scale_off)[i - na - nb - nas] = lb.Bs[e][i - na - nb - nas];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) meta[lb.slot[e]] = SlotMeta{lb.rank[e], lb.scale[e], 1, 0};
}

__global__ void pool_clear_err_kernel(int *err)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        err[0] = 0;
        err[1] = INT_MAX;
    }
}

}  // namespace

PoolView elora_pool::view() const
{
    PoolView v;
    v.meta = reinterpret_cast<const SlotMeta *>(storage + meta_offset);
    v.slots = storage + slots_offset;
    v.err = reinterpret_cast<int *>(storage);
    v.slot_bytes = slot_bytes;
    v.b_offset = b_offset;
    v.capacity = capacity;
    v.max_rank = max_rank;
    v.q8 = q8;
    v.a_scale_off = a_scale_off;
    v.b_scale_off = b_scale_off;
    v.n_odd_ranks = n_odd_ranks;
    return v;
}

int elora::pool_ensure_cleared(elora_pool *pool, hipStream_t stream)
{
    if (pool->device_cleared) return ELORA_OK;
    int blocks = (pool->capacity + 255) / 256;
    hipLaunchKernelGGL(pool_clear_kernel, dim3(blocks), dim3(256), 0, stream,
                       reinterpret_cast<int *>(pool->storage),
                       reinterpret_cast<SlotMeta *>(pool->storage + pool->meta_offset), pool->capacity);
    ELORA_HIP_TRY(hipGetLastError());
    pool->device_cleared = true;
    return ELORA_OK;
}

extern "C" {

size_t elora_pool_storage_bytes(int d_in, int d_out, int max_rank, int capacity, int dtype)
{
    if (!pool_dims_ok(d_in, d_out, max_rank, capacity, dtype)) return 0;
    size_t e = elem_bytes(dtype);
    size_t a_bytes = align_up((size_t)max_rank * d_in * e);
    size_t b_bytes = align_up((size_t)max_rank * d_out * e);
    return kAlign + align_up(sizeof(SlotMeta) * (size_t)capacity) + (a_bytes + b_bytes) * (size_t)capacity;
}

int elora_pool_create(int d_in, int d_out, int max_rank, int capacity, int dtype, void *dev_storage,
                      size_t storage_bytes, elora_pool_t **out)
{
    if (out == nullptr || dev_storage == nullptr) return ELORA_E_NULL;
    if (dtype != ELORA_F32 && dtype != ELORA_BF16) return ELORA_E_DTYPE;
    if (d_in <= 0 || d_out <= 0 || capacity <= 0) return ELORA_E_SHAPE;
    if (max_rank < 1 || max_rank > kMaxRank) return ELORA_E_RANK;
    if (reinterpret_cast<uintptr_t>(dev_storage) % kAlign) return ELORA_E_ALIGN;
    size_t need = elora_pool_storage_bytes(d_in, d_out, max_rank, capacity, dtype);
    if (storage_bytes < need) return ELORA_E_STORAGE;

    elora_pool *p = new (std::nothrow) elora_pool;
    if (p == nullptr) return ELORA_E_STORAGE;  // out of host memory
    p->host_meta = new (std::nothrow) SlotMeta[capacity];
    if (p->host_meta == nullptr) {
        delete p;
        return ELORA_E_STORAGE;
    }
    for (int i = 0; i < capacity; ++i) p->host_meta[i] = SlotMeta{0, 0.0f, 0, 0};
    p->n_odd_ranks = 0;
    size_t e = elem_bytes(dtype);
    p->d_in = d_in;
    p->d_out = d_out;
    p->max_rank = max_rank;
    p->capacity = capacity;
    p->dtype = dtype;
    p->storage = static_cast<char *>(dev_storage);
    p->storage_bytes = storage_bytes;
    p->meta_offset = kAlign;
    p->slots_offset = kAlign + align_up(sizeof(SlotMeta) * (size_t)capacity);
    p->q8 = 0;
    p->a_scale_off = p->b_scale_off = 0;
    p->b_offset = align_up((size_t)max_rank * d_in * e);
    p->slot_bytes = p->b_offset + align_up((size_t)max_rank * d_out * e);
    p->device_cleared = false;
    *out = p;
    return ELORA_OK;
}

// block of a pool whose adapters stay in 8-bit blocks: A codes [max_rank, d_in], A scales, B codes [d_out, max_rank], B scales
static void q8_block_layout(int d_in, int d_out, int max_rank, size_t *a_scale_off, size_t *b_offset, size_t *b_scale_off, size_t *slot_bytes)
{
    const size_t a_vals = (size_t)max_rank * d_in, b_vals = (size_t)max_rank * d_out;
    *a_scale_off = align_up(a_vals);
    *b_offset = *a_scale_off + align_up(a_vals / 32 * 2);
    *b_scale_off = *b_offset + align_up(b_vals);
    *slot_bytes = *b_scale_off + align_up((b_vals + 31) / 32 * 2);
}

static bool q8_dims_ok(int d_in, int d_out, int max_rank, int capacity)
{
    return pool_dims_ok(d_in, d_out, max_rank, capacity, ELORA_BF16) && d_in % 32 == 0 && d_out % 4 == 0 && max_rank % 8 == 0;
}

size_t elora_pool_storage_bytes_q8(int d_in, int d_out, int max_rank, int capacity)
{
    if (!q8_dims_ok(d_in, d_out, max_rank, capacity)) return 0;
    size_t aso, bo, bso, sb;
    q8_block_layout(d_in, d_out, max_rank, &aso, &bo, &bso, &sb);
    return kAlign + align_up(sizeof(SlotMeta) * (size_t)capacity) + sb * (size_t)capacity;
}

int elora_pool_create_q8(int d_in, int d_out, int max_rank, int capacity, void *dev_storage, size_t storage_bytes,
                         elora_pool_t **out)
{
    if (out == nullptr || dev_storage == nullptr) return ELORA_E_NULL;
    if (d_in <= 0 || d_out <= 0 || capacity <= 0 || d_in % 32 != 0 || d_out % 4 != 0) return ELORA_E_SHAPE;
    if (max_rank < 8 || max_rank > kMaxRank || max_rank % 8 != 0) return ELORA_E_RANK;
    if (reinterpret_cast<uintptr_t>(dev_storage) % kAlign) return ELORA_E_ALIGN;
    if (storage_bytes < elora_pool_storage_bytes_q8(d_in, d_out, max_rank, capacity)) return ELORA_E_STORAGE;
    elora_pool *p = new (std::nothrow) elora_pool;
    if (p == nullptr) return ELORA_E_STORAGE;
    p->host_meta = new (std::nothrow) SlotMeta[capacity];
    if (p->host_meta == nullptr) {
        delete p;
        return ELORA_E_STORAGE;
    }
    for (int i = 0; i < capacity; ++i) p->host_meta[i] = SlotMeta{0, 0.0f, 0, 0};
    p->n_odd_ranks = 0;
    p->d_in = d_in;
    p->d_out = d_out;
    p->max_rank = max_rank;
    p->capacity = capacity;
    p->dtype = ELORA_BF16;
    p->q8 = 1;
    p->storage = static_cast<char *>(dev_storage);
    p->storage_bytes = storage_bytes;
    p->meta_offset = kAlign;
    p->slots_offset = kAlign + align_up(sizeof(SlotMeta) * (size_t)capacity);
    q8_block_layout(d_in, d_out, max_rank, &p->a_scale_off, &p->b_offset, &p->b_scale_off, &p->slot_bytes);
    p->device_cleared = false;
    *out = p;
    return ELORA_OK;
}

int elora_pool_destroy(elora_pool_t *pool)
{
    if (pool == nullptr) return ELORA_E_NULL;
    delete[] pool->host_meta;
    delete pool;
    return ELORA_OK;
}

int elora_pool_load_adapter(elora_pool_t *pool, int slot, int rank, float scale, const void *A, const void *B,
                            int src_on_device, elora_stream_t stream_)
{
    if (pool == nullptr || A == nullptr || B == nullptr) return ELORA_E_NULL;
    if (pool->q8) return ELORA_E_DTYPE;  // this pool holds 8-bit blocks: elora_pool_load_adapters_q8
    if (slot < 0 || slot >= pool->capacity) return ELORA_E_SLOT;
    if (rank < 1 || rank > pool->max_rank) return ELORA_E_RANK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = pool_ensure_cleared(pool, stream);
    if (rc != ELORA_OK) return rc;
    size_t e = elem_bytes(pool->dtype);
    char *block = pool->storage + pool->slots_offset + (size_t)slot * pool->slot_bytes;
    hipMemcpyKind kind = src_on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
    SlotMeta *dmeta = reinterpret_cast<SlotMeta *>(pool->storage + pool->meta_offset);
    // the slot reads as empty while its content is being replaced
    hipLaunchKernelGGL(pool_set_meta_kernel, dim3(1), dim3(64), 0, stream, dmeta, slot, 0, 0.0f, 0);
    ELORA_HIP_TRY(hipGetLastError());
    pool->set_host_meta(slot, SlotMeta{0, 0.0f, 0, 0});
    ELORA_HIP_TRY(hipMemcpyAsync(block, A, (size_t)rank * pool->d_in * e, kind, stream));
    ELORA_HIP_TRY(hipMemcpyAsync(block + pool->b_offset, B, (size_t)rank * pool->d_out * e, kind, stream));
    hipLaunchKernelGGL(pool_set_meta_kernel, dim3(1), dim3(64), 0, stream, dmeta, slot, rank, scale, 1);
    ELORA_HIP_TRY(hipGetLastError());
    pool->set_host_meta(slot, SlotMeta{rank, scale, 1, 0});
    return ELORA_OK;
}

// Where the device can read `p` from: p itself for device memory, the device-side address for pinned host memory,
// nullptr for anything else (ordinary host memory).
static const void *device_readable(const void *p, bool *is_device)
{
    hipPointerAttribute_t attr;
    *is_device = false;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (attr.type == hipMemoryTypeDevice) {
        *is_device = true;
        return p;
    }
    if (attr.type == hipMemoryTypeHost) return attr.devicePointer;
    return nullptr;
}

int elora_pool_load_adapters(elora_pool_t *pool, int n, const int *slots, const int *ranks, const float *scales,
                             const void *const *A, const void *const *B, elora_stream_t stream_)
{
    if (pool == nullptr || (n > 0 && (!slots || !ranks || !scales || !A || !B))) return ELORA_E_NULL;
    if (n < 0) return ELORA_E_SHAPE;
    if (pool->q8) return ELORA_E_DTYPE;
    for (int i = 0; i < n; ++i) {
        if (A[i] == nullptr || B[i] == nullptr) return ELORA_E_NULL;
        if (slots[i] < 0 || slots[i] >= pool->capacity) return ELORA_E_SLOT;
        if (ranks[i] < 1 || ranks[i] > pool->max_rank) return ELORA_E_RANK;
        for (int j = 0; j < i; ++j)
            if (slots[j] == slots[i]) return ELORA_E_SLOT;  // one block, two adapters
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = pool_ensure_cleared(pool, stream);
    if (rc != ELORA_OK) return rc;
    const size_t e = elem_bytes(pool->dtype);
    SlotMeta *dmeta = reinterpret_cast<SlotMeta *>(pool->storage + pool->meta_offset);
    for (int i0 = 0; i0 < n; i0 += kLoadBatch) {
        LoadBatch lb;
        lb.n = n - i0 < kLoadBatch ? n - i0 : kLoadBatch;
        bool direct = true, on_device[kLoadBatch], b_on_device = false;
        size_t most = 0;
        for (int i = 0; i < lb.n; ++i) {
            const size_t a_bytes = (size_t)ranks[i0 + i] * pool->d_in * e, b_bytes = (size_t)ranks[i0 + i] * pool->d_out * e;
            const void *a = device_readable(A[i0 + i], &on_device[i]), *b = device_readable(B[i0 + i], &b_on_device);
            if (on_device[i] != b_on_device) direct = false;  // (then the copy engine sorts it out, or reports it)
            direct = direct && a && b && a_bytes % 16 == 0 && b_bytes % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(a) % 16 == 0 && reinterpret_cast<uintptr_t>(b) % 16 == 0;
            lb.slot[i] = slots[i0 + i];
            lb.rank[i] = ranks[i0 + i];
            lb.scale[i] = scales[i0 + i];
            lb.A[i] = static_cast<const uint4 *>(a);
            lb.B[i] = static_cast<const uint4 *>(b);
            lb.a_vecs[i] = (unsigned)(a_bytes / 16);
            lb.b_vecs[i] = (unsigned)(b_bytes / 16);
            most = a_bytes + b_bytes > most ? a_bytes + b_bytes : most;
        }
        if (!direct) {
            // ordinary host memory, or sizes that are no multiple of 16 bytes: one by one through the copy engine
            for (int i = 0; i < lb.n; ++i) {
                rc = elora_pool_load_adapter(pool, slots[i0 + i], ranks[i0 + i], scales[i0 + i], A[i0 + i], B[i0 + i],
                                             on_device[i] ? 1 : 0, stream_);
                if (rc != ELORA_OK) return rc;
            }
            continue;
        }
        unsigned per = (unsigned)((most / 16 + 256 * 4 - 1) / (256 * 4));  // four pieces per thread
        per = per < 1 ? 1 : per > 64 ? 64 : per;
        hipLaunchKernelGGL(pool_load_batch_kernel, dim3(per, lb.n), dim3(256), 0, stream, lb, pool->storage + pool->slots_offset,
                           pool->slot_bytes, pool->b_offset, dmeta);
        ELORA_HIP_TRY(hipGetLastError());
        for (int i = 0; i < lb.n; ++i) pool->set_host_meta(slots[i0 + i], SlotMeta{ranks[i0 + i], scales[i0 + i], 1, 0});
    }
    return ELORA_OK;
}

int elora_pool_load_adapters_q8(elora_pool_t *pool, int n, const int *slots, const int *ranks, const float *scales,
                                const void *const *A_codes, const void *const *A_scales, const void *const *B_codes,
                                const void *const *B_scales, elora_stream_t stream_)
{
    if (pool == nullptr || (n > 0 && (!slots || !ranks || !scales || !A_codes || !A_scales || !B_codes || !B_scales))) return ELORA_E_NULL;
    if (n < 0) return ELORA_E_SHAPE;
    if (pool->dtype != ELORA_BF16) return ELORA_E_DTYPE;
    for (int i = 0; i < n; ++i) {
        if (!A_codes[i] || !A_scales[i] || !B_codes[i] || !B_scales[i]) return ELORA_E_NULL;
        if (slots[i] < 0 || slots[i] >= pool->capacity) return ELORA_E_SLOT;
        if (ranks[i] < 1 || ranks[i] > pool->max_rank) return ELORA_E_RANK;
        if (((size_t)ranks[i] * pool->d_in) % 32 || ((size_t)ranks[i] * pool->d_out) % 32) return ELORA_E_SHAPE;
        if (pool->q8 && ranks[i] % 8 != 0) return ELORA_E_RANK;  // resident blocks: 8 values of a row never straddle a block
        for (int j = 0; j < i; ++j)
            if (slots[j] == slots[i]) return ELORA_E_SLOT;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    // every source must be readable by the device (device memory or pinned host memory), codes 8-byte aligned:
    // all of them are looked at before anything is enqueued
    for (int i = 0; i < n; ++i) {
        bool dev = false;
        const void *a = device_readable(A_codes[i], &dev), *as = device_readable(A_scales[i], &dev);
        const void *b = device_readable(B_codes[i], &dev), *bs = device_readable(B_scales[i], &dev);
        if (!a || !as || !b || !bs) return ELORA_E_ALIGN;
        if (reinterpret_cast<uintptr_t>(a) % 8 || reinterpret_cast<uintptr_t>(b) % 8 || reinterpret_cast<uintptr_t>(as) % 2 ||
            reinterpret_cast<uintptr_t>(bs) % 2)
            return ELORA_E_ALIGN;
    }
    if (pool->q8) {
        // the blocks stay as they are: codes and scales are copied into the pool
        for (int i0 = 0; i0 < n; i0 += kLoadBatch) {
            LoadBatchQ8Keep lb;
            lb.n = n - i0 < kLoadBatch ? n - i0 : kLoadBatch;
            size_t most = 0;
            for (int i = 0; i < lb.n; ++i) {
                bool dev = false;
                lb.slot[i] = slots[i0 + i];
                lb.rank[i] = ranks[i0 + i];
                lb.scale[i] = scales[i0 + i];
                lb.A[i] = static_cast<const uint2 *>(device_readable(A_codes[i0 + i], &dev));
                lb.B[i] = static_cast<const uint2 *>(device_readable(B_codes[i0 + i], &dev));
                lb.As[i] = static_cast<const uint16_t *>(device_readable(A_scales[i0 + i], &dev));
                lb.Bs[i] = static_cast<const uint16_t *>(device_readable(B_scales[i0 + i], &dev));
                lb.a_vals[i] = (unsigned)((size_t)ranks[i0 + i] * pool->d_in);
                lb.b_vals[i] = (unsigned)((size_t)ranks[i0 + i] * pool->d_out);
                most = (size_t)lb.a_vals[i] + lb.b_vals[i] > most ? (size_t)lb.a_vals[i] + lb.b_vals[i] : most;
            }
            if (i0 == 0) {
                const int rc = pool_ensure_cleared(pool, stream);
                if (rc != ELORA_OK) return rc;
            }
            unsigned per = (unsigned)((most / 8 + 256 * 4 - 1) / (256 * 4));
            per = per < 1 ? 1 : per > 64 ? 64 : per;
            hipLaunchKernelGGL(pool_keep_q8_batch_kernel, dim3(per, lb.n), dim3(256), 0, stream, lb, pool->storage + pool->slots_offset,
                               pool->slot_bytes, pool->a_scale_off, pool->b_offset, pool->b_scale_off,
                               reinterpret_cast<SlotMeta *>(pool->storage + pool->meta_offset));
            ELORA_HIP_TRY(hipGetLastError());
            for (int i = 0; i < lb.n; ++i) pool->set_host_meta(slots[i0 + i], SlotMeta{ranks[i0 + i], scales[i0 + i], 1, 0});
        }
        return ELORA_OK;
    }
    for (int i0 = 0; i0 < n; i0 += kLoadBatch) {
        LoadBatchQ8 lb;
        lb.n = n - i0 < kLoadBatch ? n - i0 : kLoadBatch;
        size_t most = 0;
        for (int i = 0; i < lb.n; ++i) {
            bool dev = false;
            const void *a = device_readable(A_codes[i0 + i], &dev), *as = device_readable(A_scales[i0 + i], &dev);
            const void *b = device_readable(B_codes[i0 + i], &dev), *bs = device_readable(B_scales[i0 + i], &dev);
            if (!a || !as || !b || !bs) return ELORA_E_ALIGN;
            if (reinterpret_cast<uintptr_t>(a) % 8 || reinterpret_cast<uintptr_t>(b) % 8 || reinterpret_cast<uintptr_t>(as) % 2 ||
                reinterpret_cast<uintptr_t>(bs) % 2)
                return ELORA_E_ALIGN;
            const size_t a_vals = (size_t)ranks[i0 + i] * pool->d_in, b_vals = (size_t)ranks[i0 + i] * pool->d_out;
            lb.slot[i] = slots[i0 + i];
            lb.rank[i] = ranks[i0 + i];
            lb.scale[i] = scales[i0 + i];
            lb.A[i] = static_cast<const uint2 *>(a);
            lb.B[i] = static_cast<const uint2 *>(b);
            lb.As[i] = static_cast<const uint16_t *>(as);
            lb.Bs[i] = static_cast<const uint16_t *>(bs);
            lb.a_vecs[i] = (unsigned)(a_vals / 8);
            lb.b_vecs[i] = (unsigned)(b_vals / 8);
            most = a_vals + b_vals > most ? a_vals + b_vals : most;
        }
        if (i0 == 0) {
            const int rc = pool_ensure_cleared(pool, stream);
            if (rc != ELORA_OK) return rc;
        }
        unsigned per = (unsigned)((most / 8 + 256 * 4 - 1) / (256 * 4));
        per = per < 1 ? 1 : per > 64 ? 64 : per;
        hipLaunchKernelGGL(pool_load_q8_batch_kernel, dim3(per, lb.n), dim3(256), 0, stream, lb, pool->storage + pool->slots_offset,
                           pool->slot_bytes, pool->b_offset, reinterpret_cast<SlotMeta *>(pool->storage + pool->meta_offset));
        ELORA_HIP_TRY(hipGetLastError());
        for (int i = 0; i < lb.n; ++i) pool->set_host_meta(slots[i0 + i], SlotMeta{ranks[i0 + i], scales[i0 + i], 1, 0});
    }
    return ELORA_OK;
}

int elora_pool_evict(elora_pool_t *pool, int slot, elora_stream_t stream_)
{
    if (pool == nullptr) return ELORA_E_NULL;
    if (slot < 0 || slot >= pool->capacity) return ELORA_E_SLOT;
    if (!pool->host_meta[slot].loaded) return ELORA_E_NOT_LOADED;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = pool_ensure_cleared(pool, stream);
    if (rc != ELORA_OK) return rc;
    hipLaunchKernelGGL(pool_set_meta_kernel, dim3(1), dim3(64), 0, stream,
                       reinterpret_cast<SlotMeta *>(pool->storage + pool->meta_offset), slot, 0, 0.0f, 0);
    ELORA_HIP_TRY(hipGetLastError());
    pool->set_host_meta(slot, SlotMeta{0, 0.0f, 0, 0});
    return ELORA_OK;
}

int elora_pool_slot_info(const elora_pool_t *pool, int slot, int *rank, float *scale)
{
    if (pool == nullptr || rank == nullptr || scale == nullptr) return ELORA_E_NULL;
    if (slot < 0 || slot >= pool->capacity) return ELORA_E_SLOT;
    *rank = pool->host_meta[slot].loaded ? pool->host_meta[slot].rank : 0;
    *scale = pool->host_meta[slot].loaded ? pool->host_meta[slot].scale : 0.0f;
    return ELORA_OK;
}

int elora_pool_poll_error(elora_pool_t *pool, int clear, int *n_bad_rows, int *first_bad_row, elora_stream_t stream_)
{
    if (pool == nullptr || n_bad_rows == nullptr || first_bad_row == nullptr) return ELORA_E_NULL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    int rc = pool_ensure_cleared(pool, stream);
    if (rc != ELORA_OK) return rc;
    int rec[2] = {0, INT_MAX};
    ELORA_HIP_TRY(hipStreamSynchronize(stream));
    ELORA_HIP_TRY(hipMemcpy(rec, pool->storage, sizeof rec, hipMemcpyDeviceToHost));
    if (clear && rec[0] != 0) {
        hipLaunchKernelGGL(pool_clear_err_kernel, dim3(1), dim3(64), 0, stream, reinterpret_cast<int *>(pool->storage));
        ELORA_HIP_TRY(hipGetLastError());
    }
    *n_bad_rows = rec[0];
    *first_bad_row = rec[0] > 0 ? rec[1] : -1;
    return ELORA_OK;
}

}  // extern "C"
