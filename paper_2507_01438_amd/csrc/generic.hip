// Plain-ALU kernels for any dtype and shape: the fp32 parity configuration, odd shapes, and the
// fallback for everything the MFMA paths do not take.  Three launches:
//   route   per row: which pool slot, which scale (Sec. 3.4: each request names its adapter)
//   shrink  v_t = A_i x_t                          (Sec. 2.1 shapes: A [r, d_in])
//   base    y_t = W x_t + s * B_i v_t, written at row t (Sec. 3.4 closing equation)
#include "common.h"

using namespace elora;

namespace {

__global__ void route_kernel(int T, RouteView route, PoolView pool, int has_pool, int32_t *row_slot, float *row_scale)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    RowRoute r{-1, 0, 0.0f};
    if (has_pool) r = resolve_row(t, route, pool, true);
    row_slot[t] = r.slot;
    row_scale[t] = r.scale;
}

// one workgroup per row; wave w reduces rank rows w, w+4, ...
template <typename E>
__global__ __launch_bounds__(256) void shrink_generic_kernel(int K, const E *__restrict__ x, PoolView pool,
                                                             const int32_t *__restrict__ row_slot,
                                                             float *__restrict__ V, int R)
{
    int t = blockIdx.x;
    int slot = row_slot[t];
    if (slot < 0) return;
    int rank = pool.meta[slot].rank;
    const E *A = reinterpret_cast<const E *>(slot_A(pool, slot));
    const uint16_t *As = slot_A_scales(pool, slot);  // (adapters kept in 8-bit blocks: value = block scale * code)
    const E *xt = x + (size_t)t * K;
    int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = wave; j < rank; j += 4) {
        float s = 0.0f;
        for (int k = lane; k < K; k += 64) {
            const float a = pool.q8 ? q8_elem(reinterpret_cast<const char *>(A), As, (size_t)j * K + k) : load_elem(A, (size_t)j * K + k);
            s += a * load_elem(xt, (size_t)k);
        }
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
        if (lane == 0) V[(size_t)t * R + j] = s;
    }
}

template <int WFMT, typename E>
__device__ __forceinline__ float weight_elem(const void *W, const uint16_t *w_scales, int K, int n, int k)
{
    if (WFMT == ELORA_W_SAME) {
        return load_elem(static_cast<const E *>(W), (size_t)n * K + k);
    } else if (WFMT == ELORA_W_INT8_G32) {
        return fp16_to_f32(w_scales[(size_t)n * (K >> 5) + (k >> 5)]) * (float)static_cast<const int8_t *>(W)[(size_t)n * K + k];
    } else {
        uint8_t byte = static_cast<const uint8_t *>(W)[(size_t)n * (K >> 1) + (k >> 1)];
        int code = (k & 1) ? (byte >> 4) : (byte & 15);
        return fp16_to_f32(w_scales[(size_t)n * (K >> 5) + (k >> 5)]) * (float)(code - 8);
    }
}

// 64 x 64 output tile per workgroup, 4 x 4 outputs per thread, K in steps of 16 through LDS.
template <int WFMT, typename E>
__global__ __launch_bounds__(256) void base_generic_kernel(int T, int K, int N, const E *__restrict__ x,
                                                           const void *__restrict__ W,
                                                           const uint16_t *__restrict__ w_scales, PoolView pool,
                                                           const int32_t *__restrict__ row_slot,
                                                           const float *__restrict__ row_scale,
                                                           const float *__restrict__ V, int R, E *__restrict__ y)
{
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float xs[BK][BM + 4];
    __shared__ float ws[BK][BN + 4];
    int t0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    int tid = threadIdx.x;
    int ty = tid >> 4, tx = tid & 15;
    float acc[4][4] = {};
    int lr = tid >> 2, lk = (tid & 3) * 4;  // loader: row lr of the tile, 4 consecutive k
    for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int k = k0 + lk + i;
            int t = t0 + lr, n = n0 + lr;
            xs[lk + i][lr] = (t < T && k < K) ? load_elem(x, (size_t)t * K + k) : 0.0f;
            ws[lk + i][lr] = (n < N && k < K) ? weight_elem<WFMT, E>(W, w_scales, K, n, k) : 0.0f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float xv[4], wv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                xv[i] = xs[kk][ty * 4 + i];
                wv[i] = ws[kk][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(xv[i], wv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int t = t0 + ty * 4 + i;
        if (t >= T) continue;
        int slot = row_slot[t];
        int rank = 0;
        const E *B = nullptr;
        const uint16_t *Bs = nullptr;
        float scale = 0.0f;
        if (slot >= 0) {
            rank = pool.meta[slot].rank;
            B = reinterpret_cast<const E *>(slot_B(pool, slot));
            Bs = slot_B_scales(pool, slot);
            scale = row_scale[t];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float d = 0.0f;
            for (int q = 0; q < rank; ++q) {
                const float b = pool.q8 ? q8_elem(reinterpret_cast<const char *>(B), Bs, (size_t)n * rank + q) : load_elem(B, (size_t)n * rank + q);
                d = fmaf(V[(size_t)t * R + q], b, d);
            }
            store_elem(y, (size_t)t * N + n, acc[i][j] + scale * d);
        }
    }
}

template <int WFMT, typename E>
int launch_typed(const LinearArgs &a, hipStream_t stream)
{
    int32_t *row_slot = reinterpret_cast<int32_t *>(a.ws + a.wsl.row_slot);
    float *row_scale = reinterpret_cast<float *>(a.ws + a.wsl.row_scale);
    float *V = reinterpret_cast<float *>(a.ws + a.wsl.v);
    int R = a.pool.max_rank;
    hipLaunchKernelGGL(route_kernel, dim3((a.T + 255) / 256), dim3(256), 0, stream, a.T, a.route, a.pool,
                       a.has_pool ? 1 : 0, row_slot, row_scale);
    ELORA_HIP_TRY(hipGetLastError());
    if (a.has_pool) {
        hipLaunchKernelGGL((shrink_generic_kernel<E>), dim3(a.T), dim3(256), 0, stream, a.K,
                           static_cast<const E *>(a.x), a.pool, row_slot, V, R);
        ELORA_HIP_TRY(hipGetLastError());
    }
    dim3 grid((a.N + 63) / 64, (a.T + 63) / 64);
    profile_mark_begin(stream);
    hipLaunchKernelGGL((base_generic_kernel<WFMT, E>), grid, dim3(256), 0, stream, a.T, a.K, a.N,
                       static_cast<const E *>(a.x), a.W, static_cast<const uint16_t *>(a.w_scales), a.pool, row_slot,
                       row_scale, V, R, static_cast<E *>(a.y));
    ELORA_HIP_TRY(hipGetLastError());
    profile_mark_end(stream);
    return ELORA_OK;
}

}  // namespace

int elora::launch_generic(const LinearArgs &a, hipStream_t stream)
{
    if (a.dtype == ELORA_F32) return launch_typed<ELORA_W_SAME, float>(a, stream);
    if (a.wfmt == ELORA_W_SAME) return launch_typed<ELORA_W_SAME, uint16_t>(a, stream);
    if (a.wfmt == ELORA_W_INT8_G32) return launch_typed<ELORA_W_INT8_G32, uint16_t>(a, stream);
    return launch_typed<ELORA_W_INT4_G32, uint16_t>(a, stream);
}
