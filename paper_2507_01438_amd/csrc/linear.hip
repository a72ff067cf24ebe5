// Host side of elora_batched_lora_linear: validation, workspace layout, kernel-family selection.
#include <unordered_map>

#include "common.h"

using namespace elora;

namespace {

constexpr size_t kAlign = 256;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
int g_forced_path = -1;

// Which d_out a workspace serves.  The mailboxes of the decode kernel sit at the start of a workspace and their size
// follows d_out; what the other kernels write lies behind them.  A call with a smaller d_out would write into the
// area a decode call with a larger one takes for mailboxes, so a workspace is tied to the d_out of the first call that
// uses it after its initialisation, and calls with another one are refused.
std::unordered_map<const void *, int> g_ws_d_out;

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// profiling hook state
hipEvent_t *g_prof_events = nullptr;
int g_prof_calls = 0;     // armed calls
int g_prof_begun = 0;     // calls whose begin event was recorded
int g_prof_ended = 0;

void profile_release()
{
    if (g_prof_events) {
        for (int i = 0; i < 2 * g_prof_calls; ++i) (void)hipEventDestroy(g_prof_events[i]);
        delete[] g_prof_events;
    }
    g_prof_events = nullptr;
    g_prof_calls = g_prof_begun = g_prof_ended = 0;
}

}  // namespace

void elora::profile_mark_begin(hipStream_t stream)
{
    if (g_prof_events && g_prof_begun < g_prof_calls && g_prof_begun == g_prof_ended)
        if (hipEventRecord(g_prof_events[2 * g_prof_begun], stream) == hipSuccess) ++g_prof_begun;
}

void elora::profile_mark_end(hipStream_t stream)
{
    if (g_prof_events && g_prof_ended < g_prof_begun)
        if (hipEventRecord(g_prof_events[2 * g_prof_ended + 1], stream) == hipSuccess) ++g_prof_ended;
}

WsLayout elora::ws_layout(int T, int K, int N, int R, int wfmt)
{
    WsLayout l;
    size_t t = (size_t)(T > 0 ? T : 1);
    size_t off = 0;
    l.sync = off;
    off += align_up(sizeof(int) * kSyncInts);
    l.vmail = off;
    off += align_up(sizeof(float) * kDecodeMaxTokens * kMaxRank);
    l.mail = off;
    off += align_up(decode_mail_bytes(N));
    l.row_slot = off;
    off += align_up(t * sizeof(int32_t));
    l.row_scale = off;
    off += align_up(t * sizeof(float));
    l.row_rank = off;
    off += align_up(t * sizeof(int32_t));
    l.v = off;
    size_t v_full = t * (size_t)R * sizeof(float);
    size_t v_gemm = gemm_v_bytes((int)t, R);
    off += align_up(v_full > v_gemm ? v_full : v_gemm);
    // last, and zero bytes for small row counts: a workspace sized for more rows holds every smaller layout
    l.wdeq = off;
    l.wdeq_bytes = gemm_wcopy_bytes(wfmt, T, K, N);
    off += align_up(l.wdeq_bytes);
    l.total = off;
    return l;
}

static int validate(const elora_linear_desc_t *d, WsLayout *wsl_out)
{
    if (d == nullptr) return ELORA_E_NULL;
    if (d->dtype != ELORA_F32 && d->dtype != ELORA_BF16) return ELORA_E_DTYPE;
    const bool grouped = d->wfmt == ELORA_W_INT4_G32 || d->wfmt == ELORA_W_INT8_G32;
    if (d->wfmt != ELORA_W_SAME && !grouped) return ELORA_E_DTYPE;
    if (grouped && d->dtype != ELORA_BF16) return ELORA_E_DTYPE;
    if (d->n_tokens < 0 || d->d_in <= 0 || d->d_out <= 0) return ELORA_E_SHAPE;
    if (grouped && (d->d_in % 32) != 0) return ELORA_E_SHAPE;
    if (d->x == nullptr || d->W == nullptr || d->y == nullptr || d->workspace == nullptr) return ELORA_E_NULL;
    if (grouped && d->w_scales == nullptr) return ELORA_E_NULL;
    int max_rank = 1;
    if (d->pool != nullptr) {
        const elora_pool *p = d->pool;
        if (p->dtype != d->dtype) return ELORA_E_DTYPE;
        if (p->d_in != d->d_in || p->d_out != d->d_out) return ELORA_E_SHAPE;
        bool decode_form = d->adapter_idx != nullptr;
        bool prefill_form = d->seg_offsets != nullptr || d->seg_adapter != nullptr;
        if (decode_form == prefill_form) return ELORA_E_SEGMENTS;
        if (prefill_form && (d->seg_offsets == nullptr || d->seg_adapter == nullptr || d->n_segments < 0))
            return ELORA_E_SEGMENTS;
        max_rank = p->max_rank;
    }
    if (!aligned16(d->x) || !aligned16(d->W) || !aligned16(d->y)) return ELORA_E_ALIGN;
    if (d->w_scales != nullptr && !aligned16(d->w_scales)) return ELORA_E_ALIGN;
    if (reinterpret_cast<uintptr_t>(d->workspace) % kAlign) return ELORA_E_ALIGN;
    WsLayout wsl = ws_layout(d->n_tokens, d->d_in, d->d_out, max_rank, d->wfmt);
    if (d->workspace_bytes < wsl.total) return ELORA_E_STORAGE;
    const auto bound = g_ws_d_out.find(d->workspace);
    if (bound != g_ws_d_out.end() && bound->second != d->d_out) return ELORA_E_STORAGE;
    if (wsl_out) *wsl_out = wsl;
    return ELORA_OK;
}

static void make_plan(const elora_linear_desc_t *d, elora_plan_t *plan)
{
    int max_rank = d->pool ? d->pool->max_rank : 1;
    bool dec = decode_eligible(*d, max_rank);
    bool gem = gemm_eligible(*d, max_rank);
    if (d->pool && d->pool->q8) {
        // adapters kept in 8-bit blocks: read as they are by the decode kernel (ranks up to 64), by
        // the MFMA GEMM path's shrink and expand blocks, and by the generic kernels
        dec = dec && max_rank <= 64;
    }
    int path = ELORA_PATH_GENERIC;
    if (g_forced_path >= 0) {
        if (g_forced_path == ELORA_PATH_DECODE && dec) path = ELORA_PATH_DECODE;
        if (g_forced_path == ELORA_PATH_GEMM && gem) path = ELORA_PATH_GEMM;
    } else if (dec) {
        path = ELORA_PATH_DECODE;
    } else if (gem) {
        path = ELORA_PATH_GEMM;
    }
    plan->path = path;
    plan->split_k = 1;
    plan->tile_rows = 0;
    plan->tile_cols = 0;
    if (path == ELORA_PATH_DECODE) {
        decode_plan(*d, plan);
    } else if (path == ELORA_PATH_GEMM) {
        gemm_plan(*d, plan);
    } else {
        plan->n_launches = d->pool ? 3 : 1;
        plan->grid = ((d->n_tokens + 63) / 64) * ((d->d_out + 63) / 64);
    }
}

namespace {
// counters to zero, everything behind them to all-ones (the idle state of the decode kernel's mailboxes)
__global__ void ws_init_kernel(uint32_t *ws, size_t n_words, size_t n_sync)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_words; i += (size_t)gridDim.x * blockDim.x)
        ws[i] = i < n_sync ? 0u : 0xFFFFFFFFu;
}
}  // namespace

extern "C" {

const char *elora_status_string(int status)
{
    switch (status) {
    case ELORA_OK: return "ok";
    case ELORA_E_NULL: return "required pointer is NULL";
    case ELORA_E_ALIGN: return "device pointer is misaligned";
    case ELORA_E_DTYPE: return "unsupported dtype or weight format";
    case ELORA_E_SHAPE: return "invalid or inconsistent shape";
    case ELORA_E_RANK: return "rank out of range";
    case ELORA_E_SLOT: return "slot out of range";
    case ELORA_E_NOT_LOADED: return "slot holds no adapter";
    case ELORA_E_STORAGE: return "pool storage or workspace too small";
    case ELORA_E_SEGMENTS: return "routing tables: give exactly one of adapter_idx / segment tables";
    case ELORA_E_HIP: return "HIP runtime call failed";
    case ELORA_E_BUSY: return "every cached adapter is in use";
    default: return "unknown status";
    }
}

int elora_version(void) { return 1; }

size_t elora_workspace_bytes_w(int n_tokens_max, int d_in, int d_out, int max_rank, int wfmt)
{
    if (n_tokens_max < 0 || d_in <= 0 || d_out <= 0 || max_rank < 1 || max_rank > kMaxRank) return 0;
    if (wfmt != ELORA_W_SAME && wfmt != ELORA_W_INT4_G32 && wfmt != ELORA_W_INT8_G32) return 0;
    return ws_layout(n_tokens_max, d_in, d_out, max_rank, wfmt).total;
}

size_t elora_workspace_bytes(int n_tokens_max, int d_in, int d_out, int max_rank)
{
    return elora_workspace_bytes_w(n_tokens_max, d_in, d_out, max_rank, ELORA_W_SAME);
}

int elora_workspace_init(void *workspace, size_t workspace_bytes, elora_stream_t stream)
{
    if (workspace == nullptr) return ELORA_E_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return ELORA_E_ALIGN;
    if (workspace_bytes < align_up(sizeof(int) * kSyncInts)) return ELORA_E_STORAGE;
    g_ws_d_out.erase(workspace);  // free again for any d_out
    // (before the fill: the probe borrows a corner of this workspace)
    const int rc = decode_probe_device(static_cast<char *>(workspace) + align_up(sizeof(int) * kSyncInts),
                                       workspace_bytes - align_up(sizeof(int) * kSyncInts), static_cast<hipStream_t>(stream));
    if (rc != ELORA_OK) return rc;
    const size_t n_words = workspace_bytes / sizeof(uint32_t);
    const size_t blocks = (n_words + 255) / 256;
    hipLaunchKernelGGL(ws_init_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<uint32_t *>(workspace), n_words, (size_t)kSyncInts);
    ELORA_HIP_TRY(hipGetLastError());
    return ELORA_OK;
}

int elora_debug_spin_limit(int limit)
{
    if (limit < 0) return ELORA_E_SHAPE;
    decode_set_spin_limit(limit);
    return ELORA_OK;
}

int elora_debug_wait_limit_us(int us)
{
    if (us < 1 || us > 10000000) return ELORA_E_SHAPE;
    decode_set_wait_us(us);
    return ELORA_OK;
}

int elora_debug_w4_copy_rows(int rows)
{
    if (rows < 1) return ELORA_E_SHAPE;
    gemm_set_w4_copy_rows(rows);
    return ELORA_OK;
}

int elora_debug_xcd_local(int mode)
{
    if (mode != 0 && mode != -1) return ELORA_E_SHAPE;
    decode_set_local_override(mode);
    return ELORA_OK;
}

int elora_debug_decode_passes(int mode)
{
    if (mode < -1 || mode > 1) return ELORA_E_SHAPE;
    decode_set_passes(mode);
    return ELORA_OK;
}

int elora_debug_decode_wide(int mode)
{
    if (mode < -1 || mode > 1) return ELORA_E_SHAPE;
    decode_set_wide(mode);
    return ELORA_OK;
}

int elora_debug_k_rotate(int on)
{
    if (on != 0 && on != 1) return ELORA_E_SHAPE;
    decode_set_k_rotate(on);
    return ELORA_OK;
}

int elora_force_path(int path)
{
    if (path < -1 || path > ELORA_PATH_GEMM) return ELORA_E_DTYPE;
    g_forced_path = path;
    return ELORA_OK;
}

int elora_profile_arm(int n_calls)
{
    if (n_calls < 0 || n_calls > 65536) return ELORA_E_SHAPE;
    profile_release();
    if (n_calls == 0) return ELORA_OK;
    g_prof_events = new hipEvent_t[2 * n_calls];
    for (int i = 0; i < 2 * n_calls; ++i) {
        if (hipEventCreate(&g_prof_events[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(g_prof_events[j]);
            delete[] g_prof_events;
            g_prof_events = nullptr;
            (void)hipGetLastError();
            return ELORA_E_HIP;
        }
    }
    g_prof_calls = n_calls;
    return ELORA_OK;
}

int elora_profile_read(float *ms, int n, int *n_out)
{
    if (ms == nullptr || n_out == nullptr) return ELORA_E_NULL;
    int have = g_prof_ended < n ? g_prof_ended : n;
    for (int i = 0; i < have; ++i) {
        ELORA_HIP_TRY(hipEventSynchronize(g_prof_events[2 * i + 1]));
        ELORA_HIP_TRY(hipEventElapsedTime(&ms[i], g_prof_events[2 * i], g_prof_events[2 * i + 1]));
    }
    *n_out = have;
    return ELORA_OK;
}

int elora_linear_plan(const elora_linear_desc_t *desc, elora_plan_t *plan)
{
    if (plan == nullptr) return ELORA_E_NULL;
    int rc = validate(desc, nullptr);
    if (rc != ELORA_OK) return rc;
    make_plan(desc, plan);
    return ELORA_OK;
}

// ties the workspace of a validated descriptor to its d_out (see g_ws_d_out)
static int bind_workspace(const elora_linear_desc_t *d)
{
    try {
        g_ws_d_out.emplace(d->workspace, d->d_out);
    } catch (...) {  // out of host memory
        return ELORA_E_STORAGE;
    }
    return ELORA_OK;
}

// everything a launch needs of a validated descriptor
static int fill_args(const elora_linear_desc_t *d, const WsLayout &wsl, hipStream_t stream, LinearArgs &a)
{
    int rc = ELORA_OK;
    a.T = d->n_tokens;
    a.K = d->d_in;
    a.N = d->d_out;
    a.dtype = d->dtype;
    a.wfmt = d->wfmt;
    a.x = d->x;
    a.W = d->W;
    a.w_scales = d->w_scales;
    a.y = d->y;
    a.has_pool = d->pool != nullptr;
    a.ws = static_cast<char *>(d->workspace);
    a.wsl = wsl;
    if (a.has_pool) {
        // the pool handle is const in the descriptor; clearing its device table on first use is
        // the one mutation a linear call may need
        rc = pool_ensure_cleared(const_cast<elora_pool *>(d->pool), stream);
        if (rc != ELORA_OK) return rc;
        a.pool = d->pool->view();
        a.route = RouteView{d->adapter_idx, d->seg_offsets, d->seg_adapter, d->n_segments, d->scales, 0};
    } else {
        a.pool = PoolView{nullptr, nullptr, nullptr, 0, 0, 0, 1, 0, 0, 0};
        a.route = RouteView{nullptr, nullptr, nullptr, 0, nullptr, 0};
    }
    return ELORA_OK;
}

// the launches of a validated descriptor with at least one row
static int enqueue_linear(const elora_linear_desc_t *d, const WsLayout &wsl, hipStream_t stream)
{
    elora_plan_t plan;
    make_plan(d, &plan);
    LinearArgs a;
    const int rc = fill_args(d, wsl, stream, a);
    if (rc != ELORA_OK) return rc;
    switch (plan.path) {
    case ELORA_PATH_DECODE: {
        if (a.T <= kDecodeMaxTokens) return launch_decode(a, plan, stream);
        // more rows than one launch takes: balanced row ranges, one launch each, on the same workspace one after the other
        const int passes = plan.n_launches, es = 2;  // (bf16)
        int row = 0;
        for (int p = 0; p < passes; ++p) {
            const int rows = a.T / passes + (p < a.T % passes ? 1 : 0);
            LinearArgs b = a;
            b.T = rows;
            b.x = static_cast<const char *>(a.x) + (size_t)row * a.K * es;
            b.y = static_cast<char *>(a.y) + (size_t)row * a.N * es;
            b.route.row_base = row;
            const int rc2 = launch_decode(b, plan, stream);
            if (rc2 != ELORA_OK) return rc2;
            row += rows;
        }
        return ELORA_OK;
    }
    case ELORA_PATH_GEMM: return launch_gemm(a, plan, stream);
    default: return launch_generic(a, stream);
    }
}

int elora_batched_lora_linear(const elora_linear_desc_t *d, elora_stream_t stream_)
{
    WsLayout wsl;
    int rc = validate(d, &wsl);
    if (rc != ELORA_OK) return rc;
    if (d->n_tokens == 0) return ELORA_OK;
    rc = bind_workspace(d);
    if (rc != ELORA_OK) return rc;
    return enqueue_linear(d, wsl, static_cast<hipStream_t>(stream_));
}

// ---- the same call for callers that cannot allocate: the workspace is an array of this library ---------------------
namespace {
constexpr size_t kScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];  // one copy per device, held until the process ends
struct ScratchState {
    char *ptr;     // this device's copy of `scratch` (hipGetSymbolAddress; the array's name is no device address in host code)
    size_t idle;   // bytes from the start that are known to be in a workspace's idle state, 0: none yet
    size_t used;   // bytes from the start that calls so far may have written
    int d_out;     // the d_out the idle state was last used with
};
ScratchState g_scratch[64];
}  // namespace

int elora_batched_lora_linear_noalloc(const elora_linear_desc_t *desc, elora_stream_t stream_)
{
    if (desc == nullptr) return ELORA_E_NULL;
    int dev = 0;
    ELORA_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return ELORA_E_HIP;
    ScratchState &st = g_scratch[dev];
    if (st.ptr == nullptr) {
        void *p = nullptr;
        ELORA_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (p == nullptr) return ELORA_E_HIP;
        st.ptr = static_cast<char *>(p);
    }
    elora_linear_desc_t d = *desc;
    d.workspace = st.ptr;
    d.workspace_bytes = kScratchBytes;
    WsLayout wsl;
    const int rc = validate(&d, &wsl);  // E_STORAGE: the call needs more than the array holds
    if (rc != ELORA_OK) return rc;
    if (d.n_tokens == 0) return ELORA_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    // The idle state (counters zero, everything else all-ones) is written by a fill kernel on the call's stream: over
    // what this call's layout covers before the first call, and again, over everything calls have written so far, when
    // d_out changes (what a call with another d_out wrote may lie where this one's mailboxes are).
    if (st.idle < wsl.total || st.d_out != d.d_out) {
        const size_t bytes = st.used > wsl.total ? st.used : wsl.total;
        const size_t n_words = bytes / sizeof(uint32_t), blocks = (n_words + 255) / 256;
        hipLaunchKernelGGL(ws_init_kernel, dim3((unsigned)(blocks < 4096 ? blocks : 4096)), dim3(256), 0, stream,
                           reinterpret_cast<uint32_t *>(st.ptr), n_words, (size_t)kSyncInts);
        ELORA_HIP_TRY(hipGetLastError());
        st.idle = bytes;
        st.d_out = d.d_out;
    }
    if (wsl.total > st.used) st.used = wsl.total;
    return enqueue_linear(&d, wsl, stream);
}

// How a group goes out: as one decode launch, as calls of the GEMM path that share route and shrink launches, or call
// by call.  Fills the launch arguments of the first two forms.
enum GroupForm { kGroupSingles = 0, kGroupDecode = 1, kGroupGemmShared = 2 };
constexpr int kMaxGroup = 3;

static int group_form(const elora_linear_desc_t *descs, int n, hipStream_t stream, bool fill, LinearArgs *a, int *form)
{
    *form = kGroupSingles;
    if (n < 2 || n > kMaxGroup || descs[0].n_tokens <= 0) return ELORA_OK;
    int path0 = -1;
    for (int i = 0; i < n; ++i) {
        elora_plan_t plan;
        make_plan(&descs[i], &plan);
        if (i == 0) path0 = plan.path;
        if (plan.path != path0 || descs[i].n_tokens != descs[0].n_tokens) return ELORA_OK;
        // (the decode kernel that carries several calls has one weight format and one storage format of the pools per launch)
        if (plan.path == ELORA_PATH_DECODE && descs[i].wfmt != descs[0].wfmt) return ELORA_OK;
    }
    if (path0 == ELORA_PATH_DECODE) {
        bool q8 = false;
        for (int i = 0; i < n; ++i) q8 = q8 || (descs[i].pool && descs[i].pool->q8);
        for (int i = 0; i < n; ++i)
            if (descs[i].pool && (descs[i].pool->q8 != 0) != q8) return ELORA_OK;
    }
    if (path0 != ELORA_PATH_DECODE && path0 != ELORA_PATH_GEMM) return ELORA_OK;
    if (path0 == ELORA_PATH_GEMM) {
        // the same activations and routing tables, a pool each (all in the dtype of x, or all in 8-bit blocks)
        for (int i = 0; i < n; ++i) {
            const elora_linear_desc_t &d = descs[i], &d0 = descs[0];
            if (d.pool == nullptr || d0.pool == nullptr || (d.pool->q8 != 0) != (d0.pool->q8 != 0)) return ELORA_OK;
            if (d.x != d0.x || d.d_in != d0.d_in || d.adapter_idx != d0.adapter_idx ||
                d.seg_offsets != d0.seg_offsets || d.seg_adapter != d0.seg_adapter || d.n_segments != d0.n_segments ||
                d.scales != d0.scales)
                return ELORA_OK;
        }
    }
    if (fill) {
        for (int i = 0; i < n; ++i) {
            WsLayout wsl;
            (void)validate(&descs[i], &wsl);
            int rc = bind_workspace(&descs[i]);
            if (rc == ELORA_OK) rc = fill_args(&descs[i], wsl, stream, a[i]);
            if (rc != ELORA_OK) return rc;
        }
    }
    *form = path0 == ELORA_PATH_DECODE ? kGroupDecode : kGroupGemmShared;
    return ELORA_OK;
}

int elora_batched_lora_linear_group(const elora_linear_desc_t *descs, int n, elora_stream_t stream_)
{
    if (descs == nullptr) return ELORA_E_NULL;
    if (n < 1) return ELORA_E_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    // everything is validated before anything is enqueued
    for (int i = 0; i < n; ++i) {
        const int rc = validate(&descs[i], nullptr);
        if (rc != ELORA_OK) return rc;
        for (int j = 0; j < i; ++j)
            if (descs[i].workspace == descs[j].workspace || descs[i].y == descs[j].y) return ELORA_E_STORAGE;
    }
    LinearArgs a[kMaxGroup];
    int form = kGroupSingles;
    int rc = group_form(descs, n, stream, true, a, &form);
    if (rc != ELORA_OK) return rc;
    if (form == kGroupDecode) {
        rc = launch_decode_group(a, n, stream);
        if (rc >= 0) return rc;
    } else if (form == kGroupGemmShared) {
        return launch_gemm_group(a, n, stream);
    }
    for (int i = 0; i < n; ++i) {
        rc = elora_batched_lora_linear(&descs[i], stream_);
        if (rc != ELORA_OK) return rc;
    }
    return ELORA_OK;
}

int elora_linear_group_launches(const elora_linear_desc_t *descs, int n, int *n_launches)
{
    if (descs == nullptr || n_launches == nullptr) return ELORA_E_NULL;
    if (n < 1) return ELORA_E_SHAPE;
    int sum = 0;
    for (int i = 0; i < n; ++i) {
        const int rc = validate(&descs[i], nullptr);
        if (rc != ELORA_OK) return rc;
        elora_plan_t plan;
        make_plan(&descs[i], &plan);
        sum += descs[i].n_tokens > 0 ? plan.n_launches : 0;
    }
    int form = kGroupSingles;
    (void)group_form(descs, n, nullptr, false, nullptr, &form);
    if (form == kGroupDecode) {
        int K[kMaxGroup], N[kMaxGroup], split[kMaxGroup];
        bool wlds = true;
        for (int i = 0; i < n; ++i) {
            K[i] = descs[i].d_in;
            N[i] = descs[i].d_out;
        }
        bool q8 = false;
        for (int i = 0; i < n; ++i) q8 = q8 || (descs[i].pool && descs[i].pool->q8);
        if (decode_group_splits(descs[0].n_tokens, n, K, N, split, &wlds, descs[0].wfmt == ELORA_W_INT8_G32, q8)) sum = 1;
    } else if (form == kGroupGemmShared) {
        sum -= 2 * (n - 1);  // one route and one shrink launch for all of them
    }
    *n_launches = sum;
    return ELORA_OK;
}

}  // extern "C"
