/*
 * elora.h -- C ABI of libelora: the batched multi-adapter LoRA linear layer
 * ("batch LoRA inference", Sec. 3.4 and Sec. 4.3 of the EdgeLoRA paper) for
 * one AMD MI355X (gfx950).
 *
 *     y_t = W x_t + s * B_i (A_i x_t)          i = adapter of row t
 *
 * for every row t of a batch in which each request carries its own adapter
 * index into a pool of resident adapters (closing equation of Sec. 3.4;
 * shapes W [d_out, d_in], A_i [r_i, d_in], B_i [d_out, r_i] from Sec. 2.1).
 * The adapters live in a pre-allocated pool of fixed-size blocks, one block
 * per adapter, so that no memory is allocated while serving (Sec. 3.3 and
 * Sec. 4.2, "pre-allocated memory pool").
 *
 * General conventions
 *   - Plain C types only.  `elora_stream_t` is a hipStream_t passed as void*.
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are ordinary process memory.  Every device buffer (x, W, y,
 *     pool storage, workspace) is allocated, owned and freed by the caller;
 *     the library never allocates or frees device memory.
 *   - All tensors are dense row-major.  bf16 is the 16-bit brain float; fp16
 *     is IEEE binary16.
 *   - Every function returns an elora_status_t (0 = success) unless it returns
 *     a size.  Nothing aborts, throws or prints.  On failure no work has been
 *     enqueued by that call and out-parameters are untouched (the one exception, a
 *     HIP error in the middle of a batch of loads, is stated where it applies).
 *   - All device work is enqueued on the caller's stream and the call returns
 *     without waiting.  Calls that use the same pool must be ordered by the
 *     caller (same stream, or events).
 */
#ifndef ELORA_H
#define ELORA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void *elora_stream_t; /* hipStream_t; NULL = the default stream */

typedef struct elora_pool elora_pool_t; /* opaque host object; holds metadata only */
typedef struct elora_cache elora_cache_t; /* opaque host object: which adapter sits in which block */

typedef enum {
    ELORA_OK = 0,
    ELORA_E_NULL = 1,       /* a required pointer is NULL */
    ELORA_E_ALIGN = 2,      /* a device pointer is not 16-byte aligned (pool storage: 256) */
    ELORA_E_DTYPE = 3,      /* unknown dtype / weight format, or a combination that is not supported */
    ELORA_E_SHAPE = 4,      /* non-positive or inconsistent dimension (e.g. desc vs pool d_in/d_out) */
    ELORA_E_RANK = 5,       /* rank < 1 or rank > the pool's max_rank */
    ELORA_E_SLOT = 6,       /* slot < 0 or slot >= capacity */
    ELORA_E_NOT_LOADED = 7, /* the slot holds no adapter */
    ELORA_E_STORAGE = 8,    /* pool storage or workspace smaller than required */
    ELORA_E_SEGMENTS = 9,   /* routing tables: both or neither of adapter_idx / seg_offsets given, or n_segments < 0 */
    ELORA_E_HIP = 10,       /* a HIP runtime call failed (no device, bad launch, ...) */
    ELORA_E_BUSY = 11       /* adapter cache: every cached adapter is in use by an outstanding request */
} elora_status_t;

typedef enum { ELORA_F32 = 0, ELORA_BF16 = 1 } elora_dtype_t; /* element type of x, y, A, B (and W if ELORA_W_SAME) */

typedef enum {
    ELORA_W_SAME = 0,    /* W [d_out, d_in] has the dtype of x */
    ELORA_W_INT4_G32 = 1, /* W is 4-bit, symmetric, groups of 32 along d_in (the block format the paper's
                            settings name "Q4_0", Sec. 5 "Model"; byte order is this library's own):
                            uint8 [d_out, d_in/2], byte b of a row = code(k=2b) | code(k=2b+1) << 4,
                            w = scale * (code - 8), scales fp16 [d_out, d_in/32].  Needs dtype bf16,
                            d_in % 32 == 0. */
    ELORA_W_INT8_G32 = 2  /* W is 8-bit, symmetric, groups of 32 along d_in (the "Q8_0" base model of the
                            paper's setting S1, Sec. 5 "Model"): int8 [d_out, d_in], w = scale * code,
                            scales fp16 [d_out, d_in/32].  Needs dtype bf16, d_in % 32 == 0. */
} elora_wfmt_t;

/* Kernel family a call is dispatched to (reported by elora_linear_plan). */
typedef enum {
    ELORA_PATH_GENERIC = 0, /* plain-ALU tiled kernels: any dtype / shape */
    ELORA_PATH_DECODE = 1,  /* few rows (up to 64 per launch, up to 256 in several launches): HBM-streaming split-K MFMA
                               contraction with the shrink before and the expand after it in the same kernel */
    ELORA_PATH_GEMM = 2     /* many rows: LDS-tiled bf16 MFMA GEMM with the expand as a K-extension */
} elora_path_t;

const char *elora_status_string(int status);
int elora_version(void);

/* ------------------------------------------------------------------ pool ---
 * The resident adapter pool of Sec. 3.3 / 4.2: `capacity` blocks of equal size,
 * each able to hold one adapter of rank <= max_rank for ONE linear layer
 * (d_in, d_out).  Block i ("slot" i) is what adapter index i in a batch refers to.
 */

/* Bytes of device memory a pool needs; 0 if an argument is invalid. */
size_t elora_pool_storage_bytes(int d_in, int d_out, int max_rank, int capacity, int dtype);

/*
 * Create the host object for a pool that lives in caller-owned device memory
 * `dev_storage` (256-byte aligned, >= elora_pool_storage_bytes()).  Touches no
 * device memory: the pool's device-side slot table is cleared by the first
 * stream-carrying call on this pool (load / evict / linear), on that call's
 * stream.  *out receives the handle.
 * Errors: E_NULL, E_ALIGN, E_DTYPE, E_SHAPE, E_RANK (max_rank < 1 or > 256), E_STORAGE (storage too small, or out of
 * host memory).
 */
int elora_pool_create(int d_in, int d_out, int max_rank, int capacity, int dtype,
                      void *dev_storage, size_t storage_bytes, elora_pool_t **out);

/* Free the host object.  The device storage stays with the caller; pending work must have finished. */
int elora_pool_destroy(elora_pool_t *pool);

/*
 * Place an adapter in block `slot` (Sec. 3.3: a new adapter is assigned to a
 * free block of the pool): A [rank, d_in], B [d_out, rank], both row-major in
 * the pool's dtype, scale = alpha / rank.  Copies are asynchronous on `stream`;
 * `src_on_device` says whether A and B are device (1) or host (0) pointers.
 * Host sources must stay valid until the stream has passed the copy.
 * Reloading an occupied slot replaces its content.  Linear calls enqueued
 * later on the same stream see the new adapter.
 * Errors: E_NULL, E_SLOT, E_RANK, E_HIP.
 */
int elora_pool_load_adapter(elora_pool_t *pool, int slot, int rank, float scale,
                            const void *A, const void *B, int src_on_device, elora_stream_t stream);

/*
 * The same for n adapters at once (host arrays of n entries; slots distinct), as the misses of a batch come: when
 * every source is device memory or pinned host memory (hipHostMalloc) and 16-byte aligned, with sizes that are
 * multiples of 16 bytes, the GPU reads the sources itself and one launch per 16 adapters fills the blocks and
 * their table entries; otherwise the adapters are placed one by one as above.  Nothing enqueued on other streams
 * may read or write these blocks until this call's work on `stream` is done (elora_cache_load_begin / _end do
 * that ordering).  Errors: E_NULL, E_SHAPE (n < 0), E_SLOT (out of range, or one slot twice), E_RANK: nothing is
 * enqueued; E_HIP (a launch or copy failed): adapters earlier in the arrays may already be enqueued and count as
 * loaded, the one that failed and those after it do not.
 */
int elora_pool_load_adapters(elora_pool_t *pool, int n, const int *slots, const int *ranks, const float *scales,
                             const void *const *A, const void *const *B, elora_stream_t stream);

/*
 * The same for adapters that are kept in 8-bit blocks, the storage format of the paper's adapters (Sec. 5 "Model"
 * names it "Q8_0"; the layout here is this library's own): A_codes[i] int8 [rank, d_in] and B_codes[i] int8
 * [d_out, rank], row-major, cut into blocks of 32 consecutive values in that order; A_scales[i] / B_scales[i] one
 * fp16 per block; value = scale * code.  Into a pool created by elora_pool_create (dtype bf16) the blocks are
 * converted on the way in: the pool receives bf16(scale * code), the product exact, one rounding to nearest even, so
 * the linear calls see an ordinary bf16 adapter while half the bytes cross the bus.  Into a pool created by
 * elora_pool_create_q8 they are copied as they are (ranks then multiples of 8: E_RANK otherwise).  Sources: device memory or pinned host memory, codes 8-byte aligned;
 * rank * d_in and rank * d_out multiples of 32.  One launch per 16 adapters.
 * Errors: E_NULL, E_SHAPE, E_DTYPE (pool is not bf16), E_SLOT, E_RANK, E_ALIGN (a source the device cannot read, or
 * misaligned), E_HIP.
 */
int elora_pool_load_adapters_q8(elora_pool_t *pool, int n, const int *slots, const int *ranks, const float *scales,
                                const void *const *A_codes, const void *const *A_scales, const void *const *B_codes,
                                const void *const *B_scales, elora_stream_t stream);

/*
 * A pool whose adapters STAY in 8-bit blocks (the paper's adapter storage, Sec. 5 "Model"): the blocks placed by
 * elora_pool_load_adapters_q8 are kept as they are (int8 codes and fp16 block scales), and the linear kernels read
 * them directly, value = scale * code formed in registers, so an adapter costs half the memory and half the traffic
 * of its bf16 form.  x and y of calls that use the pool are bf16, W is bf16 or in one of the grouped formats (with
 * ELORA_W_INT8_G32 base and adapters are both stored as in the paper's setting S1).  d_in % 32 == 0, d_out % 4 == 0,
 * max_rank and every loaded rank multiples of 8.  Calls with such a pool take the decode path (up to 256 rows,
 * max_rank <= 64), the GEMM path, or else the generic kernels; elora_pool_load_adapter / _load_adapters (sources in
 * bf16) answer E_DTYPE.
 * Errors: as elora_pool_create, E_SHAPE / E_RANK for the divisibility rules above.
 */
size_t elora_pool_storage_bytes_q8(int d_in, int d_out, int max_rank, int capacity);
int elora_pool_create_q8(int d_in, int d_out, int max_rank, int capacity, void *dev_storage, size_t storage_bytes,
                         elora_pool_t **out);

/* Mark `slot` empty (its block returns to the pool, Sec. 4.2).  Rows that still refer to it are
 * treated like rows with an invalid index.  Errors: E_NULL, E_SLOT, E_NOT_LOADED, E_HIP. */
int elora_pool_evict(elora_pool_t *pool, int slot, elora_stream_t stream);

/* Host-side view of a slot: *rank = 0 if empty.  Errors: E_NULL, E_SLOT. */
int elora_pool_slot_info(const elora_pool_t *pool, int slot, int *rank, float *scale);

/*
 * Rows whose adapter index was out of range (not -1, not in [0, capacity)) or
 * named an empty slot are computed as base-model-only rows and counted in a
 * sticky device-side record.  This call SYNCHRONISES `stream`, copies the
 * record to the host, and (if `clear`) resets it.  *n_bad_rows = how many
 * such rows since the last clear, *first_bad_row = the smallest such row
 * index (-1 if none).  Errors: E_NULL, E_HIP.
 */
int elora_pool_poll_error(elora_pool_t *pool, int clear, int *n_bad_rows, int *first_bad_row,
                          elora_stream_t stream);

/* ----------------------------------------------------------------- cache ---
 * The adapter memory manager of Sec. 3.3 / 4.2: a memory cache C of at most l
 * adapters over the l blocks of the pre-allocated pool.  An adapter that is
 * requested and cached is served from the cache; otherwise it is assigned to a
 * free block, and when none is free the least recently used adapter is evicted
 * and its block is reused (Sec. 4.2 states LRU).  Free blocks form a stack
 * (Sec. 4.2) that hands out 0, 1, 2, ... at first.  Block numbers are the slot
 * numbers of elora_pool_*: one cache can stand for the pools of all linear
 * layers of a model, each holding that layer's part of an adapter in the same
 * slot.  Host logic only: the cache decides, the caller loads
 * (elora_pool_load_adapter) what it reports as missing.  Not thread-safe.
 *
 * A request pins its adapter until elora_cache_release: a pinned adapter is
 * never the victim (its rows may still be waiting to run).
 */

/* Errors: E_NULL, E_SHAPE (capacity < 1), E_STORAGE (out of host memory). */
int elora_cache_create(int capacity, elora_cache_t **out);
int elora_cache_destroy(elora_cache_t *cache);

/*
 * One request for adapter `adapter_id` (>= 0).  *slot = its block; *hit = 1 if it was cached (no load needed),
 * 0 if the block was just assigned and the caller has to load the adapter into it; *evicted_id = the adapter that
 * lost the block, -1 if none did.  The adapter becomes the most recently used one and its pin count rises by one.
 * Errors: E_NULL, E_SHAPE (adapter_id < 0), E_BUSY (not cached, no free block, all cached adapters pinned:
 * nothing changes and the request is not counted), E_STORAGE (out of host memory).
 */
int elora_cache_acquire(elora_cache_t *cache, int adapter_id, int *slot, int *hit, int *evicted_id);

/* The request is over.  Errors: E_NULL, E_NOT_LOADED (not cached, or not pinned). */
int elora_cache_release(elora_cache_t *cache, int adapter_id);

/*
 * The requests of one batch, row by row in order (host arrays): slots[t] = the block of row t's adapter
 * (adapter_ids[t] < 0: no adapter, slots[t] = -1, not a request).  The adapters that have to be loaded come back
 * as miss_ids[0..*n_miss) / miss_slots[0..*n_miss), each once, in the order their blocks were assigned (room for
 * n entries each).  Later rows of the batch that name an adapter assigned by an earlier row count as hits.
 * On E_BUSY (more distinct adapters in flight than blocks) the call is undone: its requests are released and not
 * counted, and the adapters it had assigned blocks to are not cached afterwards (their blocks are free again: nothing
 * was loaded into them); the arrays hold nothing of use.  Evictions it made on the way stay.
 * Errors: E_NULL, E_SHAPE (n < 0), E_BUSY.
 */
int elora_cache_acquire_batch(elora_cache_t *cache, const int *adapter_ids, int n, int *slots, int *miss_ids,
                              int *miss_slots, int *n_miss);

/* Releases what elora_cache_acquire_batch acquired for the same rows.  Errors: E_NULL, E_SHAPE, E_NOT_LOADED
 * (some row's adapter was not cached or not pinned; the other rows are still released). */
int elora_cache_release_batch(elora_cache_t *cache, const int *adapter_ids, int n);

/* *slot = the adapter's block or -1; changes nothing (no request is counted).  Errors: E_NULL. */
int elora_cache_lookup(const elora_cache_t *cache, int adapter_id, int *slot);

/* Evict on purpose; the block goes back on the stack.  Errors: E_NULL, E_NOT_LOADED, E_BUSY (pinned). */
int elora_cache_drop(elora_cache_t *cache, int adapter_id);

/*
 * Adaptive adapter selection after the router (Algorithm 1): explicit_id >= 0 names the adapter and is returned as
 * it is.  Otherwise scores[0..n) are the router's confidence scores (host fp32, one per adapter id), the k most
 * confident adapters are gone through in descending order of confidence and the first one that is cached is chosen;
 * if none is, the most confident one.  Equal scores: the lower id first; NaN ranks below every number.  *resident =
 * 1 if the chosen adapter is cached.  Only looks: the request itself is the elora_cache_acquire that follows.
 * Errors: E_NULL, E_SHAPE (n < 1 or k < 1; k > n is taken as n).
 */
int elora_cache_select(const elora_cache_t *cache, int explicit_id, const float *scores, int n, int k, int *chosen,
                       int *resident);

/* Hit rate H = hits / requests (Sec. 3.3).  Any out-pointer may be NULL.  Errors: E_NULL (cache). */
int elora_cache_stats(const elora_cache_t *cache, long long *hits, long long *requests, long long *evictions);
int elora_cache_reset_stats(elora_cache_t *cache);

/*
 * Device-side order between the stream that loads adapters and the stream that computes, so that loads overlap
 * the linear calls of other batches and neither side waits on the host.  Arrays of block numbers (host memory;
 * negative entries, rows without adapter, are skipped):
 *   load_begin   before loading into `slots` (elora_pool_load_adapter[s]): the copy stream waits for the last
 *                batch that used any of these blocks (it may still be reading an adapter that is being replaced)
 *   load_end     after it: remembers these blocks' content as arriving with this load
 *   batch_begin  before the linear calls of a batch whose rows use `slots`: the compute stream waits for the
 *                latest load into any of these blocks, unless it has already waited that far
 *   batch_end    after them: remembers the batch as the last user of these blocks
 * One cache = one copy stream and one compute stream (the same stream may play both parts): all loads are taken
 * to run in the order of these calls on the one, all batches on the other, so one event wait per call covers
 * everything earlier.  Events are created on first use (these four calls need a device; the functions above do
 * not).  Errors: E_NULL, E_SHAPE (n < 0), E_SLOT, E_HIP.
 */
int elora_cache_load_begin(elora_cache_t *cache, const int *slots, int n, elora_stream_t copy_stream);
int elora_cache_load_end(elora_cache_t *cache, const int *slots, int n, elora_stream_t copy_stream);
int elora_cache_batch_begin(elora_cache_t *cache, const int *slots, int n, elora_stream_t compute_stream);
int elora_cache_batch_end(elora_cache_t *cache, const int *slots, int n, elora_stream_t compute_stream);

/* ---------------------------------------------------------------- linear --- */

typedef struct {
    /* shapes */
    int n_tokens;          /* T >= 0 rows in the batch (0: nothing is done) */
    int d_in;              /* K */
    int d_out;             /* N */
    int dtype;             /* elora_dtype_t of x, y (and of the pool) */
    int wfmt;              /* elora_wfmt_t */
    /* tensors (device) */
    const void *x;         /* [n_tokens, d_in] */
    const void *W;         /* [d_out, d_in] (packed 4-bit: [d_out, d_in/2] bytes; 8-bit: [d_out, d_in] bytes) */
    const void *w_scales;  /* fp16 [d_out, d_in/32] for ELORA_W_INT4_G32 and ELORA_W_INT8_G32, else NULL */
    void *y;               /* [n_tokens, d_out], overwritten */
    /* adapters */
    const elora_pool_t *pool;   /* NULL: base model only (y = W x), routing tables are ignored */
    /* routing (device int32): exactly one of the two forms when pool != NULL */
    const int32_t *adapter_idx; /* [n_tokens] slot per row, -1 = no adapter for this row (decode form) */
    const int32_t *seg_offsets; /* [n_segments + 1] rows seg_offsets[s] .. seg_offsets[s+1]-1 use        */
    const int32_t *seg_adapter; /* [n_segments]     slot seg_adapter[s] (-1 = none); offsets start at 0, */
    int n_segments;             /*                  are non-decreasing and end at n_tokens (prefill form) */
    const float *scales;        /* NULL: each adapter's own scale; else device fp32, one per row (decode
                                   form) or one per segment (prefill form), replacing it */
    /* scratch (device) */
    void *workspace;            /* >= elora_workspace_bytes_w(n_tokens, d_in, d_out, max_rank, wfmt), 256-byte aligned */
    size_t workspace_bytes;
} elora_linear_desc_t;

/* Device scratch one call may use, for up to n_tokens_max rows, with W in the dtype of x (ELORA_W_SAME).
 * 0 if an argument is invalid. */
size_t elora_workspace_bytes(int n_tokens_max, int d_in, int d_out, int max_rank);
/* The same for a given weight format (elora_wfmt_t): with a 4-bit W and 768 rows or more, or an 8-bit W and more than
 * 256 rows, the workspace also holds the call's bf16 copy of W (d_out x d_in x 2 bytes). */
size_t elora_workspace_bytes_w(int n_tokens_max, int d_in, int d_out, int max_rank, int wfmt);

/*
 * A workspace must be initialised ONCE, over its whole size, before its first use in a linear call.
 * Its first 4 KiB hold counters (idle state: zero) and most of the rest are mailboxes through which the
 * workgroups of a decode call hand each other partial results (idle state: all bits set).  This call
 * writes the idle state (one fill kernel on `stream`), and every linear call leaves the workspace idle
 * again.  Call it again only after a call that used the workspace was aborted (device reset).
 * Two calls that may run at the same time (different streams) need different workspaces.
 * A workspace serves ONE d_out: the first linear call after its initialisation ties it to that call's d_out (the
 * mailboxes' size follows d_out and what other kernels write lies behind them), and calls with another d_out are
 * refused with E_STORAGE until it is initialised again.  d_in, the row count and the pool may vary from call to call.
 * Calls on the decode path should not run at the same time at all: the workgroups of such a call wait for each
 * other, which takes all of them to be on the device together, and two such launches that each hold part of the
 * compute units keep each other's remaining workgroups out.  Every wait is bounded in time (about 200 us: a
 * workgroup whose wait runs out computes what it needs from the inputs, see elora_debug_wait_limit_us), so the
 * results stay right, but such calls are slow.  Issue them on one stream, or as one group (elora_batched_lora_linear_group); kernels
 * that do not fill the device (adapter loads, copies) may overlap them freely.
 * The first call on a device also finds out how the device places workgroups on its XCDs (one tiny
 * launch into the workspace that is being initialised, a 1 KiB copy to the host and a wait for `stream`): set-up
 * work, not to be captured in a graph.  No device memory is allocated.
 * Errors: E_NULL, E_ALIGN, E_STORAGE, E_HIP.
 */
int elora_workspace_init(void *workspace, size_t workspace_bytes, elora_stream_t stream);

typedef struct {
    int path;        /* elora_path_t */
    int n_launches;  /* kernels one call enqueues */
    int split_k;     /* K-slices of the streaming contraction (decode path: 1, 2, 4 or 8), else 1 */
    int tile_rows;   /* W rows (decode) or output rows (gemm) per workgroup, 0 for the generic path */
    int tile_cols;   /* output columns per workgroup (gemm), else 0 */
    int grid;        /* workgroups of the dominant kernel */
} elora_plan_t;

/*
 * Validate a descriptor exactly as elora_batched_lora_linear does (everything
 * that can be checked on the host without touching the device) and report
 * which kernels the call would run.  Touches no device memory.
 * Errors: E_NULL, E_ALIGN, E_DTYPE, E_SHAPE, E_SEGMENTS, E_STORAGE (workspace too small, or tied to another d_out).
 */
int elora_linear_plan(const elora_linear_desc_t *desc, elora_plan_t *plan);

/*
 * The batched multi-adapter LoRA linear layer of Sec. 3.4: the base product
 * W x is shared by the whole batch; every row adds s * B_i (A_i x) with the
 * adapter its request names; results land at the rows' own positions in y.
 * Accumulation is fp32; y is rounded once (bf16: round-to-nearest-even).
 * Rows with adapter -1 get y = W x.  Invalid indices: see elora_pool_poll_error.
 * The segment table itself is trusted to be well-formed (it is device data).
 * Errors: those of elora_linear_plan, plus E_HIP.
 */
int elora_batched_lora_linear(const elora_linear_desc_t *desc, elora_stream_t stream);

/*
 * elora_batched_lora_linear for callers that cannot allocate device memory or have none to hand over as a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  desc->workspace and
 * desc->workspace_bytes are ignored; the workspace is a 32 MiB array inside this library (one copy per GPU, held until
 * the process ends), brought into its idle state by a fill kernel on `stream` where needed (before a GPU's first call,
 * and when d_out differs from the previous call's).  Nothing is allocated or freed, on the device or through any
 * library; inputs and outputs are the caller's as ever.  A call that needs more than 32 MiB of workspace
 * (elora_workspace_bytes_w: about 2 KiB per output column on the decode path; a 4-bit W with 768 rows or more needs a
 * copy of W) is refused with E_STORAGE.  Every call on a GPU uses that GPU's one array: calls that overlap in time on
 * one GPU race, so issue them on one stream.  Whether workgroups of a tile share an XCD is only found out by
 * elora_workspace_init; until some workspace has been initialised on the GPU the decode kernel hands partial sums over
 * through memory (same results).
 * Errors: those of elora_batched_lora_linear, E_STORAGE as above.
 */
int elora_batched_lora_linear_noalloc(const elora_linear_desc_t *desc, elora_stream_t stream);

/*
 * Several calls that are due at the same time (the projections that read the same activations: q / k / v, gate /
 * up; Sec. 4.3 computes base and adapters of a batch in one graph), as an array of n descriptors.  Results are those
 * of n calls of elora_batched_lora_linear up to the order of fp32 additions.  Two or three calls that all take the
 * decode path with the same n_tokens run as ONE launch when their workgroups fit on the device together (each call
 * then gets fewer K-slices than it would take alone).  Two or three calls that all take the MFMA GEMM path, each with
 * a pool, and name the SAME x, d_in and routing tables (the same pointers) share ONE route launch and ONE shrink
 * launch, A_i x for the adapters of all of them with the rows of x fetched once, followed by each call's GEMM.
 * Otherwise, and for any other mix, the calls are enqueued one after the other.  Every call needs a workspace and an
 * output of its own.
 * Errors: those of elora_batched_lora_linear for any descriptor (nothing is enqueued then), E_SHAPE (n < 1),
 * E_STORAGE (two descriptors share a workspace or y).
 */
int elora_batched_lora_linear_group(const elora_linear_desc_t *descs, int n, elora_stream_t stream);

/* How many kernels elora_batched_lora_linear_group would enqueue for these descriptors.  Errors: as above. */
int elora_linear_group_launches(const elora_linear_desc_t *descs, int n, int *n_launches);

/*
 * Test hook: when `path` is a valid elora_path_t, later calls use that kernel
 * family if the descriptor is eligible for it (otherwise the generic one);
 * -1 restores automatic selection.  Process-wide, not thread-safe.
 */
int elora_force_path(int path);

/*
 * Test hook: upper bound on the polls of each wait inside the decode kernel (a workgroup waiting for
 * results of another one).  A workgroup whose bound runs out computes what it needs from the inputs
 * by itself, and the call removes whatever was posted to it before it ends; 0 makes every waiter take
 * that route at once.  Default 4194304.  Errors: E_SHAPE (limit < 0).
 */
int elora_debug_spin_limit(int limit);

/*
 * The bound that ends such a wait in practice is one in time: about `us` microseconds (default 200; the clock is
 * looked at every 64 polls, so a wait may last a few tens of microseconds longer), whatever a poll costs on the
 * machine and however busy it is.  Errors: E_SHAPE (us < 1 or > 10000000).
 */
int elora_debug_wait_limit_us(int us);

/*
 * Test and measurement hook: the row count from which a call with a 4-bit W converts W once into its workspace
 * instead of tile by tile inside the GEMM kernel (default 768; workspaces are sized with the value in force, so set it
 * before elora_workspace_bytes_w).  Errors: E_SHAPE (rows < 1).
 */
int elora_debug_w4_copy_rows(int rows);

/*
 * Test hook: 0 makes the decode kernel run as if the device gave no guarantee that the workgroups
 * which exchange partial sums share an XCD (every hand-over then goes through memory instead of that
 * XCD's L2); -1 goes back to what the device was found to do.  Errors: E_SHAPE.
 */
int elora_debug_xcd_local(int mode);

/*
 * Test hook: calls of 65 to 256 rows (bf16, d_in a multiple of 256, d_out of 16) may run as 2 to 4 launches of the
 * decode kernel over balanced row ranges instead of on the MFMA GEMM path.  -1 (default) and 1: they do; 0: they
 * take the GEMM path.  Errors: E_SHAPE.
 */
int elora_debug_decode_passes(int mode);

/*
 * Test hook: which decode calls with more than 32 rows run the kernel whose workgroups take 128 rows of W instead
 * of 64.  -1 (default): those whose grid then still covers most of the device; 0: none; 1: all whose workgroups are
 * resident together.  Errors: E_SHAPE.
 */
int elora_debug_decode_wide(int mode);

/*
 * Test hook: 0 makes every workgroup of the decode kernel walk its K-slice from the start; 1 (default) starts
 * the workgroups of an XCD at different places of their slices, so that they do not ask the same memory channels
 * for the same rows of x at the same moment.  Results differ only in the order of fp32 additions.  Errors: E_SHAPE.
 */
int elora_debug_k_rotate(int on);

/* ------------------------------------------------------------- profiling ---
 * Kernel timing for benchmarks (the roofline figure of a run is quoted on the
 * call's dominant kernel: the streaming contraction on the decode path, the
 * MFMA GEMM on the gemm path, the tiled base kernel on the generic path).
 *
 * elora_profile_arm(n): the next n calls of elora_batched_lora_linear each
 *   record one HIP event just before and one just after their dominant kernel,
 *   on the call's stream.  Creates 2n events (host objects, no device memory);
 *   a previous set is released.  n = 0 disarms.  Errors: E_SHAPE (n < 0 or
 *   n > 65536), E_HIP.
 * elora_profile_read(ms, n): waits for the recorded events and writes the
 *   elapsed milliseconds of the first min(n, recorded) calls to the HOST array
 *   ms; returns that count through *n_out.  Errors: E_NULL, E_HIP.
 * Process-wide, not thread-safe; meant for benchmarks only.
 */
int elora_profile_arm(int n_calls);
int elora_profile_read(float *ms, int n, int *n_out);

#ifdef __cplusplus
}
#endif
#endif /* ELORA_H */
