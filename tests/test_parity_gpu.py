"""GPU parity: the HIP path, called through the C-ABI, against the fp64 oracle on the same seeded bytes.

Tolerances (max |y - ref| / max |ref|): 1e-2 for bf16 inputs with fp32 accumulation, 1e-5 for fp32.
Adapter routing is integer work and must be exact (routing probes)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2507_01438_amd import inputs as I  # noqa: E402
from gpu_harness import DeviceCase, assert_close, rel_err, to_dev, y_to_f64  # noqa: E402

TOL = {I.F32: 1e-5, I.BF16: 1e-2}
GENERIC, DECODE, GEMM = 0, 1, 2


def _check(case, y, ref, tol=None):
    e = rel_err(y, ref)
    assert e <= (tol or TOL[case.w.dtype]), f"{case.w.name}/{case.proj.name}: rel err {e:.3e} (path {case.last_plan.path})"
    return e


def test_config1_fp32_full():
    w = I.config1()
    case = DeviceCase(w, w.projections[0])
    y = case.run()
    assert case.last_plan.path == GENERIC
    _check(case, y, case.reference())
    assert case.pool.poll_error() == (0, -1)
    case.close()


@pytest.mark.parametrize("path", [DECODE, GENERIC])
def test_config2_qproj_decode_full(path):
    w = I.config2()
    case = DeviceCase(w, w.projections[0])
    y = case.run(force_path=path)
    assert case.last_plan.path == path
    ref = case.reference()
    e = _check(case, y, ref)
    print(f"config2 path {path}: rel err {e:.2e}")
    # the adapter term must be visible in the comparison: dropping it has to break the tolerance
    base_only = case.reference(row_adapter=np.full(w.T, -1, dtype=np.int32))
    assert rel_err(base_only, ref) > 5 * TOL[w.dtype]
    # same call twice: bit-identical (fixed summation order, no float atomics)
    y2 = case.run(force_path=path)
    assert np.array_equal(y, y2)
    case.close()


SMALL = [
    # (T, K, N, pool, ranks, no_adapter_rows)
    (1, 256, 16, 2, 4, ()),
    (7, 512, 48, 3, (1, 3, 8), (2,)),
    (16, 768, 80, 4, (16, 2, 5, 8), ()),
    (17, 1024, 1040, 5, (8, 16, 32, 64, 7), (0, 16)),
    (33, 2048, 272, 6, 16, (5,)),
    (64, 4096, 144, 9, (8, 16, 32, 64), (63,)),
    (50, 1280, 4096 + 64, 7, (12, 24, 40), ()),
    (32, 4096, 256, 8, 16, ()),
    (20, 256, 32, 3, (8, 100, 256), (1,)),          # ranks up to the maximum: several passes of rows in the expand
    (9, 1792, 64, 4, (40, 72, 9, 130), ()),         # 7 chunks of K: uneven K-slices
    (32, 2304, 48, 5, 64, (0, 31)),                 # last tile only three quarters there
    (48, 768, 16, 2, 8, ()),                        # one wave of the tile active
    (40, 512, 14336, 3, (16, 8, 32), (7,)),         # 224 tiles, 3 row blocks: W straight into registers, two workgroups per CU
    (24, 512, 4096, 3, 16, ()),                     # 64 tiles x 2 K-slices of 2 sub-spans: a ring that is never full
    (40, 512, 96, 4, (8, 20, 16, 3), (2,)),         # more than 32 rows, largest rank not a multiple of 8, mixed with odd ranks
    (36, 256, 32, 3, (8, 136, 72), ()),             # more than 32 rows, ranks above 64: several rounds of the expand
    (48, 512, 64, 3, (64, 8, 8), tuple(range(1, 48))),   # more than 32 rows, one of them with an adapter: 32 shrink units in all
    (48, 512, 64, 3, (64, 8, 8), tuple(range(48))),      # a pool, and no row uses it: no shrink unit at all
    (64, 1024, 128, 4, (1, 64, 3, 8), (10, 11)),         # ranks 1 to 64 side by side (one pair of rank rows to 32 per row)
    (64, 512, 32768, 3, (8, 16), (3,)),                  # 256 tiles of 128 rows: one K-slice per tile, sums straight to y
]


@pytest.mark.parametrize("path", [DECODE, GENERIC])
@pytest.mark.parametrize("shape", SMALL)
def test_small_decode_shapes(shape, path):
    T, K, N, pool, ranks, none_rows = shape
    rk = np.resize(np.asarray(ranks, dtype=np.int32), pool)
    w = I.small_workload(100 + T, I.BF16, K, N, T, pool, rk, no_adapter_rows=none_rows)
    case = DeviceCase(w, w.projections[0])
    y = case.run(force_path=path)
    assert case.last_plan.path == path
    _check(case, y, case.reference())
    assert case.pool.poll_error() == (0, -1)
    case.close()


WIDE = [
    # (T, K, N, pool, ranks, no_adapter_rows): more than 32 rows; the kernel with 128-row tiles is forced
    (33, 256, 128, 3, (8, 16), (1, 32)),                  # one tile, one K-slice: sums stored straight from the accumulators
    (64, 512, 192, 4, (8, 16, 32, 64), ()),               # last tile half there, two K-slices: adapter term on the matrix cores
    (48, 1024, 1040, 5, (16,), (0,)),                     # last tile: one wave of eight; four K-slices
    (64, 4096, 400, 6, (8, 24, 64), (63,)),               # eight K-slices, last tile an eighth there
    (37, 768, 2048, 4, (8, 24, 40), ()),                  # 3 chunks of K on two K-slices: uneven slices
    (64, 2048, 4096, 3, (64,), ()),                       # every rank 64: two matrix instructions per row
    (50, 256, 16, 2, (8,), (49,)),                        # one wave of the tile active
    (40, 512, 272, 4, (8, 20, 16, 3), (2,)),              # ranks that are no multiples of 8: the general tail
    (36, 256, 144, 3, (8, 136, 72), ()),                  # ranks above 64: the general tail, several rounds
    (64, 1024, 256, 4, (1, 64, 3, 8), (10, 11)),          # ranks 1 to 64 side by side
    (48, 512, 128, 3, (64, 8, 8), tuple(range(48))),      # a pool, and no row uses it
]


@pytest.mark.parametrize("spin", [None, 0])
@pytest.mark.parametrize("shape", WIDE)
def test_wide_decode_kernel_small_shapes(shape, spin):
    from paper_2507_01438_amd import binding as B
    T, K, N, pool, ranks, none_rows = shape
    rk = np.resize(np.asarray(ranks, dtype=np.int32), pool)
    w = I.small_workload(500 + T + N, I.BF16, K, N, T, pool, rk, no_adapter_rows=none_rows)
    case = DeviceCase(w, w.projections[0])
    ref = case.reference()
    B.elora_debug_decode_wide(1)
    if spin is not None:
        B.elora_debug_spin_limit(spin)
    try:
        y = case.run(force_path=DECODE)
        assert case.last_plan.path == DECODE and case.last_plan.tile_rows == 128
        y2 = case.run(force_path=DECODE)
    finally:
        B.elora_debug_decode_wide(-1)
        B.elora_debug_spin_limit(1 << 22)
    assert_close(y, ref, case.base_reference(), f"wide {shape}")
    if spin is None:
        assert np.array_equal(y, y2)       # fixed summation order
    else:
        _check(case, y2, ref)
    y64 = case.run(force_path=DECODE)      # the same workspace serves the 64-row kernel right after
    _check(case, y64, ref)
    assert case.pool.poll_error() == (0, -1)
    case.close()


@pytest.mark.parametrize("T", [65, 128, 130, 255, 256])
@pytest.mark.parametrize("segments", [False, True])
def test_65_to_256_rows_run_as_several_launches_of_the_decode_kernel(T, segments):
    """Balanced row ranges, one launch each, on one workspace: per-row and per-segment routing, scale overrides that
    are indexed by the batch's rows (or segments), and bad indices reported with the batch's row numbers."""
    from paper_2507_01438_amd import binding as B
    lengths = None
    if segments:
        lengths = [40, 0, 1, T - 40 - 1 - 17, 17]      # segments that straddle the row ranges
    w = I.small_workload(600 + T, I.BF16, 1024, 272, T, 9, (8, 16, 32, 64, 24), segments=lengths,
                         no_adapter_rows=(1,) if segments else (0, 64, T - 1))
    case = DeviceCase(w, w.projections[0])
    y = case.run()
    assert case.last_plan.path == DECODE and case.last_plan.n_launches == (T + 63) // 64
    ref = case.reference()
    assert_close(y, ref, case.base_reference(), f"{T} rows")
    assert np.array_equal(y, case.run())
    n_sc = len(lengths) if segments else T
    sc = np.linspace(-1.5, 2.5, n_sc).astype(np.float32)
    row_scale = np.repeat(sc, lengths).astype(np.float32) if segments else sc
    _check(case, case.run(scales=to_dev(sc)), case.reference(row_scale=row_scale))
    # the MFMA GEMM path on the same call
    B.elora_debug_decode_passes(0)
    try:
        yg = case.run()
        assert case.last_plan.path == GEMM
    finally:
        B.elora_debug_decode_passes(-1)
    _check(case, yg, ref)
    assert case.pool.poll_error() == (0, -1)
    if not segments:
        bad = w.adapter_idx.copy()
        first = T // 2 + 3                              # in the second row range, like the last row but one
        bad[first], bad[T - 2] = 99, -7
        case.adapter_idx.copy_(to_dev(bad))
        cleaned = bad.copy()
        cleaned[first] = cleaned[T - 2] = -1
        _check(case, case.run(), case.reference(row_adapter=cleaned))
        assert case.pool.poll_error() == (2, first)
    case.close()


def test_waits_that_run_out_of_time_fall_back_to_the_inputs():
    """With a time bound of one microsecond on every wait between workgroups (the poll bound left alone), waits that are
    not served at once give up and compute from the inputs; results stay right, and the workspace is clean afterwards."""
    from paper_2507_01438_amd import binding as B
    w = I.small_workload(63, I.BF16, 2048, 1040, 48, 6, (8, 16, 24, 32), no_adapter_rows=(4,))
    case = DeviceCase(w, w.projections[0])
    ref = case.reference()
    B.elora_debug_wait_limit_us(1)
    try:
        for _ in range(3):
            _check(case, case.run(force_path=DECODE), ref)
    finally:
        B.elora_debug_wait_limit_us(200)
    y = case.run(force_path=DECODE)
    _check(case, y, ref)
    assert np.array_equal(y, case.run(force_path=DECODE))
    case.close()


def test_a_workspace_serves_one_d_out_until_it_is_initialised_again():
    """The first call ties a workspace to its d_out; a call with another d_out on it is refused (what it writes would lie
    in the other's mailboxes), whatever path it takes; other row counts and d_in are fine; initialising frees it."""
    from paper_2507_01438_amd import binding as B
    wa = I.small_workload(71, I.BF16, 512, 4096, 24, 3, (8, 16))
    wb = I.small_workload(72, I.BF16, 512, 1024, 300, 3, (8, 16))      # many rows: the MFMA GEMM path, smaller d_out
    a, b = DeviceCase(wa, wa.projections[0]), DeviceCase(wb, wb.projections[0])
    big = max(a.lin.ws_bytes, b.lin.ws_bytes)
    ws = torch.empty(big, dtype=torch.uint8, device="cuda:0")
    B.elora_workspace_init(ws, big)
    da, db = a.desc(), b.desc()
    for d in (da, db):
        d.workspace, d.workspace_bytes = ws.data_ptr(), big
    B.elora_batched_lora_linear(db)                      # ties the workspace to d_out = 1024
    with pytest.raises(B.EloraError) as e:
        B.elora_batched_lora_linear(da)
    assert e.value.status == B.ELORA_E_STORAGE
    with pytest.raises(B.EloraError) as e:
        B.elora_linear_plan(da)
    assert e.value.status == B.ELORA_E_STORAGE
    torch.cuda.synchronize()
    assert rel_err(y_to_f64(b.y[: wb.T], I.BF16), b.reference()) <= 1e-2
    B.elora_workspace_init(ws, big)                      # idle again, and free for any d_out
    B.elora_batched_lora_linear(da)
    torch.cuda.synchronize()
    assert rel_err(y_to_f64(a.y[: wa.T], I.BF16), a.reference()) <= 1e-2
    with pytest.raises(B.EloraError):
        B.elora_batched_lora_linear(db)
    # same d_out, other row counts, on the tied workspace: generic and decode calls in turn
    for T in (24, 5, 1):
        wa.adapter_idx = wa.adapter_idx[:T].copy()
        a.adapter_idx = to_dev(wa.adapter_idx)
        a.x_h = a.x_h[:T]
        d = a.desc()
        d.workspace, d.workspace_bytes = ws.data_ptr(), big
        for path in (GENERIC, DECODE):
            a.y.fill_(7)
            B.elora_force_path(path)
            try:
                B.elora_batched_lora_linear(d)
            finally:
                B.elora_force_path(-1)
            torch.cuda.synchronize()
            assert rel_err(y_to_f64(a.y[:T], I.BF16), a.reference()) <= 1e-2
    a.close()
    b.close()


@pytest.mark.parametrize("dtype,K,N", [(I.F32, 100, 30), (I.BF16, 72, 19), (I.F32, 512, 130)])
def test_odd_shapes_take_the_generic_kernels(dtype, K, N):
    w = I.small_workload(7, dtype, K, N, 13, 4, (3, 5, 1, 8), no_adapter_rows=(4,), x_std=1.0)
    case = DeviceCase(w, w.projections[0])
    y = case.run()
    assert case.last_plan.path == GENERIC
    _check(case, y, case.reference())
    case.close()


@pytest.mark.parametrize("path", [DECODE, GENERIC])
def test_segment_routing_with_empty_and_adapterless_segments(path):
    lengths = [5, 0, 1, 20, 0, 0, 7, 3]
    w = I.small_workload(21, I.BF16, 512, 256, sum(lengths), 5, (8, 16, 4, 32, 2), segments=lengths,
                         no_adapter_rows=(3,))
    case = DeviceCase(w, w.projections[0])
    y = case.run(force_path=path)
    assert case.last_plan.path == path
    _check(case, y, case.reference())
    # per-segment scale override
    seg_scales = np.linspace(-1.0, 3.0, len(lengths)).astype(np.float32)
    y = case.run(scales=to_dev(seg_scales), force_path=path)
    row_scale = np.repeat(seg_scales, lengths).astype(np.float32)
    _check(case, y, case.reference(row_scale=row_scale))
    case.close()


@pytest.mark.parametrize("path", [DECODE, GENERIC])
def test_per_row_scale_override(path):
    w = I.small_workload(22, I.BF16, 512, 128, 19, 4, 8)
    case = DeviceCase(w, w.projections[0])
    rs = np.linspace(-2.0, 2.0, w.T).astype(np.float32)
    y = case.run(scales=to_dev(rs), force_path=path)
    _check(case, y, case.reference(row_scale=rs))
    case.close()


@pytest.mark.parametrize("path", [DECODE, GENERIC])
def test_routing_probes_are_bit_exact(path):
    """W = 0, x_t = e_0, A_i[0,0] = 1, B_i[0,0] = i mod 256, B_i[1,0] = i div 256, scale 1:
    y[t,0] + 256 y[t,1] spells the adapter index that was applied to row t."""
    from paper_2507_01438_amd import binding as B
    P, K, N, T = 600, 256, 16, 64
    rng = np.random.default_rng(3)
    pool = B.AdapterPool(K, N, 4, P, B.ELORA_BF16)
    for i in range(P):
        A = np.zeros((1, K), np.float32); A[0, 0] = 1
        Bm = np.zeros((N, 1), np.float32); Bm[0, 0] = i % 256; Bm[1, 0] = i // 256
        pool.load(i, torch.from_numpy(I.f32_to_bf16_bits(A).view(np.int16)),
                  torch.from_numpy(I.f32_to_bf16_bits(Bm).view(np.int16)), 1.0)
    x = np.zeros((T, K), np.float32); x[:, 0] = 1
    idx = rng.integers(0, P, size=T).astype(np.int32)
    idx[5] = -1
    lin = B.LoraLinear(K, N, B.ELORA_BF16, pool, T)
    y = torch.zeros((T, N), dtype=torch.int16, device="cuda:0")
    xd, Wd, idxd = to_dev(I.f32_to_bf16_bits(x)), to_dev(np.zeros((N, K), np.uint16)), to_dev(idx)
    B.elora_force_path(path)
    try:
        lin(xd, Wd, y, adapter_idx=idxd)
    finally:
        B.elora_force_path(-1)
    torch.cuda.synchronize()
    yh = y_to_f64(y, I.BF16)
    spelled = (yh[:, 0] + 256 * yh[:, 1]).astype(np.int64)
    want = np.where(idx >= 0, idx, 0)
    assert np.array_equal(spelled, want)
    assert np.all(yh[:, 2:] == 0)
    pool.close()


@pytest.mark.parametrize("path", [DECODE, GENERIC])
def test_bad_and_evicted_indices_fall_back_to_base_and_are_reported(path):
    w = I.small_workload(31, I.BF16, 512, 64, 12, 4, 8)
    w.adapter_idx = np.array([0, 1, 2, 3, 99, 1, -5, 2, 2, 0, 3, 1], dtype=np.int32)
    case = DeviceCase(w, w.projections[0])
    case.pool.evict(3)
    y = case.run(force_path=path)
    cleaned = np.array([0, 1, 2, -1, -1, 1, -1, 2, 2, 0, -1, 1], dtype=np.int32)
    _check(case, y, case.reference(row_adapter=cleaned))
    assert case.pool.poll_error() == (4, 3)      # rows 3, 4, 6, 10; smallest is 3
    assert case.pool.poll_error() == (0, -1)     # cleared
    case.close()


def test_empty_batch_and_base_only_calls():
    from paper_2507_01438_amd import binding as B
    w = I.small_workload(41, I.BF16, 512, 64, 9, 2, 8)
    case = DeviceCase(w, w.projections[0])
    d = case.desc()
    d.n_tokens = 0
    B.elora_batched_lora_linear(d)               # nothing to do, no error
    lin = B.LoraLinear(512, 64, B.ELORA_BF16, None, 9)
    y = torch.zeros((9, 64), dtype=torch.int16, device="cuda:0")
    lin(case.x, case.W, y)
    torch.cuda.synchronize()
    ref = case.reference(row_adapter=np.full(9, -1, dtype=np.int32))
    assert rel_err(y_to_f64(y, I.BF16), ref) <= 1e-2
    case.close()


def test_reloading_a_slot_replaces_the_adapter():
    w = I.small_workload(51, I.BF16, 512, 64, 6, 3, (8, 4, 8))
    w.adapter_idx = np.array([0, 1, 2, 1, 1, 0], dtype=np.int32)
    case = DeviceCase(w, w.projections[0])
    A, Bm, s = w.adapter(w.projections[0], 2)    # put slot 2's rank-8 adapter into slot 1 (was rank 4)
    case.pool.load(1, torch.from_numpy(A.view(np.int16)), torch.from_numpy(Bm.view(np.int16)), 0.5)
    case.adapters[1] = (A, Bm, 0.5)
    y = case.run()
    _check(case, y, case.reference())
    assert case.B.elora_pool_slot_info(case.pool.handle, 1) == (8, 0.5)
    case.close()


@pytest.mark.parametrize("name", ["q", "k", "v", "o", "gate", "up", "down"])
def test_config3_layer_decode_full_shapes(name):
    """All seven projections at their real shapes, 64 rows, 256 adapters of mixed rank; the oracle
    computes every row on a seeded sample of 256 columns plus the first and last 16 columns."""
    w = I.config3()
    proj = I.LLAMA8B[name]
    used = w.distinct_adapters()
    case = DeviceCase(w, proj, load_slots=used)
    y = case.run()
    assert case.last_plan.path == DECODE
    rng = np.random.default_rng(9)
    cols = np.unique(np.concatenate([rng.choice(proj.N, 256, replace=False), np.arange(16), np.arange(proj.N - 16, proj.N)]))
    ref = case.reference(cols=cols)
    e = assert_close(y[:, cols], ref, case.base_reference(cols=cols), f"config3 {name}")
    print(f"config3 {name}: rel err {e:.2e}, tile {case.last_plan.tile_rows}, split_k {case.last_plan.split_k}, grid {case.last_plan.grid}")
    assert case.pool.poll_error() == (0, -1)
    # the kernel with 64-row tiles on the same call (the one with 128-row tiles is the default where its grid fills the device)
    case.B.elora_debug_decode_wide(0)
    try:
        y64 = case.run()
        assert case.last_plan.tile_rows == 64
    finally:
        case.B.elora_debug_decode_wide(-1)
    assert_close(y64[:, cols], ref, case.base_reference(cols=cols), f"config3 {name}, 64-row tiles")
    case.close()


def test_decode_epilogue_without_the_shrink_hand_off():
    """With the internal wait's bound at 0 every tile epilogue recomputes A_i x_t itself; the
    result must still match, and the counters must be left clean for the next (normal) call."""
    w = I.small_workload(61, I.BF16, 1024, 528, 37, 6, (8, 16, 24, 3), no_adapter_rows=(1,))
    case = DeviceCase(w, w.projections[0])
    ref = case.reference()
    case.B.elora_debug_spin_limit(0)
    try:
        y0 = case.run(force_path=DECODE)
    finally:
        case.B.elora_debug_spin_limit(1 << 22)
    _check(case, y0, ref)
    y1 = case.run(force_path=DECODE)
    _check(case, y1, ref)
    case.close()


def test_decode_without_the_one_xcd_guarantee():
    """The hand-overs between workgroups normally meet in the L2 of the XCD they share; without that
    guarantee they go through memory.  Same results either way, also when the waits are cut short."""
    w = I.small_workload(62, I.BF16, 2048, 1040, 30, 6, (8, 16, 24, 32), no_adapter_rows=(4,))
    case = DeviceCase(w, w.projections[0])
    ref = case.reference()
    y_local = case.run(force_path=DECODE)
    case.B.elora_debug_xcd_local(0)
    try:
        y_mem = case.run(force_path=DECODE)
        assert np.array_equal(y_local, y_mem)
        case.B.elora_debug_spin_limit(0)
        try:
            y_slow = case.run(force_path=DECODE)
        finally:
            case.B.elora_debug_spin_limit(1 << 22)
        _check(case, y_slow, ref)
        y_again = case.run(force_path=DECODE)
        assert np.array_equal(y_local, y_again)
    finally:
        case.B.elora_debug_xcd_local(-1)
    _check(case, y_local, ref)
    case.close()


def test_decode_back_to_back_calls_share_one_workspace():
    """Many calls in a row on one stream and one workspace: the counters a call leaves behind
    must be exactly what the next call expects (checked on the last result and on a changed batch)."""
    w = I.config2()
    case = DeviceCase(w, w.projections[0])
    d = case.desc()
    for _ in range(50):
        case.B.elora_batched_lora_linear(d)
    torch.cuda.synchronize()
    y = y_to_f64(case.y[: w.T], w.dtype)
    ref = case.reference()
    assert rel_err(y, ref) <= 1e-2
    # smaller batch on the same workspace afterwards
    w.adapter_idx = w.adapter_idx[:9].copy()
    case.adapter_idx = to_dev(w.adapter_idx)
    case.x_h = case.x_h[:9]
    y9 = case.run()
    assert rel_err(y9, case.reference()) <= 1e-2
    case.close()


def test_decode_calls_replay_from_a_hip_graph():
    """A layer's worth of decode calls captured once and replayed: every replay must leave the mailboxes and counters
    as the next one expects them.  Replays alternate with eager work on the same workspace and a changed x, and every
    replay is checked against the oracle (the eager result of the same inputs is checked by the other tests)."""
    w = I.small_workload(777, I.BF16, 1024, 512, 24, 6, (8, 16, 16, 8, 16, 8), no_adapter_rows=(3,))
    case = DeviceCase(w, w.projections[0])
    d = case.desc()
    case.B.elora_batched_lora_linear(d)  # warm-up outside the capture: one-time set-up of the kernel happens here
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for _ in range(3):
            case.B.elora_batched_lora_linear(d, stream=side)
    rng = np.random.default_rng(5)
    for rep in range(4):
        # new activations in place (same buffers, so the captured descriptor stays valid)
        xn = I.f32_to_bf16_bits((rng.standard_normal(case.x_h.shape) * (0.5 + rep)).astype(np.float32))
        case.x_h = xn
        case.x.copy_(to_dev(xn))
        case.y.fill_(7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        y = y_to_f64(case.y[: w.T], w.dtype)
        assert rel_err(y, case.reference()) <= 1e-2, f"replay {rep}"
        # eager work between the replays
        y_eager = case.run()
        assert rel_err(y_eager, case.reference()) <= 1e-2
        np.testing.assert_array_equal(y, y_eager)  # fixed summation order: bit-identical
    assert case.pool.poll_error() == (0, -1)
    case.close()


# ---------------------------------------------------------------------------------------------
# prefill / mixed path (LDS-tiled MFMA GEMM with the expand as K-extension)
# ---------------------------------------------------------------------------------------------

GEMM_SMALL = [
    # (K, N, pool, ranks, segment lengths, adapter-less segments)
    (64, 8, 2, (8,), [1], ()),
    (320, 136, 3, (16, 8, 24), [40, 3, 17, 1, 1, 90], (2,)),
    (1024, 264, 4, (32, 16, 64, 8), [300, 20, 0, 257, 15], ()),          # runs crossing 256-row tiles
    (512, 520, 5, (5, 16, 3, 8, 12), [100, 64, 30, 16, 50], (1,)),        # odd ranks: per-row expand
    (256, 2048 + 40, 6, (16,), [1] * 70 + [130] + [1] * 60, (5, 100)),    # decode-like rows around a prompt
    (192, 72, 3, (8, 16), [70, 10, 300], ()),                             # three K blocks: one straight-line iteration
    (128, 264, 2, (16,), [260], ()),                                      # two K blocks: the general loop only
    # runs of at most 32 rows (added after the K loop) across 32-, 128- and 256-row boundaries, ranks up to 256
    (256, 264, 5, (64, 8, 256, 32, 48), [30, 3, 31, 1, 40, 23, 2, 20, 31, 32, 33, 8, 1, 1, 28, 5], (3,)),
    (64, 264, 300, (256,), [1] * 300, ()),          # a run per row, every rank 256: the step table of a 32-row block is full
    (128, 72, 7, (16, 8), [1] * 45, (4, 44)),       # short runs only, one partial tile in both directions
    (192, 776, 6, (8, 24, 40), [5, 1, 1, 32, 2, 31, 9, 1] * 9, ()),   # short runs only, four column tiles, 2.5 row tiles
    (128, 264, 3, (32,), [250, 6], ()),             # a prompt's expand block has room for the short run behind it
    (128, 264, 3, (64, 32), [250, 6], ()),          # ... and here it has not (rank 64 fills the block): added after the loop
]


@pytest.mark.parametrize("shape", GEMM_SMALL)
def test_gemm_path_small_shapes(shape):
    K, N, pool, ranks, lengths, none_segs = shape
    w = I.small_workload(300 + K, I.BF16, K, N, sum(lengths), pool, ranks, segments=lengths, no_adapter_rows=none_segs)
    case = DeviceCase(w, w.projections[0])
    y = case.run(force_path=GEMM)
    assert case.last_plan.path == GEMM
    _check(case, y, case.reference())
    assert case.pool.poll_error() == (0, -1)
    y2 = case.run(force_path=GEMM)
    assert np.array_equal(y, y2)
    case.close()


def test_gemm_path_with_per_row_indices_and_scales():
    w = I.small_workload(77, I.BF16, 512, 328, 333, 7, (16, 8, 32), no_adapter_rows=(0, 100, 332))
    w.adapter_idx[40:200] = 3          # a long run in the middle of scattered indices
    case = DeviceCase(w, w.projections[0])
    rs = np.linspace(0.5, 2.5, w.T).astype(np.float32)
    y = case.run(scales=to_dev(rs), force_path=GEMM)
    assert case.last_plan.path == GEMM
    _check(case, y, case.reference(row_scale=rs))
    case.close()


def test_gemm_path_int4_small():
    lengths = [70, 1, 1, 1, 200, 30]
    w = I.small_workload(88, I.BF16, 384, 272, sum(lengths), 4, (16, 8), wfmt=I.W_INT4_G32, segments=lengths)
    case = DeviceCase(w, w.projections[0])
    y = case.run()
    assert case.last_plan.path == GEMM
    _check(case, y, case.reference())
    case.close()


def test_gemm_path_int4_converted_once_for_many_rows():
    # from 768 rows on the 4-bit W is converted to bf16 once per call instead of tile by tile, in the shrink's launch
    lengths = [400, 1, 1, 300, 9, 60, 30]
    w = I.small_workload(89, I.BF16, 384, 272, sum(lengths), 4, (16, 8), wfmt=I.W_INT4_G32, segments=lengths)
    case = DeviceCase(w, w.projections[0])
    y = case.run()
    assert case.last_plan.path == GEMM and case.last_plan.n_launches == 3
    _check(case, y, case.reference())
    y2 = case.run()   # the copy in the workspace is rebuilt by every call
    assert np.array_equal(y, y2)
    case.close()


def test_gemm_routing_probes_are_bit_exact():
    from paper_2507_01438_amd import binding as B
    P, K, N = 300, 64, 16
    lengths = [1] * 40 + [33, 100, 17] + [1] * 25
    T = sum(lengths)
    rng = np.random.default_rng(4)
    pool = B.AdapterPool(K, N, 8, P, B.ELORA_BF16)
    for i in range(P):
        A = np.zeros((8, K), np.float32); A[0, 0] = 1
        Bm = np.zeros((N, 8), np.float32); Bm[0, 0] = i % 256; Bm[1, 0] = i // 256
        pool.load(i, torch.from_numpy(I.f32_to_bf16_bits(A).view(np.int16)),
                  torch.from_numpy(I.f32_to_bf16_bits(Bm).view(np.int16)), 1.0)
    x = np.zeros((T, K), np.float32); x[:, 0] = 1
    seg_adapter = rng.integers(0, P, size=len(lengths)).astype(np.int32)
    lin = B.LoraLinear(K, N, B.ELORA_BF16, pool, T)
    y = torch.zeros((T, N), dtype=torch.int16, device="cuda:0")
    B.elora_force_path(GEMM)
    try:
        lin(to_dev(I.f32_to_bf16_bits(x)), to_dev(np.zeros((N, K), np.uint16)), y,
            seg_offsets=to_dev(I.offsets_from_lengths(lengths)), seg_adapter=to_dev(seg_adapter))
    finally:
        B.elora_force_path(-1)
    torch.cuda.synchronize()
    yh = y_to_f64(y, I.BF16)
    assert np.array_equal((yh[:, 0] + 256 * yh[:, 1]).astype(np.int64), np.repeat(seg_adapter, lengths))
    pool.close()


def _sampled_check(case, w, proj, n_cols=64, n_rows=32, seed=5):
    """All rows on a seeded sample of columns, and all columns on the first/last row of every
    segment plus a seeded sample of rows; each sample also with the adapter term alone and row by row."""
    y = case.run()
    rng = np.random.default_rng(seed)
    cols = np.sort(rng.choice(proj.N, n_cols, replace=False))
    e1 = assert_close(y[:, cols], case.reference(cols=cols), case.base_reference(cols=cols), f"{w.name}/{proj.name} columns")
    so = w.seg_offsets
    edge = [int(so[s]) for s in range(len(so) - 1) if so[s + 1] > so[s]] + \
           [int(so[s + 1] - 1) for s in range(len(so) - 1) if so[s + 1] > so[s]]
    rows = np.unique(np.concatenate([np.array(edge, dtype=np.int64), rng.choice(w.T, n_rows, replace=False)]))
    e2 = assert_close(y[rows], case.reference(rows=rows), case.base_reference(rows=rows), f"{w.name}/{proj.name} rows")
    return max(e1, e2)


@pytest.mark.parametrize("name", ["gate", "up", "down"])
def test_config4_prefill_segments_full_shapes(name):
    w = I.config4()
    proj = I.LLAMA8B[name]
    case = DeviceCase(w, proj, load_slots=w.distinct_adapters())
    e = _sampled_check(case, w, proj)
    assert case.last_plan.path == GEMM
    print(f"config4 {name}: T={w.T} rel err {e:.2e} grid {case.last_plan.grid}")
    assert e <= 1e-2
    assert case.pool.poll_error() == (0, -1)
    case.close()


def test_config5_mixed_int4_full_shape():
    w = I.config5()
    proj = w.projections[0]
    case = DeviceCase(w, proj, load_slots=w.distinct_adapters())
    e = _sampled_check(case, w, proj, n_rows=48)
    assert case.last_plan.path == GEMM
    print(f"config5: T={w.T} rel err {e:.2e}")
    assert e <= 1e-2
    case.close()


@pytest.mark.parametrize("T,K,N", [(24, 512, 96), (64, 1024, 1040)])
def test_decode_follows_the_ranks_the_pool_holds(T, K, N):
    """The decode path has instances without the tail for ranks that are no multiples of 8; which one a call takes
    follows what the pool holds when the call is made (Sec. 3.3 / 4.2: adapters come and go between batches)."""
    w = I.small_workload(1300 + T, I.BF16, K, N, T, 4, (8, 16, 32, 5))
    idx_even = (np.arange(T) % 3).astype(np.int32)          # rows use slots 0..2: ranks 8, 16, 32
    idx_all = (np.arange(T) % 4).astype(np.int32)           # ... and slot 3: rank 5
    w.adapter_idx = idx_even
    case = DeviceCase(w, w.projections[0], load_slots=[0, 1, 2])
    assert rel_err(case.run(), case.reference()) <= TOL[w.dtype]
    # the adapter of rank 5 arrives: rows that use it, and rows that do not
    A, Bm, s = w.adapter(w.projections[0], 3)
    case.adapters[3] = (A, Bm, s)
    case.pool.load(3, torch.from_numpy(A.view(np.int16)), torch.from_numpy(Bm.view(np.int16)), s)
    w.adapter_idx = idx_all
    case.adapter_idx.copy_(torch.from_numpy(idx_all))
    y = case.run()
    assert case.last_plan.path == DECODE
    assert rel_err(y, case.reference()) <= TOL[w.dtype]
    w.adapter_idx = idx_even
    case.adapter_idx.copy_(torch.from_numpy(idx_even))
    assert rel_err(case.run(), case.reference()) <= TOL[w.dtype]
    # and leaves again
    case.pool.evict(3)
    del case.adapters[3]
    assert rel_err(case.run(), case.reference()) <= TOL[w.dtype]
    assert case.pool.poll_error() == (0, -1)
    case.close()
