"""Parity of the linear layer on a base weight kept in 8-bit groups (Sec. 5 "Model": the Q8_0 base of setting S1),
element by element against the fp64 oracle, through the C-ABI, on every path that takes such a W."""
import numpy as np
import pytest

from paper_2507_01438_amd import inputs as I

pytestmark = pytest.mark.gpu

from gpu_harness import DeviceCase, rel_err  # noqa: E402

GENERIC, DECODE, GEMM = 0, 1, 2
TOL = 1e-2


def _case(seed, K, N, T, pool, ranks, **kw):
    w = I.small_workload(seed, I.BF16, K, N, T, pool, ranks, wfmt=I.W_INT8_G32, **kw)
    return DeviceCase(w, w.projections[0])


@pytest.mark.parametrize("shape", [
    (32, 8, 3, 2, (8,)),              # one group per row
    (96, 40, 17, 3, (8, 5)),          # odd rank, rows without adapter
    (320, 136, 70, 4, (16, 8, 24)),   # several tiles and a ragged tail
])
def test_generic_kernels_read_the_8bit_base(shape):
    K, N, T, pool, ranks = shape
    case = _case(900 + K, K, N, T, pool, ranks, no_adapter_rows=(1,))
    y = case.run(force_path=GENERIC)
    assert case.last_plan.path == GENERIC
    assert rel_err(y, case.reference()) <= TOL
    # the base alone, against the oracle's W x: an error in sign, group or row order of the codes shows here
    base = case.base_reference()
    ra = case.w.row_adapter()
    none = np.where(ra < 0)[0]
    assert none.size and np.max(np.abs(y[none] - base[none])) <= 8e-3 * np.max(np.abs(base))
    case.close()


def test_gemm_path_multiplies_from_a_bf16_copy():
    # more rows than the decode kernel takes: W is converted once per call (in the shrink's launch), then the bf16 GEMM
    lengths = [300, 1, 1, 200, 9, 60, 30]
    case = _case(901, 384, 272, sum(lengths), 4, (16, 8), segments=lengths)
    y = case.run()
    assert case.last_plan.path == GEMM and case.last_plan.n_launches == 3
    assert rel_err(y, case.reference()) <= TOL
    y2 = case.run()
    assert np.array_equal(y, y2)
    case.close()


def test_gemm_path_without_pool():
    w = I.small_workload(902, I.BF16, 256, 264, 300, 2, (8,), wfmt=I.W_INT8_G32)
    case = DeviceCase(w, w.projections[0])
    case.lin.pool = None
    d = case.lin.desc(case.x[: w.T], case.W, case.y, wfmt=w.wfmt, w_scales=case.w_scales)
    from paper_2507_01438_amd import binding as B
    import torch
    plan = B.elora_linear_plan(d)
    assert plan.path == GEMM
    B.elora_batched_lora_linear(d)
    torch.cuda.synchronize()
    from gpu_harness import y_to_f64
    y = y_to_f64(case.y[: w.T], w.dtype)
    assert rel_err(y, case.base_reference()) <= TOL
    case.close()


# (K, N, T, pool, ranks): the decode kernel with W read as 8-bit codes: 1 to 4 blocks of 16 rows of x, one to eight
# K-slices per tile, a ragged last tile, rows without adapter
W8_DECODE = [
    (256, 16, 1, 2, (8,)),
    (512, 80, 5, 3, (16, 8, 24)),
    (1024, 64, 16, 4, (8, 16)),
    (2048, 208, 20, 4, (16, 64, 8, 32)),
    (1024, 144, 33, 5, (8, 16, 32)),
    (4096, 256, 48, 4, (16,)),
    (2048, 528, 64, 6, (8, 16, 32, 64)),
    (4096, 4096, 32, 8, (16,)),
    (14336, 512, 64, 4, (8, 64)),
]


@pytest.mark.parametrize("shape", W8_DECODE)
def test_decode_kernel_reads_the_8bit_base(shape):
    K, N, T, pool, ranks = shape
    case = _case(910 + K + T, K, N, T, pool, ranks, no_adapter_rows=(0,) if T > 1 else ())
    y = case.run()
    assert case.last_plan.path == DECODE and case.last_plan.n_launches == 1
    ref = case.reference()
    assert rel_err(y, ref) <= TOL
    # row by row, and the adapter term on its own
    base = case.base_reference()
    assert np.max(np.max(np.abs(y - ref), axis=1) / np.max(np.abs(ref), axis=1)) <= 2e-2
    if np.max(np.abs(ref - base)) > 0:
        assert np.max(np.abs((y - base) - (ref - base))) / np.max(np.abs(ref - base)) <= 6e-2
    y2 = case.run()
    assert np.array_equal(y, y2)
    assert case.pool.poll_error() == (0, -1)
    case.close()


def test_decode_kernel_8bit_base_against_generic_kernels():
    # two independent readers of the same codes and scales on the device
    case = _case(930, 1024, 272, 40, 4, (8, 32))
    y_dec = case.run(force_path=DECODE)
    assert case.last_plan.path == DECODE
    y_gen = case.run(force_path=GENERIC)
    assert case.last_plan.path == GENERIC
    assert rel_err(y_dec, y_gen) <= TOL
    case.close()


@pytest.mark.parametrize("T", [65, 130, 256])
def test_8bit_base_65_to_256_rows_in_passes(T):
    case = _case(940 + T, 1024, 320, T, 6, (8, 16, 32))
    y = case.run()
    assert case.last_plan.path == DECODE and case.last_plan.n_launches == (T + 63) // 64
    assert rel_err(y, case.reference()) <= TOL
    case.close()


def test_8bit_base_when_waits_run_out():
    # a workgroup that gives up on the others recomputes its columns from the inputs: the 8-bit W has to be read there too
    from paper_2507_01438_amd import binding as B
    case = _case(950, 2048, 192, 24, 4, (16, 8))
    ref = case.reference()
    B.elora_debug_spin_limit(0)
    try:
        y = case.run()
    finally:
        B.elora_debug_spin_limit(1 << 22)
    assert case.last_plan.path == DECODE
    assert rel_err(y, ref) <= TOL
    y = case.run()
    assert rel_err(y, ref) <= TOL
    case.close()


W8_WIDE = [
    # (T, K, N, pool, ranks, no_adapter_rows): more than 32 rows, the kernel with 128-row tiles forced
    (33, 256, 128, 3, (8, 16), (1, 32)),       # one tile, one K-slice: sums stored straight from the accumulators
    (64, 512, 192, 4, (8, 16, 32, 64), ()),    # last tile half there, two K-slices: adapter term on the matrix cores
    (48, 1024, 1040, 5, (16,), (0,)),          # four K-slices
    (64, 4096, 400, 6, (8, 24, 64), (63,)),    # eight K-slices, last tile an eighth there
    (37, 768, 2048, 4, (8, 24, 40), ()),       # uneven K-slices
    (40, 512, 272, 4, (8, 20, 16, 3), (2,)),   # ranks that are no multiples of 8: the general tail
]


@pytest.mark.parametrize("spin", [None, 0])
@pytest.mark.parametrize("shape", W8_WIDE)
def test_wide_decode_kernel_reads_the_8bit_base(shape, spin):
    from paper_2507_01438_amd import binding as B
    T, K, N, pool, ranks, none_rows = shape
    rk = np.resize(np.asarray(ranks, dtype=np.int32), pool)
    case = _case(960 + T + N, K, N, T, pool, rk, no_adapter_rows=none_rows)
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
    assert rel_err(y, ref) <= TOL
    base = case.base_reference()
    if np.max(np.abs(ref - base)) > 0:
        assert np.max(np.abs((y - base) - (ref - base))) / np.max(np.abs(ref - base)) <= 6e-2
    if spin is None:
        assert np.array_equal(y, y2)
    else:
        assert rel_err(y2, ref) <= TOL
    y64 = case.run(force_path=DECODE)      # the same workspace serves the 64-row kernel right after
    assert rel_err(y64, ref) <= TOL
    assert case.pool.poll_error() == (0, -1)
    case.close()


@pytest.mark.parametrize("T,K,Ns", [(40, 1024, (272, 64, 128)), (20, 512, (4096, 1024)), (64, 2048, (144, 144, 1040)),
                                    (1, 256, (16, 32)), (64, 4096, (4096, 1024, 1024))])
def test_groups_of_calls_on_8bit_bases_run_as_one_launch(T, K, Ns):
    import torch
    from paper_2507_01438_amd import binding as B
    from gpu_harness import y_to_f64
    ranks_of = [(16, 8, 32), (8,), (5, 64, 16)][: len(Ns)]
    cases = []
    for N, ranks in zip(Ns, ranks_of):
        w = I.small_workload(970 + T, I.BF16, K, N, T, 6, ranks, wfmt=I.W_INT8_G32, no_adapter_rows=(T // 2,) if T > 1 else ())
        cases.append(DeviceCase(w, w.projections[0]))
    for rep in range(2):
        for c in cases:
            c.y.fill_(7)
        descs = B.desc_array([c.desc() for c in cases])
        assert B.elora_linear_group_launches(descs) == 1
        B.elora_batched_lora_linear_group(descs)
        torch.cuda.synchronize()
        for c in cases:
            assert rel_err(y_to_f64(c.y[: c.w.T], c.w.dtype), c.reference()) <= TOL, (c.proj.N, rep)
            assert c.pool.poll_error() == (0, -1)
    for c in cases:     # one by one on the same workspaces: the mailboxes were left idle
        assert rel_err(c.run(), c.reference()) <= TOL
        c.close()


def test_group_of_mixed_weight_formats_goes_call_by_call():
    import torch
    from paper_2507_01438_amd import binding as B
    from gpu_harness import y_to_f64
    w8 = I.small_workload(980, I.BF16, 512, 144, 24, 4, (8, 16), wfmt=I.W_INT8_G32)
    wb = I.small_workload(980, I.BF16, 512, 80, 24, 4, (8, 16))
    cases = [DeviceCase(w8, w8.projections[0]), DeviceCase(wb, wb.projections[0])]
    descs = B.desc_array([c.desc() for c in cases])
    assert B.elora_linear_group_launches(descs) == 2
    B.elora_batched_lora_linear_group(descs)
    torch.cuda.synchronize()
    for c in cases:
        assert rel_err(y_to_f64(c.y[: c.w.T], c.w.dtype), c.reference()) <= TOL
        c.close()
