"""Pools whose adapters stay in 8-bit blocks (the paper keeps all adapters in the block format its settings call "Q8_0",
Sec. 5 "Model"): the linear kernels read codes and scales as they are.  Against the oracle on the same codes and scales
(value = scale * code exactly, no rounding of the adapter), through the C-ABI."""
import numpy as np
import pytest
import torch

from gpu_harness import DeviceCase, assert_close, rel_err, to_dev, y_to_f64
from paper_2507_01438_amd import inputs as I

pytestmark = pytest.mark.gpu
GENERIC, DECODE, GEMM = 0, 1, 2

SHAPES = [
    # (T, K, N, pool, ranks, no_adapter_rows)
    (1, 256, 16, 2, (8,), ()),
    (7, 512, 48, 3, (8, 16, 24), (2,)),
    (17, 1024, 1040, 5, (8, 16, 32, 64, 40), (0, 16)),
    (32, 4096, 256, 8, (16,), ()),
    (33, 2048, 272, 6, (16, 8), (5,)),
    (64, 1792, 144, 9, (8, 16, 32, 64), (63,)),       # 7 chunks of K: uneven K-slices
    (64, 2048, 4096, 4, (64, 8, 32), ()),             # 128-row tiles where they fill the device
    (50, 768, 16, 2, (8,), ()),
    (130, 1024, 272, 6, (8, 16, 32, 64, 24), (0, 64, 129)),   # several launches of the decode kernel
    (64, 512, 32768, 3, (8, 16), (3,)),               # 256 tiles of 128 rows, one K-slice per tile: the sums still go through the mailboxes
    (40, 256, 28672, 2, (16,), ()),                   # 224 such tiles
]


@pytest.mark.parametrize("path", [DECODE, GENERIC])
@pytest.mark.parametrize("shape", SHAPES)
def test_q8_pool_small_shapes(shape, path):
    T, K, N, pool, ranks, none_rows = shape
    rk = np.resize(np.asarray(ranks, dtype=np.int32), pool)
    w = I.small_workload(700 + T + N, I.BF16, K, N, T, pool, rk, no_adapter_rows=none_rows)
    case = DeviceCase(w, w.projections[0], q8=True)
    y = case.run(force_path=path)
    assert case.last_plan.path == path
    assert_close(y, case.reference(), case.base_reference(), f"q8 {shape}")
    assert np.array_equal(y, case.run(force_path=path))
    assert case.pool.poll_error() == (0, -1)
    if path == DECODE:
        case.B.elora_debug_spin_limit(0)        # every wait cut short: the fall-backs read the 8-bit blocks as well
        try:
            y0 = case.run(force_path=DECODE)
        finally:
            case.B.elora_debug_spin_limit(1 << 22)
        assert rel_err(y0, case.reference()) <= 1e-2
    case.close()


def test_q8_pool_rules_and_the_paths_it_takes():
    from paper_2507_01438_amd import binding as B
    assert B.elora_pool_storage_bytes_q8(4096, 4096, 64, 8) < 0.6 * B.elora_pool_storage_bytes(4096, 4096, 64, 8, B.ELORA_BF16)
    assert B.elora_pool_storage_bytes_q8(4096 + 16, 4096, 64, 8) == 0          # d_in a multiple of 32
    assert B.elora_pool_storage_bytes_q8(4096, 4096, 12, 8) == 0               # max_rank a multiple of 8
    w = I.small_workload(801, I.BF16, 512, 264, 300, 4, (8, 16), segments=[100, 200])
    case = DeviceCase(w, w.projections[0], q8=True)
    y = case.run()
    assert case.last_plan.path == GEMM         # many rows: the MFMA GEMM path turns the blocks into matrix-core operands
    assert rel_err(y, case.reference()) <= 1e-2
    # adapters in bf16 are refused by such a pool, and so are ranks that are no multiple of 8
    A = torch.zeros((8, 512), dtype=torch.int16)
    Bm = torch.zeros((264, 8), dtype=torch.int16)
    with pytest.raises(B.EloraError) as e:
        case.pool.load(0, A, Bm, 1.0)
    assert e.value.status == B.ELORA_E_DTYPE
    c4 = to_dev(np.zeros((4, 512), np.int8)); s4 = to_dev(np.zeros(64, np.uint16))
    b4 = to_dev(np.zeros((264, 4), np.int8)); t4 = to_dev(np.zeros(33, np.uint16))
    with pytest.raises(B.EloraError) as e:
        B.elora_pool_load_adapters_q8(case.pool.handle, [0], [4], [1.0], [c4], [s4], [b4], [t4])
    assert e.value.status == B.ELORA_E_RANK
    case.close()


@pytest.mark.parametrize("name", ["q", "k", "gate"])
def test_q8_pool_config3_full_shapes(name):
    """Config 3's projections with every adapter kept in 8-bit blocks: half the adapter bytes are read."""
    w = I.config3()
    proj = I.LLAMA8B[name]
    case = DeviceCase(w, proj, load_slots=w.distinct_adapters(), q8=True)
    y = case.run()
    assert case.last_plan.path == DECODE
    rng = np.random.default_rng(19)
    cols = np.unique(np.concatenate([rng.choice(proj.N, 128, replace=False), np.arange(8), np.arange(proj.N - 8, proj.N)]))
    e = assert_close(y[:, cols], case.reference(cols=cols), case.base_reference(cols=cols), f"q8 config3 {name}")
    print(f"config3 {name}, adapters in 8-bit blocks: rel err {e:.2e}, tile {case.last_plan.tile_rows}, split {case.last_plan.split_k}")
    assert case.pool.poll_error() == (0, -1)
    case.close()


def test_q8_pool_config2_full_shape():
    w = I.config2()
    case = DeviceCase(w, w.projections[0], q8=True)
    y = case.run()
    assert case.last_plan.path == DECODE
    e = assert_close(y, case.reference(), case.base_reference(), "q8 config2")
    print(f"config2, adapters in 8-bit blocks: rel err {e:.2e}")
    case.close()


GEMM_Q8 = [
    # (K, N, pool, ranks, segment lengths, adapter-less segments): prefill / mixed batches on a pool of 8-bit blocks
    (320, 136, 3, (16, 8, 24), [40, 3, 17, 1, 1, 90, 150], (2,)),
    (1024, 264, 4, (32, 16, 64, 8), [300, 20, 0, 257, 15], ()),        # runs crossing 256-row tiles
    (256, 520, 6, (16,), [1] * 70 + [130] + [1] * 60, (5, 100)),       # decode-like rows around a prompt: expand blocks
    (192, 72, 3, (8, 128), [70, 10, 300], ()),                         # rank 128: two expand items per run
]


@pytest.mark.parametrize("shape", GEMM_Q8)
def test_q8_pool_on_the_gemm_path(shape):
    K, N, pool, ranks, lengths, none_segs = shape
    w = I.small_workload(820 + K, I.BF16, K, N, sum(lengths), pool, ranks, segments=lengths, no_adapter_rows=none_segs)
    case = DeviceCase(w, w.projections[0], q8=True)
    y = case.run(force_path=GEMM)
    assert case.last_plan.path == GEMM
    assert_close(y, case.reference(), case.base_reference(), f"q8 gemm {shape}")
    assert np.array_equal(y, case.run(force_path=GEMM))
    # the generic kernels read the same blocks element by element
    y_gen = case.run(force_path=GENERIC)
    assert rel_err(y, y_gen) <= 1e-2
    assert case.pool.poll_error() == (0, -1)
    case.close()


def test_q8_pools_share_route_and_shrink_on_the_gemm_path():
    # gate and up of a prefill batch, each with its own pool of 8-bit blocks: one route and one shrink launch for both
    from paper_2507_01438_amd import binding as B
    lengths = [280, 40, 1, 1, 300]
    w = I.small_workload(830, I.BF16, 256, 264, sum(lengths), 4, (16, 8), segments=lengths)
    a = DeviceCase(w, w.projections[0], q8=True)
    b = DeviceCase(w, w.projections[0], q8=True, share=a)
    arr = B.desc_array([a.desc(), b.desc()])
    assert B.elora_linear_group_launches(arr) == 4          # route, shrink, two GEMMs
    B.elora_batched_lora_linear_group(arr)
    torch.cuda.synchronize()
    from gpu_harness import y_to_f64
    for c in (a, b):
        y = y_to_f64(c.y[: w.T], w.dtype)
        assert rel_err(y, c.reference()) <= 1e-2
    a.close(); b.close()


def _q8_decode_cases(T, K, Ns, ranks_of, seed, q8=(True, True, True)):
    cases = []
    for N, ranks, q in zip(Ns, ranks_of, q8):
        w = I.small_workload(seed, I.BF16, K, N, T, 6, ranks, no_adapter_rows=(T // 2,) if T > 1 else ())
        cases.append(DeviceCase(w, w.projections[0], q8=q))
    return cases


def _run_decode_group(B, cases, expect_launches):
    for c in cases:
        c.y.fill_(7)
    descs = B.desc_array([c.desc() for c in cases])
    assert B.elora_linear_group_launches(descs) == expect_launches
    B.elora_batched_lora_linear_group(descs)
    torch.cuda.synchronize()
    worst = 0.0
    for c in cases:
        e = rel_err(y_to_f64(c.y[: c.w.T], c.w.dtype), c.reference())
        assert e <= 1e-2, (c.proj.N, e)
        assert c.pool.poll_error() == (0, -1)
        worst = max(worst, e)
    return worst


@pytest.mark.parametrize("T,K,Ns", [(40, 1024, (272, 64, 128)), (20, 512, (4096, 1024)), (64, 2048, (144, 144, 1040)),
                                    (1, 256, (16, 32)), (33, 768, (80, 4096 + 64, 48))])
def test_q8_pools_in_one_decode_launch(T, K, Ns):
    # calls that are due together (Sec. 3.4: the layer's projections of one batch), each with a pool of 8-bit blocks
    from paper_2507_01438_amd import binding as B
    ranks_of = [(16, 8, 32), (8,), (8, 64, 16)][: len(Ns)]
    cases = _q8_decode_cases(T, K, Ns, ranks_of, seed=840 + T)
    e = _run_decode_group(B, cases, expect_launches=1)
    e2 = _run_decode_group(B, cases, expect_launches=1)       # mailboxes were left idle
    for c in cases:
        assert rel_err(c.run(), c.reference()) <= 1e-2        # and one by one on the same workspaces
    print(f"q8 group T={T} K={K} N={Ns}: rel err {e:.2e} / {e2:.2e}")
    for c in cases:
        c.close()


def test_pools_of_both_formats_do_not_share_a_decode_launch():
    from paper_2507_01438_amd import binding as B
    cases = _q8_decode_cases(24, 512, (96, 160), [(8, 16), (16,)], seed=850, q8=(True, False))
    _run_decode_group(B, cases, expect_launches=2)
    for c in cases:
        c.close()


@pytest.mark.parametrize("names", [("q", "k", "v"), ("gate", "up")])
def test_q8_pool_config3_groups_full_shapes(names):
    from paper_2507_01438_amd import binding as B
    w = I.config3()
    cases = [DeviceCase(w, I.LLAMA8B[n], load_slots=w.distinct_adapters(), q8=True) for n in names]
    descs = B.desc_array([c.desc() for c in cases])
    assert B.elora_linear_group_launches(descs) == 1
    B.elora_batched_lora_linear_group(descs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(19)
    for c, n in zip(cases, names):
        cols = np.sort(rng.choice(c.proj.N, 48, replace=False))
        y = y_to_f64(c.y[: w.T], w.dtype)
        e = rel_err(y[:, cols], c.reference(cols=cols))
        print(f"config3 q8 group {names}: {n} rel err {e:.2e}")
        assert e <= 1e-2
        assert c.pool.poll_error() == (0, -1)
        c.close()
