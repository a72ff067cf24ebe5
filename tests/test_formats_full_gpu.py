"""The 8-bit storage formats (Sec. 5 "Model": Q8_0 base and Q8_0 adapters) at the benchmark configurations' full
shapes, through the C-ABI, against the oracle on seeded samples of rows and columns."""
import numpy as np
import pytest

from paper_2507_01438_amd import inputs as I

pytestmark = pytest.mark.gpu

from gpu_harness import DeviceCase, assert_close, rel_err  # noqa: E402

GENERIC, DECODE, GEMM = 0, 1, 2


def _sampled(case, w, proj, n_cols=64, n_rows=32, seed=5):
    y = case.run()
    rng = np.random.default_rng(seed)
    cols = np.sort(rng.choice(proj.N, n_cols, replace=False))
    e1 = assert_close(y[:, cols], case.reference(cols=cols), case.base_reference(cols=cols), f"{w.name}/{proj.name} columns")
    if w.seg_offsets is not None:
        so = w.seg_offsets
        edge = [int(so[s]) for s in range(len(so) - 1) if so[s + 1] > so[s]] + [int(so[s + 1] - 1) for s in range(len(so) - 1) if so[s + 1] > so[s]]
    else:
        edge = [0, w.T - 1]
    rows = np.unique(np.concatenate([np.array(edge, dtype=np.int64), rng.choice(w.T, min(n_rows, w.T), replace=False)]))
    e2 = assert_close(y[rows], case.reference(rows=rows), case.base_reference(rows=rows), f"{w.name}/{proj.name} rows")
    return max(e1, e2)


@pytest.mark.parametrize("name", ["q", "k", "gate", "down"])
def test_config3_on_an_8bit_base(name):
    w = I.config3()
    w.wfmt = I.W_INT8_G32
    proj = I.LLAMA8B[name]
    case = DeviceCase(w, proj, load_slots=w.distinct_adapters())
    e = _sampled(case, w, proj, n_cols=256)
    assert case.last_plan.path == DECODE
    print(f"config3 {name}, 8-bit base: rel err {e:.2e}, tile {case.last_plan.tile_rows}, split_k {case.last_plan.split_k}")
    assert e <= 1e-2
    assert case.pool.poll_error() == (0, -1)
    case.close()


def test_config2_on_an_8bit_base():
    w = I.config2()
    w.wfmt = I.W_INT8_G32
    proj = w.projections[0]
    case = DeviceCase(w, proj)
    y = case.run()
    assert case.last_plan.path == DECODE
    e = assert_close(y, case.reference(), case.base_reference(), "config2, 8-bit base")
    print(f"config2, 8-bit base: rel err {e:.2e}")
    case.close()


@pytest.mark.parametrize("what", ["w8", "q8"])
def test_config4_gate_in_the_8bit_formats(what):
    w = I.config4()
    if what == "w8":
        w.wfmt = I.W_INT8_G32
    proj = I.LLAMA8B["gate"]
    case = DeviceCase(w, proj, load_slots=w.distinct_adapters(), q8=(what == "q8"))
    e = _sampled(case, w, proj)
    assert case.last_plan.path == GEMM
    print(f"config4 gate, {what}: T={w.T} rel err {e:.2e}")
    assert e <= 1e-2
    assert case.pool.poll_error() == (0, -1)
    case.close()


def test_config5_batch_with_adapters_in_8bit_blocks():
    # the mixed batch (prompts and 120 decode rows) on its 4-bit base, every adapter kept in 8-bit blocks: the GEMM path's
    # shrink and expand blocks read them
    w = I.config5()
    proj = w.projections[0]
    case = DeviceCase(w, proj, load_slots=w.distinct_adapters(), q8=True)
    e = _sampled(case, w, proj, n_rows=48)
    assert case.last_plan.path == GEMM
    print(f"config5, adapters in 8-bit blocks: rel err {e:.2e}")
    assert e <= 1e-2
    case.close()
