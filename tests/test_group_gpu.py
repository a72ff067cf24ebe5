"""Several decode calls in one launch (elora_batched_lora_linear_group) against the oracle, call by call."""
import numpy as np
import pytest
import torch

from gpu_harness import DeviceCase, rel_err, to_dev, y_to_f64
from paper_2507_01438_amd import inputs as I

pytestmark = pytest.mark.gpu


def _cases(T, K, Ns, ranks_of, seed):
    """One DeviceCase per projection; all share the routing of the first (same rows -> same adapters)."""
    cases = []
    for i, (N, ranks) in enumerate(zip(Ns, ranks_of)):
        w = I.small_workload(seed, I.BF16, K, N, T, 6, ranks, no_adapter_rows=(T // 2,) if T > 1 else ())
        cases.append(DeviceCase(w, w.projections[0]))
    return cases


def _run_group(B, cases, expect_launches):
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
def test_groups_of_small_calls_run_as_one_launch(T, K, Ns):
    from paper_2507_01438_amd import binding as B
    ranks_of = [(16, 8, 32), (8,), (5, 64, 16)][: len(Ns)]
    cases = _cases(T, K, Ns, ranks_of, seed=300 + T)
    e = _run_group(B, cases, expect_launches=1)
    # the same calls again on the same workspaces, then one by one: mailboxes were left idle
    e2 = _run_group(B, cases, expect_launches=1)
    for c in cases:
        y = c.run()
        assert rel_err(y, c.reference()) <= 1e-2
    print(f"group T={T} K={K} N={Ns}: rel err {e:.2e} / {e2:.2e}")
    for c in cases:
        c.close()


def test_groups_that_do_not_fit_or_mix_paths_fall_back_to_single_calls():
    from paper_2507_01438_amd import binding as B
    # three wide projections at 64 rows: 3 x 224 tiles are more workgroups than the device holds at once
    cases = _cases(64, 256, (14336, 14336, 14336), [(8,), (8,), (8,)], seed=310)
    _run_group(B, cases, expect_launches=3)
    for c in cases:
        c.close()
    # a group of one, and a call without pool next to one with
    cases = _cases(24, 512, (96,), [(8, 16)], seed=311)
    _run_group(B, cases, expect_launches=1)
    w = cases[0].w
    lin = B.LoraLinear(512, 96, I.BF16, None, 24)
    y2 = torch.zeros((24, 96), dtype=torch.int16, device="cuda:0")
    d2 = lin.desc(cases[0].x, cases[0].W, y2)
    descs = B.desc_array([cases[0].desc(), d2])
    assert B.elora_linear_group_launches(descs) == 1
    B.elora_batched_lora_linear_group(descs)
    torch.cuda.synchronize()
    base = cases[0].reference(row_adapter=np.full(24, -1, dtype=np.int32))
    assert rel_err(y_to_f64(y2, I.BF16), base) <= 1e-2
    assert rel_err(y_to_f64(cases[0].y[:24], I.BF16), cases[0].reference()) <= 1e-2
    # two descriptors on one workspace: refused
    with pytest.raises(B.EloraError):
        B.elora_batched_lora_linear_group(B.desc_array([cases[0].desc(), cases[0].desc()]))
    cases[0].close()


@pytest.mark.parametrize("names", [("q", "k", "v"), ("gate", "up")])
def test_config3_projection_groups_full_shapes(names):
    from paper_2507_01438_amd import binding as B
    w = I.config3()
    cases = [DeviceCase(w, I.LLAMA8B[n], load_slots=w.distinct_adapters()) for n in names]
    descs = B.desc_array([c.desc() for c in cases])
    assert B.elora_linear_group_launches(descs) == 1
    B.elora_batched_lora_linear_group(descs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    for c, n in zip(cases, names):
        cols = np.sort(rng.choice(c.proj.N, 48, replace=False))
        y = y_to_f64(c.y[: w.T], w.dtype)
        e = rel_err(y[:, cols], c.reference(cols=cols))
        print(f"config3 group {names}: {n} rel err {e:.2e}")
        assert e <= 1e-2
        assert c.pool.poll_error() == (0, -1)
        c.close()


def test_group_with_every_wait_cut_short_still_matches_and_leaves_the_workspaces_idle():
    """Bound of the internal waits at 0: every workgroup of every call of the group computes what it needs from the
    inputs; results still match, and the next (normal) group launch on the same workspaces does too."""
    from paper_2507_01438_amd import binding as B
    cases = _cases(37, 1024, (528, 80, 272), [(8, 16, 24, 3), (16,), (5, 64, 16)], seed=320)
    B.elora_debug_spin_limit(0)
    try:
        _run_group(B, cases, expect_launches=1)
    finally:
        B.elora_debug_spin_limit(1 << 22)
    _run_group(B, cases, expect_launches=1)
    for c in cases:
        c.close()


# ---------------------------------------------------------------------------------------------
# calls of the MFMA GEMM path that read the same activations: one route launch and one shrink launch for all
# ---------------------------------------------------------------------------------------------

def _shared_cases(w, projs):
    cases = []
    for p in projs:
        cases.append(DeviceCase(w, p, load_slots=w.distinct_adapters(), share=cases[0] if cases else None))
    return cases


@pytest.mark.parametrize("lengths,none_segs", [([70, 1, 1, 1, 200, 30, 0, 5], (2,)), ([300, 20, 257, 15, 1, 1, 1, 90], ())])
def test_gemm_calls_that_share_x_share_route_and_shrink(lengths, none_segs):
    from paper_2507_01438_amd import binding as B
    T = sum(lengths)
    w = I.small_workload(330 + T, I.BF16, 512, 264, T, 6, (16, 8, 32, 64, 5, 24), segments=lengths, no_adapter_rows=none_segs)
    w.projections = [I.Projection("a", 512, 264), I.Projection("b", 512, 1040), I.Projection("c", 512, 72)]
    cases = _shared_cases(w, w.projections)
    descs = B.desc_array([c.desc() for c in cases])
    assert [B.elora_linear_plan(c.desc()).path for c in cases] == [2, 2, 2]
    assert B.elora_linear_group_launches(descs) == 2 + 3           # route, shrink, three GEMMs (alone: 3 x 3)
    for c in cases:
        c.y.fill_(7)
    B.elora_batched_lora_linear_group(descs)
    torch.cuda.synchronize()
    together = [y_to_f64(c.y[:T], I.BF16) for c in cases]
    for c, y in zip(cases, together):
        assert rel_err(y, c.reference()) <= 1e-2, c.proj.name
        assert c.pool.poll_error() == (0, -1)
    # one by one: the same bits (the shrink of a call does not depend on who shares its launch)
    for c, y in zip(cases, together):
        np.testing.assert_array_equal(c.run(), y)
    # calls that name different copies of x do not share: 3 launches each
    other = DeviceCase(w, w.projections[1], load_slots=w.distinct_adapters())
    assert B.elora_linear_group_launches(B.desc_array([cases[0].desc(), other.desc()])) == 6
    other.close()
    for c in cases:
        c.close()


def test_config4_gate_and_up_share_their_shrink_full_shapes():
    from paper_2507_01438_amd import binding as B
    w = I.config4()
    cases = _shared_cases(w, [I.LLAMA8B["gate"], I.LLAMA8B["up"]])
    descs = B.desc_array([c.desc() for c in cases])
    assert B.elora_linear_group_launches(descs) == 4
    B.elora_batched_lora_linear_group(descs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(11)
    for c in cases:
        cols = np.sort(rng.choice(c.proj.N, 48, replace=False))
        rows = np.sort(rng.choice(w.T, 96, replace=False))
        y = y_to_f64(c.y[: w.T], w.dtype)
        e = rel_err(y[np.ix_(rows, cols)], c.reference(rows=rows, cols=cols))
        print(f"config4 gate/up with a shared shrink: {c.proj.name} rel err {e:.2e}")
        assert e <= 1e-2
        assert c.pool.poll_error() == (0, -1)
        c.close()
