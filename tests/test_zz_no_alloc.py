"""The entry point that allocates nothing (elora_batched_lora_linear_noalloc: the workspace is an array inside the
library) against the entry point with a caller-supplied workspace, through the C-ABI: same kernels, same bits."""
import numpy as np
import pytest
import torch

from gpu_harness import DeviceCase, rel_err, y_to_f64
from paper_2507_01438_amd import inputs as I

pytestmark = pytest.mark.gpu


def _both(B, case):
    """y of the existing entry point and of the one without a workspace argument, for the same descriptor."""
    case.y.fill_(7)
    d = case.desc()
    B.elora_batched_lora_linear(d)
    torch.cuda.synchronize()
    want = case.y[: case.w.T].clone()
    case.y.fill_(7)
    d.workspace, d.workspace_bytes = None, 0       # ignored by the call under test
    B.elora_batched_lora_linear_noalloc(d)
    torch.cuda.synchronize()
    return want, case.y[: case.w.T].clone()


def test_two_calls_in_a_row_the_second_smaller_match_the_call_with_a_workspace():
    from paper_2507_01438_amd import binding as B
    shapes = [
        (64, 2048, 1040, (8, 16, 32, 64)),        # decode path, 128-row tiles, several K-slices: mailboxes and counters in use
        (24, 1024, 272, (8, 16)),                 # smaller: fewer rows, fewer columns (another d_out on the same array)
        (300, 512, 328, (16, 8, 32)),             # the MFMA GEMM path: row tables and shrink results in the array
        (9, 100, 30, (3, 5)),                     # generic kernels
        (64, 2048, 1040, (8, 16, 32, 64)),        # the first shape again, after everything else has written into the array
    ]
    before = torch.cuda.memory_allocated()
    for i, (T, K, N, ranks) in enumerate(shapes):
        w = I.small_workload(900 + i, I.BF16, K, N, T, 6, ranks, no_adapter_rows=(1,))
        case = DeviceCase(w, w.projections[0])
        want, got = _both(B, case)
        assert torch.equal(want, got), f"shape {i}: the two entry points differ"
        assert rel_err(y_to_f64(got, I.BF16), case.reference()) <= 1e-2
        want2, got2 = _both(B, case)               # and once more on the array as the call left it
        assert torch.equal(want2, got2) and torch.equal(got, got2)
        assert case.pool.poll_error() == (0, -1)
        case.close()
        del case, want, got, want2, got2
    assert torch.cuda.memory_allocated() == before


def test_a_call_that_needs_more_than_the_array_holds_is_refused():
    from paper_2507_01438_amd import binding as B
    K, N, T = 256, 32768, 8                         # 2 KiB of mailboxes per output column: 64 MiB
    assert B.elora_workspace_bytes(T, K, N, 1) > (32 << 20)
    x = torch.zeros((T, K), dtype=torch.int16, device="cuda:0")
    W = torch.zeros((N, K), dtype=torch.int16, device="cuda:0")
    y = torch.zeros((T, N), dtype=torch.int16, device="cuda:0")
    d = B.make_desc(n_tokens=T, d_in=K, d_out=N, dtype=B.ELORA_BF16, x=x, W=W, y=y, workspace=None, workspace_bytes=0)
    with pytest.raises(B.EloraError) as e:
        B.elora_batched_lora_linear_noalloc(d)
    assert e.value.status == B.ELORA_E_STORAGE
    d.n_tokens = -1
    with pytest.raises(B.EloraError) as e:
        B.elora_batched_lora_linear_noalloc(d)
    assert e.value.status == B.ELORA_E_SHAPE
