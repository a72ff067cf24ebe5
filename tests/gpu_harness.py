"""Shared plumbing of the GPU parity tests: upload a seeded workload, run it through the C-ABI,
fetch y, and compute the oracle's answer for the same bytes.  No arithmetic of the layer here."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2507_01438_amd import inputs as I

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> device tensor with the same bytes (uint16 bit patterns travel as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(a).to(DEV)


def y_to_f64(y: torch.Tensor, dtype: int) -> np.ndarray:
    h = y.cpu().numpy()
    if dtype == I.F32:
        return h.astype(np.float64)
    return I.bf16_bits_to_f32(h.view(np.uint16)).astype(np.float64)


def assert_close(y: np.ndarray, ref: np.ndarray, base_ref: np.ndarray, what: str = "") -> float:
    """The stated tolerance on the whole result (max-norm 1e-2), and two sharper views of the same numbers: the
    adapter term alone, (y - W x) against (ref - W x), within 4e-2 of its own largest entry (one bf16 rounding of y is
    2^-9 of |y|, and the adapter term is about a fifth of y), and every row within 2e-2 of its own largest entry."""
    e = rel_err(y, ref)
    assert e <= 1e-2, f"{what}: rel err {e:.3e}"
    lora_ref = ref - base_ref
    if np.abs(lora_ref).max() > 0:
        el = float(np.abs((y - base_ref) - lora_ref).max() / np.abs(lora_ref).max())
        assert el <= 4e-2, f"{what}: adapter term off by {el:.3e} of its largest entry"
    row_max = np.abs(ref).max(axis=1)
    er = float((np.abs(y - ref).max(axis=1) / np.where(row_max > 0, row_max, 1.0)).max())
    assert er <= 2e-2, f"{what}: worst row off by {er:.3e} of its largest entry"
    return e


def rel_err(y: np.ndarray, ref: np.ndarray) -> float:
    """max |y - ref| / max |ref| -- the metric the tolerances are stated in."""
    return float(np.abs(y - ref).max() / np.abs(ref).max())


class DeviceCase:
    """One projection of a workload resident on the GPU, with its pool loaded."""

    def __init__(self, w: I.Workload, proj: I.Projection, *, load_slots=None, n_tokens_max=None, share=None, q8=False):
        """share: another case of the same workload and d_in whose device copies of x and of the routing tables this
        one uses as well (projections that read the same activations: their descriptors then name the same pointers).
        q8: the workload's adapters are cut into 8-bit blocks (input preparation) and the pool keeps them that way; the
        oracle then gets the same codes and scales."""
        from paper_2507_01438_amd import binding as B
        self.B = B
        self.w, self.proj = w, proj
        self.x_h = w.x(proj)
        self.W_h, self.ws_h = w.W(proj)
        if share is not None:
            assert share.w is w and share.proj.K == proj.K
        self.x = to_dev(self.x_h) if share is None else share.x
        self.W = to_dev(self.W_h)
        self.w_scales = None if self.ws_h is None else to_dev(self.ws_h)
        self.q8 = q8
        self.pool = B.AdapterPool(proj.K, proj.N, w.max_rank, w.pool, w.dtype, DEV, q8=q8)
        self.adapters = {}
        slots = range(w.pool) if load_slots is None else load_slots
        keep = []
        for i in slots:
            A, Bm, s = w.adapter(proj, int(i))
            if q8:
                Ac, As = I.quantize_q8_blocks(I.bf16_bits_to_f32(A))
                Bc, Bs = I.quantize_q8_blocks(I.bf16_bits_to_f32(Bm))
                self.adapters[int(i)] = (Ac, Bc, s, As, Bs)
                dev = [to_dev(Ac), to_dev(As), to_dev(Bc), to_dev(Bs)]
                keep.append(dev)
                B.elora_pool_load_adapters_q8(self.pool.handle, [int(i)], [Ac.shape[0]], [s], [dev[0]], [dev[1]], [dev[2]], [dev[3]])
                continue
            self.adapters[int(i)] = (A, Bm, s)
            self.pool.load(int(i), torch.from_numpy(A.view(np.int16) if A.dtype == np.uint16 else A),
                           torch.from_numpy(Bm.view(np.int16) if Bm.dtype == np.uint16 else Bm), s)
        torch.cuda.synchronize()
        del keep
        self.lin = B.LoraLinear(proj.K, proj.N, w.dtype, self.pool, n_tokens_max or max(w.T, 1), DEV, wfmt=w.wfmt)
        self.y = torch.zeros((max(w.T, 1), proj.N), dtype=torch.float32 if w.dtype == I.F32 else torch.int16, device=DEV)
        if share is not None:
            self.adapter_idx, self.seg_offsets, self.seg_adapter = share.adapter_idx, share.seg_offsets, share.seg_adapter
        else:
            self.adapter_idx = None if w.adapter_idx is None else to_dev(w.adapter_idx)
            self.seg_offsets = None if w.seg_offsets is None else to_dev(w.seg_offsets)
            self.seg_adapter = None if w.seg_adapter is None else to_dev(w.seg_adapter)

    def desc(self, scales=None):
        return self.lin.desc(self.x[: self.w.T], self.W, self.y, adapter_idx=self.adapter_idx,
                             seg_offsets=self.seg_offsets, seg_adapter=self.seg_adapter, scales=scales,
                             wfmt=self.w.wfmt, w_scales=self.w_scales)

    def run(self, scales=None, force_path=None) -> np.ndarray:
        B = self.B
        self.y.fill_(7 if self.w.dtype != I.F32 else 7.0)  # stale content must be overwritten
        d = self.desc(scales)
        if force_path is not None:
            B.elora_force_path(force_path)
        try:
            plan = B.elora_linear_plan(d)
            B.elora_batched_lora_linear(d)
        finally:
            if force_path is not None:
                B.elora_force_path(-1)
        torch.cuda.synchronize()
        self.last_plan = plan
        return y_to_f64(self.y[: self.w.T], self.w.dtype)

    def oracle_adapters(self):
        ads = [None] * self.w.pool
        for i in self.w.distinct_adapters():
            if int(i) in self.adapters:
                if self.q8:
                    Ac, Bc, s, As, Bs = self.adapters[int(i)]
                    ads[int(i)] = oracle.Adapter(Ac, Bc, s, A_scales=As, B_scales=Bs)
                    continue
                A, Bm, s = self.adapters[int(i)]
                ads[int(i)] = oracle.Adapter(A, Bm, s)
        return ads

    def reference(self, rows=None, cols=None, row_scale=None, row_adapter=None) -> np.ndarray:
        """The oracle's y for this case.  Routing comes from the workload's own tables: the per-row index as it is,
        a segment table through the oracle's own segment -> row expansion; `row_adapter` replaces either."""
        kw = dict(wfmt=self.w.wfmt, w_scales=self.ws_h, rows=rows, cols=cols, row_scale=row_scale)
        if row_adapter is None and self.w.adapter_idx is None:
            return oracle.linear_segments(self.w.dtype, self.x_h, self.W_h, self.oracle_adapters(), self.w.seg_offsets,
                                          self.w.seg_adapter, **kw)
        ra = self.w.adapter_idx if row_adapter is None else row_adapter
        return oracle.linear(self.w.dtype, self.x_h, self.W_h, self.oracle_adapters(), ra, **kw)

    def base_reference(self, rows=None, cols=None) -> np.ndarray:
        """The oracle's W x alone (every row without adapter)."""
        return self.reference(rows=rows, cols=cols, row_adapter=np.full(self.w.T, -1, dtype=np.int32))

    def close(self):
        self.pool.close()
