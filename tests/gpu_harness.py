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


def rel_err(y: np.ndarray, ref: np.ndarray) -> float:
    """max |y - ref| / max |ref| -- the metric the tolerances are stated in."""
    return float(np.abs(y - ref).max() / np.abs(ref).max())


class DeviceCase:
    """One projection of a workload resident on the GPU, with its pool loaded."""

    def __init__(self, w: I.Workload, proj: I.Projection, *, load_slots=None, n_tokens_max=None):
        from paper_2507_01438_amd import binding as B
        self.B = B
        self.w, self.proj = w, proj
        self.x_h = w.x(proj)
        self.W_h, self.ws_h = w.W(proj)
        self.x = to_dev(self.x_h)
        self.W = to_dev(self.W_h)
        self.w_scales = None if self.ws_h is None else to_dev(self.ws_h)
        self.pool = B.AdapterPool(proj.K, proj.N, w.max_rank, w.pool, w.dtype, DEV)
        self.adapters = {}
        slots = range(w.pool) if load_slots is None else load_slots
        for i in slots:
            A, Bm, s = w.adapter(proj, int(i))
            self.adapters[int(i)] = (A, Bm, s)
            self.pool.load(int(i), torch.from_numpy(A.view(np.int16) if A.dtype == np.uint16 else A),
                           torch.from_numpy(Bm.view(np.int16) if Bm.dtype == np.uint16 else Bm), s)
        torch.cuda.synchronize()
        self.lin = B.LoraLinear(proj.K, proj.N, w.dtype, self.pool, n_tokens_max or max(w.T, 1), DEV, wfmt=w.wfmt)
        self.y = torch.zeros((max(w.T, 1), proj.N), dtype=torch.float32 if w.dtype == I.F32 else torch.int16, device=DEV)
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
                A, Bm, s = self.adapters[int(i)]
                ads[int(i)] = oracle.Adapter(A, Bm, s)
        return ads

    def reference(self, rows=None, cols=None, row_scale=None, row_adapter=None) -> np.ndarray:
        ra = self.w.row_adapter() if row_adapter is None else row_adapter
        return oracle.linear(self.w.dtype, self.x_h, self.W_h, self.oracle_adapters(), ra, wfmt=self.w.wfmt,
                             w_scales=self.ws_h, rows=rows, cols=cols, row_scale=row_scale)

    def close(self):
        self.pool.close()
