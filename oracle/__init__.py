"""fp64 CPU oracle for the batched multi-adapter LoRA linear layer.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only ``tests/``, the smoke check and
the benchmark's ``cpu_baseline`` leg may import this package; the product
package never does, and this package never imports the product.

The arithmetic lives in ``elora_oracle.c`` (plain C loops in double, written
from Sec. 2.1, Sec. 3.4 and Sec. 4.3 of the paper); this module only compiles
that file with gcc and marshals numpy arrays into it.

Array conventions (row-major): ``x [T,K]``, ``W [N,K]``, ``A_i [r_i,K]``,
``B_i [N,r_i]``.  bf16 tensors are ``uint16`` arrays of bit patterns, fp32
tensors are ``float32`` arrays.  4-bit W is ``uint8 [N,K/2]`` plus fp16 scales
as ``uint16 [N,K/32]`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "elora_oracle.c")
_LIB = os.path.join(_HERE, "libelora_oracle.so")

F32 = 0
BF16 = 1
W_SAME = 0
W_INT4_G32 = 1
W_INT8_G32 = 2


def build(force: bool = False) -> str:
    """Compile elora_oracle.c into libelora_oracle.so next to it (gcc, OpenMP)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", tmp, _SRC, "-lm"],
            check=True,
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.elora_oracle_widen_bf16.restype = ctypes.c_double
        lib.elora_oracle_widen_bf16.argtypes = [ctypes.c_uint16]
        lib.elora_oracle_widen_fp16.restype = ctypes.c_double
        lib.elora_oracle_widen_fp16.argtypes = [ctypes.c_uint16]
        lib.elora_oracle_weight_at.restype = ctypes.c_double
        lib.elora_oracle_rows_from_segments.restype = ctypes.c_int
        lib.elora_oracle_ubatches.restype = ctypes.c_int
        lib.elora_oracle_linear.restype = ctypes.c_int
        lib.elora_oracle_linear_grouped.restype = ctypes.c_int
        _lib = lib
    return _lib


@dataclass
class Adapter:
    """One pool entry: A [rank, K], B [N, rank], scale = alpha / rank.  With A_scales / B_scales (uint16 fp16 bit
    patterns, one per block of 32 consecutive values in row-major order) A and B are int8 codes: the 8-bit block
    format the paper keeps its adapters in (Sec. 5 "Model"), value = scale * code."""

    A: np.ndarray
    B: np.ndarray
    scale: float
    A_scales: Optional[np.ndarray] = None
    B_scales: Optional[np.ndarray] = None

    @property
    def rank(self) -> int:
        return int(self.A.shape[0])


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_tensor(a: np.ndarray, dtype: int, name: str) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16
    if a.dtype != want:
        raise TypeError(f"{name}: expected {want} for dtype code {dtype}, got {a.dtype}")
    return np.ascontiguousarray(a)


def widen_bf16(bits: int) -> float:
    return float(_load().elora_oracle_widen_bf16(int(bits)))


def widen_fp16(bits: int) -> float:
    return float(_load().elora_oracle_widen_fp16(int(bits)))


def weight_at(dtype: int, wfmt: int, W: np.ndarray, w_scales: Optional[np.ndarray],
              K: int, n: int, k: int) -> float:
    W = np.ascontiguousarray(W)
    ws = None if w_scales is None else np.ascontiguousarray(w_scales, dtype=np.uint16)
    return float(_load().elora_oracle_weight_at(
        ctypes.c_int(dtype), ctypes.c_int(wfmt), _ptr(W), _ptr(ws),
        ctypes.c_int(K), ctypes.c_int(n), ctypes.c_int(k)))


def rows_from_segments(T: int, seg_offsets: Sequence[int], seg_adapter: Sequence[int]) -> np.ndarray:
    """Adapter id per row from a CSR segment table (Sec. 3.4: requests of a batch)."""
    so = np.ascontiguousarray(seg_offsets, dtype=np.int32)
    sa = np.ascontiguousarray(seg_adapter, dtype=np.int32)
    n_seg = int(sa.shape[0])
    if so.shape[0] != n_seg + 1:
        raise ValueError("seg_offsets must have n_segments + 1 entries")
    out = np.full(T, -1, dtype=np.int32)
    rc = _load().elora_oracle_rows_from_segments(
        ctypes.c_int(T), ctypes.c_int(n_seg), _ptr(so), _ptr(sa), _ptr(out))
    if rc != 0:
        raise ValueError("malformed segment table")
    return out


def ubatches(row_adapter: Sequence[int], P: int):
    """adapter id -> sample indices (Sec. 3.4 / 4.3).  Returns (perm, group_offsets, n_distinct)."""
    ra = np.ascontiguousarray(row_adapter, dtype=np.int32)
    T = int(ra.shape[0])
    perm = np.zeros(max(T, 1), dtype=np.int32)
    offs = np.zeros(P + 1, dtype=np.int32)
    d = _load().elora_oracle_ubatches(ctypes.c_int(T), ctypes.c_int(P), _ptr(ra), _ptr(perm), _ptr(offs))
    return perm[:T], offs, int(d)


def _pool_args(dtype: int, adapters: Sequence[Optional[Adapter]], K: int, N: int):
    P = len(adapters)
    ranks = np.zeros(max(P, 1), dtype=np.int32)
    scales = np.zeros(max(P, 1), dtype=np.float64)
    A_ptrs = (ctypes.c_void_p * max(P, 1))()
    B_ptrs = (ctypes.c_void_p * max(P, 1))()
    As_ptrs = (ctypes.c_void_p * max(P, 1))()
    Bs_ptrs = (ctypes.c_void_p * max(P, 1))()
    keep = []
    for i, ad in enumerate(adapters):
        if ad is None:
            A_ptrs[i] = None
            B_ptrs[i] = None
            continue
        if ad.A_scales is not None or ad.B_scales is not None:
            A, B = np.ascontiguousarray(ad.A), np.ascontiguousarray(ad.B)
            As, Bs = np.ascontiguousarray(ad.A_scales), np.ascontiguousarray(ad.B_scales)
            if A.dtype != np.int8 or B.dtype != np.int8 or As.dtype != np.uint16 or Bs.dtype != np.uint16:
                raise TypeError(f"adapter {i}: 8-bit blocks are int8 codes with uint16 (fp16 bit pattern) scales")
            if A.size % 32 or B.size % 32 or As.size != A.size // 32 or Bs.size != B.size // 32:
                raise ValueError(f"adapter {i}: one scale per block of 32 values")
            keep += [As, Bs]
            As_ptrs[i] = As.ctypes.data
            Bs_ptrs[i] = Bs.ctypes.data
        else:
            A = _check_tensor(ad.A, dtype, f"A[{i}]")
            B = _check_tensor(ad.B, dtype, f"B[{i}]")
        r = A.shape[0]
        if A.shape != (r, K) or B.shape != (N, r):
            raise ValueError(f"adapter {i}: A {A.shape} / B {B.shape} do not fit K={K}, N={N}")
        keep += [A, B]
        ranks[i] = r
        scales[i] = float(ad.scale)
        A_ptrs[i] = A.ctypes.data
        B_ptrs[i] = B.ctypes.data
    return P, ranks, scales, (A_ptrs, As_ptrs), (B_ptrs, Bs_ptrs), keep


def _w_args(dtype: int, wfmt: int, W: np.ndarray, w_scales: Optional[np.ndarray], K: int):
    if wfmt == W_SAME:
        Wc = _check_tensor(W, dtype, "W")
        if Wc.ndim != 2 or Wc.shape[1] != K:
            raise ValueError("W must be [N, K]")
        return Wc, None, int(Wc.shape[0])
    if K % 32:
        raise ValueError("group-wise W needs K % 32 == 0")
    Wc = np.ascontiguousarray(W)
    if wfmt == W_INT8_G32:
        if Wc.dtype != np.int8 or Wc.ndim != 2 or Wc.shape[1] != K:
            raise ValueError("8-bit W must be int8 [N, K]")
    elif wfmt != W_INT4_G32:
        raise ValueError("unknown weight format")
    elif Wc.dtype != np.uint8 or Wc.ndim != 2 or Wc.shape[1] != K // 2:
        raise ValueError("4-bit W must be uint8 [N, K/2]")
    ws = np.ascontiguousarray(w_scales)
    if ws.dtype != np.uint16 or ws.shape != (Wc.shape[0], K // 32):
        raise ValueError("w_scales must be uint16 fp16 bit patterns [N, K/32]")
    return Wc, ws, int(Wc.shape[0])


def linear(dtype: int, x: np.ndarray, W: np.ndarray, adapters: Sequence[Optional[Adapter]],
           row_adapter: Sequence[int], *, wfmt: int = W_SAME,
           w_scales: Optional[np.ndarray] = None, row_scale: Optional[np.ndarray] = None,
           rows: Optional[Sequence[int]] = None, cols: Optional[Sequence[int]] = None,
           n_threads: int = 0, return_threads: bool = False):
    """Per-sample form: y_t = W x_t + s * B_i (A_i x_t), i = row_adapter[t] (< 0: base only).

    Returns float64 [len(rows) or T, len(cols) or N].
    """
    xc = _check_tensor(x, dtype, "x")
    T, K = xc.shape
    Wc, ws, N = _w_args(dtype, wfmt, W, w_scales, K)
    P, ranks, scales, A_ptrs, B_ptrs, keep = _pool_args(dtype, adapters, K, N)
    ra = np.ascontiguousarray(row_adapter, dtype=np.int32)
    if ra.shape != (T,):
        raise ValueError("row_adapter must have one entry per row of x")
    rs = None if row_scale is None else np.ascontiguousarray(row_scale, dtype=np.float32)
    rsel = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    csel = None if cols is None else np.ascontiguousarray(cols, dtype=np.int32)
    if rsel is not None and rsel.size and (rsel.min() < 0 or rsel.max() >= T):
        raise ValueError("rows out of range")
    if csel is not None and csel.size and (csel.min() < 0 or csel.max() >= N):
        raise ValueError("cols out of range")
    nr = T if rsel is None else int(rsel.shape[0])
    nc = N if csel is None else int(csel.shape[0])
    y = np.zeros((nr, nc), dtype=np.float64)
    used = _load().elora_oracle_linear(
        ctypes.c_int(dtype), ctypes.c_int(wfmt), ctypes.c_int(T), ctypes.c_int(K), ctypes.c_int(N),
        _ptr(xc), _ptr(Wc), _ptr(ws),
        ctypes.c_int(P), _ptr(ranks), _ptr(scales), A_ptrs[0], B_ptrs[0], A_ptrs[1], B_ptrs[1],
        _ptr(ra), _ptr(rs),
        ctypes.c_int(nr), _ptr(rsel), ctypes.c_int(nc), _ptr(csel),
        _ptr(y), ctypes.c_int(n_threads))
    del keep
    if used < 1:
        raise ValueError(f"oracle rejected its arguments (code {used})")
    return (y, used) if return_threads else y


def linear_segments(dtype: int, x: np.ndarray, W: np.ndarray, adapters, seg_offsets, seg_adapter, **kw):
    """Prefill form: row t takes the adapter of the segment that contains it."""
    ra = rows_from_segments(int(x.shape[0]), seg_offsets, seg_adapter)
    return linear(dtype, x, W, adapters, ra, **kw)


def linear_grouped(dtype: int, x: np.ndarray, W: np.ndarray, adapters, row_adapter, *,
                   wfmt: int = W_SAME, w_scales=None, row_scale=None) -> np.ndarray:
    """Grouped ("u-batch") form in the order of Sec. 3.4: base, group, gather, per-adapter products, scatter."""
    xc = _check_tensor(x, dtype, "x")
    T, K = xc.shape
    Wc, ws, N = _w_args(dtype, wfmt, W, w_scales, K)
    P, ranks, scales, A_ptrs, B_ptrs, keep = _pool_args(dtype, adapters, K, N)
    ra = np.ascontiguousarray(row_adapter, dtype=np.int32)
    rs = None if row_scale is None else np.ascontiguousarray(row_scale, dtype=np.float32)
    y = np.zeros((T, N), dtype=np.float64)
    rc = _load().elora_oracle_linear_grouped(
        ctypes.c_int(dtype), ctypes.c_int(wfmt), ctypes.c_int(T), ctypes.c_int(K), ctypes.c_int(N),
        _ptr(xc), _ptr(Wc), _ptr(ws),
        ctypes.c_int(P), _ptr(ranks), _ptr(scales), A_ptrs[0], B_ptrs[0], A_ptrs[1], B_ptrs[1], _ptr(ra), _ptr(rs), _ptr(y))
    del keep
    if rc < 1:
        raise ValueError(f"oracle rejected its arguments (code {rc})")
    return y
