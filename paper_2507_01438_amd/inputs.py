"""Seeded synthetic inputs for the batched multi-adapter LoRA linear layer.

This module only DRAWS and STORES numbers (Gaussian tensors, adapter
popularity, prompt lengths, storage-format conversions of the inputs).  It
contains none of the layer's arithmetic and is the one module that both the
HIP path's tests/benchmark and the CPU oracle's tests are fed from, so that
both sides see the same bytes.

Workload shapes follow the paper's evaluation set-up: Llama3.1-8B projection
sizes and adapter ranks 16/32 (Sec. 5 "Model", Table "exp_setting"), adapter
popularity P(i) = i^-alpha / sum_j j^-alpha (Sec. 5.1 "Workload trace") and
uniformly distributed prompt lengths (Table "default_parameters").  The
paper's own adapters and models are not available, so seeded N(0, 0.02)
weights stand in for them.

Storage conventions (numpy, row-major):
  fp32 tensors  -> float32 arrays
  bf16 tensors  -> uint16 arrays holding the bit patterns
  4-bit W       -> uint8 [N, K/2] (k even in the low nibble, k odd in the high
                   nibble) + fp16 scales as uint16 bit patterns [N, K/32]
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

F32 = 0
BF16 = 1
W_SAME = 0
W_INT4_G32 = 1
W_INT8_G32 = 2


# ----------------------------------------------------------------------------
# storage-format helpers (inputs only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(a: np.ndarray, dtype: int) -> np.ndarray:
    """Round a float array to the storage dtype (float32 array or bf16 bit patterns)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a if dtype == F32 else f32_to_bf16_bits(a)


def as_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    """Stored tensor -> float64 values (exact)."""
    return (a if dtype == F32 else bf16_bits_to_f32(a)).astype(np.float64)


def normal(rng: np.random.Generator, shape, std: float, dtype: int) -> np.ndarray:
    """N(0, std^2) draws rounded to the storage dtype."""
    return store(rng.standard_normal(shape, dtype=np.float32) * np.float32(std), dtype)


def quantize_int4_g32(w: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric 4-bit group-wise storage of W [N, K]: groups of 32 along K,
    scale = absmax / 7 rounded to fp16, code = clamp(rne(w / scale) + 8, 0, 15).
    Returns (packed uint8 [N, K/2], fp16 scale bit patterns uint16 [N, K/32]).
    The layer consumes (code, scale); how they were chosen is not part of it."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, K = w.shape
    if K % 32:
        raise ValueError("K must be a multiple of 32")
    g = w.reshape(N, K // 32, 32)
    scale = (np.abs(g).max(axis=2) / np.float32(7.0)).astype(np.float16)
    sf = scale.astype(np.float32)
    sf_safe = np.where(sf == 0, np.float32(1.0), sf)
    q = np.clip(np.rint(g / sf_safe[:, :, None]) + 8, 0, 15).astype(np.uint8).reshape(N, K)
    packed = (q[:, 0::2] | (q[:, 1::2] << 4)).astype(np.uint8)
    return np.ascontiguousarray(packed), np.ascontiguousarray(scale.view(np.uint16))


def quantize_int8_g32(w: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Symmetric 8-bit group-wise storage of W [N, K] (the "Q8_0" base of Sec. 5's
    setting S1): groups of 32 along K, scale = absmax / 127 rounded to fp16,
    code = clamp(rne(w / scale), -127, 127).  Returns (int8 [N, K], fp16 scale bit
    patterns uint16 [N, K/32]).  The layer consumes (code, scale) as they are."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    N, K = w.shape
    if K % 32:
        raise ValueError("K must be a multiple of 32")
    g = w.reshape(N, K // 32, 32)
    scale = (np.abs(g).max(axis=2) / np.float32(127.0)).astype(np.float16)
    sf = scale.astype(np.float32)
    sf_safe = np.where(sf == 0, np.float32(1.0), sf)
    q = np.clip(np.rint(g / sf_safe[:, :, None]), -127, 127).astype(np.int8).reshape(N, K)
    return np.ascontiguousarray(q), np.ascontiguousarray(scale.view(np.uint16))


# ----------------------------------------------------------------------------
# routing draws
# ----------------------------------------------------------------------------

def power_law_probs(n: int, alpha: float) -> np.ndarray:
    """P(i) = i^-alpha / sum_j j^-alpha for popularity ranks i = 1..n (Sec. 5.1)."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-float(alpha))
    return w / w.sum()


def draw_adapters(rng: np.random.Generator, n_draws: int, pool: int, alpha: Optional[float]) -> np.ndarray:
    """One pool slot per request.  alpha None: uniform; otherwise power law over
    popularity ranks, with rank -> slot through a seeded permutation so that
    popular adapters are not neighbours in the pool."""
    if alpha is None:
        return rng.integers(0, pool, size=n_draws).astype(np.int32)
    slot_of_rank = rng.permutation(pool)
    ranks = rng.choice(pool, size=n_draws, p=power_law_probs(pool, alpha))
    return slot_of_rank[ranks].astype(np.int32)


def quantize_q8_blocks(a: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """8-bit block storage of an adapter matrix (the paper's adapters are kept in such blocks, Sec. 5 "Model"): blocks of
    32 consecutive values in row-major order, scale = absmax / 127 rounded to fp16, code = clamp(rne(a / scale), -127,
    127).  Returns (int8 codes of a's shape, fp16 scale bit patterns uint16 [a.size / 32]).  How codes and scales were
    chosen is input preparation: the library and the oracle both consume (codes, scales)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.size % 32:
        raise ValueError("the number of values must be a multiple of 32")
    g = a.reshape(-1, 32)
    scale = (np.abs(g).max(axis=1) / np.float32(127.0)).astype(np.float16)
    sf = scale.astype(np.float32)
    sf_safe = np.where(sf == 0, np.float32(1.0), sf)
    codes = np.clip(np.rint(g / sf_safe[:, None]), -127, 127).astype(np.int8)
    return codes.reshape(a.shape), scale.view(np.uint16)


def request_trace(seed: int, n_adapters: int, alpha: Optional[float], length: int) -> np.ndarray:
    """Adapter ids of `length` successive requests: power law over popularity ranks (Sec. 5.1; alpha None: uniform),
    ranks mapped to ids through a seeded permutation."""
    return draw_adapters(np.random.default_rng(seed), length, n_adapters, alpha)


def draw_lengths(rng: np.random.Generator, n: int, lo: int, hi: int) -> np.ndarray:
    """Integer lengths uniform on [lo, hi] inclusive (Table "default_parameters": U[I_l, I_u])."""
    return rng.integers(lo, hi + 1, size=n).astype(np.int32)


def offsets_from_lengths(lengths: Sequence[int]) -> np.ndarray:
    out = np.zeros(len(lengths) + 1, dtype=np.int32)
    out[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return out


# ----------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class Projection:
    name: str
    K: int  # d_in
    N: int  # d_out


LLAMA8B = {
    "q": Projection("q", 4096, 4096),
    "k": Projection("k", 4096, 1024),
    "v": Projection("v", 4096, 1024),
    "o": Projection("o", 4096, 4096),
    "gate": Projection("gate", 4096, 14336),
    "up": Projection("up", 4096, 14336),
    "down": Projection("down", 14336, 4096),
}


@dataclass
class Workload:
    """One benchmark/parity configuration.  Tensors are generated on demand and
    deterministically from (seed, what, which), so any subset can be rebuilt."""

    name: str
    seed: int
    dtype: int
    wfmt: int
    projections: List[Projection]
    pool: int                      # adapters resident in the pool
    max_rank: int
    ranks: np.ndarray              # [pool]
    scale: float                   # alpha / r, the same for every adapter of a config
    x_std: float
    w_std: float = 0.02
    # routing: exactly one of the two forms
    adapter_idx: Optional[np.ndarray] = None       # [T] decode: one adapter per token
    seg_offsets: Optional[np.ndarray] = None       # [n_seg + 1] prefill / mixed
    seg_adapter: Optional[np.ndarray] = None       # [n_seg]
    note: str = ""
    _cache: Dict = field(default_factory=dict, repr=False)

    @property
    def T(self) -> int:
        if self.adapter_idx is not None:
            return int(self.adapter_idx.shape[0])
        return int(self.seg_offsets[-1])

    def row_adapter(self) -> np.ndarray:
        """Adapter per row, written out from the routing tables (input bookkeeping, not the layer)."""
        if self.adapter_idx is not None:
            return self.adapter_idx.copy()
        out = np.full(self.T, -1, dtype=np.int32)
        for s in range(len(self.seg_adapter)):
            out[self.seg_offsets[s]:self.seg_offsets[s + 1]] = self.seg_adapter[s]
        return out

    def _rng(self, *key: int) -> np.random.Generator:
        return np.random.default_rng([self.seed, *key])

    def proj_id(self, proj: Projection) -> int:
        return [p.name for p in self.projections].index(proj.name)

    def x(self, proj: Projection) -> np.ndarray:
        """Activations [T, K]; projections with the same d_in share them."""
        key = ("x", proj.K)
        if key not in self._cache:
            self._cache[key] = normal(self._rng(1, proj.K), (self.T, proj.K), self.x_std, self.dtype)
        return self._cache[key]

    def W_float(self, proj: Projection) -> np.ndarray:
        return self._rng(2, self.proj_id(proj)).standard_normal((proj.N, proj.K), dtype=np.float32) * np.float32(self.w_std)

    def W(self, proj: Projection):
        """Base weight [N, K] in storage form: (W, None), (packed int4, fp16 scale bits) or (int8, fp16 scale bits)."""
        key = ("W", proj.name)
        if key not in self._cache:
            wf = self.W_float(proj)
            if self.wfmt == W_SAME:
                self._cache[key] = (store(wf, self.dtype), None)
            elif self.wfmt == W_INT8_G32:
                self._cache[key] = quantize_int8_g32(wf)
            else:
                self._cache[key] = quantize_int4_g32(wf)
        return self._cache[key]

    def adapter(self, proj: Projection, slot: int) -> Tuple[np.ndarray, np.ndarray, float]:
        """(A [r, K], B [N, r], scale) of pool slot `slot` for this projection."""
        r = int(self.ranks[slot])
        rng = self._rng(3, self.proj_id(proj), int(slot))
        A = normal(rng, (r, proj.K), self.w_std, self.dtype)
        B = normal(rng, (proj.N, r), self.w_std, self.dtype)
        return A, B, float(self.scale)

    def distinct_adapters(self) -> np.ndarray:
        ra = self.row_adapter()
        return np.unique(ra[ra >= 0])

    def algorithmic_bytes(self, proj: Projection, q8_adapters: bool = False) -> int:
        """Bytes one call must move: W once, x once, y once, and the used rows
        (r_i, not max_rank) of every DISTINCT adapter once, in the format they are stored in (q8_adapters: one byte per
        value plus one fp16 scale per 32 values)."""
        e = 4 if self.dtype == F32 else 2
        if self.wfmt == W_SAME:
            wb = proj.N * proj.K * e
        elif self.wfmt == W_INT8_G32:
            wb = proj.N * proj.K + proj.N * (proj.K // 32) * 2
        else:
            wb = proj.N * proj.K // 2 + proj.N * (proj.K // 32) * 2
        if q8_adapters:
            ab = sum((proj.K + proj.N) * int(self.ranks[i]) * 17 // 16 for i in self.distinct_adapters())
        else:
            ab = sum((proj.K + proj.N) * int(self.ranks[i]) * e for i in self.distinct_adapters())
        return wb + self.T * proj.K * e + self.T * proj.N * e + ab

    def algorithmic_flops(self, proj: Projection) -> int:
        """2*T*K*N for the base product plus 2*r*(K+N) per row that has an adapter."""
        ra = self.row_adapter()
        lora = sum(2 * int(self.ranks[i]) * (proj.K + proj.N) for i in ra if i >= 0)
        return 2 * self.T * proj.K * proj.N + lora


def _uniform_ranks(pool: int, r: int) -> np.ndarray:
    return np.full(pool, r, dtype=np.int32)


def config1(seed: int = 1001) -> Workload:
    """fp32, d_in = d_out = 512, 8 decode tokens, 4 adapters of rank 8, alpha = 16 (scale 2)."""
    rng = np.random.default_rng([seed, 0])
    return Workload("c1_fp32_512", seed, F32, W_SAME, [Projection("sq", 512, 512)], pool=4, max_rank=8,
                    ranks=_uniform_ranks(4, 8), scale=16.0 / 8.0, x_std=0.02,
                    adapter_idx=draw_adapters(rng, 8, 4, None))


def config2(seed: int = 1002, T: int = 32) -> Workload:
    """Llama3.1-8B q_proj decode, bf16: 32 tokens, 64 adapters of rank 16, power-law(1.1) popularity, scale 2."""
    rng = np.random.default_rng([seed, 0])
    return Workload("c2_qproj_decode", seed, BF16, W_SAME, [LLAMA8B["q"]], pool=64, max_rank=16,
                    ranks=_uniform_ranks(64, 16), scale=2.0, x_std=1.0,
                    adapter_idx=draw_adapters(rng, T, 64, 1.1))


def config3(seed: int = 1003, T: int = 64, pool: int = 256) -> Workload:
    """Llama3.1-8B, all seven projections of a layer, decode, bf16: 64 tokens,
    256 adapters with ranks drawn from {8,16,32,64}, uniform adapter choice."""
    rng = np.random.default_rng([seed, 0])
    ranks = rng.choice(np.array([8, 16, 32, 64], dtype=np.int32), size=pool).astype(np.int32)
    return Workload("c3_layer_decode", seed, BF16, W_SAME,
                    [LLAMA8B[n] for n in ("q", "k", "v", "o", "gate", "up", "down")],
                    pool=pool, max_rank=64, ranks=ranks, scale=2.0, x_std=1.0,
                    adapter_idx=draw_adapters(rng, T, pool, None))


def config4(seed: int = 1004, n_seg: int = 16, lo: int = 64, hi: int = 1024, pool: int = 128) -> Workload:
    """Llama3.1-8B prefill segments, bf16: 16 prompts with lengths U{64..1024},
    each with its own rank-32 adapter out of 128; gate/up and down projections."""
    rng = np.random.default_rng([seed, 0])
    lengths = draw_lengths(rng, n_seg, lo, hi)
    return Workload("c4_prefill_segments", seed, BF16, W_SAME,
                    [LLAMA8B["gate"], LLAMA8B["up"], LLAMA8B["down"]],
                    pool=pool, max_rank=32, ranks=_uniform_ranks(pool, 32), scale=2.0, x_std=1.0,
                    seg_offsets=offsets_from_lengths(lengths),
                    seg_adapter=rng.choice(pool, size=n_seg, replace=False).astype(np.int32))


def config5(seed: int = 1005, n_prefill: int = 4, prefill_len: int = 512, n_decode: int = 120,
            pool: int = 1024) -> Workload:
    """Mixed batch on a 4-bit base: 4 prefill segments of 512 rows followed by 120
    decode rows (segments of length 1), W 4096 -> 14336 in 4-bit groups of 32,
    bf16 adapters of rank 16 out of 1024, power-law(1.0) popularity."""
    rng = np.random.default_rng([seed, 0])
    lengths = [prefill_len] * n_prefill + [1] * n_decode
    return Workload("c5_mixed_int4", seed, BF16, W_INT4_G32, [LLAMA8B["gate"]],
                    pool=pool, max_rank=16, ranks=_uniform_ranks(pool, 16), scale=2.0, x_std=1.0,
                    seg_offsets=offsets_from_lengths(lengths),
                    seg_adapter=draw_adapters(rng, n_prefill + n_decode, pool, 1.0))


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def small_workload(seed: int, dtype: int, K: int, N: int, T: int, pool: int, ranks: Sequence[int],
                   *, wfmt: int = W_SAME, segments: Optional[Sequence[int]] = None,
                   alpha: Optional[float] = None, scale: float = 2.0, x_std: float = 1.0,
                   no_adapter_rows: Sequence[int] = ()) -> Workload:
    """Free-form small case for parity tests: any shape, any rank mix, decode or
    segment routing, optional rows/segments with adapter -1 (base model only)."""
    rng = np.random.default_rng([seed, 0])
    ranks = np.asarray(ranks, dtype=np.int32)
    ranks = np.resize(ranks, pool).astype(np.int32)  # a shorter list repeats
    w = Workload(f"small_{seed}", seed, dtype, wfmt, [Projection("p", K, N)], pool=pool,
                 max_rank=int(ranks.max()) if ranks.size else 1, ranks=ranks, scale=scale, x_std=x_std)
    if segments is None:
        idx = draw_adapters(rng, T, pool, alpha)
        for t in no_adapter_rows:
            idx[t] = -1
        w.adapter_idx = idx
    else:
        if int(np.sum(segments)) != T:
            raise ValueError("segment lengths must sum to T")
        w.seg_offsets = offsets_from_lengths(segments)
        sa = draw_adapters(rng, len(segments), pool, alpha)
        for s in no_adapter_rows:
            sa[s] = -1
        w.seg_adapter = sa
    return w
