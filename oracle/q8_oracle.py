"""What a pool block holds after an adapter stored in 8-bit blocks has been placed in it.

TEST INFRASTRUCTURE, NOT PRODUCT CODE (only ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this package; it imports nothing of the product).

The paper keeps all adapters in the block format its settings call "Q8_0" (Sec. 5 "Model"): blocks of 32 consecutive
values, one fp16 scale per block, signed 8-bit codes, value = scale * code.  The pool of this library holds bf16, so
placing such an adapter means: every value scale * code (exact in binary32: an 11-bit times an 8-bit significand),
rounded once to bfloat16, round to nearest, ties to even.  Written out with Python integers so that the rounding
can be read off the code.
"""
from __future__ import annotations

import struct

import numpy as np


def _fp16_to_float(bits: int) -> float:
    return struct.unpack("<e", struct.pack("<H", bits & 0xFFFF))[0]


def round_to_bf16_bits(value: float) -> int:
    """Bit pattern of the bfloat16 nearest to `value` (a double that is exactly representable in binary32),
    ties to the even significand."""
    u = struct.unpack("<I", struct.pack("<f", value))[0]
    if struct.unpack("<f", struct.pack("<I", u))[0] != value and value == value:
        raise ValueError("not a binary32 value")
    lower, rest = u >> 16, u & 0xFFFF
    if rest > 0x8000 or (rest == 0x8000 and (lower & 1)):
        lower += 1                      # carries into the exponent where it should
    return lower & 0xFFFF


def dequant_q8_to_bf16(codes: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """codes: int8, any shape with a multiple of 32 elements, blocks of 32 in row-major order; scales: uint16 bit
    patterns of fp16, one per block.  Returns uint16 bf16 bit patterns of the same shape as `codes`."""
    flat = np.ascontiguousarray(codes, dtype=np.int8).reshape(-1)
    sc = np.ascontiguousarray(scales, dtype=np.uint16).reshape(-1)
    assert flat.size % 32 == 0 and sc.size == flat.size // 32
    out = np.empty(flat.size, dtype=np.uint16)
    for i in range(flat.size):
        out[i] = round_to_bf16_bits(_fp16_to_float(int(sc[i // 32])) * int(flat[i]))
    return out.reshape(np.shape(codes))
