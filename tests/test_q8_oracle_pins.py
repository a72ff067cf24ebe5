"""The 8-bit block dequantisation oracle against what the formats fix (no GPU, no product code)."""
import numpy as np

from oracle.q8_oracle import dequant_q8_to_bf16, round_to_bf16_bits


def _bf16(bits):
    return float(np.array([bits << 16], dtype=np.uint32).view(np.float32)[0])


def test_rounding_to_bf16_known_values():
    assert round_to_bf16_bits(1.0) == 0x3F80 and round_to_bf16_bits(-2.0) == 0xC000 and round_to_bf16_bits(0.0) == 0
    # bf16 has 8 significand bits: neighbours of 1.0 are 1.0 and 1.0078125
    assert round_to_bf16_bits(1.00390625) == 0x3F80          # exactly halfway: ties to the even significand (1.0)
    assert round_to_bf16_bits(1.01171875) == 0x3F82          # halfway between 0x3F81 (odd) and 0x3F82: up to even
    assert round_to_bf16_bits(1.00390625 + 2.0 ** -20) == 0x3F81   # just above halfway
    assert round_to_bf16_bits(1.00390625 - 2.0 ** -20) == 0x3F80   # just below
    assert round_to_bf16_bits(1.99609375 + 2.0 ** -9) == 0x4000     # rounds up into the next binade (2.0)
    for v in (3.0, -0.15625, 96.0, 2.0 ** -20):               # representable: unchanged
        assert _bf16(round_to_bf16_bits(v)) == v


def test_unit_and_power_of_two_scales_give_the_codes_back():
    codes = np.arange(-128, 128, dtype=np.int8).reshape(8, 32)
    one = np.full(8, 0x3C00, dtype=np.uint16)                 # fp16 1.0
    out = dequant_q8_to_bf16(codes, one)
    assert all(_bf16(int(b)) == float(c) for b, c in zip(out.reshape(-1), codes.reshape(-1)))   # |code| <= 128: exact in bf16
    quarter = np.full(8, 0x3400, dtype=np.uint16)             # fp16 0.25
    out = dequant_q8_to_bf16(codes, quarter)
    assert all(_bf16(int(b)) == 0.25 * float(c) for b, c in zip(out.reshape(-1), codes.reshape(-1)))


def test_block_scales_apply_to_their_own_32_values_and_ties_follow_the_rule():
    codes = np.ones((2, 64), dtype=np.int8)
    codes[1, 40] = 3
    # fp16 1 + 2^-8 = 0x3C04: times 1 it is halfway between bf16 1.0 and 1.0078125; times 3 it is 3.01171875,
    # halfway between 3.0 (0x4040) and 3.015625 (0x4041): both go to the even one
    scales = np.array([0x3C00, 0x4000, 0x3C04, 0xBC00], dtype=np.uint16)   # 1, 2, 1 + 2^-8, -1
    out = dequant_q8_to_bf16(codes, scales)
    assert set(out[0, :32]) == {0x3F80} and set(out[0, 32:]) == {0x4000}
    assert out[1, 0] == 0x3F80 and set(out[1, 32:40]) == {0xBF80} and out[1, 40] == 0xC040


def test_against_numpy_float32_products_on_random_blocks():
    rng = np.random.default_rng(5)
    codes = rng.integers(-128, 128, size=(16, 96), dtype=np.int8)
    scales = rng.uniform(1e-3, 0.2, size=48).astype(np.float16)
    out = dequant_q8_to_bf16(codes, scales.view(np.uint16))
    prod = (np.repeat(scales.astype(np.float32), 32) * codes.reshape(-1).astype(np.float32))     # exact in binary32
    got = (out.reshape(-1).astype(np.uint32) << 16).view(np.float32)
    # the nearest bf16: as close as the closer of the two bf16 values that bracket the product (truncation and the
    # next one away from zero), and never further than half a unit in the last place (2^-8 relative)
    trunc_bits = prod.view(np.uint32) & np.uint32(0xFFFF0000)
    lower = trunc_bits.view(np.float32).astype(np.float64)
    upper = (trunc_bits + np.uint32(0x10000)).view(np.float32).astype(np.float64)
    p64, g64 = prod.astype(np.float64), got.astype(np.float64)
    assert np.all(np.abs(g64 - p64) == np.minimum(np.abs(lower - p64), np.abs(upper - p64)))
    assert np.all(np.abs(g64 - p64) <= np.abs(p64) * 2.0 ** -8)
    assert np.all(np.sign(got) == np.sign(prod))
