"""Pins for the fp64 CPU oracle (no GPU, no product code).

The oracle is only trusted because these tests tie it to things other than
itself: a hand-expanded instance of the paper's equation (Sec. 3.4), closed
forms, library routines (numpy float64 matmul) on special cases, and
invariants the method's definition implies.  Each test names the mistake it
would catch.
"""
import json
import os

import numpy as np
import pytest

import oracle
from oracle import Adapter
from paper_2507_01438_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _f32(a):
    return np.asarray(a, dtype=np.float32)


def _bf16(a):
    return I.f32_to_bf16_bits(_f32(a))


def _mk(dtype, a):
    return _f32(a) if dtype == I.F32 else _bf16(a)


def _random_case(seed, dtype=I.F32, K=24, N=20, T=9, P=5, ranks=(1, 2, 3, 4, 5), scale=None):
    rng = np.random.default_rng(seed)
    x = I.normal(rng, (T, K), 1.0, dtype)
    W = I.normal(rng, (N, K), 0.5, dtype)
    ads = []
    for i in range(P):
        r = ranks[i % len(ranks)]
        ads.append(Adapter(I.normal(rng, (r, K), 0.5, dtype), I.normal(rng, (N, r), 0.5, dtype),
                           float(scale if scale is not None else 0.25 * (i + 1))))
    ra = rng.integers(-1, P, size=T).astype(np.int32)
    return x, W, ads, ra


def _numpy_reference(dtype, x, W, ads, ra, row_scale=None):
    """Independent statement with numpy float64 matmuls (library routine), row by row."""
    xd, Wd = I.as_f64(x, dtype), I.as_f64(W, dtype)
    y = xd @ Wd.T
    for t, i in enumerate(ra):
        if i >= 0:
            A, B = I.as_f64(ads[i].A, dtype), I.as_f64(ads[i].B, dtype)
            s = ads[i].scale if row_scale is None else float(row_scale[t])
            y[t] += s * (B @ (A @ xd[t]))
    return y


# --------------------------------------------------------------------------
# widening of stored formats
# --------------------------------------------------------------------------

def test_bf16_widening_matches_bit_definition():
    # every bf16 pattern that is finite: value == float32 with the low 16 bits zero
    bits = np.arange(0, 1 << 16, 7, dtype=np.uint32).astype(np.uint16)
    with np.errstate(invalid="ignore"):   # signalling NaN patterns are among the bits; they are masked out below
        ref = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    got = np.array([oracle.widen_bf16(int(b)) for b in bits])
    finite = np.isfinite(ref)
    assert np.array_equal(got[finite], ref[finite])
    assert oracle.widen_bf16(0x3F80) == 1.0 and oracle.widen_bf16(0xC000) == -2.0


def test_fp16_widening_matches_numpy_half():
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.widen_fp16(int(b)) for b in bits[::5]])
    r = ref[::5]
    finite = np.isfinite(r)
    assert np.array_equal(got[finite], r[finite])  # normals, subnormals, signed zeros
    assert oracle.widen_fp16(0x3C00) == 1.0 and oracle.widen_fp16(0x0001) == 2.0 ** -24


def test_int4_nibble_order_and_offset():
    # byte b holds k=2b in the LOW nibble and k=2b+1 in the HIGH nibble; w = scale * (code - 8)
    K, N = 64, 2
    packed = np.zeros((N, K // 2), dtype=np.uint8)
    packed[0, 0] = 0x3A          # k=0 -> code 10, k=1 -> code 3
    packed[1, 17] = 0xF0         # k=34 -> code 0, k=35 -> code 15
    scales = np.array([[np.float16(0.5), np.float16(2.0)], [np.float16(1.0), np.float16(-3.0)]]).view(np.uint16)
    at = lambda n, k: oracle.weight_at(I.BF16, I.W_INT4_G32, packed, scales, K, n, k)
    assert at(0, 0) == 0.5 * (10 - 8)
    assert at(0, 1) == 0.5 * (3 - 8)
    assert at(0, 2) == 0.5 * (0 - 8)
    assert at(1, 34) == -3.0 * (0 - 8)     # group 1 of row 1
    assert at(1, 35) == -3.0 * (15 - 8)
    assert at(1, 31) == 1.0 * (0 - 8)      # last element of group 0


# --------------------------------------------------------------------------
# P1: hand-expanded instance of the Sec. 3.4 equation
# --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
def test_hand_expanded_tiny(dtype):
    g = json.load(open(os.path.join(GOLDEN, "hand_expanded_tiny.json")))
    x, W = _mk(dtype, g["x"]), _mk(dtype, g["W"])
    ads = [Adapter(_mk(dtype, a["A"]), _mk(dtype, a["B"]), a["scale"]) for a in g["adapters"]]
    y = oracle.linear(dtype, x, W, ads, g["row_adapter"])
    assert np.array_equal(y, np.array(g["y"], dtype=np.float64))
    assert np.array_equal(oracle.linear_grouped(dtype, x, W, ads, g["row_adapter"]), np.array(g["y"]))


# --------------------------------------------------------------------------
# P2: closed form with all-ones operands
# --------------------------------------------------------------------------

def test_all_ones_closed_form():
    g = json.load(open(os.path.join(GOLDEN, "closed_forms.json")))
    for c in g["all_ones"]:
        for dtype in (I.F32, I.BF16):
            K, N, T, r = c["K"], c["N"], c["T"], c["r"]
            one = lambda *s: _mk(dtype, np.ones(s))
            ads = [Adapter(one(r, K), one(N, r), c["scale"])] * 3
            y = oracle.linear(dtype, one(T, K), one(N, K), ads, np.arange(T) % 3)
            assert np.all(y == c["y"]), (c, dtype)


def test_int4_unit_scale_integer_closed_form():
    g = json.load(open(os.path.join(GOLDEN, "closed_forms.json")))["int4_unit_scale"]
    K, N = g["K"], g["N"]
    code = (np.arange(N)[:, None] + np.arange(K)[None, :]) % 16
    packed = (code[:, 0::2] | (code[:, 1::2] << 4)).astype(np.uint8)
    scales = np.full((N, K // 32), np.float16(1.0)).view(np.uint16)
    x = _bf16(np.ones((2, K)))
    y = oracle.linear(I.BF16, x, packed, [], [-1, -1], wfmt=I.W_INT4_G32, w_scales=scales)
    assert np.all(y == g["y_all_ones"])
    # P10: integer x, unit scales -> exact integer result sum_k x_k (code - 8)
    rng = np.random.default_rng(5)
    xi = rng.integers(-4, 5, size=(3, K)).astype(np.float32)
    y = oracle.linear(I.BF16, _bf16(xi), packed, [], [-1] * 3, wfmt=I.W_INT4_G32, w_scales=scales)
    assert np.array_equal(y, xi.astype(np.int64) @ (code.astype(np.int64) - 8).T)


def test_int8_base_sign_group_and_row_order():
    # int8 code per weight, row-major; one fp16 scale per 32 consecutive k of a row; w = scale * code
    K, N = 64, 2
    codes = np.zeros((N, K), dtype=np.int8)
    codes[0, 0], codes[0, 31], codes[0, 32], codes[1, 5], codes[1, 63] = -128, 127, -3, 9, -77
    scales = np.array([[np.float16(0.5), np.float16(2.0)], [np.float16(1.0), np.float16(-3.0)]]).view(np.uint16)
    at = lambda n, k: oracle.weight_at(I.BF16, I.W_INT8_G32, codes, scales, K, n, k)
    assert at(0, 0) == 0.5 * -128       # signed, not a byte 0..255
    assert at(0, 31) == 0.5 * 127       # last element of group 0
    assert at(0, 32) == 2.0 * -3        # first element of group 1
    assert at(1, 5) == 1.0 * 9          # row 1 starts K codes and K/32 scales later
    assert at(1, 63) == -3.0 * -77
    assert at(1, 6) == 0.0


def test_int8_base_unit_scale_integer_closed_form():
    g = json.load(open(os.path.join(GOLDEN, "closed_forms.json")))["int8_unit_scale"]
    K, N = g["K"], g["N"]
    code = (((np.arange(N)[:, None] + 3 * np.arange(K)[None, :]) % 255) - 127).astype(np.int8)
    scales = np.full((N, K // 32), np.float16(1.0)).view(np.uint16)
    y = oracle.linear(I.BF16, _bf16(np.ones((2, K))), code, [], [-1, -1], wfmt=I.W_INT8_G32, w_scales=scales)
    assert np.all(y == g["y0_all_ones"] + g["slope"] * np.arange(N)[None, :])
    # integer x, unit scales -> exact integer result sum_k x_k code[n, k]
    rng = np.random.default_rng(6)
    xi = rng.integers(-4, 5, size=(3, K)).astype(np.float32)
    y = oracle.linear(I.BF16, _bf16(xi), code, [], [-1] * 3, wfmt=I.W_INT8_G32, w_scales=scales)
    assert np.array_equal(y, xi.astype(np.int64) @ code.astype(np.int64).T)


def test_int8_base_matches_dequantised_dense():
    # the 8-bit base must equal the dense path run on the matrix dequantised by numpy, adapters on top as before
    rng = np.random.default_rng(12)
    K, N, T = 96, 10, 4
    codes, sb = I.quantize_int8_g32(rng.standard_normal((N, K)).astype(np.float32))
    wd = codes.astype(np.float64) * np.repeat(sb.view(np.float16).astype(np.float64), 32, axis=1)
    x = I.normal(rng, (T, K), 1.0, I.BF16)
    ad = Adapter(I.normal(rng, (3, K), 1.0, I.BF16), I.normal(rng, (N, 3), 1.0, I.BF16), 0.5)
    y = oracle.linear(I.BF16, x, codes, [ad], [0, -1, 0, 0], wfmt=I.W_INT8_G32, w_scales=sb)
    xd = I.as_f64(x, I.BF16)
    ref = xd @ wd.T
    for t in (0, 2, 3):
        ref[t] += 0.5 * (I.as_f64(ad.B, I.BF16) @ (I.as_f64(ad.A, I.BF16) @ xd[t]))
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)
    yg = oracle.linear_grouped(I.BF16, x, codes, [ad], [0, -1, 0, 0], wfmt=I.W_INT8_G32, w_scales=sb)
    np.testing.assert_allclose(yg, y, rtol=1e-13, atol=1e-13)


def test_int8_quantiser_round_trip_bound():
    # the generator's codes reproduce w within half a step of its group's scale (what the test inputs rely on)
    rng = np.random.default_rng(13)
    w = rng.standard_normal((6, 128)).astype(np.float32)
    codes, sb = I.quantize_int8_g32(w)
    s = np.repeat(sb.view(np.float16).astype(np.float64), 32, axis=1)
    assert np.all(np.abs(codes.astype(np.float64) * s - w) <= 0.5 * s + 1e-12)
    assert codes.min() >= -127 and codes.max() <= 127


def test_int4_matches_dequantised_dense():
    # the 4-bit path must equal the dense path run on the dequantised matrix (library decode via numpy)
    rng = np.random.default_rng(11)
    K, N, T = 96, 10, 4
    packed, sb = I.quantize_int4_g32(rng.standard_normal((N, K)).astype(np.float32))
    code = np.stack([packed & 0xF, packed >> 4], axis=2).reshape(N, K).astype(np.float64)
    wd = (code - 8.0) * np.repeat(sb.view(np.float16).astype(np.float64), 32, axis=1)
    x = I.normal(rng, (T, K), 1.0, I.BF16)
    ad = Adapter(I.normal(rng, (3, K), 1.0, I.BF16), I.normal(rng, (N, 3), 1.0, I.BF16), 0.5)
    y = oracle.linear(I.BF16, x, packed, [ad], [0, -1, 0, 0], wfmt=I.W_INT4_G32, w_scales=sb)
    xd = I.as_f64(x, I.BF16)
    ref = xd @ wd.T
    for t in (0, 2, 3):
        ref[t] += 0.5 * (I.as_f64(ad.B, I.BF16) @ (I.as_f64(ad.A, I.BF16) @ xd[t]))
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)


# --------------------------------------------------------------------------
# library-routine reference on random rectangular cases (catches transposes,
# wrong strides, wrong adapter, dropped scale)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_numpy_matmul(dtype, seed):
    x, W, ads, ra = _random_case(seed, dtype, K=24 + 8 * seed, N=20 - 3 * seed, T=9 + seed)
    y = oracle.linear(dtype, x, W, ads, ra)
    ref = _numpy_reference(dtype, x, W, ads, ra)
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    assert np.abs(ref).max() > 1.0  # the comparison is not vacuous


def test_row_scale_override():
    x, W, ads, ra = _random_case(7)
    rs = np.linspace(-1, 2, len(ra)).astype(np.float32)
    y = oracle.linear(I.F32, x, W, ads, ra, row_scale=rs)
    np.testing.assert_allclose(y, _numpy_reference(I.F32, x, W, ads, ra, rs), rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------
# P3..P9 invariants
# --------------------------------------------------------------------------

def test_P3_zero_B_gives_exactly_base():
    x, W, ads, ra = _random_case(3)
    zero = [Adapter(a.A, np.zeros_like(a.B), a.scale) for a in ads]
    y = oracle.linear(I.F32, x, W, zero, ra)
    base = oracle.linear(I.F32, x, W, zero, np.full(len(ra), -1))
    assert np.array_equal(y, base)
    np.testing.assert_allclose(base, I.as_f64(x, I.F32) @ I.as_f64(W, I.F32).T, rtol=1e-13, atol=1e-13)


def test_P4_identical_adapters_equal_merged_weights():
    # merged inference (Sec. 2.1): folding s*B*A into W gives the same output
    x, W, ads, _ = _random_case(4, ranks=(3,))
    same = [ads[0]] * len(ads)
    ra = np.arange(x.shape[0]) % len(ads)
    y = oracle.linear(I.F32, x, W, same, ra)
    Wm = I.as_f64(W, I.F32) + ads[0].scale * (I.as_f64(ads[0].B, I.F32) @ I.as_f64(ads[0].A, I.F32))
    np.testing.assert_allclose(y, I.as_f64(x, I.F32) @ Wm.T, rtol=1e-12, atol=1e-12)


def test_P5_rank_one_closed_form():
    rng = np.random.default_rng(5)
    K, N, T = 16, 12, 6
    x, W = I.normal(rng, (T, K), 1, I.F32), I.normal(rng, (N, K), 1, I.F32)
    a, b = I.normal(rng, (1, K), 1, I.F32), I.normal(rng, (N, 1), 1, I.F32)
    y = oracle.linear(I.F32, x, W, [Adapter(a, b, 1.5)], np.zeros(T, dtype=np.int32))
    xd = x.astype(np.float64)
    ref = xd @ W.astype(np.float64).T + 1.5 * np.outer(xd @ a[0].astype(np.float64), b[:, 0].astype(np.float64))
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_P6_permuting_rows_permutes_outputs_bit_exactly():
    x, W, ads, ra = _random_case(6, I.BF16)
    perm = np.random.default_rng(0).permutation(len(ra))
    y = oracle.linear(I.BF16, x, W, ads, ra)
    yp = oracle.linear(I.BF16, x[perm], W, ads, ra[perm])
    assert np.array_equal(yp, y[perm])


def test_P7_segments_equal_per_token_and_grouped_equals_per_sample():
    rng = np.random.default_rng(8)
    x, W, ads, _ = _random_case(8, T=12)
    lengths = [3, 0, 1, 5, 0, 3]
    so = I.offsets_from_lengths(lengths)
    sa = np.array([2, 4, -1, 0, 1, 2], dtype=np.int32)
    ra = oracle.rows_from_segments(12, so, sa)
    assert ra.tolist() == [2, 2, 2, -1, 0, 0, 0, 0, 0, 2, 2, 2]
    y_seg = oracle.linear_segments(I.F32, x, W, ads, so, sa)
    assert np.array_equal(y_seg, oracle.linear(I.F32, x, W, ads, ra))
    # Sec. 4.3: the grouped (u-batch) computation gives what the per-sample baseline gives
    yg = oracle.linear_grouped(I.F32, x, W, ads, ra)
    np.testing.assert_allclose(yg, y_seg, rtol=1e-13, atol=1e-13)
    with pytest.raises(ValueError):
        oracle.rows_from_segments(12, [0, 5, 4, 12], [0, 1, 2])
    with pytest.raises(ValueError):
        oracle.rows_from_segments(12, [0, 5, 11], [0, 1])


def test_P8_zero_padding_the_rank_changes_nothing():
    x, W, ads, ra = _random_case(9, I.BF16)
    R = 8
    padded = []
    for a in ads:
        Ap = np.zeros((R, a.A.shape[1]), dtype=a.A.dtype); Ap[: a.rank] = a.A
        Bp = np.zeros((a.B.shape[0], R), dtype=a.B.dtype); Bp[:, : a.rank] = a.B
        padded.append(Adapter(Ap, Bp, a.scale))
    assert np.array_equal(oracle.linear(I.BF16, x, W, padded, ra), oracle.linear(I.BF16, x, W, ads, ra))


def test_P9_linear_in_scale():
    x, W, ads, ra = _random_case(10)
    at = lambda s: oracle.linear(I.F32, x, W, [Adapter(a.A, a.B, s) for a in ads], ra)
    y0, y1, y3 = at(0.0), at(1.0), at(3.0)
    np.testing.assert_allclose(y3 - y0, 3.0 * (y1 - y0), rtol=1e-11, atol=1e-12)
    assert np.abs(y1 - y0).max() > 0.1


def test_routing_probe_spells_the_adapter_index():
    # W = 0, x_t = e_0, A_i[0,0] = 1, B_i[0,0] = i mod 256, B_i[1,0] = i div 256, s = 1
    P, K, N, T = 700, 8, 4, 50
    rng = np.random.default_rng(12)
    ads = []
    for i in range(P):
        A = np.zeros((1, K), np.float32); A[0, 0] = 1
        B = np.zeros((N, 1), np.float32); B[0, 0] = i % 256; B[1, 0] = i // 256
        ads.append(Adapter(_bf16(A), _bf16(B), 1.0))
    x = np.zeros((T, K), np.float32); x[:, 0] = 1
    ra = rng.integers(0, P, size=T).astype(np.int32)
    y = oracle.linear(I.BF16, _bf16(x), _bf16(np.zeros((N, K))), ads, ra)
    assert np.array_equal((y[:, 0] + 256 * y[:, 1]).astype(np.int64), ra)


# --------------------------------------------------------------------------
# u-batch map and output selection
# --------------------------------------------------------------------------

def test_ubatches_is_a_stable_counting_sort():
    rng = np.random.default_rng(13)
    P = 9
    ra = rng.integers(-1, P, size=200).astype(np.int32)
    perm, offs, distinct = oracle.ubatches(ra, P)
    key = np.where(ra < 0, P, ra)
    assert np.array_equal(perm, np.argsort(key, kind="stable"))
    assert np.array_equal(offs, np.concatenate([[0], np.cumsum(np.bincount(ra[ra >= 0], minlength=P))]))
    assert distinct == len(np.unique(ra[ra >= 0]))


def test_row_and_column_selection_is_a_submatrix():
    x, W, ads, ra = _random_case(14, I.BF16, K=40, N=33, T=17)
    full = oracle.linear(I.BF16, x, W, ads, ra)
    rows, cols = [16, 0, 5, 5], [32, 1, 0, 7, 31]
    sub = oracle.linear(I.BF16, x, W, ads, ra, rows=rows, cols=cols)
    assert np.array_equal(sub, full[np.ix_(rows, cols)])
    one, used = oracle.linear(I.BF16, x, W, ads, ra, n_threads=1, return_threads=True)
    assert used == 1 and np.array_equal(one, full)  # threads only pick who computes a row


def test_bad_arguments_are_rejected():
    x, W, ads, ra = _random_case(15)
    ra[0] = len(ads)
    with pytest.raises(ValueError):
        oracle.linear(I.F32, x, W, ads, ra)
    ra[0] = 0
    with pytest.raises(ValueError):
        oracle.linear(I.F32, x, W, [None] + ads[1:], ra)
    with pytest.raises(TypeError):
        oracle.linear(I.BF16, x, W, ads, ra)


# ---------------------------------------------------------------------------------------------
# adapters kept in 8-bit blocks (Sec. 5 "Model": all adapters in the block format called Q8_0):
# value = fp16 scale of the block * int8 code, blocks of 32 consecutive values in row-major order
# ---------------------------------------------------------------------------------------------

def _fp16_bits(v):
    return np.array(v, dtype=np.float16).view(np.uint16)


def _dequant_independent(codes, scales_bits):
    """scale * code with numpy's own fp16 decoding, as float64 (exact)."""
    sc = np.asarray(scales_bits, dtype=np.uint16).view(np.float16).astype(np.float64)
    return (np.asarray(codes, dtype=np.int8).reshape(-1).astype(np.float64) * np.repeat(sc, 32)).reshape(np.shape(codes))


def test_q8_adapters_unit_scales_integer_closed_form():
    # unit scales, integer x, W = 0: y = s * B_codes (A_codes x) in integers, exactly
    rng = np.random.default_rng(81)
    K, N, T, r = 64, 12, 5, 8
    x = rng.integers(-3, 4, size=(T, K)).astype(np.float32)
    W = np.zeros((N, K), np.float32)
    Ac = rng.integers(-127, 128, size=(r, K), dtype=np.int8)
    Bc = rng.integers(-127, 128, size=(N, r), dtype=np.int8)
    one = lambda n: np.full(n // 32, 0x3C00, dtype=np.uint16)
    ad = oracle.Adapter(Ac, Bc, 2.0, A_scales=one(Ac.size), B_scales=one(Bc.size))
    y = oracle.linear(I.F32, x, W, [ad], np.zeros(T, np.int32))
    want = 2 * (Bc.astype(np.int64) @ (Ac.astype(np.int64) @ x.astype(np.int64).T)).T
    assert np.array_equal(y, want.astype(np.float64))


def test_q8_adapter_blocks_run_across_rows_and_carry_their_own_scales():
    # B [8, 8]: 64 values = two blocks of four rows each.  Only B[5, 2] = 3 and A[2, 40] = 5 are non-zero, x = e_40:
    # y[5] = s * (scale of B's second block) * 3 * (scale of A's block 2 * 2 + 1 = 5: row 2, columns 32..63) * 5.
    K, N, r = 64, 8, 8
    Ac = np.zeros((r, K), np.int8); Ac[2, 40] = 5
    Bc = np.zeros((N, r), np.int8); Bc[5, 2] = 3
    As = _fp16_bits(np.arange(1, 17, dtype=np.float32) * 0.25)      # block b of A has scale (b + 1) / 4
    Bs = _fp16_bits([0.5, -1.5])
    x = np.zeros((1, K), np.float32); x[0, 40] = 1
    ad = oracle.Adapter(Ac, Bc, 1.0, A_scales=As, B_scales=Bs)
    y = oracle.linear(I.F32, x, np.zeros((N, K), np.float32), [ad], np.zeros(1, np.int32))
    want = np.zeros((1, N)); want[0, 5] = (-1.5 * 3) * ((6 / 4) * 5)
    assert np.array_equal(y, want)


def _b2d(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_q8_adapters_equal_the_dense_product_of_their_dequantised_values():
    # against numpy float64 on independently dequantised matrices; mixed with an adapter in bf16, ranks 8 and 16,
    # bf16 x and W; per-sample and grouped forms agree
    rng = np.random.default_rng(82)
    K, N, T = 96, 20, 7
    x = _bf16((rng.standard_normal((T, K))).astype(np.float32))
    W = _bf16((rng.standard_normal((N, K)) * 0.05).astype(np.float32))
    ads, dense = [], []
    for r in (8, 16):
        Ac = rng.integers(-127, 128, size=(r, K), dtype=np.int8)
        Bc = rng.integers(-127, 128, size=(N, r), dtype=np.int8)
        As = _fp16_bits(rng.uniform(1e-3, 2e-2, Ac.size // 32).astype(np.float32))
        Bs = _fp16_bits(rng.uniform(1e-3, 2e-2, Bc.size // 32).astype(np.float32))
        ads.append(oracle.Adapter(Ac, Bc, 1.5, A_scales=As, B_scales=Bs))
        dense.append((_dequant_independent(Ac, As), _dequant_independent(Bc, Bs), 1.5))
    A2 = _bf16((rng.standard_normal((4, K)) * 0.05).astype(np.float32))
    B2 = _bf16((rng.standard_normal((N, 4)) * 0.05).astype(np.float32))
    ads.append(oracle.Adapter(A2, B2, 0.5))
    dense.append((_b2d(A2), _b2d(B2), 0.5))
    ra = np.array([0, 1, 2, -1, 1, 0, 2], dtype=np.int32)
    y = oracle.linear(I.BF16, x, W, ads, ra)
    xf, Wf = _b2d(x), _b2d(W)
    want = xf @ Wf.T
    for t, i in enumerate(ra):
        if i >= 0:
            A, B, s = dense[i]
            want[t] += s * (B @ (A @ xf[t]))
    assert np.abs(y - want).max() <= 1e-12 * np.abs(want).max()
    yg = oracle.linear_grouped(I.BF16, x, W, ads, ra)
    assert np.abs(yg - y).max() <= 1e-12 * np.abs(y).max()
