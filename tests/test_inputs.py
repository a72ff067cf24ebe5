"""Seeded input generators: reproducible, right shapes, right distributions (no GPU)."""
import numpy as np
import torch

from paper_2507_01438_amd import inputs as I


def test_bf16_rounding_is_rne_and_matches_torch():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(20000) * 10 ** rng.uniform(-6, 6, 20000)).astype(np.float32)
    bits = I.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert I.f32_to_bf16_bits(np.array([1 + 2.0 ** -8], np.float32))[0] == 0x3F80
    assert I.f32_to_bf16_bits(np.array([1 + 3 * 2.0 ** -8], np.float32))[0] == 0x3F82
    assert np.array_equal(I.f32_to_bf16_bits(I.bf16_bits_to_f32(bits)), bits)


def test_power_law_matches_formula_and_draws():
    p = I.power_law_probs(64, 1.1)
    assert abs(p.sum() - 1) < 1e-12 and abs(p[0] / p[1] - 2 ** 1.1) < 1e-12
    rng = np.random.default_rng(1)
    idx = I.draw_adapters(rng, 200000, 64, 1.1)
    freq = np.sort(np.bincount(idx, minlength=64) / 200000.0)[::-1]
    assert np.abs(freq - p).max() < 0.005
    assert 0.23 < freq[0] < 0.27  # the most popular adapter of the 64 takes about a quarter


def test_int4_pack_round_trip():
    rng = np.random.default_rng(2)
    w = (rng.standard_normal((6, 128)) * 0.02).astype(np.float32)
    packed, sb = I.quantize_int4_g32(w)
    assert packed.shape == (6, 64) and sb.shape == (6, 4)
    code = np.stack([packed & 0xF, packed >> 4], axis=2).reshape(6, 128).astype(np.float32)
    deq = (code - 8) * np.repeat(sb.view(np.float16).astype(np.float32), 32, axis=1)
    step = np.repeat(sb.view(np.float16).astype(np.float32), 32, axis=1)
    assert np.all(np.abs(deq - w) <= 0.5 * step * 1.01 + 1e-8)
    assert code.min() >= 1 and code.max() <= 15  # symmetric: code 0 (= -8) is never produced by absmax/7


def test_configs_have_the_stated_shapes():
    c1, c2, c3, c4, c5 = (I.CONFIGS[i]() for i in range(1, 6))
    assert (c1.dtype, c1.T, c1.pool, c1.max_rank, c1.scale) == (I.F32, 8, 4, 8, 2.0)
    assert (c2.T, c2.pool, c2.max_rank) == (32, 64, 16) and (c2.projections[0].K, c2.projections[0].N) == (4096, 4096)
    assert c3.T == 64 and c3.pool == 256 and set(np.unique(c3.ranks)) == {8, 16, 32, 64}
    assert [(p.K, p.N) for p in c3.projections] == [(4096, 4096), (4096, 1024), (4096, 1024), (4096, 4096),
                                                    (4096, 14336), (4096, 14336), (14336, 4096)]
    lens = np.diff(c4.seg_offsets)
    assert len(lens) == 16 and lens.min() >= 64 and lens.max() <= 1024 and len(set(c4.seg_adapter)) == 16
    assert c5.T == 4 * 512 + 120 and c5.wfmt == I.W_INT4_G32 and len(c5.seg_adapter) == 124
    assert np.array_equal(c5.row_adapter()[:512], np.full(512, c5.seg_adapter[0]))
    # same seed, same bytes
    p = c2.projections[0]
    assert np.array_equal(I.config2().x(p), c2.x(p))
    A1, B1, _ = c2.adapter(p, 5)
    A2, B2, _ = I.config2().adapter(p, 5)
    assert np.array_equal(A1, A2) and np.array_equal(B1, B2)
    # algorithmic bytes of the headline configuration: W + x + y + distinct adapters (about 38 MB)
    assert 36e6 < c2.algorithmic_bytes(p) < 43e6
