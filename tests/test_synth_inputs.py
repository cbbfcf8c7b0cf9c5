"""The seeded input recipe: deterministic, layer-sliceable, shaped as stated."""
import numpy as np

from paper_2502_02789_amd import synth


def test_workload_shapes_match_the_benchmark_definition():
    w3 = synth.workload(3)
    assert (w3.T, w3.L, w3.H, w3.H_kv, w3.d, w3.N) == (32768, 32, 32, 8, 128, 8)
    assert w3.k_bytes() == 2 * 1024 ** 3
    w4 = synth.workload(4)
    assert w4.B == 64 and min(w4.seqlens) >= 1024 and max(w4.seqlens) <= 4096
    assert w4.seqlens == synth.workload(4).seqlens
    w5 = synth.workload(5)
    assert w5.T == 131072 and w5.chunk == 64 and w5.embed_dim == 8192


def test_layers_are_reproducible_alone():
    w = synth.scaled(synth.workload(2), seqlens=(300,), L=4)
    full = synth.make_qk(w)
    part = synth.make_qk(w, layers=[2])
    assert (full["q"][2] == part["q"][0]).all()
    assert (full["k"][2] == part["k"][0]).all()
    assert full["q"].shape == (4, 1, 8, 32, 64) and full["k"][0].shape == (300, 8, 64)
    assert full["q"].dtype == np.uint16


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-40], dtype=np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie -> rounds to even (1.0); 1.01171875 = 1 + 3*2^-8 ties up to 1 + 2^-6
    got = synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(x))
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.015625 and got[3] == -2.5


def test_rope_keeps_norms_and_position_zero_is_identity():
    g = np.random.default_rng(0)
    x = g.standard_normal((5, 2, 64)).astype(np.float32)
    r = synth.rope_rotate(x, np.arange(5))
    np.testing.assert_allclose(np.linalg.norm(r, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-5)
    assert (r[0] == x[0]).all()


def test_salient_runs_and_fraction():
    w = synth.workload(3)
    m = synth.salient_mask(w)
    assert 0.005 * w.T <= m.sum() <= 0.011 * w.T
    w1 = synth.workload(1)
    assert synth.salient_mask(w1).sum() == 20
