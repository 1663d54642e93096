"""Sanity of the seeded input generators (distributions, seeds, shapes).  CPU only."""
import numpy as np

from paper_2410_16144_amd import synth


def test_weight_distributions():
    rng = synth.rng_for(5)
    w = synth.ternary_weights(rng, 400, 500)
    n = w.size
    for v in (-1, 0, 1):
        f = np.count_nonzero(w == v) / n
        assert abs(f - 1 / 3) < 4 * np.sqrt((1 / 3) * (2 / 3) / n)
    w = synth.ternary_weights(rng, 400, 500, p_zero=0.4)
    for v, p in ((-1, 0.3), (0, 0.4), (1, 0.3)):
        f = np.count_nonzero(w == v) / n
        assert abs(f - p) < 4 * np.sqrt(p * (1 - p) / n)
    assert w.dtype == np.int8 and set(np.unique(w).tolist()) == {-1, 0, 1}


def test_activation_outliers_and_determinism():
    x = synth.activations(synth.rng_for(6), 8, 20000, outlier_frac=0.01)
    assert x.dtype == np.float32
    assert abs(x.std() - np.sqrt(0.99 + 0.01 * 400)) < 0.1
    assert 0.004 < np.mean(np.abs(x) > 6.5) < 0.012      # N(0,1) almost never exceeds 6.5; x20 outliers mostly do
    y = synth.activations(synth.rng_for(6), 8, 20000, outlier_frac=0.01)
    assert np.array_equal(x, y)
    s = synth.draw_w_scale(synth.rng_for(1))
    assert s.dtype == np.float32 and 0.01 <= s <= 0.05


def test_seed_rule_and_shapes():
    assert synth.seed_for(1) == 0
    assert synth.seed_for(2, 3, 4) == 2034
    assert len(synth.PAPER_MODELS) == 12
    projs = synth.layer_projections(3200, 8640)
    assert [p.name for p in projs] == list(synth.PROJ_NAMES)
    assert sum(p.packed_bytes for p in projs) == 30_976_000
    assert sum(p.packed_bytes for p in synth.layer_projections(4096, 11008)) == 50_593_792
    assert sum(p.packed_bytes for p in synth.layer_projections(12288, 33792)) == 462_422_016
    h, f, layers = synth.PAPER_MODELS["100B"]
    total = layers * sum(p.packed_bytes for p in synth.layer_projections(h, f))
    assert abs(total - 24.99e9) < 0.01e9


def test_bf16_bits_roundtrip():
    x = np.array([1.0, -2.0, 0.5, 3.140625, 1.00390625, 1.01171875], np.float32)
    b = synth.to_bf16_bits(x)
    assert b.tolist()[:4] == [0x3F80, 0xC000, 0x3F00, 0x4049]
    assert b[4] == 0x3F80          # 1 + 2^-8 is a tie: rounds to even (1.0)
    assert b[5] == 0x3F82          # 1 + 3*2^-8 is a tie: rounds to even (1 + 2^-6)
    assert np.array_equal(synth.bf16_bits_to_f32(b)[:4], x[:4])
