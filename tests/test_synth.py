"""Shape, range and reproducibility checks of the seeded input generators."""
import numpy as np

import synth


def test_configs_follow_the_benchmark_table():
    c2, c3, c4 = synth.CONFIGS["C2"], synth.CONFIGS["C3"], synth.CONFIGS["C4"]
    assert c2.n_bits == c2.n * c2.m and c4.n_bits == c4.n * c4.m
    assert synth.CONFIGS["C1"].n_bits == 60 and synth.CONFIGS["C1"].t == 2
    # a 64-px tile of a 256-px image is 1/16 of the work (Section 7, end-to-end evaluation)
    assert c3.flops_per_image() == 16 * c2.flops_per_image()
    assert abs(c2.flops_per_image() - 2.355e9) < 1e6


def test_images_are_position_addressable():
    cfg = synth.CONFIGS["C1"]
    a = synth.images(cfg, 0, 4)
    b = synth.images(cfg, 2, 2)
    assert a.dtype == np.uint8 and a.shape == (4, 3, 256, 256)
    assert np.array_equal(a[2:], b)
    assert not np.array_equal(a[0], a[1])
    assert 120 < a.mean() < 135 and a.min() == 0 and a.max() == 255


def test_offsets_policies():
    cfg = synth.CONFIGS["C2"]
    r = synth.offsets(cfg, 0, 5000, "random")
    assert r.min() >= 0 and r.max() <= cfg.H - cfg.tile and r.max() > 150
    assert np.array_equal(r[4090:4100], synth.offsets(cfg, 4090, 10, "random"))
    g = synth.offsets(cfg, 0, 1000, "random_grid")
    assert np.all(g % cfg.tile == 0) and g.max() == cfg.H - cfg.tile
    assert not synth.offsets(cfg, 0, 10, "fixed").any()
    assert not synth.offsets(synth.CONFIGS["C3"], 0, 10, "random").any()   # full-image tile


def test_weights_statistics():
    w = synth.config_weights(synth.CONFIGS["C2"])
    assert w["conv_w"].size == 64 * 3 * 9 + 7 * 64 * 64 * 9 + 48 * 64 * 9
    mid = w["conv_w"][64 * 27:64 * 27 + 64 * 64 * 9]
    assert abs(mid.std() - np.sqrt(2 / 576)) < 2e-3
    assert abs(w["scale"].mean() - 1) < 0.03 and abs(w["bias"].mean()) < 0.03
    assert w["lin_w"].shape == (48, 48) and not w["lin_b"].any()
    w2 = synth.config_weights(synth.CONFIGS["C2"])
    assert np.array_equal(w["conv_w"], w2["conv_w"])


def test_rs_cases_error_patterns():
    msgs, err, nerr = synth.rs_cases(0, 4000, 15, 11, 4)
    assert msgs.max() < 16 and err.max() < 16
    assert np.array_equal((err != 0).sum(1), nerr)
    assert set(np.unique(nerr)) == {0, 1, 2, 3}
    counts = np.bincount(nerr, minlength=4)
    assert counts.min() > 800
    pos = np.nonzero(err)[1]
    assert np.bincount(pos, minlength=15).min() > 250            # positions roughly uniform
