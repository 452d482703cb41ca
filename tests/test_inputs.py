"""The seeded input generator: deterministic, counter based (row subsets equal the full draw), right shapes and
distributions for the five benchmark configurations."""
import numpy as np

from paper_2304_13013_amd import inputs as I


def test_deterministic_and_subset_consistent():
    a = I.make_layer_inputs("tiny", seed=0)
    b = I.make_layer_inputs("tiny", seed=0)
    c = I.make_layer_inputs("tiny", seed=1)
    for k in ("x", "w", "dy"):
        assert np.array_equal(a[k], b[k]) and not np.array_equal(a[k], c[k])
    rows = [0, 7, 511]
    sub = I.make_layer_inputs("tiny", token_rows=rows)
    assert np.array_equal(sub["x"], a["x"][rows]) and np.array_equal(sub["dy"], a["dy"][rows])
    assert np.array_equal(sub["w"], a["w"])


def test_shapes_and_moments():
    d = I.make_layer_inputs("tiny")
    assert d["x"].shape == (512, 256) and d["w"].shape == (1024, 256) and d["dy"].shape == (512, 1024)
    x, w, dy = (I.bf16_bits_to_f32(d[k]).astype(np.float64) for k in ("x", "w", "dy"))
    assert abs(x.std() - 1) < 0.02 and abs(w.std() - 1 / 16) < 0.002 and abs(dy.std() - 1) < 0.02
    assert abs(x.mean()) < 0.02
    rows = np.arange(0, 6304, 97)
    d = I.make_layer_inputs("vit_b16", 1, token_rows=rows, which=("x", "dy"))
    assert d["x"].shape == (len(rows), 3072) and d["dy"].shape == (len(rows), 768)
    assert abs(I.bf16_bits_to_f32(d["dy"]).std() - 0.1) < 0.005


def test_outlier_config():
    rows = np.arange(64)
    d = I.make_layer_inputs("outlier", 0, token_rows=rows, which=("x", "dy"))
    x = I.bf16_bits_to_f32(d["x"]).astype(np.float64)
    cols = I.outlier_columns(4096, 0, 1)
    assert len(cols) == 5 and len(set(cols.tolist())) == 5
    mask = np.zeros(4096, bool)
    mask[cols] = True
    assert x[:, mask].std() > 50 and abs(x[:, ~mask].std() - 1) < 0.05
    dy = I.bf16_bits_to_f32(d["dy"]).astype(np.float64)
    assert np.abs(dy).max() > 0.2                      # heavy tails: far beyond 6 sigma of a 0.01 normal
    assert 0.008 < np.median(np.abs(dy)) / 0.7649 < 0.012   # median |t_3| = 0.7649


def test_bf16_round_trip():
    v = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.0e-39], np.float32)
    bits = I.f32_to_bf16_bits(v)
    back = I.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625) and back[3] == -2.5
    assert np.array_equal(I.f32_to_bf16_bits(back), bits)
