"""Seeded generators: determinism, the stated outlier structure, and the smallest benchmark
layer (C1) checked end-to-end against the dense definition."""
import numpy as np

from oracle import apb_oracle as o
from oracle import capi
from paper_2306_08960_amd import synth


def test_generators_are_deterministic():
    cfg = synth.CONFIGS["C1"]
    W1, d1, X1, s1 = synth.make_layer(cfg)
    W2, d2, X2, s2 = synth.make_layer(cfg)
    assert np.array_equal(W1, W2) and np.array_equal(X1, X2) and d1 == d2 and s1 == s2
    assert W1.dtype == np.float32 and X1.dtype == np.float32 and W1.shape == (256, 256) and X1.shape == (256, 64)


def test_outlier_rates_of_quantile_configs():
    for name in ("C1", "C3_r05_b1", "C3_r50_b2"):
        cfg = synth.CONFIGS[name]
        W, delta = synth.make_weights(cfg)
        nnz = int(np.count_nonzero(np.abs(W) > delta))
        assert nnz == int(np.floor(cfg.rho * cfg.N * cfg.K))


def test_zipf_rows_are_skewed():
    cfg = synth.CONFIGS["C4"]
    W, delta = synth.make_weights(cfg)
    per_row = np.count_nonzero(np.abs(W) > delta, axis=1)
    assert abs(int(per_row.sum()) - 1475) <= 64
    assert per_row.max() > 250 and per_row.min() <= 4
    top = np.sort(per_row)[::-1]
    assert top[0] > 1.8 * top[1] > 1.8 * top[3] * 0.9     # roughly r^-1.1


def test_two_bit_code_mix():
    cfg = synth.small_variant(synth.CONFIGS["C2"], M=4096)
    X = synth.make_acts(cfg)
    c = o.quantize(X, 2, cfg.step)
    frac = np.bincount(c.ravel(), minlength=4) / c.size
    assert np.allclose(frac, [0.646, 0.223, 0.101, 0.030], atol=0.01)


def test_c1_oracle_against_dense_definition():
    cfg = synth.CONFIGS["C1"]
    W, delta, X, step = synth.make_layer(cfg)
    L = o.compress(W, delta)
    assert L["row_ptr"][-1] == 655
    c = o.quantize(X, cfg.bits, step)
    F = capi.forward(L, o.pack_acts(c, cfg.bits), c, cfg.bits, step, threads=2)
    Yb = o.brute_force(W, delta, L["alpha"], X, cfg.bits, step)
    mag = np.abs(o.apb_dense(W, delta, L["alpha"])) @ np.abs(o.dequantize(c, step))
    assert np.max(np.abs(F["Y"] - Yb) / mag) < 2.0 ** -22
    assert np.array_equal(F["D"], o.int_part_unpacked(L["bit"], c))
