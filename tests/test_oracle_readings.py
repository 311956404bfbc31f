"""Pins for the alternative row-scale readings: the built reading reproduces the main oracle bit for bit, the
three scales are ordered, and they coincide exactly where the definitions say they must."""
import numpy as np

from oracle import mixed_linear as ml
from oracle import readings as rd
from paper_2407_19775_amd import workloads as wl


def data(seed, outliers=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((24, 128)).astype(np.float32)
    if outliers:
        x[::3, 5] *= 30.0                     # a critical column whose other rows stay below the threshold
        x[:, 77] = 40.0                       # a critical column with every entry above it
    X = wl.to_fp16(x)
    Wq, c = ml.prequantize_weight(wl.to_fp16(rng.standard_normal((128, 40)).astype(np.float32) * 0.05))
    return X, Wq, c


def test_built_reading_is_the_main_oracle():
    X, Wq, c = data(0)
    a = rd.mixed_int8_linear_with_row_scale(X, Wq, c, 6.0, "sub_threshold")
    b = ml.mixed_int8_linear(X, Wq, c, 6.0)
    for k in ("flag", "r", "Xq", "acc", "Y"):
        assert np.array_equal(a[k], b[k]), k


def test_scales_are_ordered_and_meet_where_they_must():
    X, Wq, c = data(1)
    r = {k: rd.row_scale(X, 6.0, k) for k in rd.ROW_SCALES}
    assert np.all(r["non_critical"] <= r["sub_threshold"]) and np.all(r["sub_threshold"] <= r["all"])
    assert np.all(r["all"] >= 40.0)                                   # column 77 (or a larger entry of column 5)
    # by hand: the non-critical scale ignores columns 5 and 77 altogether
    ax = np.abs(X.astype(np.float32))
    assert np.array_equal(r["non_critical"], np.delete(ax, [5, 77], axis=1).max(axis=1))
    # the sub-threshold scale may pick up an entry of column 5 in a row where it is below 6
    sub = np.where(ax < 6.0, ax, 0).max(axis=1)
    assert np.array_equal(r["sub_threshold"], sub)
    # without critical columns all three are the plain row absmax and the layers agree bit for bit
    X0, Wq0, c0 = data(2, outliers=False)
    ys = [rd.mixed_int8_linear_with_row_scale(X0, Wq0, c0, np.inf, k)["Y"] for k in rd.ROW_SCALES]
    assert np.array_equal(ys[0], ys[1]) and np.array_equal(ys[0], ys[2])
    # a critical column whose every entry is above the threshold contributes nothing below it: the first two agree
    X1 = X0.copy()
    X1[:, 9] = np.float16(50.0)
    assert np.array_equal(rd.row_scale(X1, 6.0, "sub_threshold"), rd.row_scale(X1, 6.0, "non_critical"))


def test_master_rows_make_tau_zero_the_exact_fp16_product():
    # every column critical: with the original rows the layer is X W exactly (rounded once); with the re-created
    # rows it is X times the dequantized weights, within c / 254 * sum |x| of it
    rng = np.random.default_rng(5)
    X = wl.to_fp16(rng.standard_normal((7, 64)).astype(np.float32))
    W = wl.to_fp16(rng.standard_normal((64, 24)).astype(np.float32) * 0.05)
    Wq, c = ml.prequantize_weight(W)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    a = rd.mixed_int8_linear_with_row_scale(X, Wq, c, 0.0, "sub_threshold", master_W=W)
    assert np.array_equal(a["Y"], exact.astype(np.float16)) and not a["acc"].any()
    b = rd.mixed_int8_linear_with_row_scale(X, Wq, c, 0.0, "sub_threshold")
    bound = (c.astype(np.float64) / 254.0)[None, :] * np.abs(X.astype(np.float64)).sum(axis=1)[:, None]
    assert np.all(np.abs(b["Y64"] - exact) <= bound * (1 + 2.0 ** -9) + 1e-12)
    assert np.any(b["Y"] != a["Y"])
