"""Pins for the low-rank adapted layer of the oracle: special cases with a closed form, brute force,
the adapted-weight identity W' = W + B A, additivity over the rank."""
import numpy as np

from oracle import lora
from oracle import mixed_linear as ml
from paper_2407_19775_amd import workloads as wl


def case(seed, M, K, N, r, outlier_cols=(7,)):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    for k in outlier_cols:
        x[:, k] *= 20.0
    X = wl.to_fp16(x)
    W = wl.to_fp16(rng.standard_normal((K, N)).astype(np.float32) * 0.02)
    A = wl.to_fp16(rng.standard_normal((r, K)).astype(np.float32) * 0.05)
    B = wl.to_fp16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    Wq, c = ml.prequantize_weight(W)
    return X, W, Wq, c, A, B


def test_zero_factor_leaves_the_base_layer():
    X, W, Wq, c, A, B = case(1, 9, 64, 24, 4)
    base = ml.mixed_int8_linear(X, Wq, c, 6.0)
    for A_, B_ in [(np.zeros_like(A), B), (A, np.zeros_like(B))]:
        o = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A_, B_)
        assert np.array_equal(o["Y"].view(np.uint16), base["Y"].view(np.uint16))


def test_selector_rows_give_a_closed_form():
    # A picks feature dimensions k_j: T is those columns of X without rounding, and the
    # correction is sum_j X[m, k_j] B[n, j], written out here as loops
    X, W, Wq, c, _, B = case(2, 5, 48, 16, 3, outlier_cols=(7, 20))
    picks = [20, 3, 41]                                            # one critical column among them
    A = np.zeros((3, 48), np.float16)
    for j, k in enumerate(picks):
        A[j, k] = 1.0
    o = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A, B)
    assert np.array_equal(o["T"], X[:, picks])
    base = ml.mixed_int8_linear(X, Wq, c, 6.0)
    for m in range(5):
        for n in range(16):
            corr = sum(float(X[m, k]) * float(B[n, j]) for j, k in enumerate(picks))
            assert abs(o["Y64"][m, n] - (base["Y64"][m, n] + corr)) <= 1e-12 * (1 + abs(corr))


def test_brute_force_tiny():
    X, W, Wq, c, A, B = case(3, 3, 16, 8, 2, outlier_cols=())
    o = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A, B)
    base = ml.mixed_int8_linear(X, Wq, c, 6.0)
    for m in range(3):
        t = [np.float16(sum(float(X[m, k]) * float(A[j, k]) for k in range(16))) for j in range(2)]
        assert [x.view(np.uint16) for x in t] == [x.view(np.uint16) for x in o["T"][m]]
        for n in range(8):
            y = base["Y64"][m, n] + sum(float(t[j]) * float(B[n, j]) for j in range(2))
            assert np.float16(y).view(np.uint16) == o["Y"][m, n].view(np.uint16)


def test_equals_the_adapted_weight_up_to_the_rounding_of_T():
    # y = W' x with W' = W + B A (here transposed: X [M, K], W [K, N]).  The low-rank part of the
    # oracle differs from X (B A)^T only by the fp16 rounding of T: at most 2^-11 relative per entry of T
    X, W, Wq, c, A, B = case(4, 12, 128, 40, 8)
    o = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A, B)
    BA = B.astype(np.float64) @ A.astype(np.float64)               # [N, K]
    exact = X.astype(np.float64) @ BA.T
    got = o["Y64"] - o["Y64_base"]
    T64 = X.astype(np.float64) @ A.astype(np.float64).T
    bound = 2.0 ** -11 * (np.abs(T64) @ np.abs(B.astype(np.float64)).T) + 1e-12
    assert np.all(np.abs(got - exact) <= bound)
    assert np.max(np.abs(exact)) > 0.01                            # the term is not negligible in this case
    # and the whole layer is the fp64 product with the adapted weight up to the int8 error of the base part
    full = X.astype(np.float64) @ (W.astype(np.float64) + BA.T)
    base_err = np.abs(o["Y64_base"] - X.astype(np.float64) @ W.astype(np.float64))
    assert np.all(np.abs(o["Y64"] - full) <= base_err + bound)


def test_additive_over_the_rank():
    X, W, Wq, c, A, B = case(5, 6, 64, 16, 6)
    whole = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A, B)
    first = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A[:2], np.ascontiguousarray(B[:, :2]))
    rest = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A[2:], np.ascontiguousarray(B[:, 2:]))
    s = first["Y64"] + rest["Y64"] - whole["Y64_base"]
    assert np.allclose(s, whole["Y64"], rtol=0, atol=1e-12)
    assert np.array_equal(np.concatenate([first["T"], rest["T"]], axis=1), whole["T"])


def test_row_sampling_matches_full_run():
    X, W, Wq, c, A, B = case(6, 20, 64, 16, 4)
    full = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A, B)
    rows = np.array([0, 7, 19])
    part = lora.mixed_int8_linear_lora(X, Wq, c, 6.0, A, B, rows=rows)
    assert np.array_equal(part["Y"].view(np.uint16), full["Y"][rows].view(np.uint16))
    assert np.array_equal(part["T"], full["T"][rows])
