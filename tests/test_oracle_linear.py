"""Pins for the mixed int8 linear oracle: hand-worked values, brute force, special cases, bounds."""
import numpy as np
import pytest

from oracle import mixed_linear as ml
from paper_2407_19775_amd import workloads as wl


def rand_case(seed, M, K, N, outlier_cols=(), scale=20.0):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    for k in outlier_cols:
        x[:, k] *= scale
    X = wl.to_fp16(x)
    W = wl.to_fp16(rng.standard_normal((K, N)).astype(np.float32) * 0.02)
    return X, W


def test_worked_example(golden):
    g = golden("mixed_linear_worked_example.txt")
    X = g["X"].reshape(2, 4).astype(np.float16)
    W = g["W"].reshape(4, 2).astype(np.float16)
    o = ml.linear_from_fp16_weight(X, W, float(g["tau"][0]))
    assert np.array_equal(o["flag"], g["flag"].astype(bool))
    assert np.array_equal(o["outlier_idx"], [2])
    assert np.array_equal(o["r"], g["r"].astype(np.float32))
    assert np.array_equal(o["Xq"], g["Xq"].reshape(2, 4).astype(np.int8))
    assert np.array_equal(o["c"], g["c"].astype(np.float32))
    assert np.array_equal(o["Wq"], g["Wq"].reshape(4, 2).astype(np.int8))
    assert np.array_equal(o["acc"], g["acc"].reshape(2, 2).astype(np.int32))
    wt = ml.dequantized_weight_fp16(o["Wq"], o["c"])[2]
    assert np.array_equal(wt, g["Wt_row2"].astype(np.float32).astype(np.float16))
    # printed to 4 significant digits
    assert np.allclose(o["Y"].astype(np.float64).reshape(-1), g["Y"], rtol=2e-3)
    assert np.allclose(o["Y"].astype(np.float64).reshape(-1), g["Y_exact_fp16_gemm"], atol=1e-3)


def test_integer_gemm_equals_triple_loop():
    rng = np.random.default_rng(11)
    for (M, K, N) in [(1, 1, 1), (3, 16, 2), (7, 33, 5), (2, 64, 3)]:
        A = rng.integers(-127, 128, (M, K)).astype(np.int8)
        B = rng.integers(-127, 128, (K, N)).astype(np.int8)
        A[0, :] = 127
        B[:, 0] = -127                                     # extreme products
        ref = np.zeros((M, N), dtype=np.int64)
        for m in range(M):
            for n in range(N):
                s = 0
                for k in range(K):
                    s += int(A[m, k]) * int(B[k, n])
                ref[m, n] = s
        got = ml.int_gemm(A, B)
        assert got.dtype == np.int32 and np.array_equal(got, ref)


def test_int32_bound_is_tight():
    assert ml.INT32_SAFE_K == 133144
    assert ml.INT32_SAFE_K * 127 * 127 < 2 ** 31 <= (ml.INT32_SAFE_K + 1) * 127 * 127


def vectorwise_int8_linear(X, W):
    """Plain row-wise x column-wise absmax int8 product, written independently of the oracle."""
    x = X.astype(np.float64)
    w = W.astype(np.float64)
    r = np.abs(x).max(axis=1)
    c = np.abs(w).max(axis=0)
    xq = np.rint((X.astype(np.float32) * (np.float32(127) / r.astype(np.float32))[:, None]).astype(np.float64))
    wq = np.rint((W.astype(np.float32) * (np.float32(127) / c.astype(np.float32))[None, :]).astype(np.float64))
    acc = np.zeros((X.shape[0], W.shape[1]))
    for k in range(X.shape[1]):
        acc += np.outer(xq[:, k], wq[k, :])
    return acc, (acc * np.outer(r, c) / (127.0 * 127.0)).astype(np.float16)


@pytest.mark.parametrize("tau", [np.inf, 1000.0])
def test_no_outliers_reduces_to_vectorwise_int8(tau):
    X, W = rand_case(1, 9, 48, 13)
    o = ml.linear_from_fp16_weight(X, W, tau)
    assert not o["flag"].any() and o["outlier_idx"].size == 0
    assert np.array_equal(o["r"], np.abs(X.astype(np.float32)).max(axis=1))
    acc, Y = vectorwise_int8_linear(X, W)
    assert np.array_equal(o["acc"], acc.astype(np.int32))
    assert np.array_equal(o["Y"], Y)


def test_tau_zero_is_the_fp16_gemm():
    X, W = rand_case(2, 6, 40, 11)
    X[:, 5] = 0                                            # |0| >= 0 must still flag the column
    o = ml.linear_from_fp16_weight(X, W, 0.0)
    assert o["flag"].all() and not o["Xq"].any() and not o["acc"].any() and not o["r"].any()
    Wt = ml.dequantized_weight_fp16(o["Wq"], o["c"])
    ref = np.zeros((6, 11))
    for k in range(40):                                    # plain outer-product accumulation
        ref += np.outer(X[:, k].astype(np.float64), Wt[k, :].astype(np.float64))
    assert np.array_equal(o["Y"], ref.astype(np.float16))
    # against the ORIGINAL fp16 weights: each 8-bit weight is within half a step c/254 (plus the
    # fp16 rounding of the dequantized weight and of the output)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    bound = (o["c"].astype(np.float64)[None, :] / 254.0) * np.abs(X.astype(np.float64)).sum(axis=1)[:, None]
    slack = np.abs(exact) * 2.0 ** -10 + bound * 2.0 ** -9 + 1e-7
    assert np.all(np.abs(o["Y"].astype(np.float64) - exact) <= bound + slack)


def test_planted_outlier_dims_of_tiny_config():
    cfg = wl.config1()
    flag = ml.outlier_mask(cfg["X"], cfg["tau"])
    assert np.array_equal(np.flatnonzero(flag), cfg["planted"])
    r = ml.row_absmax(cfg["X"], cfg["tau"])
    assert np.all(r < 6.0) and np.all(r > 2.0)


def test_quantization_error_bound():
    X, W = rand_case(3, 12, 96, 17, outlier_cols=(4, 50))
    o = ml.linear_from_fp16_weight(X, W, 6.0)
    keep = ~o["flag"]
    assert o["flag"][[4, 50]].all()
    x = X.astype(np.float64)[:, keep]
    w = W.astype(np.float64)[keep, :]
    exact = x @ w
    r = o["r"].astype(np.float64)[:, None]
    c = o["c"].astype(np.float64)[None, :]
    Yi = o["acc"].astype(np.float64) * r * c / 16129.0
    # each code is within half a step of the scaled value: |x - r xq/127| <= r/254, same for w
    bound = (np.abs(x).sum(axis=1)[:, None] * c / 254.0 + np.abs(w).sum(axis=0)[None, :] * r / 254.0
             + x.shape[1] * r * c / 254.0 ** 2)
    assert np.all(np.abs(Yi - exact) <= bound * (1 + 1e-6))
    # and the whole layer tracks the fp16 GEMM closely on this well-conditioned case
    full = X.astype(np.float64) @ W.astype(np.float64)
    rel = np.linalg.norm(o["Y"].astype(np.float64) - full) / np.linalg.norm(full)
    assert rel < 2e-2
    assert np.abs(o["Xq"]).max() <= 127 and np.abs(o["Wq"]).max() == 127
    assert not o["Xq"][:, o["flag"]].any()


def test_row_scale_ignores_super_threshold_entries():
    X = np.array([[1.0, 7.0, -3.0, 0.0], [6.0, 5.9960938, 0.0, 0.0], [9.0, 9.0, 9.0, 9.0]], np.float16)
    assert np.array_equal(ml.outlier_mask(X, 6.0), [True, True, True, True])
    assert np.array_equal(ml.row_absmax(X, 6.0), np.array([3.0, 5.9960938, 0.0], np.float32))
    flag = np.array([False, True, False, False])
    xq = ml.quantize_activations(X, flag, ml.row_absmax(X, 6.0))
    assert np.array_equal(xq[2], [0, 0, 0, 0])             # zero scale -> zero codes
    assert np.array_equal(xq[0], [42, 0, -127, 0])         # 1*127/3 = 42.33 -> 42


def test_zero_row_and_zero_weight_column():
    X, W = rand_case(4, 5, 32, 6)
    X[2, :] = 0
    W[:, 3] = 0
    o = ml.linear_from_fp16_weight(X, W, 6.0)
    assert o["r"][2] == 0 and o["c"][3] == 0
    assert not o["Xq"][2].any() and not o["Wq"][:, 3].any()
    assert not o["Y"][2].any() and not o["Y"][:, 3].any()


def test_bias_is_added_before_the_single_rounding():
    X, W = rand_case(5, 4, 32, 8, outlier_cols=(3,))
    b = wl.to_fp16(np.linspace(-1, 1, 8).astype(np.float32))
    o0 = ml.linear_from_fp16_weight(X, W, 6.0)
    o1 = ml.linear_from_fp16_weight(X, W, 6.0, bias=b)
    assert np.array_equal(o1["Y"], (o0["Y64"] + b.astype(np.float64)[None, :]).astype(np.float16))
    exact = X.astype(np.float64) @ W.astype(np.float64) + b.astype(np.float64)[None, :]
    assert np.abs(o1["Y"].astype(np.float64) - exact).max() < 0.02     # |bias| reaches 1


def test_symmetries():
    X, W = rand_case(6, 8, 64, 10, outlier_cols=(9,))
    o = ml.linear_from_fp16_weight(X, W, 6.0)
    rng = np.random.default_rng(0)
    pm, pk = rng.permutation(8), rng.permutation(64)
    om = ml.linear_from_fp16_weight(X[pm], W, 6.0)
    for key in ("r", "Xq", "acc", "Y"):
        assert np.array_equal(om[key], o[key][pm])
    assert np.array_equal(om["flag"], o["flag"])
    ok = ml.linear_from_fp16_weight(np.ascontiguousarray(X[:, pk]), np.ascontiguousarray(W[pk, :]), 6.0)
    assert np.array_equal(ok["flag"], o["flag"][pk]) and np.array_equal(ok["acc"], o["acc"])
    assert np.allclose(ok["Y"].astype(np.float64), o["Y"].astype(np.float64), rtol=2e-3, atol=1e-4)
    # a power-of-two scaling of a row that stays sub-threshold scales r and leaves the codes alone
    Xs, Ws = rand_case(8, 8, 64, 10)
    os_ = ml.linear_from_fp16_weight(Xs, Ws, 6.0)
    assert not os_["flag"].any()
    X2 = Xs.copy()
    X2[1] = (Xs[1].astype(np.float32) * 0.25).astype(np.float16)
    assert np.array_equal(X2[1].astype(np.float32) * 4, Xs[1].astype(np.float32))   # exact scaling
    o2 = ml.linear_from_fp16_weight(X2, Ws, 6.0)
    assert o2["r"][1] == os_["r"][1] * 0.25
    assert np.array_equal(o2["Xq"], os_["Xq"]) and np.array_equal(o2["acc"], os_["acc"])
    # any split of K sums to the same integers
    a1 = ml.int_gemm(o["Xq"][:, :40], o["Wq"][:40]).astype(np.int64)
    a2 = ml.int_gemm(o["Xq"][:, 40:], o["Wq"][40:]).astype(np.int64)
    assert np.array_equal(a1 + a2, o["acc"])


def test_threshold_comparison_is_inclusive():
    X = np.array([[6.0, 5.9960938]], np.float16)
    assert np.array_equal(ml.outlier_mask(X, 6.0), [True, False])
    assert ml.row_absmax(X, 6.0)[0] == np.float32(5.9960938)


def test_row_sampling_matches_full_run():
    X, W = rand_case(9, 10, 48, 7, outlier_cols=(3,))
    full = ml.linear_from_fp16_weight(X, W, 6.0)
    rows = np.array([7, 0, 4])
    part = ml.linear_from_fp16_weight(X, W, 6.0, rows=rows)
    assert np.array_equal(part["flag"], full["flag"])
    for key in ("r", "Xq", "acc", "Y"):
        assert np.array_equal(part[key], full[key][rows])
