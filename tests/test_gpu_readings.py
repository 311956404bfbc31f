"""The layer under the other readings of the method (mmd8_mixed_int8_linear_readings): the row scale over the
non-critical columns only, and the 16-bit weights of the critical dimensions taken from the original fp16 matrix.
Against oracle/readings.py: mask, scales, codes and accumulators bit for bit, the output to the fp16 bar; the
library's own reading through the same entry point must reproduce the plain entry point bit for bit."""
import numpy as np
import pytest
import torch

from oracle import mixed_linear as ml
from oracle import readings as rd
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu

SCALES = {"sub_threshold": binding.ROW_SCALE_SUB_THRESHOLD, "non_critical": binding.ROW_SCALE_NON_CRITICAL}


def problem(M, K, N, seed, heavy=False, shared_column=True):
    rng = np.random.default_rng([M, K, N, seed])
    x = (rng.standard_t(3.0, size=(M, K)) if heavy else rng.standard_normal((M, K))).astype(np.float32)
    cols = rng.choice(K, max(2, K // 150), replace=False)
    x[:, cols] *= 25.0
    if shared_column and M > 2:
        # a critical column whose other rows stay just below the threshold: there the two row scales differ
        x[:, cols[0]] = 5.5 * np.sign(x[:, cols[0]] + 0.1)
        x[0, cols[0]] = 40.0
    W = wl.gaussian_weight(K, N, 0.02, rng)
    return wl.to_fp16(x), W, wl.gaussian_bias(N, 0.3, rng)


def check(X, W, b, tau, scale, master, expect_scales_differ=None):
    pw = binding.prequantize_weight(to_gpu(W))
    Wq, c = ml.prequantize_weight(W)
    Xg, bg = to_gpu(X), to_gpu(b)
    Wg = to_gpu(W) if master else None
    Y, taps = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, taps=True, readings=(SCALES[scale], Wg))
    Y2 = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, readings=(SCALES[scale], Wg))
    torch.cuda.synchronize()
    o = rd.mixed_int8_linear_with_row_scale(X, Wq, c, tau, scale, bias=b, master_W=W if master else None)
    assert torch.equal(Y, Y2), "tapped and untapped outputs differ"
    assert np.array_equal(to_np(taps["outlier_mask"]).astype(bool), o["flag"])
    assert np.array_equal(to_np(taps["row_absmax"]).view(np.uint32), o["r"].view(np.uint32)), "row scale"
    assert np.array_equal(to_np(taps["xq"]), o["Xq"]), "activation codes"
    assert np.array_equal(to_np(taps["acc"]), o["acc"]), "accumulators"
    assert_y_close(to_np(Y), o["Y"])
    if expect_scales_differ is not None:
        other = rd.row_scale(X, tau, "sub_threshold")
        assert bool(np.any(other != o["r"])) == expect_scales_differ
    return to_np(Y), o


@pytest.mark.parametrize("M,K,N", [(300, 1040, 520), (5, 528, 264), (64, 2048, 512), (100, 272, 1000), (1, 4096, 4096),
                                   (520, 4096, 768)])
@pytest.mark.parametrize("scale", ["sub_threshold", "non_critical"])
@pytest.mark.parametrize("master", [False, True])
def test_readings_against_the_oracle(M, K, N, scale, master):
    heavy = M in (5, 64)
    X, W, b = problem(M, K, N, 1, heavy=heavy)
    # (Gaussian rows: the planted column sits at 5.5 where the rest of a row stays below 5, so the two scales differ)
    check(X, W, b, wl.TAU, scale, master, expect_scales_differ=True if (scale == "non_critical" and M > 2 and not heavy) else None)


def test_the_librarys_own_reading_through_this_entry_point_is_the_plain_layer():
    for (M, K, N) in [(300, 1040, 520), (40, 528, 264), (2, 4096, 1024)]:
        X, W, b = problem(M, K, N, 2, heavy=(M == 40))
        pw = binding.prequantize_weight(to_gpu(W))
        Xg, bg = to_gpu(X), to_gpu(b)
        plain, t0 = binding.mixed_int8_linear(Xg, pw, wl.TAU, bias=bg, taps=True)
        same, t1 = binding.mixed_int8_linear(Xg, pw, wl.TAU, bias=bg, taps=True, readings=(binding.ROW_SCALE_SUB_THRESHOLD, None))
        torch.cuda.synchronize()
        for k in ("outlier_mask", "row_absmax", "xq", "acc", "n_outliers"):
            assert torch.equal(t0[k], t1[k]), k
        if M > 2:
            assert torch.equal(plain, same)              # (one or two rows: the plain call is the single kernel, whose
        else:                                            # 16-bit part is added in another order)
            assert_y_close(to_np(same), to_np(plain), rel=2e-3)


@pytest.mark.parametrize("M", [3, 200])
def test_master_rows_make_threshold_zero_the_fp16_product(M):
    K, N = 528, 264
    X, W, b = problem(M, K, N, 3, shared_column=False)
    Y, o = check(X, W, None if False else b, 0.0, "sub_threshold", True)
    exact = X.astype(np.float64) @ W.astype(np.float64) + b.astype(np.float64)[None, :]
    assert not o["acc"].any()
    assert_y_close(Y, exact.astype(np.float16), rel=2e-3)
    # with the re-created rows the same call is X times the dequantized weights: different numbers
    Y_codes, _ = check(X, W, b, 0.0, "sub_threshold", False)
    assert np.any(Y_codes != Y)


def test_many_critical_columns_and_thresholds():
    # more than the 32 critical columns that ride as a slab: the rest is gathered in the epilogue, from W as well
    X, W, b = problem(260, 1040, 520, 4, heavy=True)
    for tau in (2.5, np.inf):
        for master in (False, True):
            check(X, W, b, tau, "non_critical", master)
    assert int(ml.outlier_mask(X, 2.5).sum()) > 64


def test_llama7b_linear_at_full_size():
    shape = wl.LLAMA_7B_LINEARS[1]
    X, _ = wl.prefill_activation(2, 11, 2048, shape.K)
    W = wl.prefill_weight(2, 21, shape, 0.02)
    check(X, W, wl.gaussian_bias(shape.N, 0.1, np.random.default_rng(5)), wl.TAU, "non_critical", True)


def test_bad_arguments():
    X, W, b = problem(8, 128, 64, 5)
    pw = binding.prequantize_weight(to_gpu(W))
    Xg = to_gpu(X)
    with pytest.raises(binding.Mmd8Error):
        binding.mixed_int8_linear(Xg, pw, wl.TAU, readings=(7, None))
    Wg = torch.zeros((128, 72), dtype=torch.float16, device="cuda")[:, :64]      # ldw = 72: fine
    binding.mixed_int8_linear(Xg, pw, wl.TAU, readings=(0, Wg))
    Wbad = torch.zeros((128, 68), dtype=torch.float16, device="cuda")[:, :64]     # ldw % 8 != 0
    with pytest.raises(binding.Mmd8Error):
        binding.mixed_int8_linear(Xg, pw, wl.TAU, readings=(0, Wbad))
    torch.cuda.synchronize()
