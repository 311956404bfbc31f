"""GPU parity of the low-rank adapted layer (W' = W + B A on the int8 base) against the CPU oracle.

Bit-exact: everything the base layer pins (mask, index list, row absmax, codes, int32 accumulators).
T = f16(X A^T): the GPU sums in fp32 on the matrix cores, the oracle in float64, so an entry may land
on the neighbouring fp16 value: |delta| <= 2^-10 |T| + K 2^-24 sum_k |X| |A| (the fp32 accumulation bound).
Y: the 1e-2 relative bar of the base layer.
"""
import numpy as np
import pytest
import torch

from oracle import lora, mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


def check_lora(X, W, A, B, tau, bias=None, rows=None, tuning=0):
    pw = binding.prequantize_weight(to_gpu(W))
    Wq_o, c_o = ml.prequantize_weight(W)
    M, r = X.shape[0], A.shape[0]
    Xg, Ag, Bg = to_gpu(X), to_gpu(A), to_gpu(B)
    bg = to_gpu(bias) if bias is not None else None
    T = torch.full((M, r), float("nan"), dtype=torch.float16, device="cuda")
    Y, taps = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, taps=True, lora=(Ag, Bg, T), tuning=tuning)
    Y2 = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, lora=(Ag, Bg), tuning=tuning)   # untapped, no T output
    torch.cuda.synchronize()
    o = lora.mixed_int8_linear_lora(X, Wq_o, c_o, tau, A, B, bias, rows=rows)
    sel = slice(None) if rows is None else np.asarray(rows)
    assert np.array_equal(to_np(taps["outlier_mask"]).astype(bool), o["flag"]), "outlier mask"
    assert int(to_np(taps["n_outliers"])[0]) == o["outlier_idx"].size
    assert np.array_equal(to_np(taps["row_absmax"])[sel].view(np.uint32), o["r"].view(np.uint32)), "row absmax"
    assert np.array_equal(to_np(taps["xq"])[sel], o["Xq"]), "activation codes"
    assert np.array_equal(to_np(taps["acc"])[sel], o["acc"]), "int32 accumulators"
    Tg = to_np(T)[sel].astype(np.float64)
    To = o["T"].astype(np.float64)
    Xs = X[sel].astype(np.float64)
    slack = 2.0 ** -10 * np.abs(To) + X.shape[1] * 2.0 ** -24 * (np.abs(Xs) @ np.abs(A.astype(np.float64)).T) + 2.0 ** -24
    assert np.all(np.isfinite(Tg)) and np.all(np.abs(Tg - To) <= slack), ("T", float(np.max(np.abs(Tg - To) - slack)))
    Yg = to_np(Y)
    assert np.array_equal(Yg.view(np.uint16), to_np(Y2).view(np.uint16)), "tapped and untapped outputs differ"
    # the adapter's term must matter in the comparison: a layer that ignored it would fail the bar
    low = o["Y64"] - o["Y64_base"]
    assert np.linalg.norm(low) > 0.03 * np.linalg.norm(o["Y64"]), "adapter term too small to be tested"
    return assert_y_close(Yg[sel], o["Y"])


def rand_case(seed, M, K, N, r, outlier_cols=(3,), std=0.05):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    for k in outlier_cols:
        if k < K:
            x[:, k] *= 25.0
    A = wl.to_fp16(rng.standard_normal((r, K)).astype(np.float32) * std)
    B = wl.to_fp16(rng.standard_normal((N, r)).astype(np.float32) * std)
    return wl.to_fp16(x), wl.gaussian_weight(K, N, 0.02, rng), A, B


@pytest.mark.parametrize("M,K,N", [(1, 16, 8), (5, 144, 40), (77, 272, 264), (130, 1040, 520), (300, 512, 1000)])
@pytest.mark.parametrize("r", [8, 16, 24, 64])
def test_ragged_shapes_and_ranks(M, K, N, r):
    X, W, A, B = rand_case(M + r, M, K, N, r, outlier_cols=(3, 100))
    check_lora(X, W, A, B, 6.0)


@pytest.mark.parametrize("tau", [float("inf"), 0.0, 2.5])
@pytest.mark.parametrize("M", [40, 200])
def test_no_critical_column_and_many(tau, M):
    """tau = inf: the slab of critical columns is skipped and the adapter's slabs still run; tau = 2.5 and 0:
    hundreds of critical columns (gather loop, or every column in fp16) next to the adapter."""
    X, W, A, B = rand_case(17, M, 528, 264, 40)
    check_lora(X, W, A, B, tau, bias=wl.gaussian_bias(264, 0.5, np.random.default_rng(5)))


@pytest.mark.parametrize("variant", [4, 0, 5])
@pytest.mark.parametrize("n_crit,r", [(1, 64), (33, 16), (70, 40), (200, 8), (256, 64), (257, 24), (700, 16), (830, 40)])
def test_critical_column_slabs_next_to_the_adapter(n_crit, r, variant):
    """1 to 8 fp16 slabs of critical columns in use (the unused ones are skipped), then the adapter's one or two
    slabs behind them in the same ring; 257: one more column, in a ninth slab from the further ones."""
    M, K, N = 300, 1040, 520
    rng = np.random.default_rng([n_crit, r, variant])
    x = np.clip(rng.standard_normal((M, K)), -5.0, 5.0).astype(np.float32)
    cols = np.sort(rng.choice(K, n_crit, replace=False))
    for j, k in enumerate(cols):
        x[(11 * j) % M, k] = (-1.0) ** j * (7.0 + j % 40)
    X = wl.to_fp16(x)
    assert np.array_equal(np.flatnonzero(ml.outlier_mask(X, 6.0)), cols)
    A = wl.to_fp16(rng.standard_normal((r, K)).astype(np.float32) * 0.05)
    B = wl.to_fp16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    check_lora(X, wl.gaussian_weight(K, N, 0.02, rng), A, B, 6.0, tuning=binding.tune_gemm_tiles(variant))


@pytest.mark.parametrize("variant", [4, 2])
def test_dense_pass_next_to_the_adapter(variant):
    """1600 of 2096 columns critical: no slab of critical columns, the adapter's slab, then the second, fp16 pass
    over K."""
    M, K, N, n_crit, r = 300, 2096, 264, 1600, 16
    rng = np.random.default_rng([n_crit, r, variant, 3])
    x = np.clip(rng.standard_normal((M, K)), -5.0, 5.0).astype(np.float32)
    cols = np.sort(rng.choice(K, n_crit, replace=False))
    for j, k in enumerate(cols):
        x[(11 * j) % M, k] = (-1.0) ** j * (7.0 + j % 40)
    X = wl.to_fp16(x)
    assert np.array_equal(np.flatnonzero(ml.outlier_mask(X, 6.0)), cols)
    A = wl.to_fp16(rng.standard_normal((r, K)).astype(np.float32) * 0.05)
    B = wl.to_fp16(rng.standard_normal((N, r)).astype(np.float32) * 0.05)
    check_lora(X, wl.gaussian_weight(K, N, 0.02, rng), A, B, 6.0, tuning=binding.tune_gemm_tiles(variant))


@pytest.mark.parametrize("M", [1, 64])
@pytest.mark.parametrize("shape", wl.LLAMA_7B_LINEARS, ids=lambda s: s.name)
def test_decode_shapes(M, shape):
    X = wl.decode_activation(10 * M + shape.K % 7, M, shape.K)
    W = wl.prefill_weight(3, 100 + shape.K % 7, shape, 0.02)
    A, B = wl.adapter_factors(3, 200 + shape.K % 7, shape.K, shape.N, 16, 0.03)
    check_lora(X, W, A, B, wl.TAU)


@pytest.mark.parametrize("shape", wl.LLAMA_7B_LINEARS, ids=lambda s: s.name)
def test_prefill_full_size(shape):
    """The 2048-token launches with a rank-16 adapter, compared in full."""
    X, _ = wl.prefill_activation(2, 10 + shape.K % 5, 2048, shape.K)
    W = wl.prefill_weight(2, 20 + wl.LLAMA_7B_LINEARS.index(shape), shape, 0.02)
    A, B = wl.adapter_factors(2, 40 + wl.LLAMA_7B_LINEARS.index(shape), shape.K, shape.N, 16, 0.03)
    check_lora(X, W, A, B, wl.TAU)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5])
def test_every_gemm_tile_configuration(variant):
    tune = binding.tune_gemm_tiles(variant)
    X, W, A, B = rand_case(variant, 300, 1040, 520, 64, outlier_cols=(3, 777))
    check_lora(X, W, A, B, 6.0, tuning=tune)
    X, W, A, B = rand_case(variant + 50, 512, 1024, 512, 32)     # full tiles: the unchecked store path
    check_lora(X, W, A, B, 6.0, tuning=tune)


def test_one_workspace_with_and_without_the_adapter():
    """A workspace sized for the adapter serves plain calls too, in any order, and a zero B gives the plain layer."""
    X, W, A, B = rand_case(9, 300, 512, 264, 16)
    pw = binding.prequantize_weight(to_gpu(W))
    ws = binding.linear_workspace(300, 512, 264, "cuda", lora_rank=16)
    Xg, Ag, Bg = to_gpu(X), to_gpu(A), to_gpu(B)
    plain = binding.mixed_int8_linear(Xg, pw, 6.0, workspace=ws)
    with_a = binding.mixed_int8_linear(Xg, pw, 6.0, workspace=ws, lora=(Ag, Bg))
    plain2 = binding.mixed_int8_linear(Xg, pw, 6.0, workspace=ws)
    zero_b = binding.mixed_int8_linear(Xg, pw, 6.0, workspace=ws, lora=(Ag, torch.zeros_like(Bg)))
    small = binding.mixed_int8_linear(Xg[:7], pw, 6.0, workspace=ws, lora=(Ag, Bg))     # decode path, same workspace
    torch.cuda.synchronize()
    assert torch.equal(plain, plain2)
    assert torch.equal(plain, zero_b)
    assert not torch.equal(plain, with_a)
    Wq_o, c_o = ml.prequantize_weight(W)
    o = lora.mixed_int8_linear_lora(X[:7], Wq_o, c_o, 6.0, A, B)
    assert_y_close(to_np(small), o["Y"])
