"""Seeded sweep over random problem shapes: every entry point of the layer (plain, coded input, adapter)
and the codec against the oracle, with row strides larger than the row, biases, thresholds from "every
column critical" to "none", and sizes that leave ragged tiles in every dimension."""
import numpy as np
import pytest
import torch

from oracle import blockwise_codec as bc
from oracle import lora, mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng([seed, 77])
    M = int(rng.choice([1, 2, 7, 31, 33, 64, 65, 100, 129, 257, 300, 390]))
    K = 16 * int(rng.integers(1, 140))
    N = 8 * int(rng.integers(1, 140))
    tau = float(rng.choice([0.0, 1.0, 3.0, 6.0, 6.0, 6.0, 40.0, np.inf]))
    heavy = bool(rng.integers(0, 2))
    x = (rng.standard_t(3.0, size=(M, K)) if heavy else rng.standard_normal((M, K))).astype(np.float32)
    for k in rng.choice(K, size=min(K, int(rng.integers(0, 6))), replace=False):
        x[:, k] *= rng.uniform(8.0, 60.0)
    if rng.integers(0, 4) == 0:
        x[int(rng.integers(0, M))] = 0.0                                   # a zero row: scale 0
    X = wl.to_fp16(x)
    W = wl.gaussian_weight(K, N, 0.02, rng)
    if rng.integers(0, 4) == 0:
        W[:, int(rng.integers(0, N))] = 0                                  # a zero weight column: scale 0
    bias = wl.gaussian_bias(N, 0.3, rng) if rng.integers(0, 2) else None
    mode = ["plain", "plain", "coded", "adapter"][int(rng.integers(0, 4))]
    pad_x = 8 * int(rng.integers(0, 3)) if mode != "coded" else 0          # coded input is contiguous
    pad_y = 8 * int(rng.integers(0, 3))
    return dict(M=M, K=K, N=N, tau=tau, X=X, W=W, bias=bias, mode=mode, pad_x=pad_x, pad_y=pad_y, rng=rng)


@pytest.mark.parametrize("seed", range(48))
def test_random_layer(seed):
    c = draw_case(seed)
    M, K, N, tau, X, W, bias = c["M"], c["K"], c["N"], c["tau"], c["X"], c["W"], c["bias"]
    pw = binding.prequantize_weight(to_gpu(W))
    Wq_o, c_o = ml.prequantize_weight(W)
    assert np.array_equal(to_np(binding.unpack_weight(pw)), Wq_o)
    assert np.array_equal(to_np(pw.col_absmax).view(np.uint32), c_o.view(np.uint32))
    xbuf = torch.zeros((M, K + c["pad_x"]), dtype=torch.float16, device="cuda")
    Xg = xbuf[:, :K]
    ybuf = torch.full((M, N + c["pad_y"]), 7.0, dtype=torch.float16, device="cuda")
    Yg = ybuf[:, :N]
    bg = to_gpu(bias) if bias is not None else None
    kw = {}
    if c["mode"] == "coded":
        block = int(c["rng"].choice([64, 256, 1024, 4096]))
        codes_o, absmax_o = bc.quantize_blockwise(X.reshape(-1), block)
        X = bc.dequantize_blockwise(codes_o, absmax_o, block).reshape(M, K)     # what the layer sees
        kw["coded"] = (to_gpu(codes_o), to_gpu(absmax_o), block)
    else:
        Xg.copy_(to_gpu(X))
    if c["mode"] == "adapter":
        r = int(c["rng"].choice([8, 16, 32, 40, 64]))
        A = wl.to_fp16(c["rng"].standard_normal((r, K)).astype(np.float32) * 0.05)
        B = wl.to_fp16(c["rng"].standard_normal((N, r)).astype(np.float32) * 0.05)
        kw["lora"] = (to_gpu(A), to_gpu(B))
        o = lora.mixed_int8_linear_lora(X, Wq_o, c_o, tau, A, B, bias)
    else:
        o = ml.mixed_int8_linear(X, Wq_o, c_o, tau, bias)
    _, taps = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, out=Yg, taps=True, **kw)
    torch.cuda.synchronize()
    if c["mode"] == "coded":
        assert np.array_equal(to_np(Xg).view(np.uint16), X.view(np.uint16)), "decoded activations"
    assert np.array_equal(to_np(taps["outlier_mask"]).astype(bool), o["flag"])
    n_o = int(to_np(taps["n_outliers"])[0])
    assert n_o == o["outlier_idx"].size
    assert np.array_equal(to_np(taps["outlier_idx"])[:n_o], o["outlier_idx"])
    assert np.array_equal(to_np(taps["row_absmax"]).view(np.uint32), o["r"].view(np.uint32))
    assert np.array_equal(to_np(taps["xq"]), o["Xq"])
    assert np.array_equal(to_np(taps["acc"]), o["acc"])
    assert_y_close(to_np(Yg), o["Y"])
    if c["pad_y"]:
        assert torch.all(ybuf[:, N:] == 7.0), "columns past N were written"
    # without the taps the library may take shortcuts (up to 8 rows the decode kernel prepares its own operands):
    # the output must not change by a bit
    y_tapped = Yg.clone()
    if c["mode"] == "coded":
        Xg.zero_()
    Yg.fill_(0)
    binding.mixed_int8_linear(Xg, pw, tau, bias=bg, out=Yg, **kw)
    torch.cuda.synchronize()
    assert torch.equal(Yg, y_tapped), "output differs without taps"


@pytest.mark.parametrize("seed", range(24))
def test_random_codec(seed):
    rng = np.random.default_rng([seed, 78])
    block = int(rng.choice([64, 128, 192, 256, 320, 1024, 2048, 4096, 4032]))
    n = int(rng.choice([1, 63, 64, 65, block - 1, block, block + 1, 5 * block + 17, 100003, 262144 + 8 * int(rng.integers(0, 9))]))
    x = rng.standard_t(3.0, size=n).astype(np.float32) * float(rng.choice([1e-4, 1.0, 300.0]))
    if rng.integers(0, 3) == 0:
        x[rng.integers(0, n, size=max(1, n // 50))] = 0.0
    if rng.integers(0, 3) == 0 and n > block:
        x[:block] = 0.0                                                    # an all-zero block
    x = wl.to_fp16(x)
    codes_o, absmax_o = bc.quantize_blockwise(x, block)
    codes_g, absmax_g = binding.quantize_blockwise(to_gpu(x), block)
    back_g = binding.dequantize_blockwise(codes_g, absmax_g, block)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(absmax_g).view(np.uint32), absmax_o.view(np.uint32))
    assert np.array_equal(to_np(codes_g), codes_o)
    assert np.array_equal(to_np(back_g).view(np.uint16), bc.dequantize_blockwise(codes_o, absmax_o, block).view(np.uint16))
