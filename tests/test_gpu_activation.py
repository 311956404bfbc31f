"""The int8 layer followed by GELU in the same kernels, against the oracle: integers as in the plain layer
(taps), the activated output to the fp16 bar, and bit for bit against the oracle's activation applied to the
plain entry point's own output wherever the fp32 evaluation rounds like the float64 one (it must in all but a
few elements, and never differ by more than one fp16 step)."""
import numpy as np
import pytest
import torch

from oracle import activation as act
from oracle import mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


def ulp_distance(a, b):
    """distance in fp16 steps between two fp16 arrays (sign-magnitude patterns mapped to a line)"""
    def line(x):
        u = x.view(np.uint16).astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    return np.abs(line(a) - line(b))


@pytest.mark.parametrize("M,K,N", [(1, 1024, 4096), (7, 528, 264), (64, 768, 3072), (100, 272, 520), (128, 64, 8),
                                   (197, 768, 3072), (300, 1040, 264), (1576, 1024, 4096), (130, 64, 64)])
@pytest.mark.parametrize("tau", [wl.TAU, np.inf])
def test_layer_with_gelu(M, K, N, tau):
    rng = np.random.default_rng([M, K, N])
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.integers(0, K, max(1, K // 200))] *= 20.0
    X = wl.to_fp16(x)
    W = wl.gaussian_weight(K, N, 0.05, rng)
    bias = wl.gaussian_bias(N, 0.5, rng)
    pw = binding.prequantize_weight(to_gpu(W))
    Wq_o, c_o = ml.prequantize_weight(W)
    Xg, bg = to_gpu(X), to_gpu(bias)
    ybuf = torch.full((M, N + 8), 7.0, dtype=torch.float16, device="cuda")
    G, taps = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, out=ybuf[:, :N], taps=True, gelu=True)
    Y = binding.mixed_int8_linear(Xg, pw, tau, bias=bg)
    torch.cuda.synchronize()
    o = act.mixed_int8_linear_gelu(X, Wq_o, c_o, tau, bias)
    assert np.array_equal(to_np(taps["outlier_mask"]).astype(bool), o["flag"])
    assert np.array_equal(to_np(taps["xq"]), o["Xq"])
    assert np.array_equal(to_np(taps["acc"]), o["acc"])
    assert_y_close(to_np(G), o["G"])
    assert torch.all(ybuf[:, N:] == 7.0), "columns past N were written"
    # the activation itself, on the layer output the GPU produced
    want = act.gelu_fp16(to_np(Y))
    d = ulp_distance(to_np(G), want)
    assert d.max() <= 1, ("fp16 steps", int(d.max()))
    assert np.mean(d > 0) < 0.01
    # the activation did something, and the test data reaches both tails
    yv = to_np(Y).astype(np.float32)
    assert yv.min() < -2 and yv.max() > 2 and not np.array_equal(to_np(G), to_np(Y))


@pytest.mark.parametrize("M", [3, 130])
def test_gelu_of_every_fp16_value(M):
    """Zero weights and a bias that holds every finite fp16 value: the layer returns the bias exactly, so the
    activation is checked on every input it can see, on the decode path and in the tiled GEMM's epilogue."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bits.view(np.float16)
    vals = vals[np.isfinite(vals)]
    N = (vals.size + 7) // 8 * 8
    bias = np.zeros(N, np.float16)
    bias[:vals.size] = vals
    K = 64
    pw = binding.prequantize_weight(to_gpu(np.zeros((K, N), np.float16)))
    X = wl.to_fp16(np.random.default_rng(M).standard_normal((M, K)).astype(np.float32))
    Xg, bg = to_gpu(X), to_gpu(bias)
    G = binding.mixed_int8_linear(Xg, pw, wl.TAU, bias=bg, gelu=True)
    Y = binding.mixed_int8_linear(Xg, pw, wl.TAU, bias=bg)
    torch.cuda.synchronize()
    assert ulp_distance(to_np(Y), np.ascontiguousarray(np.broadcast_to(bias, (M, N)))).max() == 0   # (-0 comes back as +0)
    want = act.gelu_fp16(to_np(Y))
    d = ulp_distance(to_np(G), want)
    assert d.max() <= 1, int(d.max())
    assert np.mean(d > 0) < 0.01
