"""The layer added onto a residual stream in its own kernels: bit for bit the oracle's fp16 addition applied to
the plain entry point's output, close to the oracle end to end, in place or into another buffer."""
import numpy as np
import pytest
import torch

from oracle import boundary_exit as be
from oracle import mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,K,N", [(1, 4096, 4096), (3, 528, 264), (8, 1040, 520), (33, 512, 1024), (64, 528, 72), (100, 272, 520),
                                   (128, 64, 8), (130, 64, 64), (300, 1040, 264), (512, 512, 1024), (2048, 4096, 4096)])
@pytest.mark.parametrize("in_place", [False, True])
def test_layer_plus_residual(M, K, N, in_place):
    rng = np.random.default_rng([M, K, N])
    x = rng.standard_t(3.0, size=(M, K)).astype(np.float32)
    x[:, rng.integers(0, K, max(1, K // 200))] *= 20.0
    X = wl.to_fp16(x)
    W = wl.gaussian_weight(K, N, 0.02, rng)
    b = wl.gaussian_bias(N, 0.3, rng)
    R = wl.to_fp16(rng.standard_t(3.0, size=(M, N)).astype(np.float32))
    pw = binding.prequantize_weight(to_gpu(W))
    Xg, bg = to_gpu(X), to_gpu(b)
    pad = 8 if M % 2 else 0
    rbuf = torch.zeros((M, N + pad), dtype=torch.float16, device="cuda")
    Rg = rbuf[:, :N]
    Rg.copy_(to_gpu(R))
    out = Rg if in_place else torch.full((M, N), 7.0, dtype=torch.float16, device="cuda")
    Y = binding.mixed_int8_linear(Xg, pw, wl.TAU, bias=bg)
    H = binding.mixed_int8_linear(Xg, pw, wl.TAU, bias=bg, residual=Rg, out=out)
    torch.cuda.synchronize()
    assert H.data_ptr() == out.data_ptr()
    want = be.add_residual(to_np(Y), R)
    assert np.array_equal(to_np(H).view(np.uint16), want.view(np.uint16))
    if pad:
        assert torch.all(rbuf[:, N:] == 0), "columns past N were written"
    if K * N <= 4096 * 1024:
        Wq_o, c_o = ml.prequantize_weight(W)
        o = ml.mixed_int8_linear(X, Wq_o, c_o, wl.TAU, b)
        assert_y_close(to_np(H), be.add_residual(o["Y"], R))
