"""mmd8_mixed_int8_linear_static: the layer for callers that cannot allocate.  Its workspace is the library's own
device array; everything else is the code of mmd8_mixed_int8_linear, so every output must equal that entry
point's bit for bit: on two calls in a row, the second with a smaller input (the array keeps the first call's
contents), across the three kernel paths (tiled, decode, single kernel), with taps, and interleaved with calls that
bring their own workspace.  Sizes beyond the array are refused."""
import numpy as np
import pytest
import torch

from oracle import mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


def problem(M, K, N, seed, heavy=False):
    rng = np.random.default_rng([M, K, N, seed])
    x = (rng.standard_t(3.0, size=(M, K)) if heavy else rng.standard_normal((M, K))).astype(np.float32)
    x[:, rng.integers(0, K, max(1, K // 200))] *= 20.0
    return wl.to_fp16(x), wl.gaussian_weight(K, N, 0.02, rng), wl.gaussian_bias(N, 0.3, rng)


def both(Xg, pw, bg, tau=wl.TAU):
    M, N = Xg.shape[0], pw.N
    Y_ref, t_ref = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, taps=True)
    Y = torch.full((M, N), 3.0, dtype=torch.float16, device="cuda")
    _, t = binding.mixed_int8_linear_static(Xg, pw, tau, Y, bias=bg, taps=True)
    Y2 = torch.full((M, N), 5.0, dtype=torch.float16, device="cuda")
    binding.mixed_int8_linear_static(Xg, pw, tau, Y2, bias=bg)                       # untapped
    torch.cuda.synchronize()
    assert torch.equal(Y, Y_ref) and torch.equal(Y2, Y_ref)
    for k in t_ref:
        if k == "outlier_idx":
            n = int(t_ref["n_outliers"].item())
            assert torch.equal(t[k][:n], t_ref[k][:n]), k
        else:
            assert torch.equal(t[k], t_ref[k]), k
    return Y


@pytest.mark.parametrize("big,small", [((300, 1040, 520), (130, 528, 264)), ((64, 4096, 4096), (5, 1040, 264)),
                                       ((2, 4096, 12288), (1, 272, 64)), ((520, 528, 1000), (2, 11008, 4096))])
def test_two_calls_in_a_row_the_second_smaller(big, small):
    outs = []
    for i, (M, K, N) in enumerate((big, small)):
        X, W, b = problem(M, K, N, i, heavy=(M <= 64))
        pw = binding.prequantize_weight(to_gpu(W))
        Y = both(to_gpu(X), pw, to_gpu(b))
        outs.append((X, W, b, Y))
    # and against the oracle, for the smaller one (the larger ones are covered by the other entry point's tests)
    X, W, b, Y = outs[1]
    Wq, c = ml.prequantize_weight(W)
    o = ml.mixed_int8_linear(X, Wq, c, wl.TAU, b)
    assert_y_close(to_np(Y), o["Y"])


def test_interleaved_with_calls_that_bring_their_own_workspace_and_thresholds():
    X, W, b = problem(200, 528, 512, 7)
    pw = binding.prequantize_weight(to_gpu(W))
    Xg, bg = to_gpu(X), to_gpu(b)
    ws = binding.linear_workspace(200, 528, 512, "cuda")
    ws3 = binding.linear_workspace(3, 528, 512, "cuda")           # (the decode path keeps other buffers)
    for tau in (wl.TAU, 0.0, float("inf"), 2.0):
        ref = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, workspace=ws)
        Y = torch.empty_like(ref)
        binding.mixed_int8_linear_static(Xg, pw, tau, Y, bias=bg)
        ref2 = binding.mixed_int8_linear(Xg[:3], pw, tau, bias=bg, workspace=ws3)
        Y2 = torch.empty_like(ref2)
        binding.mixed_int8_linear_static(Xg[:3], pw, tau, Y2, bias=bg)
        torch.cuda.synchronize()
        assert torch.equal(Y, ref) and torch.equal(Y2, ref2), tau


def test_sizes_beyond_the_array_are_refused_and_nothing_is_written():
    L = binding.lib()
    M, K, N = 2048, 28672, 8192
    assert L.mmd8_linear_workspace_bytes(M, K, N) > binding.STATIC_WORKSPACE_BYTES
    Xg = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    # refused before any pointer is used: a small stand-in for the 235 MB of weight codes is enough
    pw = binding.PackedWeight(torch.zeros(256, dtype=torch.int8, device="cuda"), torch.zeros(N, dtype=torch.float32, device="cuda"),
                              K, N)
    Y = torch.full((M, N), 9.0, dtype=torch.float16, device="cuda")
    with pytest.raises(binding.Mmd8Error, match="workspace"):
        binding.mixed_int8_linear_static(Xg, pw, wl.TAU, Y)
    torch.cuda.synchronize()
    assert bool((Y == 9.0).all())
    # the largest decode shapes of both model sizes fit
    for shp in list(wl.LLAMA_7B_LINEARS) + list(wl.LLAMA_70B_LINEARS):
        assert L.mmd8_linear_workspace_bytes(64, shp.K, shp.N) <= binding.STATIC_WORKSPACE_BYTES, shp
