"""Pins for the oracle of the shard's exit (last linear, residual, blockwise encoding): cases whose result is
fixed by hand-worked values of the codec, by the fp16 grid, or by the codec's error bound."""
import numpy as np

from oracle import blockwise_codec as bc
from oracle import boundary_exit as be
from oracle import dynamic_code as dc
from oracle import mixed_linear as ml
from paper_2407_19775_amd import workloads as wl


def test_zero_weight_passes_the_residual_and_blocks_run_row_by_row(golden):
    # W = 0: the layer contributes nothing, H is the residual.  The residual is the codec's hand-worked
    # example laid out as [4, 2] with 4-element blocks, so a block holds two rows: the codes and scales of
    # that example must come out, in its order.
    g = golden("codec_worked_example.txt")
    R = g["x"].astype(np.float16).reshape(4, 2)
    rng = np.random.default_rng(0)
    X = wl.to_fp16(rng.standard_normal((4, 16)).astype(np.float32))
    Wq, c = ml.prequantize_weight(np.zeros((16, 2), np.float16))
    o = be.mixed_int8_linear_to_codes(X, Wq, c, 6.0, int(g["block"][0]), residual=R)
    assert np.array_equal(o["H"], R)
    assert np.array_equal(o["codes"], g["codes"].astype(np.uint8))
    assert np.array_equal(o["absmax"], g["absmax"].astype(np.float32))
    # and the transposed layout gives other blocks: flattening is by rows, not by columns
    Rt = np.ascontiguousarray(R.T)
    Wq2, c2 = ml.prequantize_weight(np.zeros((16, 4), np.float16))
    o2 = be.mixed_int8_linear_to_codes(X[:2], Wq2, c2, 6.0, 4, residual=Rt)
    assert not np.array_equal(o2["codes"], o["codes"])
    assert np.array_equal(o2["absmax"], np.array([3.0, 3.0], np.float32))


def test_residual_sum_is_rounded_to_the_nearest_even_fp16():
    # One-hot rows make the layer exact: with column maximum 2540 = 127 * 20 the weight codes are W / 20 and a
    # row that is 1 at feature k returns W[k, :] itself.  Above 2048 the fp16 grid has spacing 2, so an odd
    # sum is a tie: 2060 + 1 -> 2060 (mantissa 1030 even), 2540 + 3 -> 2544 (1272 even), 2060 + 3 -> 2064.
    W = np.zeros((16, 2), np.float16)
    W[0] = [2060.0, 2540.0]
    W[1] = [2540.0, 2060.0]
    Wq, c = ml.prequantize_weight(W)
    assert np.array_equal(c, np.array([2540.0, 2540.0], np.float32)) and Wq[0, 0] == 103 and Wq[0, 1] == 127
    X = np.zeros((2, 16), np.float16)
    X[0, 0] = 1.0
    X[1, 1] = 1.0
    R = np.array([[1.0, 3.0], [-3.0, 3.0]], np.float16)
    o = be.mixed_int8_linear_to_codes(X, Wq, c, np.inf, 4, residual=R)
    assert np.array_equal(o["Y"], W[:2])
    assert np.array_equal(o["H"], np.array([[2060.0, 2544.0], [2536.0, 2064.0]], np.float16))
    assert np.array_equal(o["absmax"], np.array([2544.0], np.float32))
    # the block maximum takes the +1.0 code; 2060 / 2544 = 0.8097.. lies in the top bracket (step 0.9 / 64)
    T = dc.code_table().astype(np.float64)
    want = [int(np.argmin(np.abs(T - v / 2544.0))) for v in (2060.0, 2544.0, 2536.0, 2064.0)]
    assert want[1] == 255 and np.array_equal(o["codes"], np.array(want, np.uint8))


def test_without_residual_the_codes_describe_the_layer_output_within_the_codec_bound():
    rng = np.random.default_rng(3)
    M, K, N, block = 12, 64, 40, 64
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, 5] *= 20.0
    X = wl.to_fp16(x)
    Wq, c = ml.prequantize_weight(wl.to_fp16(rng.standard_normal((K, N)).astype(np.float32) * 0.05))
    bias = wl.to_fp16(rng.standard_normal(N).astype(np.float32))
    o = be.mixed_int8_linear_to_codes(X, Wq, c, 6.0, block, bias=bias)
    base = ml.mixed_int8_linear(X, Wq, c, 6.0, bias)
    assert o["H"] is o["Y"] and np.array_equal(o["Y"].view(np.uint16), base["Y"].view(np.uint16))
    n = M * N
    assert o["codes"].shape == (n,) and o["absmax"].shape == ((n + block - 1) // block,)
    flat = o["H"].reshape(-1).astype(np.float64)
    # absmax is the largest magnitude of each run of `block` consecutive elements of the row-major tensor
    for b in range(o["absmax"].size):
        assert o["absmax"][b] == np.abs(flat[b * block:(b + 1) * block]).max()
    # decoding returns every element to within half the table's largest gap times the block's absmax
    # (plus the fp16 rounding of the decoded value, at most 2^-11 of the block's absmax)
    back = bc.dequantize_blockwise(o["codes"], o["absmax"], block).astype(np.float64)
    half_gap = np.diff(dc.code_table().astype(np.float64)).max() / 2
    a_el = np.repeat(o["absmax"].astype(np.float64), block)[:n]
    assert np.all(np.abs(back - flat) <= a_el * (half_gap + 2.0 ** -11) + 2.0 ** -24)
    # and with a residual the encoded tensor moves by it: H - Y = R up to one fp16 rounding of H
    R = wl.to_fp16(rng.standard_normal((M, N)).astype(np.float32) * 3.0)
    o2 = be.mixed_int8_linear_to_codes(X, Wq, c, 6.0, block, bias=bias, residual=R)
    exact = o["Y"].astype(np.float64) + R.astype(np.float64)
    assert np.all(np.abs(o2["H"].astype(np.float64) - exact) <= np.abs(exact) * 2.0 ** -11 + 2.0 ** -25)
    assert not np.array_equal(o2["codes"], o["codes"])
