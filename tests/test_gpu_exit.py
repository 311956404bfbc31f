"""The layer with its result leaving in blockwise-coded form (the shard's last linear) against the oracle.

The fp16 tensor that is encoded, H, is compared with the oracle's to the fp16 output bar.  The integer outputs
depend on H bit by bit (a code flips when H moves by one fp16 step across a decision threshold), so they are
checked in the precision the kernel took the decision in: the oracle's encoder applied to the H the GPU
produced must give the GPU's codes and scales exactly, the oracle's fp16 addition applied to the GPU's plain
layer output must give that H exactly, and H without a residual must be the plain entry point's output."""
import numpy as np
import pytest
import torch

from oracle import blockwise_codec as bc
from oracle import boundary_exit as be
from oracle import mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


def make_case(M, K, N, seed, heavy=False, bias=True, residual=True):
    rng = np.random.default_rng([M, K, N, seed])
    x = (rng.standard_t(3.0, size=(M, K)) if heavy else rng.standard_normal((M, K))).astype(np.float32)
    x[:, rng.integers(0, K, max(1, K // 200))] *= 20.0
    X = wl.to_fp16(x)
    W = wl.gaussian_weight(K, N, 0.02, rng)
    b = wl.gaussian_bias(N, 0.3, rng) if bias else None
    R = wl.to_fp16(rng.standard_t(3.0, size=(M, N)).astype(np.float32)) if residual else None
    return X, W, b, R


def run_and_check(X, W, b, R, block, tau=wl.TAU, want_h=True, taps=False, pad_r=0, tuning=0):
    M, K = X.shape
    N = W.shape[1]
    pw = binding.prequantize_weight(to_gpu(W))
    Wq_o, c_o = ml.prequantize_weight(W)
    Xg = to_gpu(X)
    bg = to_gpu(b) if b is not None else None
    Rg = None
    if R is not None:
        rbuf = torch.zeros((M, N + pad_r), dtype=torch.float16, device="cuda")
        Rg = rbuf[:, :N]
        Rg.copy_(to_gpu(R))
    Hg = torch.full((M, N), 7.0, dtype=torch.float16, device="cuda") if want_h else None
    n = M * N
    nb = (n + block - 1) // block
    codes = torch.full((n + 16,), 0xAB, dtype=torch.uint8, device="cuda")
    absmax = torch.full((nb + 4,), -1.0, dtype=torch.float32, device="cuda")
    out = binding.mixed_int8_linear_to_codes(Xg, pw, tau, block, bias=bg, residual=Rg, codes=codes, absmax=absmax,
                                             H=Hg, taps=taps, tuning=tuning)
    Y_plain = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, tuning=tuning)
    torch.cuda.synchronize()
    o = be.mixed_int8_linear_to_codes(X, Wq_o, c_o, tau, block, bias=b, residual=R)
    codes_g, absmax_g = to_np(codes), to_np(absmax)
    assert np.all(codes_g[n:] == 0xAB) and np.all(absmax_g[nb:] == -1.0), "wrote past the outputs"
    # the tensor that was encoded, as the kernel's own precision fixes it
    H_expect = to_np(Y_plain) if R is None else be.add_residual(to_np(Y_plain), R)
    if want_h:
        assert np.array_equal(to_np(Hg).view(np.uint16), H_expect.view(np.uint16)), "H"
    assert_y_close(H_expect, o["H"])
    codes_e, absmax_e = bc.quantize_blockwise(H_expect.reshape(-1), block)
    assert np.array_equal(absmax_g[:nb].view(np.uint32), absmax_e.view(np.uint32)), "block absmax"
    bad = np.flatnonzero(codes_g[:n] != codes_e)
    assert bad.size == 0, ("codes", bad[:8], codes_g[bad[:8]], codes_e[bad[:8]])
    # and against the oracle's own codes: they may differ only where H differs
    same_h = H_expect.reshape(-1).view(np.uint16) == o["H"].reshape(-1).view(np.uint16)
    blocks_same = np.add.reduceat(~same_h, np.arange(0, n, block)) == 0
    el_ok = np.repeat(blocks_same, block)[:n]
    assert np.array_equal(codes_g[:n][el_ok], o["codes"][el_ok])
    if taps:
        t = out[2]
        assert np.array_equal(to_np(t["outlier_mask"]).astype(bool), o["flag"])
        assert np.array_equal(to_np(t["xq"]), o["Xq"])
        assert np.array_equal(to_np(t["acc"]), o["acc"])
    return float(np.mean(el_ok))


# more than 128 rows: the tiled GEMM encodes in its epilogue when the block is 64, 128 or 256 and divides N
@pytest.mark.parametrize("M,K,N,block", [(300, 528, 512, 256), (300, 528, 512, 64), (257, 272, 384, 128),
                                         (256, 1024, 512, 256), (512, 512, 1024, 128), (130, 64, 64, 64),
                                         (700, 2048, 2304, 256), (300, 528, 768, 256)])
@pytest.mark.parametrize("residual", [True, False])
def test_tiled_path_encodes_in_the_epilogue(M, K, N, block, residual):
    X, W, b, R = make_case(M, K, N, block, residual=residual)
    run_and_check(X, W, b, R, block, want_h=(M + N) % 3 != 0, pad_r=8 if M % 2 else 0)


# the same shapes where a block would be shared between tiles, or does not divide N: the encoder runs afterwards
@pytest.mark.parametrize("M,K,N,block", [(300, 528, 1024, 1024), (300, 528, 520, 64), (200, 272, 512, 4096),
                                         (129, 64, 72, 192)])
def test_tiled_path_with_the_encoder_after_it(M, K, N, block):
    X, W, b, R = make_case(M, K, N, block)
    run_and_check(X, W, b, R, block, want_h=True)
    run_and_check(X, W, None, None, block, want_h=False)
    run_and_check(X, W, b, R, block, want_h=False)


# up to 128 rows: the kernel that sums the split-K partial outputs encodes, any block size
@pytest.mark.parametrize("M,K,N,block", [(1, 4096, 4096, 1024), (1, 512, 520, 64), (5, 1040, 264, 192), (64, 528, 264, 4096),
                                         (33, 512, 1024, 256), (8, 2048, 512, 2048), (65, 528, 512, 256), (128, 512, 520, 64),
                                         (100, 528, 264, 128), (2, 64, 8, 64)])
@pytest.mark.parametrize("residual", [True, False])
def test_decode_path_encodes_where_it_sums(M, K, N, block, residual):
    X, W, b, R = make_case(M, K, N, block, heavy=bool(M % 2), residual=residual)
    run_and_check(X, W, b, R, block, want_h=N % 3 != 0, pad_r=16 if M % 2 else 0)


# 65 to 128 rows whose second pass of 64 rows does not start on a block boundary: encoder afterwards
@pytest.mark.parametrize("M,K,N,block", [(100, 528, 520, 4096), (128, 64, 72, 1024)])
def test_decode_path_with_the_encoder_after_it(M, K, N, block):
    X, W, b, R = make_case(M, K, N, block)
    run_and_check(X, W, b, R, block, want_h=True)
    run_and_check(X, W, b, R, block, want_h=False)


def test_taps_and_thresholds():
    for (M, K, N, block, tau) in [(300, 528, 512, 256, 0.0), (300, 528, 512, 128, np.inf), (260, 272, 256, 64, 2.0),
                                  (40, 528, 264, 256, 0.0), (90, 272, 256, 64, np.inf)]:
        X, W, b, R = make_case(M, K, N, block, heavy=True)
        run_and_check(X, W, b, R, block, tau=tau, taps=True)


def test_every_tile_configuration_encodes_alike():
    X, W, b, R = make_case(300, 272, 768, 1)
    for variant in range(6):
        for block in (64, 256):
            run_and_check(X, W, b, R, block, want_h=bool(variant % 2), tuning=binding.tune_gemm_tiles(variant))


def test_zero_rows_and_blocks_take_the_zero_code():
    # an all-zero hidden state: every absmax is 0 and every code is the code of 0 (127)
    M, K, N, block = 260, 64, 256, 128
    X = np.zeros((M, K), np.float16)
    W = wl.gaussian_weight(K, N, 0.02, np.random.default_rng(0))
    pw = binding.prequantize_weight(to_gpu(W))
    codes, absmax = binding.mixed_int8_linear_to_codes(to_gpu(X), pw, wl.TAU, block)
    torch.cuda.synchronize()
    assert torch.all(codes == 127) and torch.all(absmax == 0)


def test_one_workspace_serves_plain_and_coded_calls():
    M, K, N, block = 300, 528, 512, 1024          # the larger workspace (encoder after the layer, H not wanted)
    X, W, b, R = make_case(M, K, N, 9)
    pw = binding.prequantize_weight(to_gpu(W))
    ws = binding.linear_workspace(M, K, N, torch.device("cuda:0"), exit_block=block)
    Xg, Rg = to_gpu(X), to_gpu(R)
    Y1 = binding.mixed_int8_linear(Xg, pw, wl.TAU, workspace=ws)
    c1, a1 = binding.mixed_int8_linear_to_codes(Xg, pw, wl.TAU, block, residual=Rg, workspace=ws)
    Y2 = binding.mixed_int8_linear(Xg, pw, wl.TAU, workspace=ws)
    c2, a2 = binding.mixed_int8_linear_to_codes(Xg, pw, wl.TAU, block, residual=Rg, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Y1, Y2) and torch.equal(c1, c2) and torch.equal(a1, a2)
    H = be.add_residual(to_np(Y1), R)
    ce, ae = bc.quantize_blockwise(H.reshape(-1), block)
    assert np.array_equal(to_np(c1), ce) and np.array_equal(to_np(a1), ae)


def test_last_linear_of_the_shard_at_full_size():
    """The down-projection of the Llama-7B-shaped shard (2048 tokens, 11008 -> 4096) with a residual, blocks of
    256: sampled rows against the oracle (a block lies inside one row), every row against the plain call."""
    M, K, N, block = 2048, 11008, 4096, 256
    rng = np.random.default_rng(5)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.choice(K, 6, replace=False)] *= rng.uniform(8.0, 60.0, 6).astype(np.float32)
    X = wl.to_fp16(x)
    W = wl.gaussian_weight(K, N, 0.02, rng)
    R = wl.to_fp16(rng.standard_normal((M, N)).astype(np.float32))
    pw = binding.prequantize_weight(to_gpu(W))
    Xg, Rg = to_gpu(X), to_gpu(R)
    Hg = torch.empty((M, N), dtype=torch.float16, device="cuda")
    codes, absmax = binding.mixed_int8_linear_to_codes(Xg, pw, wl.TAU, block, residual=Rg, H=Hg)
    Y = binding.mixed_int8_linear(Xg, pw, wl.TAU)
    c2, a2 = binding.quantize_blockwise(Hg.view(-1), block)
    torch.cuda.synchronize()
    assert torch.equal(Hg, Y + Rg)                                   # fp16 addition, every row
    assert torch.equal(codes, c2) and torch.equal(absmax, a2)        # the codec's own kernel on the same tensor
    rows = np.array([0, 1, 255, 256, 1023, 2047])
    Wq_o, c_o = ml.prequantize_weight(W)
    o = ml.mixed_int8_linear(X, Wq_o, c_o, wl.TAU, rows=rows)
    H_rows = to_np(Hg)[rows]
    assert_y_close(H_rows, be.add_residual(o["Y"], R[rows]))
    cg, ag = to_np(codes).reshape(M, N)[rows], to_np(absmax).reshape(M, N // block)[rows]
    for i in range(rows.size):
        ce, ae = bc.quantize_blockwise(H_rows[i], block)
        assert np.array_equal(cg[i], ce) and np.array_equal(ag[i].view(np.uint32), ae.view(np.uint32)), rows[i]
