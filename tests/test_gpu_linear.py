"""GPU parity of the mixed int8 linear layer against the CPU oracle.

Bit-exact: outlier mask and index list, row absmax, activation codes, weight codes and scales,
int32 accumulators.  Tolerance (fp16 output): 1e-2 relative, see gpu_util.assert_y_close.
"""
import numpy as np
import pytest
import torch

from oracle import mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import critical_column_plan, assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


def check_weight(W: np.ndarray):
    pw = binding.prequantize_weight(to_gpu(W))
    Wq_o, c_o = ml.prequantize_weight(W)
    assert np.array_equal(to_np(pw.col_absmax).view(np.uint32), c_o.view(np.uint32)), "column absmax"
    Wq_g = to_np(binding.unpack_weight(pw))
    bad = np.argwhere(Wq_g != Wq_o)
    assert bad.shape[0] == 0, ("weight codes", bad[:5])
    return pw, Wq_o, c_o


def check_linear(X, W, tau, bias=None, rows=None, pw_pack=None, tuning=0, row_chunks=None):
    """Runs the layer on the GPU with all taps and compares with the oracle: every row, or the rows of `rows`,
    or chunk after chunk of `row_chunks` (a list of index arrays: full-size problems whose float64 oracle would
    not fit in memory at once).  Mask and index list are always compared in full."""
    pw, Wq_o, c_o = pw_pack if pw_pack is not None else check_weight(W)
    Xg = to_gpu(X)
    bg = to_gpu(bias) if bias is not None else None
    Y, taps = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, taps=True, tuning=tuning)
    Y2 = binding.mixed_int8_linear(Xg, pw, tau, bias=bg, tuning=tuning)   # the untapped path
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2), "tapped and untapped outputs differ"
    del Y2
    Yg = to_np(Y)
    n_o = int(to_np(taps["n_outliers"])[0])
    worst = (0.0, 0.0)
    for rows in (row_chunks if row_chunks is not None else [rows]):
        o = ml.mixed_int8_linear(X, Wq_o, c_o, tau, bias, rows=rows)
        sel = slice(None) if rows is None else torch.from_numpy(np.asarray(rows)).cuda()
        sel_np = slice(None) if rows is None else np.asarray(rows)
        assert np.array_equal(to_np(taps["outlier_mask"]).astype(bool), o["flag"]), "outlier mask"
        assert n_o == o["outlier_idx"].size
        assert np.array_equal(to_np(taps["outlier_idx"])[:n_o], o["outlier_idx"]), "outlier index list"
        assert np.array_equal(to_np(taps["row_absmax"][sel]).view(np.uint32), o["r"].view(np.uint32)), "row absmax"
        assert np.array_equal(to_np(taps["xq"][sel]), o["Xq"]), "activation codes"
        bad = np.argwhere(to_np(taps["acc"][sel]) != o["acc"])
        assert bad.shape[0] == 0, ("int32 accumulators", bad[:5])
        fro, w = assert_y_close(Yg[sel_np], o["Y"])
        worst = (max(worst[0], fro), max(worst[1], w))
        del o
    return worst


def test_config1_tiny():
    cfg = wl.config1()
    check_linear(cfg["X"], cfg["W"], cfg["tau"])
    mask = ml.outlier_mask(cfg["X"], cfg["tau"])
    assert np.array_equal(np.flatnonzero(mask), cfg["planted"])


@pytest.mark.parametrize("M,K,N", [(1, 16, 8), (5, 144, 40), (77, 272, 264), (130, 1040, 520), (300, 512, 1000)])
@pytest.mark.parametrize("tau", [6.0, float("inf"), 0.0, 2.5])
def test_ragged_shapes_and_thresholds(M, K, N, tau):
    rng = np.random.default_rng([M, K, N])
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.integers(0, K, max(1, K // 100))] *= 15.0
    W = wl.gaussian_weight(K, N, 0.02, rng)
    bias = wl.gaussian_bias(N, 0.1, rng) if N % 16 == 8 else None
    check_linear(wl.to_fp16(x), W, tau, bias=bias)


def test_zero_row_zero_column_and_all_zero_input():
    rng = np.random.default_rng(1)
    X = wl.to_fp16(rng.standard_normal((40, 256)).astype(np.float32))
    W = wl.gaussian_weight(256, 72, 0.02, rng)
    X[3, :] = 0
    W[:, 5] = 0
    check_linear(X, W, 6.0)
    check_linear(np.zeros((9, 64), np.float16), wl.gaussian_weight(64, 16, 0.02, rng), 6.0)


def test_row_stride_larger_than_k():
    rng = np.random.default_rng(2)
    big = wl.to_fp16(rng.standard_normal((33, 512)).astype(np.float32) * 3)
    W = wl.gaussian_weight(256, 64, 0.02, rng)
    pw = binding.prequantize_weight(to_gpu(W))
    Xg = to_gpu(big)[:, :256]
    assert Xg.stride(0) == 512
    Y = to_np(binding.mixed_int8_linear(Xg, pw, 6.0))
    Wq_o, c_o = ml.prequantize_weight(W)
    o = ml.mixed_int8_linear(np.ascontiguousarray(big[:, :256]), Wq_o, c_o, 6.0)
    assert_y_close(Y, o["Y"])


@pytest.mark.parametrize("M", [3, 70])
def test_k_too_large_for_one_pass_preparation(M):
    """K above 32768: the rows no longer fit the one-pass preparation kernel, so the scan and pack
    kernels run instead (for the decode kernel and for the tiled one)."""
    K, N = 32768 + 64, 72
    rng = np.random.default_rng([M, K])
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, rng.integers(0, K, 40)] *= 12.0
    check_linear(wl.to_fp16(x), wl.gaussian_weight(K, N, 0.02, rng), 6.0)


@pytest.mark.parametrize("M", [2, 130])
def test_largest_k(M):
    """K = MMD8_MAX_K (65536): the int32 accumulators stay far from overflow (K * 127^2 < 2^31), the column
    flags fill their region of the workspace head."""
    K, N = 65536, 40
    rng = np.random.default_rng([M, K, 1])
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[0, [0, K - 1, 40000]] = [9.0, -11.0, 200.0]                   # first, last and a middle column critical
    X = wl.to_fp16(x)
    o_flag = ml.outlier_mask(X, 6.0)
    assert o_flag[0] and o_flag[K - 1]
    check_linear(X, wl.gaussian_weight(K, N, 0.02, rng), 6.0)


def test_many_row_panels():
    """20001 rows: 79 panels of 256 rows, the last one with a single row; several rounds of tiles per CU."""
    M, K, N = 20001, 528, 264
    rng = np.random.default_rng([M, K, N])
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, [5, 300]] *= 12.0
    x[20000, 17] = 300.0                                            # a column made critical by the very last row only
    X = wl.to_fp16(x)
    assert ml.outlier_mask(X, 6.0)[17]
    check_linear(X, wl.gaussian_weight(K, N, 0.02, rng), 6.0)


def test_two_streams_with_their_own_workspaces():
    """Calls on different streams with different workspaces do not share state: interleaved on two streams they
    give what each gives alone."""
    rng = np.random.default_rng(12)
    cases = []
    for (M, K, N) in [(300, 1040, 520), (40, 2048, 264)]:
        x = rng.standard_t(3.0, size=(M, K)).astype(np.float32)
        X, W = to_gpu(wl.to_fp16(x)), wl.gaussian_weight(K, N, 0.02, rng)
        pw = binding.prequantize_weight(to_gpu(W))
        cases.append(dict(X=X, pw=pw, ws=binding.linear_workspace(M, K, N, "cuda"),
                          Y=torch.empty((M, N), dtype=torch.float16, device="cuda")))
    alone = []
    for c in cases:
        alone.append(binding.mixed_int8_linear(c["X"], c["pw"], 6.0, workspace=c["ws"]).clone())
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(5):
        for c, st in zip(cases, streams):
            with torch.cuda.stream(st):
                for _ in range(3):
                    binding.mixed_int8_linear(c["X"], c["pw"], 6.0, out=c["Y"], workspace=c["ws"])
        torch.cuda.synchronize()
        for c, ref in zip(cases, alone):
            assert torch.equal(c["Y"], ref), rep


def test_empty_batch():
    pw = binding.prequantize_weight(to_gpu(wl.gaussian_weight(64, 16, 0.02, np.random.default_rng(0))))
    Y = binding.mixed_int8_linear(torch.empty((0, 64), dtype=torch.float16, device="cuda"), pw, 6.0)
    assert Y.shape == (0, 16)


def test_repeated_calls_are_deterministic():
    cfg = wl.config1()
    pw = binding.prequantize_weight(to_gpu(cfg["W"]))
    Xg = to_gpu(cfg["X"])
    ws = binding.linear_workspace(16, 1024, 1024, "cuda")
    ref = None
    for _ in range(3):
        Y, taps = binding.mixed_int8_linear(Xg, pw, 6.0, workspace=ws, taps=True)
        h = (to_np(Y).tobytes(), to_np(taps["acc"]).tobytes(), to_np(taps["xq"]).tobytes())
        ref = ref or h
        assert h == ref


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 32, 64])
@pytest.mark.parametrize("shape", wl.LLAMA_7B_LINEARS, ids=lambda s: s.name)
def test_config3_decode_shapes(M, shape):
    """Student-t decode activations: up to ~45 % of the feature dimensions are critical."""
    X = wl.decode_activation(10 * M + shape.K % 7, M, shape.K)
    W = wl.prefill_weight(3, 100 + shape.K % 7, shape, 0.02)
    check_linear(X, W, wl.TAU)


@pytest.mark.parametrize("M", [96, 128, 256])
@pytest.mark.parametrize("shape", wl.LLAMA_7B_LINEARS, ids=lambda s: s.name)
def test_heavy_tailed_rows_around_the_change_of_path(M, shape):
    """The heavy-tailed launches the benchmark times on both sides of the change from the decode kernels to the
    tiled GEMM (Student-t activations at 128 and 256 rows: nearly every feature dimension is critical), and 96 rows
    (two passes of the decode kernels, the second a ragged one)."""
    X = wl.decode_activation(900 + M, M, shape.K)
    W = wl.prefill_weight(2, 20 + wl.LLAMA_7B_LINEARS.index(shape), shape, 0.02)
    check_linear(X, W, wl.TAU)


@pytest.mark.parametrize("shape", wl.LLAMA_7B_LINEARS, ids=lambda s: s.name)
def test_config2_prefill_full_size(shape):
    """The launches the benchmark times (2048 tokens), compared in full."""
    X, dims = wl.prefill_activation(2, 10 + shape.K % 5, 2048, shape.K)
    W = wl.prefill_weight(2, 20 + wl.LLAMA_7B_LINEARS.index(shape), shape, 0.02)
    fro, worst = check_linear(X, W, wl.TAU)
    flag = ml.outlier_mask(X, wl.TAU)
    assert set(dims.tolist()) <= set(np.flatnonzero(flag).tolist())


@pytest.mark.parametrize("shape", wl.LLAMA_70B_LINEARS, ids=lambda s: s.name)
def test_config5_prefill_full_size(shape):
    """70B-shaped linears at full size (4096 tokens): the launches the benchmark's step times.  Everything is
    compared in full: weight codes, mask, index list, and every row of the scales, codes, accumulators and Y, the
    oracle taking 512 rows at a time (1024 for gate/up, whose weight matrix is the costly part of a chunk)."""
    M = 4096
    X, _ = wl.prefill_activation(5, 10 + shape.K % 5, M, shape.K)
    W = wl.prefill_weight(5, 20 + wl.LLAMA_70B_LINEARS.index(shape), shape, 0.015)
    step = 1024 if shape.name == "gate_up" else 512
    chunks = [np.arange(m0, m0 + step) for m0 in range(0, M, step)]
    check_linear(X, W, wl.TAU, row_chunks=chunks)


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5])
def test_every_gemm_tile_configuration(variant):
    """All tile configurations of the GEMM kernel give the same integers (and pass the output bar)."""
    tune = binding.tune_gemm_tiles(variant)
    rng = np.random.default_rng(variant)
    x = rng.standard_normal((300, 1040)).astype(np.float32)
    x[:, [3, 777]] *= 25.0
    check_linear(wl.to_fp16(x), wl.gaussian_weight(1040, 520, 0.02, rng), 6.0, tuning=tune)
    X, _ = wl.prefill_activation(2, 99, 512, 4096)       # full tiles: the unchecked store path
    check_linear(X, wl.gaussian_weight(4096, 512, 0.02, rng), 6.0, tuning=tune)


def exactly_n_critical(rng, M, K, n_crit):
    """Activations in (-5, 5) except `n_crit` columns (chosen at random, first and last column among them when
    n_crit >= 2) that hold one entry above tau = 6 each, in different rows, and ordinary values otherwise."""
    x = np.clip(rng.standard_normal((M, K)), -5.0, 5.0).astype(np.float32)
    cols = rng.choice(np.arange(1, K - 1), max(0, n_crit - 2), replace=False) if n_crit >= 2 else \
        rng.choice(K, n_crit, replace=False)
    cols = np.sort(np.concatenate([cols, [0, K - 1]])) if n_crit >= 2 else cols
    for j, k in enumerate(cols):
        x[(7 * j) % M, k] = (-1.0) ** j * (8.0 + j % 50)
    return wl.to_fp16(x), cols


@pytest.mark.parametrize("variant", [4, 0, 2])
@pytest.mark.parametrize("n_crit", [0, 1, 31, 32, 33, 64, 65, 100, 255, 256, 257, 300])
def test_counts_of_critical_columns_around_the_slab_limits(n_crit, variant):
    """The tiled GEMM takes critical columns 32 at a time as fp16 slabs, up to 256 of them, and adds the rest from
    rows the preparation gathered: counts on both sides of every border between those paths, over several row
    panels and a ragged tail."""
    M, K, N = 600, 1040, 520
    rng = np.random.default_rng([n_crit, variant])
    X, cols = exactly_n_critical(rng, M, K, n_crit)
    flag = ml.outlier_mask(X, 6.0)
    assert np.array_equal(np.flatnonzero(flag), cols)
    bias = wl.gaussian_bias(N, 0.1, rng) if n_crit % 2 else None
    check_linear(X, wl.gaussian_weight(K, N, 0.05, rng), 6.0, bias=bias, tuning=binding.tune_gemm_tiles(variant))


@pytest.mark.parametrize("variant", [4, 5, 0])
@pytest.mark.parametrize("n_crit", [257, 300, 1312, 1344, 1345, 1485, 1486, 1550])
def test_counts_of_critical_columns_around_the_change_to_the_dense_pass(n_crit, variant):
    """34 slabs of K: up to 1344 critical columns travel as fp16 slabs (8, then up to 34 further ones), up to 1485
    the ones beyond are gathered in the GEMM's epilogue, from 1486 on all of them go through the second, fp16 pass
    over K."""
    M, K, N = 300, 2096, 264
    assert critical_column_plan(K, N) == (1344, 1486)
    rng = np.random.default_rng([n_crit, variant, 7])
    X, cols = exactly_n_critical(rng, M, K, n_crit)
    assert np.array_equal(np.flatnonzero(ml.outlier_mask(X, 6.0)), cols)
    check_linear(X, wl.gaussian_weight(K, N, 0.05, rng), 6.0, bias=wl.gaussian_bias(N, 0.1, rng),
                 tuning=binding.tune_gemm_tiles(variant))


@pytest.mark.parametrize("variant", [4, 3, 0])
@pytest.mark.parametrize("K", [16, 64, 128, 192, 320])
@pytest.mark.parametrize("tau", [6.0, 0.0])
def test_short_rows_in_the_tiled_gemm(K, tau, variant):
    """Two to five slabs of codes: fewer than the ring holds ahead, so the first requests already reach into the fp16
    slabs (tau = 0: every column critical, up to ten fp16 slabs behind two to five slabs of codes)."""
    M, N = 300, 264
    rng = np.random.default_rng([K, variant])
    x = rng.standard_normal((M, K)).astype(np.float32)
    x[:, K // 2] *= 20.0
    check_linear(wl.to_fp16(x), wl.gaussian_weight(K, N, 0.05, rng), tau, bias=wl.gaussian_bias(N, 0.1, rng),
                 tuning=binding.tune_gemm_tiles(variant))


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 4, 5])
@pytest.mark.parametrize("M,K,N", [(260, 2096, 304), (600, 1040, 520), (1030, 4096, 264)])
def test_most_columns_critical_over_many_rows(M, K, N, variant):
    """Heavy-tailed rows (Student-t, 3 degrees of freedom) over more rows than the decode kernels take: most
    columns are critical, far more than the fp16 slabs hold, with and without the master-weight reading."""
    rng = np.random.default_rng([M, K, variant])
    X = wl.to_fp16(rng.standard_t(3.0, size=(M, K)).astype(np.float32))
    n = int(ml.outlier_mask(X, wl.TAU).sum())
    assert n >= critical_column_plan(K, N)[1], n               # the dense pass
    W = wl.gaussian_weight(K, N, 0.05, rng)
    check_linear(X, W, wl.TAU, bias=wl.gaussian_bias(N, 0.1, rng), tuning=binding.tune_gemm_tiles(variant))


def test_moderate_share_of_critical_columns_full_size():
    """A 7B-shaped projection at 2048 tokens with 3 % of its dimensions critical (123 columns: four slabs)."""
    shape = wl.LLAMA_7B_LINEARS[0]
    rng = np.random.default_rng(31)
    X, _ = wl.gaussian_with_outlier_dims(2048, shape.K, 0.03, 8.0, 40.0, rng)
    n = int(ml.outlier_mask(X, wl.TAU).sum())
    assert 64 < n <= 256, n
    rows = np.concatenate([np.arange(0, 300), np.arange(2048 - 130, 2048)])
    check_linear(X, wl.prefill_weight(2, 77, shape, 0.02), wl.TAU, rows=rows)


@pytest.mark.parametrize("shape", wl.VIT_L_LINEARS, ids=lambda s: s.name)
def test_vit_shaped_linears_with_bias(shape):
    """ViT-L-shaped linears (width 1024, 4 images of 197 tokens: a ragged M) with a bias vector."""
    rng = np.random.default_rng([197, shape.K, shape.N])
    M = 4 * 197
    x = rng.standard_normal((M, shape.K)).astype(np.float32)
    x[:, rng.choice(shape.K, max(1, shape.K // 500), replace=False)] *= rng.uniform(8.0, 40.0)
    W = wl.gaussian_weight(shape.K, shape.N, 0.02, rng)
    check_linear(wl.to_fp16(x), W, wl.TAU, bias=wl.gaussian_bias(shape.N, 0.1, rng))


def test_one_workspace_serves_calls_of_different_shapes():
    """The head of the workspace (column flags) is standing state: every call must leave it
    ready for the next one, whatever the shapes and however many columns were flagged."""
    rng = np.random.default_rng(42)
    shapes = [(70, 2064, 72), (5, 144, 40), (300, 512, 264), (33, 2064, 72), (1, 16, 8)]
    ws = binding.linear_workspace(300, 2064, 264, "cuda")
    for rep in range(2):
        for (M, K, N) in shapes:
            x = rng.standard_normal((M, K)).astype(np.float32)
            x[:, rng.integers(0, K, max(1, K // 50))] *= 15.0
            X = wl.to_fp16(x)
            W = wl.gaussian_weight(K, N, 0.02, rng)
            tau = [6.0, 0.0, 2.0][(rep + M) % 3]
            pw = binding.prequantize_weight(to_gpu(W))
            Y, taps = binding.mixed_int8_linear(to_gpu(X), pw, tau, workspace=ws, taps=True)
            Wq_o, c_o = ml.prequantize_weight(W)
            o = ml.mixed_int8_linear(X, Wq_o, c_o, tau)
            assert np.array_equal(to_np(taps["outlier_mask"]).astype(bool), o["flag"]), (rep, M, K, N)
            assert np.array_equal(to_np(taps["acc"]), o["acc"]), (rep, M, K, N)
            assert_y_close(to_np(Y), o["Y"])


@pytest.mark.parametrize("M,K,N,block", [(300, 1040, 264, 64), (2048, 4096, 512, 1024), (40, 512, 72, 256), (130, 272, 40, 4096),
                                         (130, 16384, 40, 1024), (130, 16448, 40, 64), (100, 528, 72, 256)])
def test_layer_on_blockwise_coded_activations(M, K, N, block):
    """The layer fed with a coded hidden state: identical, bit for bit, to decoding first and
    calling the layer on the result (for more than 128 rows the decoding happens inside the
    preparation kernel), and equal to the oracle's two steps."""
    from oracle import blockwise_codec as bc
    rng = np.random.default_rng([M, K, N, block])
    h = rng.standard_t(3, (M, K)).astype(np.float32)
    h[:, rng.integers(0, K, max(1, K // 200))] *= 20.0
    H = wl.to_fp16(h)
    W = wl.gaussian_weight(K, N, 0.02, rng)
    codes_o, absmax_o = bc.quantize_blockwise(H.reshape(-1), block)
    X_o = bc.dequantize_blockwise(codes_o, absmax_o, block).reshape(M, K)
    pw, Wq_o, c_o = check_weight(W)
    codes, absmax = to_gpu(codes_o), to_gpu(absmax_o)
    Xd = torch.empty((M, K), dtype=torch.float16, device="cuda")
    Y, taps = binding.mixed_int8_linear(Xd, pw, wl.TAU, taps=True, coded=(codes, absmax, block))
    # the two separate calls
    X2 = binding.dequantize_blockwise(codes, absmax, block).view(M, K)
    Y2 = binding.mixed_int8_linear(X2, pw, wl.TAU)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(Xd).view(np.uint16), X_o.view(np.uint16)), "decoded activations"
    assert np.array_equal(to_np(Y).view(np.uint16), to_np(Y2).view(np.uint16)), "fused and two-step outputs differ"
    o = ml.mixed_int8_linear(X_o, Wq_o, c_o, wl.TAU)
    assert np.array_equal(to_np(taps["outlier_mask"]).astype(bool), o["flag"])
    assert np.array_equal(to_np(taps["row_absmax"]).view(np.uint32), o["r"].view(np.uint32))
    assert np.array_equal(to_np(taps["xq"]), o["Xq"])
    assert np.array_equal(to_np(taps["acc"]), o["acc"])
    assert_y_close(to_np(Y), o["Y"])
