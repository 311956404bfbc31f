"""Up to eight rows: the decode GEMM kernel prepares its own operands (row scales, codes, critical columns) and
the scan and pack kernels are left out.  The result must equal, bit for bit, the one obtained with those kernels
(forced through the call's tuning word, or by asking for their taps), the int32 accumulators must equal the oracle's, and
the output must meet the oracle's to the fp16 bar; with every companion of the layer (bias, adapter, activation,
coded input, coded output).  One or two rows (while their operands fit in LDS) go through a single kernel that shares K out between the waves of a
workgroup: same integers, and an output that may differ from the split-K kernels' in the last fp16 bit (another
order of fp32 additions), so it is compared with theirs to a fifth of the usual bar and with the oracle to the usual bar."""
import numpy as np
import pytest
import torch

from oracle import blockwise_codec as bc
from oracle import mixed_linear as ml
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import assert_y_close, to_gpu, to_np

pytestmark = pytest.mark.gpu


class Tune:
    """The kernel choice handed to every call of this module (mmd8_debug_taps.tuning): per call, no library state."""
    value = 0


def lin(*args, **kw):
    return binding.mixed_int8_linear(*args, tuning=Tune.value, **kw)


def lin_to_codes(*args, **kw):
    return binding.mixed_int8_linear_to_codes(*args, tuning=Tune.value, **kw)


def rows_kernel(on):
    Tune.value = (Tune.value & ~binding.TUNE_NO_ROWS_KERNEL) | (0 if on else binding.TUNE_NO_ROWS_KERNEL)


def own_prep(on):
    Tune.value = (Tune.value & ~binding.TUNE_SEPARATE_PREP) | (0 if on else binding.TUNE_SEPARATE_PREP)


@pytest.fixture(autouse=True)
def own_prep_on():
    Tune.value = 0
    yield
    Tune.value = 0


def fp16_steps(a, b):
    def line(t):
        u = t.view(torch.int16).to(torch.int32) & 0xffff
        return torch.where(u >= 0x8000, -(u & 0x7fff), u)
    return (line(a) - line(b)).abs().max().item() if a.numel() else 0


def case(M, K, N, seed, heavy):
    rng = np.random.default_rng([M, K, N, seed])
    x = (rng.standard_t(3.0, size=(M, K)) if heavy else rng.standard_normal((M, K))).astype(np.float32)
    x[:, rng.integers(0, K, max(1, K // 200))] *= 20.0
    return wl.to_fp16(x), wl.gaussian_weight(K, N, 0.02, rng), wl.gaussian_bias(N, 0.3, rng), rng


@pytest.mark.parametrize("K,N", [(64, 8), (528, 264), (4096, 4096), (4096, 12288), (11008, 4096), (1040, 22016),
                                 (16448, 72), (65536, 32), (8192, 57344)])
def test_own_preparation_equals_the_separate_kernels(K, N):
    rng = np.random.default_rng([K, N])
    W = wl.gaussian_weight(K, N, 0.02, rng)
    b = wl.gaussian_bias(N, 0.3, rng)
    pw = binding.prequantize_weight(to_gpu(W))
    bg = to_gpu(b)
    # the oracle on every output column, or (large weights) on 256 of them spread over the whole width, the first and
    # the last included: columns are independent of each other in every step of the layer
    cols = np.arange(N) if K * N <= 4096 * 4096 else np.unique(np.concatenate([np.linspace(0, N - 1, 250).astype(np.int64),
                                                                               rng.integers(0, N, 6)]))
    Wq_o, c_o = ml.prequantize_weight(np.ascontiguousarray(W[:, cols]))
    cols_g = torch.from_numpy(cols).cuda()
    for M in (1, 2, 3, 4, 5, 8):
        for rep, tau in enumerate([wl.TAU, 0.0, np.inf, 2.0]):
            X = case(M, K, 8, rep, heavy=bool(rep % 2))[0]
            if rep == 2:
                X[M - 1] = 0                                         # a zero row: scale 0
            Xbuf = torch.zeros((M, K + 8), dtype=torch.float16, device="cuda")
            Xg = Xbuf[:, :K]
            Xg.copy_(to_gpu(X))
            rows_kernel(0)
            Y_taps, taps = lin(Xg, pw, tau, bias=bg, taps=True)     # scan + pack (their taps asked for)
            own_prep(0)
            Y_off = lin(Xg, pw, tau, bias=bg)                       # scan + pack (hook)
            own_prep(1)
            Y, t_acc = lin(Xg, pw, tau, bias=bg, taps=("acc",))   # own preparation in the panel kernel
            rows_kernel(1)
            torch.cuda.synchronize()
            assert torch.equal(Y, Y_off) and torch.equal(Y, Y_taps), (M, K, N, tau)
            assert torch.equal(t_acc["acc"], taps["acc"]), (M, K, N, tau)
            if M <= 2 and 3 * M * ((K + 63) // 64 * 64) <= 66 * 1024:                     # the single kernel
                Y, t_acc = lin(Xg, pw, tau, bias=bg, taps=("acc",))
                Y_all, t_all = lin(Xg, pw, tau, bias=bg, taps=True)   # scan + pack for their taps only
                torch.cuda.synchronize()
                assert torch.equal(t_acc["acc"], taps["acc"]), (M, K, N, tau)
                assert torch.equal(Y, Y_all), (M, K, N, tau)
                for name in ("outlier_mask", "row_absmax", "xq", "acc", "n_outliers", "outlier_idx"):
                    assert torch.equal(t_all[name], taps[name]), name
                assert_y_close(to_np(Y), to_np(Y_off), rel=2e-3)                           # another order of fp32 additions
            o = ml.mixed_int8_linear(X, Wq_o, c_o, tau, np.ascontiguousarray(b[cols]))
            assert np.array_equal(to_np(t_acc["acc"][:, cols_g]), o["acc"])
            assert_y_close(to_np(Y[:, cols_g]), o["Y"])


@pytest.mark.parametrize("M", [1, 2, 4, 7, 8])
def test_companions_of_the_layer(M):
    K, N = 2048, 1024
    X, W, b, rng = case(M, K, N, 7, heavy=True)
    pw = binding.prequantize_weight(to_gpu(W))
    Xg, bg = to_gpu(X), to_gpu(b)
    A = to_gpu(wl.to_fp16(rng.standard_normal((16, K)).astype(np.float32) * 0.05))
    B = to_gpu(wl.to_fp16(rng.standard_normal((N, 16)).astype(np.float32) * 0.05))
    R = to_gpu(wl.to_fp16(rng.standard_normal((M, N)).astype(np.float32)))
    codes_o, absmax_o = bc.quantize_blockwise(X.reshape(-1), 256)
    cg, ag = to_gpu(codes_o), to_gpu(absmax_o)

    def run_all():
        out = [lin(Xg, pw, wl.TAU, bias=bg, lora=(A, B)),
               lin(Xg, pw, wl.TAU, bias=bg, gelu=True)]
        Xd = torch.empty((M, K), dtype=torch.float16, device="cuda")
        out.append(lin(Xd, pw, wl.TAU, bias=bg, coded=(cg, ag, 256)))
        out.append(Xd)
        out.extend(lin_to_codes(Xg, pw, wl.TAU, 1024, bias=bg, residual=R))
        torch.cuda.synchronize()
        return out

    on = run_all()
    own_prep(0)
    off = run_all()
    own_prep(1)
    for i, (a, b_) in enumerate(zip(on, off)):
        if a.dtype == torch.float16 and i == 1 and M <= 2:
            # GELU of a pre-activation that moved by one fp16 step: many steps of the much smaller output
            assert torch.allclose(a.float(), b_.float(), rtol=1e-2, atol=1e-3), i
        elif a.dtype == torch.float16 and M <= 2:
            assert_y_close(to_np(a), to_np(b_), rel=2e-3)             # (one or two rows: the single kernel where it applies)
        elif a.dtype == torch.float16:
            assert torch.equal(a, b_), i
        elif i < len(on) - 2:
            assert torch.equal(a, b_), i
    # the coded output (last two entries) is encoded by the kernel that sums the partial outputs on both ways
    assert torch.equal(on[-2], off[-2]) and torch.equal(on[-1], off[-1])
    Rplain = lin(Xg, pw, wl.TAU, bias=bg, residual=R)
    rows_kernel(0)
    Rpanel = lin(Xg, pw, wl.TAU, bias=bg, residual=R)
    rows_kernel(1)
    torch.cuda.synchronize()
    assert_y_close(to_np(Rplain), to_np(Rpanel), rel=2e-3)


def test_same_workspace_alternates_between_both_ways():
    M, K, N = 1, 4096, 4096
    X, W, b, _ = case(M, K, N, 3, heavy=True)
    pw = binding.prequantize_weight(to_gpu(W))
    ws = binding.linear_workspace(64, K, N, torch.device("cuda:0"))
    Xg = to_gpu(X)
    X64 = to_gpu(wl.to_fp16(np.random.default_rng(1).standard_t(3.0, size=(64, K)).astype(np.float32)))
    ys = []
    for i in range(3):
        ys.append(lin(Xg, pw, wl.TAU, workspace=ws))
        y64 = lin(X64, pw, wl.TAU, workspace=ws)           # scan + pack, leaves the flags zero again
        if i == 0:
            y64_first = y64
        else:
            assert torch.equal(y64, y64_first)
    torch.cuda.synchronize()
    assert torch.equal(ys[0], ys[1]) and torch.equal(ys[0], ys[2])
