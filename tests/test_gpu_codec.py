"""GPU parity of the blockwise codec against the CPU oracle: everything bit-exact."""
import numpy as np
import pytest
import torch

from oracle import blockwise_codec as bc
from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import to_gpu, to_np

pytestmark = pytest.mark.gpu


def run_both(x: np.ndarray, block: int):
    xg = to_gpu(x)
    codes, absmax = binding.quantize_blockwise(xg, block)
    dec = binding.dequantize_blockwise(codes, absmax, block)
    torch.cuda.synchronize()
    oc, oa = bc.quantize_blockwise(x, block)
    od = bc.dequantize_blockwise(oc, oa, block)
    return (to_np(codes), to_np(absmax), to_np(dec)), (oc, oa, od)


def check(x, block):
    (c, a, d), (oc, oa, od) = run_both(x, block)
    assert np.array_equal(a.view(np.uint32), oa.view(np.uint32)), "block absmax"
    bad = np.flatnonzero(c != oc)
    assert bad.size == 0, ("codes", bad[:8], c[bad[:8]], oc[bad[:8]])
    assert np.array_equal(d.view(np.uint16), od.view(np.uint16)), "decoded"


def test_config1_hidden_state():
    cfg = wl.config1()
    check(cfg["X"], cfg["block"])


@pytest.mark.parametrize("block", [64, 128, 192, 256, 512, 1024, 2048, 4032, 4096])
def test_block_sizes_with_ragged_tail(block):
    rng = np.random.default_rng(block)
    n = 37 * block + block // 2 + 3                  # several spans, short last block, n % 8 != 0
    x = rng.standard_t(3, n).astype(np.float32) * rng.choice([1e-4, 1.0, 30.0], n).astype(np.float32)
    x[rng.integers(0, n, 50)] = 0
    x[5 * block:6 * block] = 0                       # an all-zero block
    x[7 * block:8 * block] = -np.abs(x[7 * block:8 * block])   # a block whose maximum is negative
    check(wl.to_fp16(x), block)


def test_every_finite_fp16_value():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    allv = bits.view(np.float16)
    allv = allv[np.isfinite(allv)]
    for a in (65504.0, 1.0, 3.0, 0.0123, 777.5, 6.1e-5, 5.96e-8):
        a16 = np.float16(a)
        x = allv[np.abs(allv.astype(np.float32)) <= np.float32(a16)]
        # 4095 values per block plus the maximum itself, so that every block has absmax a16
        nblk = (x.size + 4094) // 4095
        data = np.zeros(nblk * 4095, np.float16)
        data[:x.size] = x
        xs = np.full((nblk, 4096), a16, np.float16)
        xs[:, :4095] = data.reshape(nblk, 4095)
        xs = xs.reshape(-1)
        check(xs, 4096)


def test_tiny_and_empty_inputs():
    for n in (1, 7, 8, 63, 64, 65):
        x = wl.to_fp16(np.random.default_rng(n).standard_normal(n).astype(np.float32))
        check(x, 64)
    e = torch.empty(0, dtype=torch.float16, device="cuda")
    c, a = binding.quantize_blockwise(e, 256)
    assert c.numel() == 0 and a.numel() == 0
    assert binding.dequantize_blockwise(c, a, 256).numel() == 0


def test_unsupported_block_raises():
    x = torch.zeros(1024, dtype=torch.float16, device="cuda")
    for block in (0, 32, 100, 8192):
        with pytest.raises(binding.Mmd8Error):
            binding.quantize_blockwise(x, block)


def test_round_trip_of_codes_on_gpu():
    rng = np.random.default_rng(5)
    block, nblk = 256, 300
    q = rng.integers(0, 256, size=block * nblk).astype(np.uint8)
    q[np.arange(nblk) * block + rng.integers(0, block, nblk)] = 255
    a = rng.uniform(0.25, 1000.0, nblk).astype(np.float16).astype(np.float32)
    x = binding.dequantize_blockwise(to_gpu(q), to_gpu(a), block)
    q2, a2 = binding.quantize_blockwise(x, block)
    assert np.array_equal(to_np(q2), q) and np.array_equal(to_np(a2), a)


@pytest.mark.parametrize("block", wl.CODEC_BLOCKS_BOUNDARY)
def test_config4_full_size(block):
    """[8192, 8192] Student-t hidden state, the launch the benchmark times, compared in full."""
    x, dims = wl.boundary_hidden_state()
    assert dims.size == 4
    check(x, block)


@pytest.mark.parametrize("n,block", [(8192 * 64, 256), (70000, 4096), (5000, 64), (4096 * 3 + 40, 1024), (130, 128), (7, 64),
                                     (262144, 2048), (100000, 192)])
def test_block_scales_stored_as_fp16(n, block):
    """The other storage of the block scales: same codes, same decoded values, scales as fp16 bit patterns; against
    the oracle and against the library's fp32 form."""
    rng = np.random.default_rng([n, block])
    x = (rng.standard_t(3.0, size=n) * rng.uniform(0.01, 300.0)).astype(np.float16)
    x[rng.integers(0, n, 3)] = 0
    xg = torch.from_numpy(x).cuda()
    nb = (n + block - 1) // block
    codes = torch.full((n + 16,), 0xAB, dtype=torch.uint8, device="cuda")
    scales = torch.full((nb + 8,), -1.0, dtype=torch.float16, device="cuda")
    binding.quantize_blockwise(xg, block, codes=codes[:n], absmax=scales[:nb], fp16_scales=True)
    c32, a32 = binding.quantize_blockwise(xg, block)
    dec = binding.dequantize_blockwise(codes[:n], scales[:nb], block)
    dec32 = binding.dequantize_blockwise(c32, a32, block)
    torch.cuda.synchronize()
    oc, oa = bc.quantize_blockwise(x, block, fp16_scales=True)
    assert np.array_equal(codes[:n].cpu().numpy(), oc)
    assert np.array_equal(scales[:nb].cpu().numpy().view(np.uint16), oa.view(np.uint16))
    assert bool((codes[n:] == 0xAB).all()) and bool((scales[nb:] == -1.0).all()), "wrote past the outputs"
    assert torch.equal(codes[:n], c32) and torch.equal(scales[:nb].float(), a32)
    assert np.array_equal(dec.cpu().numpy().view(np.uint16), bc.dequantize_blockwise(oc, oa, block).view(np.uint16))
    assert torch.equal(dec, dec32)
