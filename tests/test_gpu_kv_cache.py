"""The codec on a key/value cache: one block per (token, head), tokens appended in pieces at their place in
preallocated buffers, any token range decoded on its own; bit-exact against the oracle."""
import numpy as np
import pytest
import torch

from oracle import kv_cache as kvo
from paper_2407_19775_amd import binding
from gpu_util import to_gpu, to_np

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("T,H,D,pieces", [(300, 32, 128, (255, 1, 1, 43)), (70, 8, 64, (1, 1, 1, 67)), (33, 5, 256, (32, 1)),
                                          (2048, 32, 128, (2048,))])
def test_cache_appended_in_pieces(T, H, D, pieces):
    assert sum(pieces) == T
    rng = np.random.default_rng([T, H, D])
    x = (rng.standard_t(3.0, size=(T, H, D)) * 0.7).astype(np.float32)
    x[:, :, 3] *= 12.0                                   # a large channel, as rotary-embedded keys have
    x = x.astype(np.float16)
    codes = torch.full((T, H, D), 0xAB, dtype=torch.uint8, device="cuda")
    absmax = torch.full((T, H), -1.0, dtype=torch.float32, device="cuda")
    xg = to_gpu(x)
    t0 = 0
    for n in pieces:
        binding.quantize_blockwise(xg[t0:t0 + n].reshape(-1), D, codes=codes[t0:t0 + n].view(-1), absmax=absmax[t0:t0 + n].view(-1))
        t0 += n
        torch.cuda.synchronize()
        assert torch.all(codes[t0:] == 0xAB) and torch.all(absmax[t0:] == -1.0), "wrote past the appended tokens"
    codes_o, absmax_o = kvo.encode_tokens(x)
    assert np.array_equal(to_np(absmax).view(np.uint32), absmax_o.view(np.uint32))
    assert np.array_equal(to_np(codes), codes_o)
    # a token range on its own
    a, b = T // 3, T // 3 + max(1, T // 5)
    back = binding.dequantize_blockwise(codes[a:b].view(-1), absmax[a:b].view(-1), D)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(back).reshape(b - a, H, D).view(np.uint16), kvo.decode_tokens(codes_o[a:b], absmax_o[a:b]).view(np.uint16))
