"""Pins for the coded key/value cache of the oracle: the paper's size equation on known models, independence of
tokens and heads, and the codec's hand-worked example as one head."""
import numpy as np

from oracle import blockwise_codec as bc
from oracle import kv_cache as kv


def test_size_equation_on_known_shapes():
    # a 32-layer model with 32 heads of 128 dimensions: 2 * 128 * 32 * 32 = 262144 elements, 512 KiB in fp16
    assert kv.cache_elements_per_token(128, 32, 32) == 262144
    assert kv.cache_elements_per_token(128, 64, 80) == 1310720
    assert kv.cache_elements_per_token(64, 16, 24) == 49152
    # coded: one byte per element and one fp32 scale per head vector: (1 + 4 / head_dim) / 2 of the fp16 size
    assert kv.coded_bytes_per_token(128, 32, 32) == 262144 + 8192
    assert kv.coded_bytes_per_token(128, 32, 32) / (2 * 262144) == (1 + 4 / 128) / 2
    assert bc.compressed_fraction(262144, 128) == kv.coded_bytes_per_token(128, 32, 32) / (2 * 262144)


def test_tokens_and_heads_are_encoded_independently(golden):
    rng = np.random.default_rng(1)
    x = (rng.standard_t(3.0, size=(6, 4, 64)) * 0.5).astype(np.float16)
    codes, absmax = kv.encode_tokens(x)
    assert codes.shape == x.shape and absmax.shape == (6, 4)
    assert np.array_equal(absmax, np.abs(x.astype(np.float32)).max(axis=2))
    # appending token by token, or head by head, gives the same cache as encoding everything at once
    for t in range(6):
        c1, a1 = kv.encode_tokens(x[t:t + 1])
        assert np.array_equal(c1[0], codes[t]) and np.array_equal(a1[0], absmax[t])
        for h in range(4):
            c2, a2 = bc.quantize_blockwise(x[t, h], 64)
            assert np.array_equal(c2, codes[t, h]) and a2[0] == absmax[t, h]
    # changing one head of one token changes nothing else
    y = x.copy()
    y[2, 1] *= np.float16(3.0)
    c3, a3 = kv.encode_tokens(y)
    keep = np.ones((6, 4), bool)
    keep[2, 1] = False
    assert np.array_equal(c3[keep], codes[keep]) and np.array_equal(a3[keep], absmax[keep])
    back = kv.decode_tokens(codes, absmax)
    assert back.shape == x.shape and np.array_equal(back[3], kv.decode_tokens(codes[3:4], absmax[3:4])[0])
    # the codec's hand-worked 4-element blocks as two heads of dimension 4
    g = golden("codec_worked_example.txt")
    c4, a4 = kv.encode_tokens(g["x"].astype(np.float16).reshape(1, 2, 4))
    assert np.array_equal(c4.reshape(-1), g["codes"].astype(np.uint8)) and np.array_equal(a4.reshape(-1), g["absmax"].astype(np.float32))
