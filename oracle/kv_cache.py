"""Key/value cache held in blockwise-coded form (oracle; test infrastructure).

Section "Cache optimization to enhance efficiency" gives the size of the cache: per token,
2 * head_dim * n_heads * n_layers elements (one key and one value vector per head and layer).  The paper
does not compress the cache; applying its hidden-state codec ("Compression techniques", item 1) to it is this
library's extension, with the natural block: the head_dim elements of one token and one head, so that a
token is encoded when it is appended and never touched again, and any token range decodes on its own.

  K1  cache_elements_per_token = 2 * head_dim * n_heads * n_layers                      (the paper's equation)
  K2  a cache tensor of one layer is [T, n_heads, head_dim] fp16, contiguous; its coded form is
      quantize_blockwise(flattened, block = head_dim): codes uint8 [T, n_heads, head_dim], absmax fp32 [T, n_heads]
"""
import numpy as np

from . import blockwise_codec


def cache_elements_per_token(head_dim: int, n_heads: int, n_layers: int) -> int:
    """K1."""
    return 2 * head_dim * n_heads * n_layers


def coded_bytes_per_token(head_dim: int, n_heads: int, n_layers: int) -> int:
    """One byte per element plus one fp32 scale per (key or value, head, layer)."""
    return cache_elements_per_token(head_dim, n_heads, n_layers) + 4 * 2 * n_heads * n_layers


def encode_tokens(kv: np.ndarray):
    """K2 for a run of tokens: kv fp16 [t, n_heads, head_dim] -> (codes uint8 same shape, absmax fp32 [t, n_heads])."""
    assert kv.dtype == np.float16 and kv.ndim == 3
    t, h, d = kv.shape
    codes, absmax = blockwise_codec.quantize_blockwise(np.ascontiguousarray(kv).reshape(-1), d)
    return codes.reshape(t, h, d), absmax.reshape(t, h)


def decode_tokens(codes: np.ndarray, absmax: np.ndarray) -> np.ndarray:
    t, h, d = codes.shape
    return blockwise_codec.dequantize_blockwise(codes.reshape(-1), absmax.reshape(-1), d).reshape(t, h, d)
