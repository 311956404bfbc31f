"""Dynamic blockwise 8-bit codec for shard-boundary hidden states (oracle; test infrastructure).

Section "Compression techniques", item 1: the hidden state handed from one node to the next is
quantized block by block to 8 bits, halving the bytes on the wire.  Steps, in order:

1. the tensor is flattened (row-major); block ``b`` is elements ``[b*B, min((b+1)*B, n))``;
2. ``a[b] = max |x_i|`` over the block, held as fp32 (exact: it is an fp16 value);
3. ``inv = 1.0f / a[b]`` (one fp32 division; 0 when ``a[b] == 0``), ``v_i = f32(x_i) * inv``
   (one fp32 multiplication);
4. ``code_i = #{ j in 0..254 : v_i > Mid[j] }`` (strict), i.e. the nearest table entry with
   exact ties going to the lower index;
5. decoding is ``f16( T[code_i] * a[b] )``: one fp32 multiplication, one rounding to fp16.

All arithmetic is IEEE binary32, round to nearest even, no fused operations.  The full blocks
are handled as the rows of an ``[n // B, B]`` array and a short last block on its own; each row
goes through exactly the steps above.

Another reading of step 2 stores ``a[b]`` as the fp16 number it is (2 bytes per block instead of 4): with
``fp16_scales=True`` the encoder returns the scales as fp16 and the decoder takes them as such; every other
value is unchanged because the conversion is exact in both directions.
"""
import numpy as np

from . import dynamic_code


def _split(flat: np.ndarray, block: int):
    """Views of the full blocks ([nfull, block]) and of the short last block ([1, tail] or None)."""
    n = flat.size
    nfull = n // block
    full = flat[:nfull * block].reshape(nfull, block)
    tail = flat[nfull * block:].reshape(1, -1) if n % block else None
    return full, tail


def _absmax_rows(rows: np.ndarray) -> np.ndarray:
    if rows.shape[0] == 0:
        return np.zeros(0, dtype=np.float32)
    return np.max(np.abs(rows.astype(np.float32)), axis=1)


def block_absmax(x: np.ndarray, block: int) -> np.ndarray:
    flat = np.ascontiguousarray(x).reshape(-1)
    assert flat.dtype == np.float16 and block >= 1
    full, tail = _split(flat, block)
    parts = [_absmax_rows(full)]
    if tail is not None:
        parts.append(_absmax_rows(tail))
    return np.concatenate(parts).astype(np.float32)


def _encode_rows(rows: np.ndarray, a: np.ndarray, mid: np.ndarray) -> np.ndarray:
    one = np.float32(1.0)
    with np.errstate(divide="ignore"):
        inv = np.where(a == 0, np.float32(0.0), one / a).astype(np.float32)   # fp32 division
    v = rows.astype(np.float32) * inv[:, None]                                 # fp32 product
    assert v.dtype == np.float32
    # number of midpoints strictly below v
    return np.searchsorted(mid, v.reshape(-1), side="left").astype(np.uint8)


def quantize_blockwise(x: np.ndarray, block: int, fp16_scales: bool = False):
    """x: fp16, any shape -> (codes uint8 [n], absmax float32 [ceil(n/block)]; float16 with fp16_scales)."""
    flat = np.ascontiguousarray(x).reshape(-1)
    assert flat.dtype == np.float16 and block >= 1
    mid = dynamic_code.midpoints()
    a = block_absmax(flat, block)
    full, tail = _split(flat, block)
    nfull = full.shape[0]
    parts = [_encode_rows(full, a[:nfull], mid)]
    if tail is not None:
        parts.append(_encode_rows(tail, a[nfull:], mid))
    if fp16_scales:
        a16 = a.astype(np.float16)
        assert np.array_equal(a16.astype(np.float32), a)                       # the magnitude of an fp16 element
        return np.concatenate(parts), a16
    return np.concatenate(parts), a


def dequantize_blockwise(codes: np.ndarray, absmax: np.ndarray, block: int) -> np.ndarray:
    """codes uint8 [n], absmax float32 (or float16: the other storage of the scales) [ceil(n/block)] -> fp16 [n]."""
    if absmax.dtype == np.float16:
        absmax = absmax.astype(np.float32)                                     # exact
    t = dynamic_code.code_table()
    codes = np.ascontiguousarray(codes).reshape(-1)
    n = codes.size
    assert codes.dtype == np.uint8
    assert absmax.dtype == np.float32 and absmax.size == (n + block - 1) // block
    full, tail = _split(codes, block)
    nfull = full.shape[0]
    outs = []
    for rows, a in ((full, absmax[:nfull]), (tail, absmax[nfull:])):
        if rows is None:
            continue
        prod = t[rows] * a[:, None]                                            # fp32 product
        assert prod.dtype == np.float32
        outs.append(prod.astype(np.float16).reshape(-1))                       # round to nearest even
    return np.concatenate(outs) if outs else np.zeros(0, np.float16)


def compressed_fraction(n: int, block: int, scale_bytes: int = 4) -> float:
    """Bytes after / bytes before for an fp16 tensor of n elements (codes + absmax of scale_bytes each)."""
    nblk = (n + block - 1) // block
    return (n + scale_bytes * nblk) / (2 * n)
