"""The shard's last linear with the hidden state leaving in coded form (oracle; test infrastructure).

Section "Compression techniques": item 2 gives the int8 layer, item 1 compresses the hidden state that
one node hands to the next.  At the end of a shard the two meet: the last layer's output, plus the
residual stream where the model has one, is what gets encoded.  The composition, in this library's
row layout (X is [M, K], the layer maps K features to N):

  E1  Y = the int8 layer's fp16 output (as in mixed_linear.mixed_int8_linear)
  E2  H[m, n] = f16( Y[m, n] + R[m, n] )      R: fp16 residual [M, N]; without one H = Y
  E3  (codes, absmax) = quantize_blockwise(H flattened row by row, block)

The paper names the two techniques, not how they join.  Readings: the hidden state is an fp16 tensor
before it is encoded (E1 keeps its own rounding: encoding sees exactly what an implementation that
runs the two steps one after the other sees), and the residual is added as an fp16 addition (a second
rounding, to nearest even).  Blocks run over the flattened tensor, so they cross row ends whenever
the block size does not divide N.
"""
import numpy as np

from . import blockwise_codec, mixed_linear


def add_residual(Y: np.ndarray, R: np.ndarray) -> np.ndarray:
    """E2: the fp16 sum, formed exactly (float64 holds any sum of two fp16 values) and rounded once."""
    assert Y.dtype == np.float16 and R.dtype == np.float16 and Y.shape == R.shape
    with np.errstate(over="ignore"):
        return (Y.astype(np.float64) + R.astype(np.float64)).astype(np.float16)


def mixed_int8_linear_to_codes(X, Wq, c, tau, block, bias=None, residual=None):
    """The base layer's dict plus H (fp16 [M, N]), codes (uint8 [M N]) and absmax (float32)."""
    out = mixed_linear.mixed_int8_linear(X, Wq, c, tau, bias)
    H = out["Y"] if residual is None else add_residual(out["Y"], residual)
    codes, absmax = blockwise_codec.quantize_blockwise(np.ascontiguousarray(H).reshape(-1), block)
    out.update(H=H, codes=codes, absmax=absmax)
    return out
