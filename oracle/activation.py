"""The int8 layer followed by GELU (oracle; test infrastructure).

The paper's shards hold transformer blocks (language models and vision transformers); the first linear of
an MLP block is followed by the GELU activation, gelu(x) = x Phi(x) with Phi the standard normal
distribution function.  The paper does not say which form of GELU its models use; the reading here is
the exact one (not the tanh approximation), written with the complementary error function:

  G1  Y = the int8 layer's fp16 output (mixed_linear.mixed_int8_linear, bias included)
  G2  G[m, n] = f16( Y[m, n] * erfc(-Y[m, n] / sqrt 2) / 2 )          evaluated in float64

so that G is what the layer followed by an fp16 activation kernel holds (Y keeps its own rounding).
"""
import numpy as np
from scipy.special import erfc

from . import mixed_linear


def gelu_fp16(Y: np.ndarray) -> np.ndarray:
    """G2 on an fp16 tensor: exact GELU in float64, one rounding to fp16."""
    assert Y.dtype == np.float16
    y = Y.astype(np.float64)
    with np.errstate(over="ignore", invalid="ignore"):
        return (0.5 * y * erfc(-y / np.sqrt(2.0))).astype(np.float16)


def mixed_int8_linear_gelu(X, Wq, c, tau, bias=None, rows=None):
    """The base layer's dict plus G (fp16 [M, N])."""
    out = mixed_linear.mixed_int8_linear(X, Wq, c, tau, bias, rows)
    out.update(G=gelu_fp16(out["Y"]))
    return out
