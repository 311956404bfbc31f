"""Low-rank adapted mixed int8 linear layer (oracle; test infrastructure).

Section "BSNS with parameter-efficient fine-tuning via adapters": a weight matrix of the frozen
base model is adapted as W' = W + B A with A in R^{r x n}, B in R^{n x r}, r << n.  The shard keeps
W in its 8-bit form (section "Compression techniques", item 2) and the two small factors in
fp16, so that y = W' x is evaluated as the int8 layer plus a rank-r correction.  In the row
layout of this library (X is [M, K], one token per row; the layer maps K features to N):

  L1  T[m, j] = f16( sum_k X[m, k] * A[j, k] )        A is [r, K] fp16; the low-rank activation
                                                       is an fp16 tensor like any other activation
  L2  Y[m, n] = f16( Yi + Yo + bias[n] + sum_j T[m, j] * B[n, j] )
                                                       B is [N, r] fp16; Yi, Yo as in the base
                                                       layer; one final rounding

The sums are evaluated in float64.  A scale factor (alpha / r in the usual formulation) is
the caller's to fold into B.  The paper states only W' = W + B A; L1 (the fp16 rounding of the
intermediate) and L2 (joining the single final rounding) are readings.
"""
import numpy as np

from . import mixed_linear


def lora_down(X: np.ndarray, A: np.ndarray) -> np.ndarray:
    """L1: T = f16(X A^T), [M, r]."""
    assert X.dtype == np.float16 and A.dtype == np.float16 and X.shape[1] == A.shape[1]
    T64 = X.astype(np.float64) @ A.astype(np.float64).T
    with np.errstate(over="ignore"):
        return T64.astype(np.float16)


def mixed_int8_linear_lora(X, Wq, c, tau, A, B, bias=None, rows=None):
    """The base layer's dict with Y and Y64 replaced by the adapted ones, plus T (fp16 [M, r])."""
    assert B.dtype == np.float16 and B.shape == (Wq.shape[1], A.shape[0])
    out = mixed_linear.mixed_int8_linear(X, Wq, c, tau, bias, rows)
    Xr = X if rows is None else np.ascontiguousarray(X[np.asarray(rows)])
    T = lora_down(Xr, A)
    Y64 = out["Y64"] + T.astype(np.float64) @ B.astype(np.float64).T
    with np.errstate(over="ignore"):
        Y = Y64.astype(np.float16)
    out.update(T=T, Y64=Y64, Y=Y, Y_base=out["Y"], Y64_base=out["Y64"])
    return out
