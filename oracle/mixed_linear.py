"""Mixed-matrix-decomposition int8 linear layer (oracle; test infrastructure).

Section "Compression techniques", item 2: weights are held as 8-bit values and a small fraction
of critical entries is kept at 16-bit precision.  The paper gives no equations; the reading
implemented here, step by step (X is [M, K] fp16, W is [K, N] fp16, Y = X W is [M, N] fp16):

weights, once per matrix
  W1  c[n]    = max_k |f32(W[k, n])|                                    (exact)
  W2  sw[n]   = 127.0f / c[n]  (fp32 division; 0 when c[n] == 0)
      Wq[k,n] = clamp(rint(f32(W[k, n]) * sw[n]), -127, 127)             (fp32 product, ties to even)

activations, per call
  A1  flag[k] = any_m ( |f32(X[m, k])| >= tau )                          (a feature dimension is
                                                                          critical if any token exceeds tau)
  A2  r[m]    = max( {0} u { |f32(X[m, k])| : |f32(X[m, k])| < tau } )   (row scale from sub-threshold entries)
  A3  sx[m]   = 127.0f / r[m]  (0 when r[m] == 0)
      Xq[m,k] = 0 if flag[k] else clamp(rint(f32(X[m, k]) * sx[m]), -127, 127)
  A4  acc[m,n]= sum_k int(Xq[m, k]) * int(Wq[k, n])                      (exact integer sum)
  A5  Yi[m,n] = acc[m, n] * r[m] * c[n] / 127**2                         (outer-product dequantization)
      Wt[k,n] = f16( f32(Wq[k, n]) * (c[n] / 127.0f) )                   (16-bit weights of critical rows)
      Yo[m,n] = sum_{k : flag[k]} X[m, k] * Wt[k, n]                     (fp16 operands, exact products)
      Y[m,n]  = f16( Yi + Yo + bias[n] )                                 (one final rounding)

A5 is evaluated in float64; A1..A3 and W1..W2 in fp32 exactly as written.  The integer sum A4
is defined by the triple loop; it is evaluated here with a float64 matrix product, which is
exact because every partial sum is an integer below K * 127**2 <= 2**31 << 2**53.
"""
import numpy as np

INT32_SAFE_K = (2 ** 31 - 1) // (127 * 127)      # largest K whose accumulators cannot overflow int32


def _f32(a):
    return np.asarray(a).astype(np.float32)


def _scale_to_127(absmax: np.ndarray) -> np.ndarray:
    """127.0f / absmax as an fp32 division, 0 where absmax is 0."""
    absmax = _f32(absmax)
    q = np.float32(127.0)
    with np.errstate(divide="ignore"):
        return np.where(absmax == 0, np.float32(0.0), q / absmax).astype(np.float32)


def _to_int8(scaled: np.ndarray) -> np.ndarray:
    assert scaled.dtype == np.float32
    return np.clip(np.rint(scaled), -127, 127).astype(np.int8)


# ---------------------------------------------------------------- weights (W1, W2)
def prequantize_weight(W: np.ndarray):
    """W fp16 [K, N] -> (Wq int8 [K, N], c float32 [N])."""
    assert W.dtype == np.float16 and W.ndim == 2
    w32 = _f32(W)
    c = np.max(np.abs(w32), axis=0).astype(np.float32) if W.shape[0] else np.zeros(W.shape[1], np.float32)
    sw = _scale_to_127(c)
    prod = w32 * sw[None, :]
    assert prod.dtype == np.float32
    return _to_int8(prod), c


def dequantized_weight_fp16(Wq: np.ndarray, c: np.ndarray) -> np.ndarray:
    """Wt[k, n] = f16( f32(Wq[k, n]) * (c[n] / 127.0f) )."""
    step = (_f32(c) / np.float32(127.0)).astype(np.float32)
    prod = Wq.astype(np.float32) * step[None, :]
    assert prod.dtype == np.float32
    return prod.astype(np.float16)


# ---------------------------------------------------------------- activations (A1..A3)
def outlier_mask(X: np.ndarray, tau: float) -> np.ndarray:
    assert X.dtype == np.float16 and X.ndim == 2
    ax = np.abs(_f32(X))
    return np.any(ax >= np.float32(tau), axis=0) if X.shape[0] else np.zeros(X.shape[1], bool)


def row_absmax(X: np.ndarray, tau: float) -> np.ndarray:
    ax = np.abs(_f32(X))
    sub = np.where(ax < np.float32(tau), ax, np.float32(0.0))
    return np.max(sub, axis=1, initial=np.float32(0.0)).astype(np.float32)


def quantize_activations(X: np.ndarray, flag: np.ndarray, r: np.ndarray) -> np.ndarray:
    sx = _scale_to_127(r)
    prod = _f32(X) * sx[:, None]
    assert prod.dtype == np.float32
    xq = _to_int8(prod)
    xq[:, flag] = 0
    return xq


# ---------------------------------------------------------------- integer GEMM (A4)
def int_gemm(Xq: np.ndarray, Wq: np.ndarray) -> np.ndarray:
    assert Xq.dtype == np.int8 and Wq.dtype == np.int8
    K = Xq.shape[1]
    assert K == Wq.shape[0] and K <= INT32_SAFE_K
    acc = Xq.astype(np.float64) @ Wq.astype(np.float64)
    out = acc.astype(np.int64)
    assert np.all(out == acc)
    return out.astype(np.int32)


# ---------------------------------------------------------------- whole layer
def mixed_int8_linear(X, Wq, c, tau, bias=None, rows=None):
    """Returns a dict with every intermediate: flag, outlier_idx, r, Xq, acc, Y (fp16) and the
    float64 value Y64 before the final rounding.

    rows: optional index array.  The critical-dimension mask is always taken over every row of
    X (step A1); with ``rows`` given, the per-row quantities (r, Xq, acc, Y) are produced for
    those rows only, which is how full-size problems are spot-checked."""
    assert X.dtype == np.float16 and Wq.dtype == np.int8 and c.dtype == np.float32
    flag = outlier_mask(X, tau)
    if rows is not None:
        X = np.ascontiguousarray(X[np.asarray(rows)])
    M, K = X.shape
    N = Wq.shape[1]
    r = row_absmax(X, tau)
    Xq = quantize_activations(X, flag, r)
    acc = int_gemm(Xq, Wq)
    Yi = acc.astype(np.float64) * r.astype(np.float64)[:, None] * c.astype(np.float64)[None, :] / 16129.0
    idx = np.flatnonzero(flag)
    if idx.size:
        Wt = dequantized_weight_fp16(Wq[idx, :], c)
        Yo = X[:, idx].astype(np.float64) @ Wt.astype(np.float64)
    else:
        Yo = np.zeros((M, N), np.float64)
    Y64 = Yi + Yo
    if bias is not None:
        assert bias.dtype == np.float16 and bias.shape == (N,)
        Y64 = Y64 + bias.astype(np.float64)[None, :]
    with np.errstate(over="ignore"):
        Y = Y64.astype(np.float16)
    return dict(flag=flag, outlier_idx=idx.astype(np.int32), r=r, Xq=Xq, acc=acc, Y=Y, Y64=Y64)


def linear_from_fp16_weight(X, W, tau, bias=None, rows=None):
    """Convenience: pre-quantize W (W1, W2) then run the layer."""
    Wq, c = prequantize_weight(W)
    out = mixed_int8_linear(X, Wq, c, tau, bias, rows)
    out["Wq"], out["c"] = Wq, c
    return out
