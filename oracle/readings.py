"""Alternative readings of the int8 layer (oracle; test infrastructure; CPU only).

"Compression techniques", item 2, keeps "a small fraction of critical weights at 16-bit precision" and says no
more about how the 8-bit part is scaled.  The library scales a row by the largest magnitude below the threshold
(mixed_linear.row_absmax).  Two other readings are written out here so that what the choice costs can be
measured and the library's switchable variants of them can be checked.

  sub_threshold   r[m] = max{ |X[m,k]| : |X[m,k]| < tau }                  the library's reading
  non_critical    r[m] = max{ |X[m,k]| : column k not critical }           needs the flags of all rows first
  all             r[m] = max_k |X[m,k]|                                     plain row absmax: outliers set the scale

And two readings of where the 16-bit weights of the critical dimensions come from:

  dequantized     f16(Wq[k,n] c[n] / 127) re-created from the 8-bit codes      the library's reading: 1 byte per weight
  master          the original fp16 W[k,n]                                     needs a second, fp16 copy of W (3 bytes)

Entries of a critical column never reach the 8-bit product, so the first two differ only through
sub-threshold entries that sit in critical columns: non_critical <= sub_threshold <= all, elementwise.
"""
import numpy as np

from . import mixed_linear as ml

ROW_SCALES = ("sub_threshold", "non_critical", "all")


def row_scale(X: np.ndarray, tau: float, reading: str) -> np.ndarray:
    assert X.dtype == np.float16 and reading in ROW_SCALES
    ax = np.abs(X.astype(np.float32))
    if reading == "sub_threshold":
        return ml.row_absmax(X, tau)
    if reading == "all":
        return np.max(ax, axis=1, initial=np.float32(0.0)).astype(np.float32)
    keep = ~ml.outlier_mask(X, tau)
    return np.max(ax[:, keep], axis=1, initial=np.float32(0.0)).astype(np.float32)


def mixed_int8_linear_with_row_scale(X, Wq, c, tau, reading, bias=None, master_W=None):
    """The layer of mixed_linear.mixed_int8_linear with the row scale of `reading`; same steps otherwise
    (codes, exact integer product, outer-product dequantization, fp16 product on the critical columns).
    master_W: the original fp16 weights [K, N]; if given, their rows multiply the critical columns."""
    flag = ml.outlier_mask(X, tau)
    r = row_scale(X, tau, reading)
    Xq = ml.quantize_activations(X, flag, r)
    acc = ml.int_gemm(Xq, Wq)
    Y64 = acc.astype(np.float64) * r.astype(np.float64)[:, None] * c.astype(np.float64)[None, :] / 16129.0
    idx = np.flatnonzero(flag)
    if idx.size:
        Wt = ml.dequantized_weight_fp16(Wq[idx, :], c) if master_W is None else master_W[idx, :]
        assert Wt.dtype == np.float16
        Y64 = Y64 + X[:, idx].astype(np.float64) @ Wt.astype(np.float64)
    if bias is not None:
        Y64 = Y64 + bias.astype(np.float64)[None, :]
    with np.errstate(over="ignore"):
        return dict(flag=flag, r=r, Xq=Xq, acc=acc, Y64=Y64, Y=Y64.astype(np.float16))
