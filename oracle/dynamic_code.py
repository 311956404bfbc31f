"""The 8-bit signed dynamic code used by the blockwise codec (oracle; test infrastructure).

Section "Compression techniques", item 1 names "dynamic blockwise quantization" without
printing a code table.  The reading taken here is the dynamic (variable-exponent) data type
of the 8-bit-quantization literature written as a closed form:

* a magnitude is ``10**-e * (0.1 + 0.9 * (j + 1/2) / 2**f)`` with a decimal exponent
  ``e = 0..6`` and ``f = 6 - e`` fraction bits, ``j = 0 .. 2**f - 1``; the fraction is the
  midpoint of one of ``2**f`` equal slices of ``[0.1, 1]``.  That is 1+2+...+64 = 127
  magnitudes;
* the table holds the 127 negated magnitudes, an exact 0, the 127 magnitudes and an exact
  +1.0: 256 strictly ascending fp32 values (-1.0 is *not* a code).

Written over a common denominator, a magnitude is the ratio of two integers
``(2**(f+1) + 9*(2j+1)) / (10**(e+1) * 2**(f+1))``; it is evaluated as one float64 division
of two exactly representable integers and then rounded once to fp32.
"""
import numpy as np

N_CODES = 256
ZERO_CODE = 127


def magnitudes() -> np.ndarray:
    """The 127 positive magnitudes, ascending, as float32."""
    vals = []
    for e in range(6, -1, -1):          # smallest decade first -> ascending order
        f = 6 - e
        for j in range(2 ** f):
            num = 2 ** (f + 1) + 9 * (2 * j + 1)
            den = 10 ** (e + 1) * 2 ** (f + 1)
            vals.append(np.float32(np.float64(num) / np.float64(den)))
    out = np.array(vals, dtype=np.float32)
    assert out.shape == (127,)
    return out


def code_table() -> np.ndarray:
    """T[0..255]: fp32, strictly ascending."""
    p = magnitudes()
    t = np.concatenate([-p[::-1], np.zeros(1, np.float32), p, np.ones(1, np.float32)])
    return t.astype(np.float32)


def midpoints(table: np.ndarray | None = None) -> np.ndarray:
    """Mid[j] = fp32((T[j] + T[j+1]) / 2) for j = 0..254 (sum and halving exact in float64)."""
    t = code_table() if table is None else table
    t64 = t.astype(np.float64)
    return ((t64[:-1] + t64[1:]) / 2.0).astype(np.float32)
