"""What the reading of the row scale costs in accuracy (CPU only; prints a table).  python -m oracle.study_row_scale

Output error of the int8 layer, as the relative Frobenius distance to the exact product of X with the fp16
weights, for the three row scales of readings.py, for critical weight rows taken from an fp16 master copy instead of the
codes, for the pure 8-bit layer (no critical columns: tau = inf) and
for the fp16 rounding of the exact result alone.  Inputs as in the parity workloads: Gaussian activations with a
few feature dimensions scaled by 8-60 (the prefill recipe), and Student-t(3) activations (the decode recipe)."""
import numpy as np

from . import mixed_linear as ml
from . import readings as rd


def fp16(a):
    return np.clip(a, -65504, 65504).astype(np.float16)


def inputs(kind, M, K, rng):
    if kind == "gaussian + outlier dims":
        x = rng.standard_normal((M, K)).astype(np.float32)
        for k in rng.choice(K, size=max(1, round(0.001 * K)), replace=False):
            x[:, k] *= rng.uniform(8.0, 60.0)
        return fp16(x)
    return fp16(rng.standard_t(3.0, size=(M, K)).astype(np.float32))


def main():
    rng = np.random.default_rng(0)
    M, K, N, tau = 256, 4096, 512, 6.0
    W = fp16(rng.standard_normal((K, N)).astype(np.float32) * 0.02)
    Wq, c = ml.prequantize_weight(W)
    print("%-26s %-22s %12s %14s" % ("activations", "layer", "rel. error", "mean scale r"))
    for kind in ("gaussian + outlier dims", "student-t(3)"):
        X = inputs(kind, M, K, rng)
        exact = X.astype(np.float64) @ W.astype(np.float64)
        norm = np.linalg.norm(exact)
        rows = [("fp16 rounding only", np.linalg.norm(fp16(exact).astype(np.float64) - exact) / norm, float("nan"))]
        for reading in rd.ROW_SCALES:
            o = rd.mixed_int8_linear_with_row_scale(X, Wq, c, tau, reading)
            rows.append(("mixed, r = " + reading, np.linalg.norm(o["Y64"] - exact) / norm, float(o["r"].mean())))
        o = rd.mixed_int8_linear_with_row_scale(X, Wq, c, tau, "sub_threshold", master_W=W)
        rows.append(("mixed, fp16 master rows", np.linalg.norm(o["Y64"] - exact) / norm, float(o["r"].mean())))
        o = rd.mixed_int8_linear_with_row_scale(X, Wq, c, np.inf, "all")
        rows.append(("8-bit only (tau = inf)", np.linalg.norm(o["Y64"] - exact) / norm, float(o["r"].mean())))
        crit = int(ml.outlier_mask(X, tau).sum())
        for name, err, r in rows:
            print("%-26s %-22s %12.3e %14.3f" % (kind, name, err, r))
        print("%-26s critical columns at tau = 6: %d of %d" % (kind, crit, K))


if __name__ == "__main__":
    main()
