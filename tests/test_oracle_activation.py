"""Pins for the oracle's GELU: textbook values of the normal distribution function, identities, brute-force
integration of the normal density, and the layer composition."""
import math

import numpy as np

from oracle import activation as act
from oracle import mixed_linear as ml
from paper_2407_19775_amd import workloads as wl


def all_finite_fp16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = bits.view(np.float16)
    return x[np.isfinite(x)]


def test_textbook_values():
    # Phi(1) = 0.8413447..., Phi(2) = 0.9772499..., Phi(-1) = 0.1586553... (standard normal table)
    x = np.array([0.0, 1.0, 2.0, -1.0, -2.0, 0.5], np.float16)
    want = np.array([0.0, 0.8413447, 2 * 0.9772499, -0.1586553, -2 * 0.0227501, 0.5 * 0.6914625])
    got = act.gelu_fp16(x).astype(np.float64)
    assert np.all(np.abs(got - want) <= np.abs(want) * 2.0 ** -11 + 1e-7)


def test_identities_over_every_fp16_value():
    x = all_finite_fp16()
    g = act.gelu_fp16(x).astype(np.float64)
    gm = act.gelu_fp16(-x).astype(np.float64)
    xf = x.astype(np.float64)
    # gelu(x) - gelu(-x) = x (Phi(x) + Phi(-x)) = x, up to the two roundings
    assert np.all(np.abs(g - gm - xf) <= (np.abs(g) + np.abs(gm)) * 2.0 ** -11 + 2.0 ** -24)
    # x Phi(x) lies between min(x, 0) and max(x, 0); equals x for large x and 0 for very negative x
    assert np.all(g <= np.maximum(xf, 0) + 1e-12) and np.all(g >= np.minimum(xf, 0) - 0.17 - 1e-12)
    assert np.all(g[xf >= 6] == xf[xf >= 6]) and np.all(g[xf <= -13] == 0)
    # the minimum of gelu is about -0.16997 near x = -0.7518 (flat there: several fp16 inputs share the rounded minimum)
    i = np.argmin(g)
    assert abs(xf[i] + 0.7518) < 0.05 and abs(g[i] + 0.16997) < 2e-4
    # monotone increasing to the right of the minimum
    order = np.argsort(xf)
    right = order[xf[order] > -0.75]
    assert np.all(np.diff(g[right]) >= 0)


def test_against_numerical_integration_of_the_normal_density():
    # Phi(x) = 1/2 + integral_0^x exp(-t^2/2)/sqrt(2 pi) dt by Simpson's rule
    for x in (-3.0, -0.3, 0.25, 1.5, 3.25):
        n = 20000
        t = np.linspace(0.0, x, n + 1)
        f = np.exp(-t * t / 2) / math.sqrt(2 * math.pi)
        integral = (x / n) / 3 * (f[0] + f[-1] + 4 * f[1:-1:2].sum() + 2 * f[2:-1:2].sum())
        want = x * (0.5 + integral)
        got = float(act.gelu_fp16(np.array([x], np.float16))[0])
        assert abs(got - want) <= abs(want) * 2.0 ** -11 + 1e-9, (x, got, want)


def test_layer_composition_uses_the_rounded_layer_output():
    rng = np.random.default_rng(0)
    X = wl.to_fp16(rng.standard_normal((6, 64)).astype(np.float32))
    Wq, c = ml.prequantize_weight(wl.to_fp16(rng.standard_normal((64, 24)).astype(np.float32) * 0.2))
    bias = wl.to_fp16(rng.standard_normal(24).astype(np.float32))
    o = act.mixed_int8_linear_gelu(X, Wq, c, 6.0, bias)
    base = ml.mixed_int8_linear(X, Wq, c, 6.0, bias)
    assert np.array_equal(o["Y"].view(np.uint16), base["Y"].view(np.uint16))
    y = base["Y"].astype(np.float64)
    want = np.array([[v * 0.5 * math.erfc(-v / math.sqrt(2.0)) for v in row] for row in y])
    assert np.array_equal(o["G"], want.astype(np.float16))
    assert np.any(o["G"] != base["Y"])
