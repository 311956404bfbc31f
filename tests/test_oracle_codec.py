"""Pins for the blockwise-codec oracle: closed forms, hand-worked values, brute force, bounds."""
import numpy as np
import pytest

from oracle import blockwise_codec as bc
from oracle import dynamic_code as dc


def all_finite_fp16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = bits.view(np.float16)
    return x[np.isfinite(x)]


def test_table_closed_form_facts(golden):
    g = golden("dynamic_code_facts.txt")
    T = dc.code_table()
    assert T.dtype == np.float32 and T.size == int(g["n_codes"][0])
    assert dc.magnitudes().size == int(g["n_magnitudes"][0])
    assert np.all(np.diff(T.astype(np.float64)) > 0)
    for i, v in zip(g["index"].astype(int), g["value"]):
        assert T[i] == np.float32(v), (i, T[i], v)
    # mirrored magnitudes: index(-t) = 254 - index(t); only +1.0 has no mirror
    assert np.array_equal(T[:127], -T[254:127:-1])
    assert T[int(g["zero_index"][0])] == 0 and T[255] == 1 and T[0] > -1
    gaps = np.diff(T.astype(np.float64))
    assert gaps.max() == pytest.approx(g["largest_gap"][0], rel=1e-5)
    # bracket e starts at 128 + 2^f - 1 and holds 2^f equally spaced values
    for e, first in zip(g["bracket_e"].astype(int), g["bracket_first_index"].astype(int)):
        f = 6 - e
        assert first == 128 + 2 ** f - 1
        vals = T[first:first + 2 ** f].astype(np.float64)
        assert vals[0] >= 10.0 ** (-e - 1) and vals[-1] <= 10.0 ** (-e)
        if f:
            assert np.allclose(np.diff(vals), 0.9 * 10.0 ** (-e) / 2 ** f, rtol=1e-5)


def test_table_values_against_decimal_arithmetic():
    """Every magnitude equals 10^-e (0.1 + 0.9 (j+1/2)/2^f) evaluated with exact rationals."""
    from fractions import Fraction
    p = dc.magnitudes()
    i = 0
    for e in range(6, -1, -1):
        f = 6 - e
        for j in range(2 ** f):
            exact = Fraction(1, 10 ** e) * (Fraction(1, 10) + Fraction(9, 10) * Fraction(2 * j + 1, 2 ** (f + 1)))
            assert abs(Fraction(float(p[i])) - exact) <= abs(exact) * Fraction(1, 2 ** 24)
            i += 1
    assert i == 127


def test_midpoints_are_between_neighbours():
    T, Mid = dc.code_table(), dc.midpoints()
    assert Mid.size == 255 and Mid.dtype == np.float32
    assert np.all(Mid > T[:-1]) and np.all(Mid < T[1:])
    exact = (T[:-1].astype(np.float64) + T[1:].astype(np.float64)) / 2
    assert np.all(np.abs(Mid.astype(np.float64) - exact) <= np.abs(exact) * 2.0 ** -24)


def test_worked_example(golden):
    g = golden("codec_worked_example.txt")
    B = int(g["block"][0])
    x = g["x"].astype(np.float16)
    codes, a = bc.quantize_blockwise(x, B)
    assert np.array_equal(codes, g["codes"].astype(np.uint8))
    assert np.array_equal(a, g["absmax"].astype(np.float32))
    dec = bc.dequantize_blockwise(codes, a, B)
    assert np.array_equal(dec, g["decoded"].astype(np.float32).astype(np.float16))
    codes2, a2 = bc.quantize_blockwise(dec, B)
    assert np.array_equal(codes2, codes) and np.array_equal(a2, a)
    # block whose maximum is negative: -1.0 is not a code, the decoded absmax shrinks
    xn = g["neg_x"].astype(np.float16)
    cn, an = bc.quantize_blockwise(xn, B)
    assert np.array_equal(cn, g["neg_codes"].astype(np.uint8)) and an[0] == g["neg_absmax"][0]
    dn = bc.dequantize_blockwise(cn, an, B)
    assert np.array_equal(dn, g["neg_decoded"].astype(np.float32).astype(np.float16))
    _, an2 = bc.quantize_blockwise(dn, B)
    assert an2[0] == np.float32(g["neg_reencoded_absmax"][0])


@pytest.mark.parametrize("a", [65504.0, 1.0, 3.0, 0.0123, 777.5, 6.1e-5])
def test_code_is_nearest_table_entry_brute_force(a):
    """Brute force over every finite fp16 value with |x| <= a: the code is the float64 argmin of
    |v - T[j]|, except where the two best distances differ by less than 2^-29 (the midpoint is
    rounded to fp32, so a float64 near-tie may legitimately resolve either way)."""
    a16 = np.float16(a)
    x = all_finite_fp16()
    x = x[np.abs(x.astype(np.float32)) <= np.float32(a16)]
    block = x.size + 1
    xs = np.concatenate([x, np.array([a16], np.float16)])           # force absmax = a16
    codes, am = bc.quantize_blockwise(xs, block)
    assert am.size == 1 and am[0] == np.float32(a16)
    inv = np.float32(1.0) / np.float32(a16)
    v = (xs.astype(np.float32) * inv).astype(np.float64)
    T = dc.code_table().astype(np.float64)
    d = np.abs(v[:, None] - T[None, :])
    best = np.argmin(d, axis=1)                                     # first minimum = lower index
    bad = np.flatnonzero(best != codes)
    dist_best = d[bad, best[bad]]
    dist_code = d[bad, codes[bad].astype(np.int64)]
    assert np.all(np.abs(dist_best - dist_code) <= 2.0 ** -29), bad[:10]
    assert bad.size <= 4


def test_strict_tie_goes_to_lower_index():
    Mid = dc.midpoints()
    # v exactly on a midpoint that is representable in fp16 scale: use a = 1 and x = Mid if fp16-exact
    exact = [j for j in range(255) if np.float32(np.float16(Mid[j])) == Mid[j]]
    assert exact, "no fp16-representable midpoint to test ties with"
    for j in exact:
        x = np.array([Mid[j], 1.0], np.float32).astype(np.float16)
        codes, _ = bc.quantize_blockwise(x, 2)
        assert codes[0] == j


@pytest.mark.parametrize("block", [64, 256, 1000, 4096])
def test_error_bound_and_exact_points(block):
    rng = np.random.default_rng(block)
    n = 5 * block + 37                                              # ragged tail
    x = (rng.standard_t(3, n) * rng.choice([1e-3, 1.0, 50.0], n)).astype(np.float32)
    x[rng.integers(0, n, 20)] = 0
    x = np.clip(x, -65504, 65504).astype(np.float16)
    codes, a = bc.quantize_blockwise(x, block)
    assert codes.size == n and a.size == 6
    dec = bc.dequantize_blockwise(codes, a, block).astype(np.float64)
    xa = x.astype(np.float64)
    a_el = np.repeat(a.astype(np.float64), block)[:n]
    ulp16 = np.maximum(np.abs(xa), 2.0 ** -14) * 2.0 ** -10
    assert np.all(np.abs(dec - xa) <= a_el * 0.00703125 * (1 + 2.0 ** -10) + ulp16)
    assert np.all(dec[xa == 0] == 0)
    for b in range(a.size):                                         # a positive block maximum is exact
        seg = slice(b * block, min((b + 1) * block, n))
        pos_max = xa[seg] == a[b]
        assert np.all(dec[seg][pos_max] == a[b])
        # absmax really is the block's largest magnitude
        assert a[b] == np.abs(xa[seg]).max()


def test_round_trip_of_codes_invariant():
    """quantize(dequantize(q)) == q when every block holds a 255 and absmax >= 0.25."""
    rng = np.random.default_rng(7)
    block, nblk = 128, 40
    q = rng.integers(0, 256, size=block * nblk).astype(np.uint8)
    q[np.arange(nblk) * block + rng.integers(0, block, nblk)] = 255
    a = rng.uniform(0.25, 1000.0, nblk).astype(np.float16).astype(np.float32)
    x = bc.dequantize_blockwise(q, a, block)
    q2, a2 = bc.quantize_blockwise(x, block)
    assert np.array_equal(a2, a)
    assert np.array_equal(q2, q)


def test_zero_block_and_short_last_block():
    x = np.zeros(10, np.float16)
    x[8] = -0.0
    x[9] = 2.0
    codes, a = bc.quantize_blockwise(x, 8)
    assert np.array_equal(a, np.array([0, 2], np.float32))
    assert np.all(codes[:9] == dc.ZERO_CODE) and codes[9] == 255
    dec = bc.dequantize_blockwise(codes, a, 8)
    assert np.array_equal(dec, np.array([0] * 9 + [2], np.float16))
    c0, a0 = bc.quantize_blockwise(np.zeros(0, np.float16), 64)
    assert c0.size == 0 and a0.size == 0


def test_compression_ratio_halves_the_bytes():
    """The paper's claim that the codec halves the bandwidth: (1 + 4/B) / 2."""
    n = 8192 * 8192
    assert bc.compressed_fraction(n, 256) == 0.5078125
    assert bc.compressed_fraction(n, 1024) == 0.501953125
    assert bc.compressed_fraction(n, 4096) == 0.50048828125
    assert bc.compressed_fraction(16 * 1024, 2048) == pytest.approx(0.5009765625)
    x = np.ones(n // 4096, np.float16)
    codes, a = bc.quantize_blockwise(x, 256)
    assert (codes.nbytes + a.nbytes) / x.nbytes == 0.5078125


def test_monotone_and_power_of_two_scale_invariant():
    rng = np.random.default_rng(3)
    x = np.sort(rng.standard_normal(512).astype(np.float16))
    codes, a = bc.quantize_blockwise(x, 512)
    assert np.all(np.diff(codes.astype(int)) >= 0)
    for j in (-3, 2, 5):
        cs, as_ = bc.quantize_blockwise((x.astype(np.float32) * 2.0 ** j).astype(np.float16), 512)
        assert as_[0] == a[0] * 2.0 ** j
        # scaling by 2^j is exact unless a value drops into the fp16 subnormal range
        normal = np.abs(x.astype(np.float32)) * 2.0 ** min(j, 0) >= 2.0 ** -14
        assert np.array_equal(cs[normal], codes[normal])


def test_block_scales_are_fp16_numbers():
    # a block's absmax is the magnitude of one of its fp16 elements: keeping it in 2 bytes instead of 4 would
    # lose nothing (the library stores fp32; the note in the design document gives the byte counts)
    rng = np.random.default_rng(11)
    x = (rng.standard_t(3.0, size=5000) * 7.0).astype(np.float16)
    _, a = bc.quantize_blockwise(x, 64)
    assert np.array_equal(a, a.astype(np.float16).astype(np.float32))


def test_fp16_scales_change_nothing_but_the_bytes():
    """The other storage of the block scales (2 bytes each): the scales are the same numbers, the codes are the
    same, decoding from them gives the same values, and the hand-worked example of the golden file still holds."""
    rng = np.random.default_rng(12)
    for n, block in [(5000, 64), (4096, 256), (70000, 4096), (130, 128)]:
        x = (rng.standard_t(3.0, size=n) * rng.uniform(0.01, 300.0)).astype(np.float16)
        x[rng.integers(0, n, 5)] = 0
        c32, a32 = bc.quantize_blockwise(x, block)
        c16, a16 = bc.quantize_blockwise(x, block, fp16_scales=True)
        assert a16.dtype == np.float16 and a16.nbytes * 2 == a32.nbytes
        assert np.array_equal(c16, c32) and np.array_equal(a16.astype(np.float32), a32)
        # the scale is the largest magnitude of the block, read straight off the fp16 data
        full = np.abs(x[: n // block * block].reshape(-1, block)).max(axis=1)
        assert np.array_equal(a16[: n // block], full)
        assert np.array_equal(bc.dequantize_blockwise(c16, a16, block), bc.dequantize_blockwise(c32, a32, block))
    g = np.array([1, -0.5, 0.25, 0, -3, 0.003, 1.5, 3], dtype=np.float16)        # the worked example of the codec, blocks of 4
    codes, a = bc.quantize_blockwise(g, 4, fp16_scales=True)
    assert codes.tolist() == [255, 35, 201, 127, 0, 142, 219, 255] and a.tolist() == [1.0, 3.0]
    assert bc.compressed_fraction(1 << 20, 256, scale_bytes=2) == (1 + 2 / 256) / 2
    assert bc.compressed_fraction(1 << 20, 4096, scale_bytes=2) == (1 + 2 / 4096) / 2
