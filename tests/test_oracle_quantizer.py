"""Pins of the oracle's quantisation encoder (Section III-D) and its half-precision helpers."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

R = 512


def _adversarial(eb, rng, n=4000):
    e2 = 2.0 * eb
    k = rng.integers(-R - 3, R + 3, n)
    edges = (k + 0.5) * e2                                     # bin edges
    ulp = np.spacing(np.abs(edges).astype(np.float32)).astype(np.float64)
    near = edges + rng.integers(-3, 4, n) * ulp                # a few ulps around every edge
    centre = k * e2
    specials = np.array([0.0, -0.0, np.nan, np.inf, -np.inf, 1e-45, -1e-45, 1.1754942e-38, 3.4e38, -3.4e38,
                         (R - 0.5) * e2, (R - 1) * e2, R * e2, -(R - 0.5) * e2, -R * e2])
    rnd = rng.standard_normal(n) * eb * 40
    return np.concatenate([edges, near, centre, specials, rnd]).astype(np.float32)


@pytest.mark.parametrize("eb", [1e-3, 0.01, 0.03, 0.05, 3.7e-5, 0.5, 1e-30])
def test_bound_holds_on_every_element_f32(eb):
    rng = np.random.default_rng(int(eb * 1e6) % 97)
    x = _adversarial(eb, rng)
    sym, rec = oracle.quantize(x, eb, R)
    eb32 = float(np.float32(eb))
    fin = np.isfinite(x)
    err = np.abs(x[fin].astype(np.float64) - rec[fin].astype(np.float64))
    assert np.all(err <= eb32 * (1 + 1e-6))
    # escapes reproduce the input bit for bit
    esc = sym == 0
    assert np.array_equal(rec[esc].view(np.uint32), x[esc].view(np.uint32))
    assert np.all(esc[~fin])
    assert np.all((sym[~esc] >= 1) & (sym[~esc] <= 2 * R - 1))
    # non-escapes reconstruct to (c - R) * 2eb computed in binary32
    want = (sym[~esc].astype(np.int32) - R).astype(np.float32) * (np.float32(eb) * np.float32(2))
    assert np.array_equal(rec[~esc].view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("eb", [1e-3, 0.02, 0.4])
def test_symbols_against_exact_rational_rounding(eb):
    """Bin = round_half_even(x / (2 eb)) in exact arithmetic, except within a few binary32 ulps of a bin edge."""
    rng = np.random.default_rng(5)
    x = _adversarial(eb, rng, 1500)
    x = x[np.isfinite(x)]
    sym, rec = oracle.quantize(x, eb, R)
    e2 = Fraction(float(np.float32(eb) * np.float32(2)))
    eb_f = Fraction(float(np.float32(eb)))
    n_edge = 0
    for xi, c, ri in zip(x, sym, rec):
        q = Fraction(float(xi)) / e2
        fl = q.numerator // q.denominator
        frac = q - fl
        exact = fl + (1 if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and fl % 2 == 1) else 0)
        dist_to_edge = abs(frac - Fraction(1, 2))
        tol = max(abs(q), 1) * Fraction(4, 2 ** 23)
        if c == 0:
            # escape: out of range, or (rarely) a reconstruction just over the bound at a bin edge
            assert abs(exact) >= R or dist_to_edge <= tol, (xi, exact)
            continue
        got = int(c) - R
        if got != exact:
            n_edge += 1
            assert abs(got - exact) == 1 and dist_to_edge <= tol, (xi, got, exact)
        # the bound holds on the reconstructed value, in exact arithmetic, with no slack at all
        assert abs(Fraction(float(xi)) - Fraction(float(ri))) <= eb_f
        # and the reconstruction is the binary32 product nearest to got * 2eb
        assert abs(Fraction(float(ri)) - got * e2) <= abs(got * e2) * Fraction(1, 2 ** 24)
    assert n_edge < len(x) // 10


def test_special_cases():
    x = np.array([0.0, -0.0, 0.3, -0.3], np.float32)
    sym, rec = oracle.quantize(x, 1.0, R)                      # eb >= max|x| -> every symbol is R
    assert np.all(sym == R) and np.all(rec == 0.0)
    assert not np.signbit(rec[1])                              # -0.0 reconstructs to +0.0
    sym, _ = oracle.quantize(np.array([np.nan, np.inf, -np.inf], np.float32), 0.1, R)
    assert np.all(sym == 0)
    # ties go to the even bin: x = 0.5 * 2eb and 1.5 * 2eb with eb a power of two (exact products)
    eb = 2.0 ** -6
    sym, _ = oracle.quantize(np.array([0.5, 1.5, 2.5, -0.5, -1.5], np.float32) * np.float32(2 * eb), eb, R)
    assert list(sym.astype(int) - R) == [0, 2, 2, 0, -2]
    # range limit: |bin| < R is coded, |bin| >= R escapes
    sym, _ = oracle.quantize(np.array([(R - 1), R, -(R - 1), -R], np.float32) * np.float32(2 * eb), eb, R)
    assert list(sym) == [2 * R - 1, 0, 1, 0]
    # subnormal inputs quantise like any other small value (not flushed to a different symbol)
    sub = np.array([1e-45, -1e-45, 5e-39], np.float32)
    sym, rec = oracle.quantize(sub, 1e-3, R)
    assert np.all(sym == R)
    sym, rec = oracle.quantize(sub, 2e-45, R)                  # bound itself subnormal
    assert np.all(np.abs(sub.astype(np.float64) - rec.astype(np.float64)) <= float(np.float32(2e-45)) * (1 + 1e-6))


def test_half_to_float_all_values():
    h = np.arange(65536, dtype=np.uint16)
    want = h.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(v)) for v in h], np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_float_to_half_matches_numpy_rne():
    rng = np.random.default_rng(11)
    h = np.arange(65536, dtype=np.uint16).view(np.float16).astype(np.float32)
    h = h[np.isfinite(h)]
    mid = ((h[:-1].astype(np.float64) + np.sort(h)[1:].astype(np.float64)) / 2).astype(np.float32)
    hs = np.sort(h)
    mids = ((hs[:-1].astype(np.float64) + hs[1:].astype(np.float64)) / 2).astype(np.float32)   # exact ties
    around = np.concatenate([np.nextafter(mids, np.float32(np.inf)), np.nextafter(mids, np.float32(-np.inf))])
    rnd = (rng.standard_normal(20000) * 10.0 ** rng.uniform(-9, 5, 20000)).astype(np.float32)
    x = np.concatenate([h, mid, mids, around, rnd, np.array([65504, 65519.99, 65520, 1e6, -1e6, 2.0 ** -25,
                                                              np.nextafter(np.float32(2.0 ** -25), np.float32(1)),
                                                              2.0 ** -24, np.inf, -np.inf], np.float32)])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.float_to_half(float(v)) for v in x], np.uint16)
    assert np.array_equal(got, want)
    assert (oracle.float_to_half(float("nan")) & 0x7C00) == 0x7C00 and (oracle.float_to_half(float("nan")) & 0x3FF)


@pytest.mark.parametrize("rel", [2.0 ** -10, 2.0 ** -8])
def test_bound_holds_on_every_element_f16(rel):
    rng = np.random.default_rng(3)
    x = rng.laplace(0, 0.05, 20000).astype(np.float16)
    x[:6] = np.array([0.0, -0.0, np.nan, np.inf, 6e-8, 65504], np.float16)
    fin = np.isfinite(x)
    eb = float(np.float32(rel * (float(x[fin & (np.abs(x) < 100)].max()) - float(x[fin].min()))))
    sym, rec = oracle.quantize(x, eb, R)
    assert rec.dtype == np.float16
    err = np.abs(x[fin].astype(np.float64) - rec[fin].astype(np.float64))
    assert np.all(err <= float(np.float32(eb)) * (1 + 1e-6))
    esc = sym == 0
    assert np.array_equal(rec[esc].view(np.uint16), x[esc].view(np.uint16))
    want = ((sym[~esc].astype(np.int32) - R).astype(np.float32) * (np.float32(eb) * np.float32(2))).astype(np.float16)
    assert np.array_equal(rec[~esc].view(np.uint16), want.view(np.uint16))
    # half precision rounding of the reconstruction makes bin-edge escapes a visible fraction
    assert 0 < esc.mean() < 0.5


# bounds (binary32 bit patterns) for which some bin centre r * 2eb, rounded to binary32, lands exactly half way between
# two binary16 numbers while the exact product does not: rounding the product to binary16 in one step (what a fused
# multiply-convert instruction does) gives another reconstruction than binary32-then-binary16
TIE_BOUNDS = [1037035110, 994589847, 1009301586, 1050593819, 982489498]


def half_tie_payload():
    """every finite binary16 value in [-2, 2], one table per bound"""
    pos = np.arange(0, 0x4001, dtype=np.uint16)
    vals = np.concatenate([pos, pos | np.uint16(0x8000)]).view(np.float16)
    n = 514 * 64
    x = np.zeros((len(TIE_BOUNDS), n), np.float16)
    x[:, :vals.size] = vals
    ebs = np.array(TIE_BOUNDS, np.uint32).view(np.float32)
    return x.reshape(len(TIE_BOUNDS), 514, 64), ebs


def test_f16_reconstruction_is_rounded_twice():
    """Section III-D fixes no number format; the reading taken is: bin centre as a binary32 product, then rounded to
    binary16 (ties to even).  The oracle must follow it where the one-step rounding differs, and the symbol decision
    (inside the bound or escape) must be the one that reading gives."""
    x, ebs = half_tie_payload()
    differ = 0
    for t, eb in enumerate(ebs):
        sym, rec = oracle.quantize(x[t:t + 1], float(eb), R)
        xs = x[t].reshape(-1).astype(np.float32)
        ebx2 = np.float32(eb * np.float32(2))
        inv = np.float32(1.0 / np.float64(ebx2))
        r = np.rint((xs * inv).astype(np.float32)).astype(np.float32)
        two = (r * ebx2).astype(np.float32).astype(np.float16)                       # the reading
        one = (r.astype(np.float64) * np.float64(ebx2)).astype(np.float16)           # a fused multiply-convert
        ok = (np.abs(r) < R) & (np.abs(xs - two.astype(np.float32)) <= eb)
        want = np.where(ok, r.astype(np.int32) + R, 0).astype(np.uint16)
        assert np.array_equal(sym.reshape(-1), want)
        got = rec.reshape(-1)
        ri = (want.astype(np.int32) - R).astype(np.float32)      # what the decoder sees (bin 0 gives +0.0)
        two_dec = (ri * ebx2).astype(np.float32).astype(np.float16)
        assert np.array_equal(got[ok].view(np.uint16), two_dec[ok].view(np.uint16))
        ok1 = (np.abs(r) < R) & (np.abs(xs - one.astype(np.float32)) <= eb)
        differ += int(np.count_nonzero(ok != ok1))
    assert differ > 0          # the case separates the two definitions
