"""Pins for the oracle's quantiser (constants, pre-quantisation, de-quantisation).

What fixes the expected values here, independently of the oracle's own code:
exact rational arithmetic (fractions) for the fp32 constants; the error-bound
guarantee of Section 2.2 checked in fp64; zero and sign preservation
(Sections 3.2 and 4.4); the uniform error model of Section 3.1.
"""
from fractions import Fraction

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

EBS = [1e-1, 1e-2, 5e-3, 1e-3, 1e-4]


def round_fraction_to_f32(v: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) binary32 value of a positive rational."""
    assert v > 0
    e = 0
    while v >= 2:
        v /= 2; e += 1
    while v < 1:
        v *= 2; e -= 1
    m = v * (1 << 23)                      # in [2^23, 2^24)
    fl = m.numerator // m.denominator
    rem = m - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    assert -126 <= e <= 126                # normal range only
    return np.float32(float(Fraction(fl, 1 << 23) * Fraction(2) ** e))


@pytest.mark.parametrize("eb", EBS + [0.5, 3.0, 2.0 ** -40, 2.0 ** 40])
def test_constants_match_exact_rational_arithmetic(orc, eb):
    eb32 = np.float32(eb)
    E = Fraction(float(eb32))
    eb_in = round_fraction_to_f32(E - E / 128)
    s = round_fraction_to_f32(2 * Fraction(float(eb_in)))
    r = round_fraction_to_f32(1 / Fraction(float(s)))
    rc, o_eb_in, o_s, o_r = orc.constants(eb32, 7)
    assert rc == 0
    assert (o_eb_in, o_s, o_r) == (eb_in, s, r)
    assert float(o_s) == 2 * float(o_eb_in)          # doubling is exact
    assert float(o_eb_in) < float(eb32)


def test_constants_reject_bad_eb(orc):
    for bad in [0.0, -1e-2, float("nan"), float("inf"), 2.0 ** -61, 2.0 ** 61]:
        assert orc.constants(bad, 7)[0] == orc.E_ARG
    assert orc.constants(1e-2, 0)[0] == orc.E_ARG
    assert orc.constants(1e-2, 24)[0] == orc.E_ARG


def adversarial_values(s: np.float32) -> np.ndarray:
    """Quantiser midpoints (k+1/2)s, grid points k*s, each +-{0,1,2} ulp, both signs,
    plus zeros, denormals and the edge of the representable range."""
    k = np.arange(0, 16385, dtype=np.float64)
    base = np.concatenate([(k + 0.5) * float(s), k * float(s)]).astype(np.float32)
    outs = [base]
    up = base.copy(); dn = base.copy()
    for _ in range(2):
        up = np.nextafter(up, np.float32(np.inf)); dn = np.nextafter(dn, np.float32(-np.inf))
        outs += [up.copy(), dn.copy()]
    v = np.concatenate(outs)
    v = np.concatenate([v, -v, np.array([0.0, -0.0, 1e-45, -1e-45, 1e-39, -1e-39], np.float32)])
    return v


@pytest.mark.parametrize("eb", EBS)
def test_error_bound_zero_and_sign_on_adversarial_values(orc, eb):
    rc, eb_in, s, r = orc.constants(eb)
    x = adversarial_values(s)
    q, events = orc.prequant(x, r)
    xr = (x * r)                                                   # the fp32 product the oracle sees
    inside = np.abs(xr) <= np.float32(16384.0)
    assert events == int((~inside).sum())
    xp = orc.dequant(q, s)
    err = np.abs(x.astype(np.float64) - xp.astype(np.float64))
    assert err[inside].max() <= float(np.float32(eb))              # Section 2.2: absolute bound
    assert np.all(np.abs(q) <= 16384)
    zero = x == 0
    assert np.all(xp[zero].view(np.uint32) == 0)                   # zeros stay +0.0 exactly
    assert np.all(x.astype(np.float64) * xp.astype(np.float64) >= 0)   # sign never flips
    assert not np.any(np.signbit(xp[q == 0]))


@settings(max_examples=40, deadline=None)
@given(st.floats(min_value=2.0 ** -30, max_value=2.0 ** 20, allow_nan=False), st.integers(0, 2 ** 31))
def test_error_bound_random_eb(orc, eb, seed):
    eb32 = np.float32(eb)
    rc, eb_in, s, r = orc.constants(eb32)
    assert rc == 0
    rng = np.random.default_rng(seed)
    x = (rng.uniform(-16000, 16000, 20000) * float(s)).astype(np.float32)
    q, events = orc.prequant(x, r)
    assert events == 0
    xp = orc.dequant(q, s)
    assert np.abs(x.astype(np.float64) - xp.astype(np.float64)).max() <= float(eb32)


def test_out_of_range_nan_inf_are_clamped_and_counted(orc):
    rc, eb_in, s, r = orc.constants(1e-2)
    big = np.float32(16384.75) * s
    x = np.array([np.nan, np.inf, -np.inf, 1e30, -1e30, big, -big, 0.0, 1.0], dtype=np.float32)
    q, events = orc.prequant(x, r)
    assert list(q[:7]) == [0, 16384, -16384, 16384, -16384, 16384, -16384]
    assert events == 7
    assert q[7] == 0 and abs(q[8] - round(1.0 / float(s))) <= 1


def test_round_half_to_even(orc):
    # with s = 1 exactly (eb_in = 0.5 is not reachable; use r directly) ties must go to even
    x = np.array([0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 1e-30], dtype=np.float32)
    q, _ = orc.prequant(x, np.float32(1.0))
    assert list(q) == [0, 2, 2, 4, 0, -2, -2, 0]


@pytest.mark.parametrize("eb", EBS)
def test_quantiser_fixed_point(orc, eb):
    """Every reconstructed value q*s quantises back to q: recompression is lossless."""
    rc, eb_in, s, r = orc.constants(eb)
    q = np.arange(-16384, 16385, dtype=np.int32)
    x = orc.dequant(q, s)
    q2, events = orc.prequant(x, r)
    assert events == 0
    assert np.array_equal(q2, q)
    assert np.array_equal(orc.dequant(q2, s).view(np.uint32), x.view(np.uint32))


def test_dequant_is_single_rounded_product(orc):
    rc, eb_in, s, r = orc.constants(1e-3)
    q = np.arange(-16384, 16385, dtype=np.int32)
    x = orc.dequant(q, s)
    exact = [Fraction(int(k)) * Fraction(float(s)) for k in q[::257]]
    want = [float(round_fraction_to_f32(abs(e))) * (1 if e > 0 else -1) if e != 0 else 0.0 for e in exact]
    assert [float(v) for v in x[::257]] == want


def test_error_is_uniform_on_nonzero_inputs(orc):
    """Section 3.1: the error of the linear-scaling quantiser is uniform on [-eb, +eb]
    (here eb_in): mean 0, variance eb_in^2/3, flat histogram."""
    eb = 1e-2
    rc, eb_in, s, r = orc.constants(eb)
    rng = np.random.default_rng(7)
    x = rng.uniform(0.5, 4.0, 400000).astype(np.float32)
    q, _ = orc.prequant(x, r)
    e = orc.dequant(q, s).astype(np.float64) - x.astype(np.float64)
    h = float(eb_in)
    assert abs(e.mean()) < 0.01 * h
    assert abs(e.var() / (h * h / 3) - 1) < 0.02
    hist, _ = np.histogram(e, bins=20, range=(-h, h))
    assert hist.sum() >= 0.999 * e.size
    assert hist.min() > 0.9 * e.size / 20 and hist.max() < 1.1 * e.size / 20
