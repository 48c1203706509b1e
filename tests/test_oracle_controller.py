"""Pins for the oracle's error-bound estimator (Sections 4.1-4.3; Eq. 5, 7, 8, 9)."""
import numpy as np
import pytest


def test_closed_form_with_powers_of_two(orc):
    """Every quantity a power of two, so the expected value is exact and needs no formula of its own:
    Mavg = 32, sigma_frac = 2^-7 -> sigma = 1/4; a = 1/4, Lbar = 2, N = 16, R = 1/4 -> denominator
    1/4 * 2 * sqrt(4) = 1; eb = 1/4."""
    act = np.zeros((16, 1, 4, 4), np.float32)
    act.reshape(-1)[::4] = 3.0                                   # one element in four is non-zero
    loss = np.zeros((16, 8), np.float32)
    loss[:, 3] = -2.0                                            # largest magnitude of every sample
    loss[:, 5] = 1.0
    mom = np.full(1000, -32.0, np.float32)
    rc, eb, (R, Lbar, Mavg) = orc.estimate_eb(act, loss, mom, sigma_frac=2.0 ** -7, a=0.25, eb_min=2.0 ** -20,
                                              eb_max=8.0)
    assert rc == 0 and (R, Lbar, Mavg) == (0.25, 2.0, 32.0)
    assert eb == np.float32(0.25)


def test_paper_constants_on_a_unit_case(orc):
    """sigma = 0.01 * Mavg (Eq. 7) and a = 0.32 (Section 5.1): with Mavg = 32, Lbar = 1, N = 1, R = 1
    the bound is 0.32 / 0.32 = 1 up to the fp32 rounding of the two constants."""
    rc, eb, _ = orc.estimate_eb(np.ones((1, 1, 2, 2), np.float32), np.array([[1.0, -0.5]], np.float32),
                                np.array([32.0, -32.0], np.float32), eb_max=4.0)
    assert rc == 0 and abs(float(eb) - 1.0) < 1e-6


def test_scaling_laws(orc):
    """Section 3.2: twice the batch -> sigma grows by sqrt(2), so the bound shrinks by sqrt(2);
    Eq. 9: sigma' = sigma * sqrt(R); Eq. 8: linear in Mavg, inverse in Lbar."""
    rng = np.random.default_rng(7)
    act = rng.standard_normal((8, 4, 6, 6)).astype(np.float32)
    loss = rng.standard_normal((8, 144)).astype(np.float32)
    mom = rng.standard_normal(500).astype(np.float32)
    kw = dict(eb_min=1e-12, eb_max=1e6)
    _, eb0, (R0, L0, M0) = orc.estimate_eb(act, loss, mom, **kw)
    assert R0 == 1.0
    # batch doubled by repeating the samples: same Lbar, N twice as large
    _, eb1, (_, L1, _) = orc.estimate_eb(np.concatenate([act, act]), np.concatenate([loss, loss]), mom, **kw)
    assert L1 == pytest.approx(L0, rel=1e-15) and float(eb1) == pytest.approx(float(eb0) / np.sqrt(2.0), rel=3e-7)
    # three quarters of the activations zeroed: R = 1/4, bound doubles
    act_z = act.copy().reshape(-1)
    act_z[np.arange(act_z.size) % 4 != 0] = 0.0
    _, eb2, (R2, _, _) = orc.estimate_eb(act_z.reshape(act.shape), loss, mom, **kw)
    assert R2 == 0.25 and float(eb2) == pytest.approx(2.0 * float(eb0), rel=3e-7)
    _, eb3, _ = orc.estimate_eb(act, loss, 4.0 * mom, **kw)
    assert float(eb3) == pytest.approx(4.0 * float(eb0), rel=3e-7)
    _, eb4, _ = orc.estimate_eb(act, 8.0 * loss, mom, **kw)
    assert float(eb4) == pytest.approx(float(eb0) / 8.0, rel=3e-7)


def test_statistics_against_numpy(orc):
    rng = np.random.default_rng(11)
    act = np.maximum(rng.standard_normal((5, 3, 9, 7)), 0).astype(np.float32)
    loss = (rng.standard_normal((5, 3, 9, 7)) * 1e-3).astype(np.float32)
    mom = (rng.standard_normal((3, 3, 3, 3)) * 1e-2).astype(np.float32)
    rc, eb, (R, Lbar, Mavg) = orc.estimate_eb(act, loss, mom)
    assert rc == 0
    assert R == np.count_nonzero(act) / act.size
    assert Lbar == pytest.approx(np.abs(loss.astype(np.float64)).reshape(5, -1).max(axis=1).mean(), rel=1e-14)
    assert Mavg == pytest.approx(np.abs(mom.astype(np.float64)).mean(), rel=1e-13)
    expect = 0.01 * Mavg / (0.32 * Lbar * np.sqrt(5 * R))
    assert float(eb) == pytest.approx(expect, rel=3e-7)


def test_clamping_and_degenerate_inputs(orc):
    one = np.ones((2, 1, 2, 2), np.float32)
    loss = np.ones((2, 4), np.float32)
    mom = np.ones(4, np.float32)
    rc, eb, _ = orc.estimate_eb(one, loss, 1e6 * mom, eb_max=0.5)
    assert rc == 0 and eb == np.float32(0.5)
    rc, eb, _ = orc.estimate_eb(one, loss, 1e-9 * mom, eb_min=1e-4)
    assert rc == 0 and eb == np.float32(1e-4)
    # nothing to estimate from: the tightest bound and a warning
    one_nan = loss.copy()
    one_nan[1, 1] = np.nan                              # a single NaN, followed by ordinary values
    for a_, l_, m_ in ((0 * one, loss, mom), (one, 0 * loss, mom), (one, loss * np.nan, mom), (one, one_nan, mom),
                       (one, loss, mom * np.inf)):
        rc, eb, _ = orc.estimate_eb(a_, l_, m_, eb_min=1e-4)
        assert rc == 1 and eb == np.float32(1e-4)
    # bad configuration
    assert orc.estimate_eb(one, loss, mom, eb_min=0.0)[0] == -1
    assert orc.estimate_eb(one, loss, mom, eb_min=1.0, eb_max=0.5)[0] == -1
