"""Pins for the Lorenzo predictor, its inverse, the outlier split and the histogram.

Fixed independently of the oracle: the rectangle-sum definition of the inverse,
numpy's cumsum along both axes (textbook reduction), closed forms for constant
and affine planes, numpy.bincount.
"""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

SHAPES = [(3, 1, 1), (2, 1, 9), (2, 9, 1), (4, 7, 7), (2, 55, 55), (1, 13, 31), (1, 31, 13)]


@pytest.mark.parametrize("shape", SHAPES)
def test_prefix_of_lorenzo_is_identity(orc, shape):
    rng = np.random.default_rng(sum(shape))
    q = rng.integers(-16384, 16385, size=shape, dtype=np.int32)
    d = orc.lorenzo2d(q)
    assert np.array_equal(orc.prefix2d(d), q)
    assert np.array_equal(np.cumsum(np.cumsum(d, axis=1), axis=2), q)
    assert np.abs(d).max() <= 4 * 16384


@pytest.mark.parametrize("shape", [(2, 1, 1), (2, 5, 6), (1, 7, 7), (1, 1, 12), (1, 12, 1)])
def test_recurrence_equals_rectangle_sum_definition(orc, shape):
    rng = np.random.default_rng(11)
    d = rng.integers(-600, 600, size=shape, dtype=np.int32)
    a = orc.prefix2d(d)
    b = orc.prefix2d(d, definition=True)
    assert np.array_equal(a, b)
    assert np.array_equal(a, np.cumsum(np.cumsum(d, axis=1), axis=2))
    assert np.array_equal(orc.lorenzo2d(a), d)


def test_planes_are_independent(orc):
    rng = np.random.default_rng(3)
    q = rng.integers(-100, 100, size=(3, 6, 5), dtype=np.int32)
    whole = orc.lorenzo2d(q)
    for p in range(3):
        assert np.array_equal(orc.lorenzo2d(q[p:p + 1]), whole[p:p + 1])


def test_closed_form_constant_plane(orc):
    q = np.full((1, 6, 9), 37, dtype=np.int32)
    d = orc.lorenzo2d(q)
    want = np.zeros_like(q); want[0, 0, 0] = 37
    assert np.array_equal(d, want)


def test_closed_form_affine_plane(orc):
    a, b, c = 5, -3, 11
    h, w = np.meshgrid(np.arange(8), np.arange(10), indexing="ij")
    q = (a * h + b * w + c).astype(np.int32)[None]
    d = orc.lorenzo2d(q)[0]
    assert d[0, 0] == c
    assert np.all(d[0, 1:] == b) and np.all(d[1:, 0] == a) and np.all(d[1:, 1:] == 0)


def test_single_spike_delta_fills_lower_right_rectangle(orc):
    d = np.zeros((1, 5, 7), np.int32); d[0, 2, 3] = 9
    q = orc.prefix2d(d)[0]
    want = np.zeros((5, 7), np.int32); want[2:, 3:] = 9
    assert np.array_equal(q, want)


def test_asymmetry_catches_transposition(orc):
    # a plane that varies along w only: deltas live in the first row
    q = np.tile(np.arange(1, 8, dtype=np.int32) ** 2, (4, 1))[None]
    d = orc.lorenzo2d(q)[0]
    assert np.array_equal(d[0], np.diff(np.concatenate([[0], q[0, 0]])))
    assert np.all(d[1:] == 0)


@settings(max_examples=60, deadline=None)
@given(st.integers(1, 4), st.integers(1, 20), st.integers(1, 20), st.integers(0, 2 ** 31))
def test_identity_random_shapes(orc, p, h, w, seed):
    rng = np.random.default_rng(seed)
    q = rng.integers(-16384, 16385, size=(p, h, w), dtype=np.int32)
    assert np.array_equal(orc.prefix2d(orc.lorenzo2d(q)), q)


def test_split_boundaries_and_order(orc):
    R = 512
    d = np.array([0, 511, -511, 512, -512, 513, 65536, -65536, 1, -1], dtype=np.int32)
    sym, oi, ov = orc.split(d, R)
    assert list(sym) == [512, 1023, 1, 0, 0, 0, 0, 0, 513, 511]
    assert list(oi) == [3, 4, 5, 6, 7]
    assert list(ov) == [512, -512, 513, 65536, -65536]


@pytest.mark.parametrize("radius", [1, 2, 8, 512])
def test_split_and_histogram_against_numpy(orc, radius):
    rng = np.random.default_rng(radius)
    d = np.rint(rng.normal(0, radius / 2 + 1, 50000)).astype(np.int32)
    sym, oi, ov = orc.split(d, radius)
    inside = np.abs(d) < radius
    assert np.array_equal(sym[inside].astype(np.int64), d[inside].astype(np.int64) + radius)
    assert np.all(sym[~inside] == 0)
    assert np.array_equal(oi, np.nonzero(~inside)[0].astype(np.uint32))
    assert np.all(np.diff(oi.astype(np.int64)) > 0)
    assert np.array_equal(ov, d[~inside])
    cnt = orc.histogram(sym, 2 * radius)
    assert np.array_equal(cnt, np.bincount(sym, minlength=2 * radius).astype(np.uint32))
    assert cnt.sum() == d.size and cnt[0] == oi.size
