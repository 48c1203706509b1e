"""Pins for the codebook stage: Huffman lengths and canonical codes.

Fixed independently of the oracle: the RFC 1951 section 3.2.2 worked example,
Kraft equality, brute-force minimum cost over all feasible length vectors on
tiny alphabets, the cost of an independent heap-based Huffman construction,
closed forms, and hand-worked tie-break cases (tests/golden/huffman_lengths.txt).
"""
import heapq
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rows(name):
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                yield line


def test_canonical_codes_rfc1951_example(orc):
    syms, lens, codes = [], [], []
    for line in rows("rfc1951_canonical.txt"):
        a, b, c = line.split()
        syms.append(int(a)); lens.append(int(b)); codes.append(c)
    rc, got = orc.canonical_codes(np.array(lens, np.uint8))
    assert rc == 0
    for k, L, want in zip(syms, lens, codes):
        assert format(int(got[k]), "0%db" % L) == want


@pytest.mark.parametrize("line", list(rows("huffman_lengths.txt")))
def test_lengths_golden(orc, line):
    kind, counts, lens = [t.strip() for t in line.split("|")]
    cnt = np.array(counts.split(), np.uint32)
    got, mx = orc.codebook_lengths(cnt)
    assert list(got) == [int(v) for v in lens.split()]
    assert mx == max(int(v) for v in lens.split())


def test_tiebreak_example_codes(orc):
    # counts (1,1,2): lengths (2,2,1); canonical order (len, symbol): sym2=0, sym0=10, sym1=11
    lens, _ = orc.codebook_lengths(np.array([1, 1, 2], np.uint32))
    rc, codes = orc.canonical_codes(lens)
    assert list(lens) == [2, 2, 1] and list(codes) == [0b10, 0b11, 0b0]


def kraft(lens):
    return sum(Fraction(1, 2 ** int(L)) for L in lens if L > 0)


def heap_cost(cnt):
    """Total coded bits of an optimal prefix code = sum of all internal node weights."""
    h = [int(c) for c in cnt if c > 0]
    if len(h) == 1:
        return h[0]
    heapq.heapify(h)
    total = 0
    while len(h) > 1:
        a = heapq.heappop(h); b = heapq.heappop(h)
        total += a + b
        heapq.heappush(h, a + b)
    return total


def brute_force_cost(cnt):
    n = len(cnt)
    best = None
    for lens in itertools.product(range(1, n), repeat=n):
        if kraft(lens) <= 1:
            c = sum(int(a) * b for a, b in zip(cnt, lens))
            best = c if best is None else min(best, c)
    return best


@settings(max_examples=120, deadline=None)
@given(st.lists(st.integers(1, 40), min_size=2, max_size=6))
def test_cost_equals_brute_force_minimum_on_tiny_alphabets(orc, counts):
    cnt = np.array(counts, np.uint32)
    lens, mx = orc.codebook_lengths(cnt)
    assert kraft(lens) == 1
    assert sum(int(a) * int(b) for a, b in zip(cnt, lens)) == brute_force_cost(counts)


@settings(max_examples=60, deadline=None)
@given(st.integers(0, 2 ** 31), st.sampled_from(["geometric", "uniform", "sparse", "flat", "huge"]))
def test_cost_equals_heap_huffman_and_kraft_on_1024_bins(orc, seed, kind):
    rng = np.random.default_rng(seed)
    if kind == "geometric":
        k = np.arange(1024) - 512
        cnt = np.floor(3e7 * np.exp(-np.abs(k) / rng.uniform(1, 60))).astype(np.uint32)
    elif kind == "uniform":
        cnt = rng.integers(0, 1000, 1024).astype(np.uint32)
    elif kind == "sparse":
        cnt = np.zeros(1024, np.uint32)
        idx = rng.choice(1024, rng.integers(1, 30), replace=False)
        cnt[idx] = rng.integers(1, 10 ** 6, idx.size)
    elif kind == "flat":
        cnt = np.full(1024, rng.integers(1, 5), np.uint32)
    else:
        cnt = rng.integers(0, 2 ** 32 - 1, 1024, dtype=np.uint64).astype(np.uint32)
    lens, mx = orc.codebook_lengths(cnt)
    used = cnt > 0
    assert np.all(lens[~used] == 0) and np.all(lens[used] > 0)
    assert mx == lens.max()
    if used.sum() >= 2:
        assert kraft(lens) == 1
    assert int((cnt.astype(np.uint64) * lens).sum()) == heap_cost(cnt)
    rc, codes = orc.canonical_codes(lens)
    assert rc == 0
    # prefix-free: sorted by (len, sym) the codes, left-aligned, are strictly increasing and
    # no code is a prefix of a later one
    order = sorted(np.nonzero(used)[0], key=lambda k: (lens[k], k))
    aligned = [int(codes[k]) << (64 - int(lens[k])) for k in order]
    assert all(a < b for a, b in zip(aligned, aligned[1:]))
    for a, b in zip(order, order[1:]):
        assert (int(codes[b]) >> (int(lens[b]) - int(lens[a]))) != int(codes[a])


def test_fibonacci_counts_give_deepest_tree(orc):
    fib = [1, 1]
    while len(fib) < 40:
        fib.append(fib[-1] + fib[-2])
    lens, mx = orc.codebook_lengths(np.array(fib, np.uint32))
    assert mx == 39 and list(lens) == [39, 39] + list(range(38, 0, -1))
    rc, codes = orc.canonical_codes(lens)
    assert rc == 0 and kraft(lens) == 1


def test_oversubscribed_lengths_rejected(orc):
    rc, _ = orc.canonical_codes(np.array([1, 1, 1], np.uint8))
    assert rc == orc.E_FORMAT


def test_planted_mistake_internal_first_is_detected():
    """The (1,1,2,2) case separates leaf-first from internal-first tie-breaking: the latter
    yields (3,3,2,1) with the same cost 12, so the golden row does pin the rule."""
    assert 1 * 3 + 1 * 3 + 2 * 2 + 2 * 1 == 1 * 2 + 1 * 2 + 2 * 2 + 2 * 2 == 12
