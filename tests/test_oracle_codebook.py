"""Pins of the oracle's histogram and Huffman codebook (the entropy encoder of Section III-D)."""
import heapq
import itertools
import math

import numpy as np
import pytest

import oracle


def _heap_huffman_cost(counts):
    """Total bits of an optimal prefix code: independent textbook heap construction."""
    h = [int(c) for c in counts if c > 0]
    if len(h) < 2:
        return 0
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def _check_code(hist, ln, code, LMAX):
    used = np.nonzero(hist)[0]
    assert np.all(ln[hist == 0] == 0)
    if used.size == 1:
        assert ln[used[0]] == 0
        return
    assert np.all(ln[used] >= 1) and ln.max() <= LMAX
    # Kraft equality
    assert sum(2.0 ** -int(l) for l in ln[used]) == 1.0
    # prefix property, checked pair by pair on the bit strings
    words = sorted(format(int(code[s]), f"0{int(ln[s])}b") for s in used)
    assert all(len(w) == 0 or True for w in words)
    for a, b in zip(words, words[1:]):
        assert not b.startswith(a), (a, b)
    # canonical: numerically increasing in (length, symbol) order
    order = sorted(used, key=lambda s: (ln[s], s))
    vals = [int(code[s]) << (LMAX - int(ln[s])) for s in order]
    assert all(x < y for x, y in zip(vals, vals[1:]))
    assert int(code[order[0]]) == 0


def test_histogram_is_bincount():
    rng = np.random.default_rng(0)
    sym = rng.integers(0, 1024, 100000).astype(np.uint16)
    h = oracle.histogram(sym, 1024)
    assert np.array_equal(h, np.bincount(sym, minlength=1024).astype(np.uint64))
    assert h.sum() == sym.size


@pytest.mark.parametrize("seed", range(12))
def test_random_histograms_are_optimal_prefix_codes(seed):
    rng = np.random.default_rng(seed)
    K = 1024
    n_used = int(rng.integers(2, 200))
    hist = np.zeros(K, np.uint64)
    where = rng.choice(K, n_used, replace=False)
    kind = seed % 3
    if kind == 0:      # bell shaped, like quantised Gaussian data (observation 3 of Section III-B)
        hist[where] = np.maximum(1, (1e6 * np.exp(-0.5 * ((where - 512) / 30.0) ** 2))).astype(np.uint64)
    elif kind == 1:    # flat with many ties
        hist[where] = rng.integers(1, 4, n_used)
    else:
        hist[where] = rng.integers(1, 100000, n_used)
    ln, code, nu, nh = oracle.codebook(hist, 12)
    assert nu == n_used
    _check_code(hist, ln, code, 12)
    cost = int((hist * ln).sum())
    if nh == 0:
        assert cost == _heap_huffman_cost(hist)
        n = int(hist.sum())
        p = hist[hist > 0] / n
        H = float(-(p * np.log2(p)).sum())
        assert H * n <= cost + 1e-6 < (H + 1) * n
    else:
        assert cost >= _heap_huffman_cost(hist)


def _brute_force_cost(counts):
    n = len(counts)
    best = None
    for depths in itertools.product(range(1, n), repeat=n):
        if sum(2.0 ** -d for d in depths) == 1.0:
            c = sum(d * w for d, w in zip(depths, counts))
            best = c if best is None or c < best else best
    return best


def test_brute_force_small_alphabets():
    rng = np.random.default_rng(42)
    for n in range(2, 7):
        for _ in range(6):
            counts = rng.integers(1, 30, n)
            hist = np.zeros(16, np.uint64)
            pos = rng.choice(16, n, replace=False)
            hist[pos] = counts
            ln, code, _, nh = oracle.codebook(hist, 12)
            assert nh == 0
            _check_code(hist, ln, code, 12)
            assert int((hist * ln).sum()) == _brute_force_cost([int(c) for c in hist[hist > 0]])


def test_dyadic_counts_give_exact_lengths():
    counts = [1, 1, 2, 4, 8, 16, 32, 64]
    hist = np.zeros(64, np.uint64)
    hist[10:18] = counts
    ln, code, _, _ = oracle.codebook(hist, 12)
    total = sum(counts)
    assert [int(l) for l in ln[10:18]] == [int(-math.log2(c / total)) for c in counts]
    _check_code(hist, ln, code, 12)


def test_fibonacci_counts_force_the_length_limit():
    fib = [1, 1]
    while len(fib) < 24:
        fib.append(fib[-1] + fib[-2])
    hist = np.zeros(1024, np.uint64)
    hist[100:124] = fib
    ln, code, nu, nh = oracle.codebook(hist, 12)
    assert nh > 0 and nu == 24
    _check_code(hist, ln, code, 12)
    assert ln.max() <= 12
    # without the limit the same counts need 23 bits
    ln2, _, _, nh2 = oracle.codebook(np.array(fib[:12], np.uint64), 12)
    assert nh2 == 0 and ln2.max() == 11


def test_degenerate_alphabets():
    hist = np.zeros(1024, np.uint64)
    hist[512] = 12345
    ln, code, nu, _ = oracle.codebook(hist, 12)
    assert nu == 1 and ln.max() == 0 and code.max() == 0          # one symbol: zero bits
    hist[3] = 1
    ln, code, nu, _ = oracle.codebook(hist, 12)
    assert nu == 2 and ln[3] == 1 and ln[512] == 1
    assert (code[3], code[512]) == (0, 1)                          # equal lengths: smaller symbol first
    # all 1024 symbols used equally: a flat 10-bit code in symbol order
    hist[:] = 7
    ln, code, nu, _ = oracle.codebook(hist, 12)
    assert nu == 1024 and np.all(ln == 10) and np.array_equal(code, np.arange(1024, dtype=np.uint32))


def test_tie_break_is_fixed():
    """Equal counts everywhere: the construction is deterministic (leaf queue first, FIFO merges)."""
    hist = np.zeros(8, np.uint64)
    hist[[1, 2, 4, 5, 7]] = 3
    ln, code, _, _ = oracle.codebook(hist, 12)
    # leaves (3,1)(3,2)(3,4)(3,5)(3,7): merges (1,2)=6, (4,5)=6, then leaf 7 with node(1,2)=9, then 6+9
    assert [int(ln[s]) for s in (1, 2, 4, 5, 7)] == [3, 3, 2, 2, 2]
    assert [int(code[s]) for s in (4, 5, 7, 1, 2)] == [0, 1, 2, 6, 7]


@pytest.mark.parametrize("LMAX", [4, 5, 7, 12])
def test_length_limited_codes_are_valid_and_monotone(LMAX):
    """Skewed counts with a small LMAX: every result is a complete prefix code within the limit, never gives
    a more frequent symbol a longer code, and costs at least the unlimited optimum."""
    rng = np.random.default_rng(LMAX)
    K = 1 << LMAX
    hit = 0
    for trial in range(60):
        n = int(rng.integers(2, K + 1))
        hist = np.zeros(K, np.uint64)
        where = rng.choice(K, n, replace=False)
        kind = trial % 3
        if kind == 0:
            hist[where] = np.maximum(1, (2.0 ** rng.uniform(0, 30, n))).astype(np.uint64)     # huge dynamic range
        elif kind == 1:
            hist[where] = np.maximum(1, 1e6 * np.exp(-0.5 * ((np.arange(n) - n / 2) / (n / 12 + 0.3)) ** 2)).astype(
                np.uint64)                                                                     # bell with long tails
        else:
            hist[where] = 1                                                                    # flat
            hist[where[0]] = 10 ** 9
        ln, code, nu, nh = oracle.codebook(hist, LMAX)
        assert nu == n
        _check_code(hist, ln, code, LMAX)
        used = np.nonzero(hist)[0]
        if nh:
            hit += 1
            order = sorted(used, key=lambda s: (-int(hist[s]), -int(s)))
            lens = [int(ln[s]) for s in order]
            assert lens == sorted(lens)                      # most frequent first gets the shortest
            assert ln.max() == LMAX
        assert int((hist * ln).sum()) >= _heap_huffman_cost(hist)
    assert hit > 5


def test_length_limit_costs_little_on_bell_shaped_counts():
    """Quantised Gaussian data (observation 3 of Section III-B): the limit only touches the far tails."""
    k = np.arange(-40, 41)
    hist = np.zeros(1024, np.uint64)
    hist[512 + k] = np.maximum(1, np.round(1e6 * 0.25 * np.exp(-0.5 * (k * 0.52) ** 2))).astype(np.uint64)
    ln, code, nu, nh = oracle.codebook(hist, 12)
    assert nh > 0 and ln.max() == 12
    _check_code(hist, ln, code, 12)
    assert int((hist * ln).sum()) <= _heap_huffman_cost(hist) * 1.01
