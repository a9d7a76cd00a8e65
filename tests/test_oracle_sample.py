"""Pins of the oracle's sampled-codebook mode (a table coded with the codebook of the counts of a few of its own
groups).

What fixes the result without reference to the code under test: the sampled groups for shapes worked out by hand from
the rule (as many groups as hold 65536 elements, no more than a quarter of the table's, evenly spread from group 0 on); the sample's counts against numpy's
bincount over the elements whose index falls into those groups; the container against the carried-codebook mode (pinned
on its own, against the independent stream reader) given those counts; the bound on every element, and the raw value
back for an element whose symbol the sample has not seen.
"""
import numpy as np
import pytest

import oracle

R = 512
K = 2 * R


@pytest.mark.parametrize("n,S,want", [
    (8192 * 128, 256, [0, 16, 32, 48]),            # 64 groups of 16384: four groups, every sixteenth
    (4096 * 64, 256, [0, 4, 8, 12]),               # 16 groups
    (5 * 16384 - 100, 256, [0, 2]),                # 5 groups (the last ragged): a quarter, rounded up, is two; stride 2
    (7 * 16384, 256, [0, 3]),
    (9 * 16384, 256, [0, 3, 6]),
    (17 * 16384, 256, [0, 4, 8, 12]),              # four groups hold 65536 elements: no more, though a quarter would be five
    (100, 256, [0]),                               # less than a group: the whole table
    (2 * 16384, 256, [0]),                         # two groups: the first
    (4 * 16384, 256, [0]),
    (8192 * 128, 64, list(range(0, 256, 16))),     # groups of 4096: sixteen of 256
    (8192 * 128, 128, list(range(0, 128, 16))),    # groups of 8192: eight of 128
])
def test_sampled_groups_of_shapes_worked_out_by_hand(n, S, want):
    assert oracle.sample_groups(n, S) == want


def _payload(T, B, D, seed, sigma=0.02):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, B, D)) * sigma * (1 + np.arange(T)[:, None, None])).astype(np.float32)


def _bincount_of_sampled_elements(x, ebs, S):
    T = x.shape[0]
    n = x[0].size
    gs = 64 * S
    h = np.zeros((T, K), np.uint64)
    for t in range(T):
        sym, _ = oracle.quantize(x[t].reshape(-1), float(ebs[t]), R)
        in_sample = np.isin(np.arange(n) // gs, oracle.sample_groups(n, S))
        h[t] = np.bincount(sym[in_sample], minlength=K).astype(np.uint64)
    return h


@pytest.mark.parametrize("T,B,D,S", [(2, 300, 50, 8), (1, 4096, 64, 256), (3, 1000, 40, 16), (2, 77, 13, 64)])
def test_sample_counts_and_container(T, B, D, S):
    x = _payload(T, B, D, 5 * B + D)
    x.reshape(-1)[::997] = 3e5  # true escapes, some inside the sample, some not
    ebs = np.array([1e-3 * (t + 1) for t in range(T)], np.float32)
    h = _bincount_of_sampled_elements(x, ebs, S)
    assert np.array_equal(oracle.sample_histogram(x, ebs, R, S), h)
    a = oracle.compress(x, ebs, R, S, 12, sample_codebook=True)
    b = oracle.compress(x, ebs, R, S, 12, carry_hist=h)
    assert a.rc == oracle.OK and np.array_equal(a.data, b.data) and np.array_equal(a.sizes, b.sizes)
    rc, rec = oracle.decompress(a.data, x.shape, np.float32)
    assert rc == oracle.OK
    for t in range(T):
        d = np.abs(rec[t].astype(np.float64) - x[t].astype(np.float64))
        assert d.max() <= float(ebs[t])


def test_a_symbol_the_sample_has_not_seen_comes_back_as_the_raw_value():
    S = 8                       # groups of 512 elements, every third of the first 103 sampled: elements from 65536 on are not
    T, B, D = 1, 1100, 64       # 70400 elements
    rng = np.random.default_rng(3)
    x = (rng.integers(-3, 4, (T, B, D)) * 2e-3).astype(np.float32)  # seven symbols throughout
    eb = 1e-3
    far = np.float32(0.0123456)                                       # a symbol of its own, outside the sample only
    x.reshape(-1)[[65536, 65537 + 640, 70399]] = far
    h = oracle.sample_histogram(x, eb, R, S)
    sym, _ = oracle.quantize(x.reshape(-1), eb, R)
    assert h[0][sym[65536]] == 0 and h[0].sum() == 35 * 512   # 138 groups of 512: a quarter of them, every third from group 0
    own = oracle.compress(x, eb, R, S, 12)
    smp = oracle.compress(x, eb, R, S, 12, sample_codebook=True)
    rc, rec = oracle.decompress(smp.data, x.shape, np.float32)
    assert rc == oracle.OK
    r = rec.reshape(-1)
    assert r[65536] == far and r[65537 + 640] == far and r[70399] == far   # escapes: bit for bit
    assert np.abs(rec.astype(np.float64) - x.astype(np.float64)).max() <= eb
    # three escape records of two words, the escape's code three times, seven symbols plus the escape to code
    assert smp.data.size > own.data.size


def test_a_table_of_one_group_is_coded_with_its_own_counts():
    x = _payload(2, 250, 64, 9)     # 16000 elements: one group at S = 256, the sample
    eb = 2e-3
    whole = oracle.compress(x, eb, R, 256, 12, want_hist=True)
    smp = oracle.compress(x, eb, R, 256, 12, sample_codebook=True)
    assert np.array_equal(oracle.sample_histogram(x, eb, R, 256), whole.hist)
    assert np.array_equal(smp.data, oracle.compress(x, eb, R, 256, 12, carry_hist=whole.hist).data)
    # (the escape's extra count can only lengthen codes: never smaller than with the payload's own codebook)
    assert smp.data.size >= whole.data.size


def test_ratio_on_gaussian_rows_is_within_a_percent_of_the_own_codebook():
    rng = np.random.default_rng(11)
    table = (rng.standard_normal((5000, 64)) * 0.05).astype(np.float32)
    x = table[rng.integers(0, 5000, (2, 8192))]
    eb = 0.03 * float(x.max() - x.min())
    own = oracle.compress(x, eb, R, 256, 12)
    smp = oracle.compress(x, eb, R, 256, 12, sample_codebook=True)
    assert smp.data.size <= own.data.size * 1.01
