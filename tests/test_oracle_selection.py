"""Pins of the oracle's compressor selection (Section III-D "Selection Between Two Encoders": Eq. 2 and the
algorithm "Compressor Selection"): Eq. 2 against exact rational arithmetic and hand-computed values, its limits,
the per-table maximum with ties, and the whole procedure against sizes taken from the two compressors."""
from fractions import Fraction

import numpy as np

import oracle

R = 512


def _exact(cr, net, tc, td):
    cr, net, tc, td = (Fraction(v) for v in (cr, net, tc, td))
    return 1 / (1 / cr + net * (1 / tc + 1 / td))


def test_eq2_hand_values():
    # 1 / (1/10 + 4 (1/80 + 1/40)) = 1 / (0.1 + 0.15) = 4;   1 / (1/2 + 1 (1/4 + 1/4)) = 1
    assert oracle.speedup(10, 4, 80, 40) == 4.0
    assert oracle.speedup(2, 1, 4, 4) == 1.0
    # 1 / (1/8 + 25 (1/2000 + 1/4000)) = 1 / 0.14375 = 160/23
    assert abs(oracle.speedup(8, 25, 2000, 4000) - 160 / 23) < 1e-14


def test_eq2_against_exact_rationals_and_limits():
    rng = np.random.default_rng(3)
    for _ in range(200):
        cr, net, tc, td = (float(v) for v in np.exp(rng.uniform(-3, 8, 4)))
        want = _exact(cr, net, tc, td)
        assert abs(Fraction(oracle.speedup(cr, net, tc, td)) - want) <= want * Fraction(1, 10 ** 14)
    # a free network hides nothing: the estimate tends to the ratio; an infinitely fast compressor leaves 1/(1/cr)
    assert abs(oracle.speedup(12.5, 1e-12, 100.0, 100.0) - 12.5) < 1e-9
    assert abs(oracle.speedup(12.5, 10.0, 1e30, 1e30) - 12.5) < 1e-9
    # compressing slower than the wire sends loses: below 1 whatever the ratio
    assert oracle.speedup(1e9, 100.0, 50.0, 1e30) < 0.5 + 1e-12
    # monotone: better ratio, faster compressor, slower network all help
    assert oracle.speedup(11, 25, 2000, 4000) > oracle.speedup(10, 25, 2000, 4000)
    assert oracle.speedup(10, 25, 2100, 4000) > oracle.speedup(10, 25, 2000, 4000)
    assert oracle.speedup(10, 24, 2000, 4000) > oracle.speedup(10, 25, 2000, 4000)
    for bad in ((0, 1, 1, 1), (1, 0, 1, 1), (1, 1, -1, 1), (1, 1, 1, float("nan"))):
        assert oracle.speedup(*bad) == 0.0


def test_select_is_the_per_table_maximum_ties_to_the_first():
    rng = np.random.default_rng(5)
    for n_comp in (1, 2, 3):
        T = 17
        cr = np.exp(rng.uniform(0, 4, (n_comp, T)))
        tc = np.exp(rng.uniform(3, 8, n_comp))
        td = np.exp(rng.uniform(3, 8, n_comp))
        for net in (0.5, 25.0, 400.0):
            choice, best = oracle.select(cr, tc, td, net)
            est = np.array([[oracle.speedup(cr[c, t], net, tc[c], td[c]) for t in range(T)] for c in range(n_comp)])
            assert np.array_equal(choice, np.argmax(est, axis=0))          # numpy's argmax takes the first maximum too
            assert np.array_equal(best, est.max(axis=0))
            exact = [[_exact(cr[c, t], net, tc[c], td[c]) for t in range(T)] for c in range(n_comp)]
            for t in range(T):                                              # and the maximum of the exact values
                col = [exact[c][t] for c in range(n_comp)]
                if sorted(col)[-1] - (sorted(col)[-2] if n_comp > 1 else 0) > Fraction(1, 10 ** 9):
                    assert choice[t] == col.index(max(col))
    # equal estimates: the compressor listed first
    cr = np.array([[5.0, 7.0], [5.0, 7.0], [5.0, 9.0]])
    choice, _ = oracle.select(cr, [100.0, 100.0, 100.0], [200.0, 200.0, 200.0], 10.0)
    assert list(choice) == [0, 2]


def _tables(B=600, D=16):
    rng = np.random.default_rng(11)
    unique = (rng.standard_normal((B, D)) * 0.02).astype(np.float32)            # no row occurs twice
    few = (rng.standard_normal((6, D)) * 0.02).astype(np.float32)[rng.integers(0, 6, B)]   # six rows, repeated
    return np.stack([unique, few, unique[::-1].copy(), few[::-1].copy()])


def test_the_procedure_on_a_sample():
    x = _tables()
    T, B, D = x.shape
    eb = np.full(T, 1e-3, np.float32)
    sizes = [oracle.compress(x, eb, R, 64, 12, row_match=[c] * T).sizes[1:].astype(np.float64) for c in (0, 1)]
    raw = B * D * 4
    # the references cost the tables without repeats a little, and more than halve the tables of six rows
    assert sizes[1][0] > sizes[0][0] and sizes[1][2] > sizes[0][2]
    assert sizes[1][1] < sizes[0][1] / 2 and sizes[1][3] < sizes[0][3] / 2
    for net, tc, td in ((25.0, (2000.0, 1400.0), (4000.0, 2500.0)),      # a slow network: the ratio decides
                        (5000.0, (2000.0, 1400.0), (4000.0, 2500.0)),    # a network as fast as the coder: the rates decide
                        (25.0, (2000.0, 2000.0), (4000.0, 4000.0))):     # equal rates: the ratio alone
        choice, best = oracle.select_compressors(x, eb, net, tc, td, R, 64, 12)
        for t in range(T):
            est = [_exact(raw / sizes[c][t], net, tc[c], td[c]) for c in (0, 1)]
            assert choice[t] == (1 if est[1] > est[0] else 0), (net, t)
            assert abs(Fraction(float(best[t])) - max(est)) <= max(est) * Fraction(1, 10 ** 13)
    assert list(oracle.select_compressors(x, eb, 25.0, (2000.0, 1400.0), (4000.0, 2500.0), R, 64, 12)[0]) == [0, 1, 0, 1]
    assert list(oracle.select_compressors(x, eb, 5000.0, (2000.0, 1400.0), (4000.0, 2500.0), R, 64, 12)[0]) == [0, 0, 0, 0]
