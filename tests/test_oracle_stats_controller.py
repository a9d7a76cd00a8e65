"""Pins of the oracle's statistics (Eq. 1) and error-bound controller (Algorithm 1)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _homo_rows():
    rows = []
    for line in open(os.path.join(GOLD, "homo_index_tables.txt")):
        if line.startswith("#") or not line.strip():
            continue
        ds, tid, eb, no, nq, batch, printed = line.split()
        rows.append((ds, int(tid), float(eb), int(no), int(nq), int(batch), printed))
    return rows


def _class_gold():
    bounds, letters = {}, {}
    for line in open(os.path.join(GOLD, "class_bounds.txt")):
        if line.startswith("#") or not line.strip():
            continue
        p = line.split()
        if len(p) == 2:
            bounds[p[0]] = float(p[1])
        else:
            letters[(p[0], int(p[1]))] = p[2]
    return bounds, letters


@pytest.mark.parametrize("row", _homo_rows(), ids=lambda r: f"{r[0]}-{r[1]}")
def test_homo_index_printed_values(row):
    """Tables III/IV: printed column = N_quant/N_ori = 1 - eta (Eq. 1), 6 decimals."""
    _, _, _, n_ori, n_quant, _, printed = row
    eta = oracle.homo_index(n_ori, n_quant)
    exact = 1 - Fraction(n_ori - n_quant, n_ori)
    assert abs((1.0 - eta) - float(exact)) < 1e-15
    decimals = len(printed.split(".")[1]) if "." in printed else 0
    assert f"{1.0 - eta:.{max(decimals, 6)}f}".rstrip("0").rstrip(".") == printed.rstrip("0").rstrip(".")
    assert 0.0 <= eta <= 1.0


def _build_batch(n_ori, n_quant, batch, eb, D, rng, dtype=np.float32):
    """A batch with exactly n_ori distinct rows that collapse to n_quant rows at bound eb."""
    # cluster centres: distinct integer bin vectors, rows sit well inside their bins
    centres = set()
    while len(centres) < n_quant:
        centres.add(tuple(rng.integers(-20, 21, D)))
    centres = np.array(sorted(centres), np.float64) * (2 * eb)
    members = np.ones(n_quant, np.int64)
    for _ in range(n_ori - n_quant):
        members[rng.integers(0, n_quant)] += 1
    rows = []
    for c, m in zip(centres, members):
        for j in range(m):
            jitter = np.zeros(D)
            jitter[0] = j * eb * 0.01  # distinct raw bits, same bin (|jitter| << eb)
            rows.append(c + jitter)
    rows = np.array(rows).astype(dtype)
    assert len(np.unique(rows.view(np.uint32 if dtype == np.float32 else np.uint16), axis=0)) == n_ori
    extra = rows[rng.integers(0, n_ori, batch - n_ori)]
    full = np.concatenate([rows, extra])
    return full[rng.permutation(batch)]


@pytest.mark.parametrize("row", _homo_rows(), ids=lambda r: f"{r[0]}-{r[1]}")
def test_stats_reproduce_printed_pattern_counts(row):
    """A batch built to have the printed pattern counts gives them back, and the printed index."""
    _, tid, eb, n_ori, n_quant, batch, printed = row
    rng = np.random.default_rng(1000 + tid + batch)
    payload = _build_batch(n_ori, n_quant, batch, eb, 8, rng)[None]
    st = oracle.stats(payload, eb)[0]
    assert (st.n_unique_raw, st.n_unique_quant, st.n_rows, st.count) == (n_ori, n_quant, batch, batch * 8)
    assert abs((1.0 - oracle.homo_index(st.n_unique_raw, st.n_unique_quant)) - float(printed)) < 5e-7


def test_stats_brute_force_small():
    rng = np.random.default_rng(7)
    for trial in range(30):
        T, B, D = int(rng.integers(1, 4)), int(rng.integers(1, 40)), int(rng.integers(1, 6))
        eb = float(rng.choice([1e-3, 0.02, 0.3]))
        vals = rng.choice(np.linspace(-1, 1, 9), (T, B, D)).astype(np.float32)  # few values: many duplicates
        vals += (rng.random((T, B, D)) < 0.2) * np.float32(eb * 0.3)            # merge only after quantisation
        st = oracle.stats(vals, eb)
        for t in range(T):
            raw = {tuple(r.view(np.uint32)) for r in vals[t]}
            sym, _ = oracle.quantize(vals[t], eb)
            qs = {tuple(r) for r in sym}
            assert st[t].n_unique_raw == len(raw)
            assert st[t].n_unique_quant == len(qs)
            assert st[t].min == vals[t].min() and st[t].max == vals[t].max()
            assert st[t].count == B * D and st[t].n_rows == B


def test_stats_sign_of_zero_and_nonfinite():
    x = np.array([[[0.0, 1.0], [-0.0, 1.0], [np.nan, np.inf], [np.nan, np.inf]]], np.float32)
    st = oracle.stats(x, 0.1)[0]
    assert st.n_unique_raw == 3          # +0 and -0 rows differ in raw bits
    assert st.n_unique_quant == 2        # they share a bin; the non-finite rows are all escapes
    assert st.min == 0.0 and st.max == 1.0  # over finite elements only


def _params(**kw):
    p = oracle.ControllerParams()
    p.mode, p.decay_kind = 0, 0
    p.global_eb, p.alpha, p.beta = 0.03, 5.0 / 3.0, 3.0
    p.h_large, p.h_small = 0.0, 0.05
    p.decay_start, p.decay_len, p.decay_steps, p.decay_mult0 = 0, 100, 5, 2.0
    p.eb_min = p.eb_max = p.rel_floor = 0.0
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def _stats_with(pairs, lo=-1.0, hi=1.0):
    st = (oracle.TableStats * len(pairs))()
    for s, (a, b) in zip(st, pairs):
        s.min, s.max, s.count, s.n_rows, s.n_unique_raw, s.n_unique_quant, s.probe_eb = lo, hi, 1, 1, a, b, 0.01
    return st


def test_class_bounds_of_section_iv():
    """GlobalEB 0.03 with alpha 5/3, beta 3 gives the printed 0.05 / 0.03 / 0.01."""
    bounds, _ = _class_gold()
    st = _stats_with([(100, 100)] * 3)
    eb, cls = oracle.controller(st, _params(), 0, class_override=[oracle.CLASS_LARGE, oracle.CLASS_MEDIUM,
                                                                   oracle.CLASS_SMALL])
    assert list(cls) == [oracle.CLASS_LARGE, oracle.CLASS_MEDIUM, oracle.CLASS_SMALL]
    assert eb[0] == np.float32(bounds["large"])
    assert eb[1] == np.float32(bounds["medium"])
    assert eb[2] == np.float32(bounds["small"])


def test_classification_agrees_with_table_ii():
    """eta = 1 - printed; every listed table with printed < 1 is class S, printed == 1 is M."""
    _, letters = _class_gold()
    for ds, tid, _, n_ori, n_quant, _, _ in _homo_rows():
        eta = oracle.homo_index(n_ori, n_quant)
        cls = oracle.classify(eta, 0.0, 0.05)
        want = {"S": oracle.CLASS_SMALL, "M": oracle.CLASS_MEDIUM, "L": oracle.CLASS_LARGE}[letters[(ds, tid)]]
        assert cls == want, (ds, tid, eta)


def test_classification_is_algorithm_1():
    assert oracle.classify(0.5, 0.1, 0.3) == oracle.CLASS_SMALL
    assert oracle.classify(0.05, 0.1, 0.3) == oracle.CLASS_LARGE
    assert oracle.classify(0.2, 0.1, 0.3) == oracle.CLASS_MEDIUM
    assert oracle.classify(0.3, 0.1, 0.3) == oracle.CLASS_MEDIUM   # strict comparisons
    assert oracle.classify(0.1, 0.1, 0.3) == oracle.CLASS_MEDIUM


def test_stepwise_schedule_shape():
    """Decay_kx: from k*base at the start of the initial phase to base at its end, then constant."""
    for M0, Ks, I, i0 in [(2.0, 5, 100, 0), (3.0, 4, 37, 10), (2.0, 1, 8, 0), (2.0, 7, 5, 3)]:
        p = _params(decay_kind=1, decay_mult0=M0, decay_steps=Ks, decay_len=I, decay_start=i0)
        m = [oracle.decay_multiplier(p, i) for i in range(0, i0 + I + 50)]
        assert m[i0] == M0
        assert all(v == M0 for v in m[:i0 + 1])
        assert all(v == 1.0 for v in m[i0 + I:])
        assert all(a >= b for a, b in zip(m, m[1:]))
        levels = sorted(set(m), reverse=True)
        assert levels[0] == M0 and levels[-1] == 1.0
        drops = sum(1 for a, b in zip(m, m[1:]) if b < a)
        assert drops == min(Ks, I)            # exactly K_s drops when the phase is long enough
        if Ks <= I:
            for s, lv in enumerate(levels):   # equally spaced stairs
                assert abs(lv - (M0 - (M0 - 1.0) * s / Ks)) < 1e-15


def test_drop_schedule():
    p = _params(decay_kind=2, decay_mult0=3.0, decay_len=40, decay_start=0)
    m = [oracle.decay_multiplier(p, i) for i in range(80)]
    assert m[:40] == [3.0] * 40 and m[40:] == [1.0] * 40


def test_linear_and_logarithmic_schedules():
    """The paper names a logarithmic decay next to the stepwise one and fixes only the end points (k x base at the
    start of the initial phase, base after it).  Pinned here: those end points, monotone decrease, the straight line
    for LINEAR, and for LOG the closed form on a few points plus its shape (below the line: fast at first)."""
    import math
    for M0, I, i0 in [(2.0, 100, 0), (3.0, 37, 10), (1.5, 8, 3)]:
        lin = [oracle.decay_multiplier(_params(decay_kind=3, decay_mult0=M0, decay_len=I, decay_start=i0), i)
               for i in range(0, i0 + I + 20)]
        lg = [oracle.decay_multiplier(_params(decay_kind=4, decay_mult0=M0, decay_len=I, decay_start=i0), i)
              for i in range(0, i0 + I + 20)]
        for m in (lin, lg):
            assert all(v == M0 for v in m[:i0 + 1]) and all(v == 1.0 for v in m[i0 + I:])
            assert all(a >= b for a, b in zip(m, m[1:]))
            assert all(1.0 <= v <= M0 for v in m)
        for k in range(I):
            assert abs(lin[i0 + k] - (M0 - (M0 - 1.0) * k / I)) < 1e-15
            assert abs(lg[i0 + k] - (M0 - (M0 - 1.0) * math.log1p(k) / math.log1p(I))) < 1e-12
        assert all(lg[i0 + k] < lin[i0 + k] for k in range(1, I))     # concave in log(1 + k): drops fast at first
        assert lg[i0 + I - 1] > 1.0                                    # reaches the base only at the end of the phase


def test_controller_bound_arithmetic():
    st = _stats_with([(100, 100), (100, 50), (100, 100)], lo=-0.5, hi=1.5)
    # absolute, stepwise at iteration 0 -> doubled
    eb, cls = oracle.controller(st, _params(decay_kind=1), 0)
    assert list(cls) == [oracle.CLASS_MEDIUM, oracle.CLASS_SMALL, oracle.CLASS_MEDIUM]
    assert eb[0] == np.float32(0.06) and eb[1] == np.float32(0.03 / 3.0 * 2.0)
    # after the phase -> base
    eb, _ = oracle.controller(st, _params(decay_kind=1), 100)
    assert eb[0] == np.float32(0.03) and eb[1] == np.float32(0.03 / 3.0)
    # range-relative
    eb, _ = oracle.controller(st, _params(mode=1), 0)
    assert eb[0] == np.float32(0.03 * 2.0) and eb[1] == np.float32(0.03 * 2.0 / 3.0)
    # clamp
    eb, _ = oracle.controller(st, _params(eb_min=0.02, eb_max=0.025), 0)
    assert eb[0] == np.float32(0.025) and eb[1] == np.float32(0.02)
    # relative floor (fp16 payloads): eb >= 2^-10 * range
    eb, _ = oracle.controller(st, _params(global_eb=1e-4, rel_floor=2.0 ** -10), 0)
    assert eb[0] == np.float32(2.0 ** -10 * 2.0) and eb[1] == np.float32(2.0 ** -10 * 2.0)
