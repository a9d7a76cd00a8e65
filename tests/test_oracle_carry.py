"""Pins of the oracle's carried-codebook mode (a table coded with the codebook of an earlier payload's counts).

What fixes the result without reference to the oracle itself: the independent Python stream reader decodes the
container; the symbols it finds must be the quantiser's, with every symbol the earlier counts lack turned into an
escape; the code lengths in the container must be those of the (separately pinned) codebook routine on the earlier
counts with the escape's count raised by one; the escape records must list exactly those elements, raw bits intact;
the reported counts must equal numpy's bincount; the bound must hold on every element.
"""
import numpy as np
import pytest

import container_reader as cr
import oracle

R = 512
K = 2 * R


def _batch(T, B, D, seed, sigma=0.02, shift=0.0):
    rng = np.random.default_rng(seed)
    table = (rng.standard_normal((80, D)) * sigma + shift).astype(np.float32)
    idx = rng.integers(0, 80, (T, B))
    return (table[idx] * (1 + np.arange(T, dtype=np.float32)[:, None, None])).astype(np.float32)


def _expected_symbols(sym, prev_hist):
    """quantiser symbols with everything the carried counts (escape raised by one) lack turned into an escape."""
    out = sym.copy()
    for t in range(sym.shape[0]):
        h = prev_hist[t].copy()
        h[0] += 1
        s = out[t].reshape(-1)
        s[h[s] == 0] = 0
    return out


CASES = [  # T, B, D, S, eb
    (2, 256, 16, 256, 1e-3),
    (2, 37, 13, 8, 2e-3),       # ragged
    (3, 100, 64, 16, 5e-3),
]


@pytest.mark.parametrize("T,B,D,S,eb", CASES)
def test_carried_container_is_what_the_definition_says(T, B, D, S, eb):
    x0 = _batch(T, B, D, 11 * B + D)
    x1 = _batch(T, B, D, 13 * B + D)          # same tables' distribution, other rows
    x1.reshape(-1)[::101] = 1e6                # true escapes
    first = oracle.compress(x0, eb, R, S, 12, want_hist=True)
    assert first.rc == oracle.OK
    # the counts reported are the quantiser's symbol counts
    sym0, _ = oracle.quantize(x0, eb, R)
    for t in range(T):
        assert np.array_equal(first.hist[t], np.bincount(sym0[t].reshape(-1), minlength=K).astype(np.uint64))
    # asking for the counts does not change the container
    assert np.array_equal(first.data, oracle.compress(x0, eb, R, S, 12).data)

    second = oracle.compress(x1, eb, R, S, 12, carry_hist=first.hist, want_hist=True)
    assert second.rc == oracle.OK
    sym1, rec1 = oracle.quantize(x1, eb, R)
    for t in range(T):                         # counts of the new payload, before any substitution
        assert np.array_equal(second.hist[t], np.bincount(sym1[t].reshape(-1), minlength=K).astype(np.uint64))
    want = _expected_symbols(sym1.reshape(T, -1), first.hist)
    cont = cr.parse(second.data)
    cr.check_layout(cont)
    got = cr.decode_symbols(cont)
    assert np.array_equal(got, want)
    assert (want == 0).sum() > (sym1 == 0).sum()          # the case has symbols without a code
    for t, tb in enumerate(cont.tables):
        h = first.hist[t].copy()
        h[0] += 1
        ln, _, n_used, _ = oracle.codebook(h, 12)
        nz = np.nonzero(h)[0]
        assert (tb.sym_lo, tb.sym_hi, tb.n_used) == (nz[0], nz[-1], n_used)
        assert np.array_equal(np.asarray(tb.lengths), ln[nz[0]:nz[-1] + 1])
        assert ln[0] > 0                                   # the escape always has a code
    for t, o in enumerate(cr.outliers(cont)):
        where = np.nonzero(want[t] == 0)[0]
        assert np.array_equal(o[:, 0], where)
        assert np.array_equal(o[:, 1], x1[t].reshape(-1).view(np.uint32)[where])
    # decoder: escapes bit for bit, everything else the quantiser's reconstruction; the bound on every element
    rc, out = oracle.decompress(second.data, x1.shape, np.float32)
    assert rc == oracle.OK
    esc = want.reshape(x1.shape) == 0
    assert np.array_equal(out[esc].view(np.uint32), x1[esc].view(np.uint32))
    assert np.array_equal(out[~esc].view(np.uint32), rec1[~esc].view(np.uint32))
    assert np.all(np.abs(x1.astype(np.float64) - out.astype(np.float64)) <= np.float32(eb) * (1 + 1e-6))


def test_carried_from_own_counts_costs_at_most_the_escape_code():
    """Carrying a payload's own counts changes nothing but the escape's extra count: no new escapes, and the size
    stays within one bit per symbol of the two-pass container."""
    x = _batch(2, 512, 32, 5)
    a = oracle.compress(x, 1e-3, R, 64, 12, want_hist=True)
    b = oracle.compress(x, 1e-3, R, 64, 12, carry_hist=a.hist)
    ca, cb = cr.parse(a.data), cr.parse(b.data)
    assert np.array_equal(cr.decode_symbols(ca), cr.decode_symbols(cb))
    assert abs(int(b.data.size) - int(a.data.size)) <= x.size // 8


def test_payload_unlike_the_carried_counts_is_all_escapes():
    x0 = _batch(1, 128, 16, 7)
    x1 = _batch(1, 128, 16, 8, shift=0.3)                  # far away from anything the counts contain
    a = oracle.compress(x0, 1e-3, R, 64, 12, want_hist=True)
    b = oracle.compress(x1, 1e-3, R, 64, 12, carry_hist=a.hist)
    assert b.rc == oracle.OK
    cont = cr.parse(b.data)
    assert np.all(cr.decode_symbols(cont) == 0)
    rc, out = oracle.decompress(b.data, x1.shape, np.float32)
    assert rc == oracle.OK and np.array_equal(out.view(np.uint32), x1.view(np.uint32))


def test_constant_table_gets_a_one_bit_code():
    """One symbol in the carried counts plus the escape: two codes of one bit each."""
    x = np.zeros((1, 64, 16), np.float32)
    a = oracle.compress(x, 1e-3, R, 64, 12, want_hist=True)
    assert cr.parse(a.data).tables[0].n_used == 1
    b = oracle.compress(x, 1e-3, R, 64, 12, carry_hist=a.hist)
    tb = cr.parse(b.data).tables[0]
    assert tb.n_used == 2 and (tb.sym_lo, tb.sym_hi) == (0, R)
    assert tb.lengths[0] == 1 and tb.lengths[-1] == 1


def test_carry_hist_shape_is_checked():
    x = _batch(2, 64, 16, 3)
    with pytest.raises(ValueError):
        oracle.compress(x, 1e-3, R, 64, 12, carry_hist=np.zeros((1, K), np.uint64))
