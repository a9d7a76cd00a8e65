"""Pins of the oracle's row matching (the vector-based LZ step: a row equal to an earlier row of its table in the batch
is stored as a reference to the first such row).

Independent of the oracle: numpy finds the first occurrence of every distinct row; the plain Python stream reader
decodes the container and must find exactly the quantiser's symbols in the coded rows and nothing for the others;
the layout adds up; the decoder's output must equal that of the same payload compressed without row matching.
"""
import numpy as np
import pytest

import container_reader as cr
import oracle

R = 512


def _lookups(T, B, D, seed, rows=40, sigma=0.02):
    rng = np.random.default_rng(seed)
    table = (rng.standard_normal((T, rows, D)) * sigma).astype(np.float32)
    idx = rng.integers(0, rows, (T, B))
    return np.stack([table[t][idx[t]] for t in range(T)])


def first_occurrence(x, sym):
    """ref[t][i] = smallest row index of table t whose row equals row i in symbols and, at escapes, in raw bits."""
    T, B, D = x.shape
    raw = x.view(np.uint32 if x.dtype == np.float32 else np.uint16).astype(np.uint64)
    ident = np.where(sym != 0, sym.astype(np.uint64), (np.uint64(1) << np.uint64(32)) | raw)
    ref = np.zeros((T, B), np.uint32)
    for t in range(T):
        _, first, inv = np.unique(ident[t], axis=0, return_index=True, return_inverse=True)
        ref[t] = first[inv.reshape(-1)]
    return ref


CASES = [  # T, B, D, S, eb
    (2, 300, 16, 64, 1e-3),
    (3, 257, 20, 16, 2e-3),      # ragged groups, rows that straddle chunk turns (D = 20)
    (1, 64, 64, 256, 5e-3),
]


@pytest.mark.parametrize("T,B,D,S,eb", CASES)
def test_container_is_what_the_definition_says(T, B, D, S, eb):
    x = _lookups(T, B, D, 7 * B + D)
    x[0, 3, 1] = 1e9                       # an escape ...
    x[0, 8] = x[0, 3]                      # ... in a row that is repeated with the same raw bits
    x[0, 11] = x[0, 3]
    x[0, 11, 1] = 2e9                      # same symbols (escape at the same place), other raw bits: not equal
    c = oracle.compress(x, eb, R, S, 12, row_match=True)
    assert c.rc == oracle.OK
    sym, rec = oracle.quantize(x, eb, R)
    ref = first_occurrence(x, sym)
    assert ref[0, 8] == 3 and ref[0, 11] == 11
    cont = cr.parse(c.data)
    cr.check_layout(cont)
    got = cr.decode_symbols(cont).reshape(T, B, D)
    for t, tb in enumerate(cont.tables):
        assert tb.ref_off != 0 and np.array_equal(tb.ref, ref[t])
        coded = ref[t] == np.arange(B)
        assert np.array_equal(got[t][coded], sym[t][coded])
        assert np.all(got[t][~coded] == 0xFFFF)
        h = np.bincount(sym[t][coded].reshape(-1), minlength=2 * R)      # only coded rows count
        assert (tb.sym_lo, tb.sym_hi, tb.n_used) == (np.nonzero(h)[0][0], np.nonzero(h)[0][-1], np.count_nonzero(h))
        ln, _, _, _ = oracle.codebook(h.astype(np.uint64), 12)
        assert np.array_equal(np.asarray(tb.lengths), ln[tb.sym_lo:tb.sym_hi + 1])
    for t, o in enumerate(cr.outliers(cont)):                            # escapes of coded rows only
        coded_el = np.repeat(ref[t] == np.arange(B), D)
        where = np.nonzero((sym[t].reshape(-1) == 0) & coded_el)[0]
        assert np.array_equal(o[:, 0], where)
        assert np.array_equal(o[:, 1], x[t].reshape(-1).view(np.uint32)[where])
    # the decoder gives what the plain path gives, bit for bit
    rc, out = oracle.decompress(c.data, x.shape, np.float32)
    plain = oracle.compress(x, eb, R, S, 12)
    rc2, out2 = oracle.decompress(plain.data, x.shape, np.float32)
    assert rc == 0 and rc2 == 0 and np.array_equal(out.view(np.uint32), out2.view(np.uint32))
    assert c.data.size < plain.data.size
    assert int(c.sizes[0]) == c.data.size


def test_flags_per_table_and_no_flag():
    x = _lookups(3, 200, 16, 5)
    plain = oracle.compress(x, 1e-3, R, 64, 12)
    assert np.array_equal(oracle.compress(x, 1e-3, R, 64, 12, row_match=[0, 0, 0]).data, plain.data)
    mixed = oracle.compress(x, 1e-3, R, 64, 12, row_match=[0, 1, 0])
    cont = cr.parse(mixed.data)
    cr.check_layout(cont)
    assert [tb.ref_off != 0 for tb in cont.tables] == [False, True, False]
    rc, out = oracle.decompress(mixed.data, x.shape, np.float32)
    rc2, out2 = oracle.decompress(plain.data, x.shape, np.float32)
    assert rc == 0 and np.array_equal(out.view(np.uint32), out2.view(np.uint32))


def test_no_repeats_and_all_repeats():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((1, 128, 16)) * 0.02).astype(np.float32)          # all rows different
    a = oracle.compress(x, 1e-3, R, 64, 12)
    b = oracle.compress(x, 1e-3, R, 64, 12, row_match=True)
    tb = cr.parse(b.data).tables[0]
    assert np.array_equal(tb.ref, np.arange(128))
    assert b.data.size == (a.data.size + 15) // 16 * 16 + 4 * 128             # the references are all it adds
    y = np.repeat(x[:, :1], 128, axis=1)                                        # one row, 128 times
    c = oracle.compress(y, 1e-3, R, 64, 12, row_match=True)
    cont = cr.parse(c.data)
    cr.check_layout(cont)
    assert np.all(cont.tables[0].ref == 0)
    rc, out = oracle.decompress(c.data, y.shape, np.float32)
    assert rc == 0 and np.all(out == out[:, :1])
    assert np.all(np.abs(out.astype(np.float64) - y) <= 1e-3 * (1 + 1e-6))


def test_damaged_references_are_rejected():
    x = _lookups(1, 100, 16, 9)
    c = oracle.compress(x, 1e-3, R, 64, 12, row_match=True)
    tb = cr.parse(c.data).tables[0]
    bad = c.data.copy()
    i = int(np.nonzero(tb.ref != np.arange(100))[0][0])
    bad[tb.ref_off + 4 * i:tb.ref_off + 4 * i + 4] = np.frombuffer(np.uint32(i + 1).tobytes(), np.uint8)   # points forward
    assert oracle.decompress(bad, x.shape, np.float32)[0] == oracle.ECORRUPT
    bad = c.data.copy()
    j = int(tb.ref[i])
    k = int(np.nonzero(tb.ref != np.arange(100))[0][1])
    bad[tb.ref_off + 4 * k:tb.ref_off + 4 * k + 4] = np.frombuffer(np.uint32(i).tobytes(), np.uint8) if i < k else bad[tb.ref_off + 4 * k:tb.ref_off + 4 * k + 4]
    if i < k:                                                              # points at a row that is itself a reference
        assert oracle.decompress(bad, x.shape, np.float32)[0] == oracle.ECORRUPT
