"""Pins of the oracle's chunked bitstream, container and decoder."""
import numpy as np
import pytest

import container_reader as cr
import dlc_workloads as W
import oracle

R = 512


def _payload(T, B, D, seed, sigma=0.02, dtype=np.float32):
    rng = np.random.default_rng(seed)
    table = (rng.standard_normal((50, D)) * sigma).astype(np.float32)
    idx = rng.integers(0, 50, (T, B))
    x = table[idx] * (1 + np.arange(T, dtype=np.float32)[:, None, None])
    return x.astype(dtype)


CASES = [  # T, B, D, S, eb
    (1, 256, 16, 256, 1e-3),    # less than one group
    (2, 37, 13, 8, 2e-3),       # ragged: B*D = 481, not a multiple of V, several small groups
    (3, 100, 64, 16, 5e-3),     # several groups and a partial last one
    (1, 3, 1, 4, 1e-3),         # three symbols
    (2, 64, 8, 4, 1.0),         # eb above the data: one symbol, empty payload
]


@pytest.mark.parametrize("T,B,D,S,eb", CASES)
def test_every_chunk_decodes_independently(T, B, D, S, eb):
    x = _payload(T, B, D, B + D)
    x.reshape(-1)[::97] = 1e6                                     # escapes
    c = oracle.compress(x, eb, R, S, 12)
    assert c.rc == oracle.OK
    cont = cr.parse(c.data)
    cr.check_layout(cont)
    assert (cont.T, cont.B, cont.D, cont.R, cont.S, cont.LMAX, cont.dtype) == (T, B, D, R, S, 12, 0)
    sym = cr.decode_symbols(cont)
    want, rec = oracle.quantize(x, eb, R)
    assert np.array_equal(sym, want.reshape(T, -1))
    # escapes listed in increasing index order with the input's raw bits
    for t, o in enumerate(cr.outliers(cont)):
        where = np.nonzero(want[t].reshape(-1) == 0)[0]
        assert np.array_equal(o[:, 0], where)
        assert np.array_equal(o[:, 1], x[t].reshape(-1).view(np.uint32)[where])
    # histogram in the container's code lengths: unused symbols have length 0
    for t, tb in enumerate(cont.tables):
        h = np.bincount(want[t].reshape(-1), minlength=2 * R)
        assert tb.sym_lo == np.nonzero(h)[0][0] and tb.sym_hi == np.nonzero(h)[0][-1]
        assert tb.n_used == np.count_nonzero(h)
        assert tb.eb == np.float32(eb)
    # size metadata: total, and the per-table shares plus fixed parts add up
    assert c.sizes[0] == c.data.size
    pads = cont.total_bytes - int(c.sizes[1:].sum()) - cr.HEADER
    assert 0 <= pads < 16 * 5


@pytest.mark.parametrize("T,B,D,S,eb", CASES)
def test_round_trip_and_reencode(T, B, D, S, eb):
    x = _payload(T, B, D, 3 * B + D)
    x.reshape(-1)[::53] = np.float32(np.nan)
    c = oracle.compress(x, eb, R, S, 12)
    rc, out, sym = oracle.decompress(c.data, x.shape, np.float32, want_symbols=True)
    assert rc == oracle.OK
    want_sym, want_rec = oracle.quantize(x, eb, R)
    assert np.array_equal(sym, want_sym)
    assert np.array_equal(out.view(np.uint32), want_rec.view(np.uint32))
    esc = want_sym == 0
    deq = (want_sym.astype(np.int32) - R).astype(np.float32) * (np.float32(eb) * np.float32(2))
    assert np.array_equal(out[~esc].view(np.uint32), deq[~esc].view(np.uint32))
    assert np.array_equal(out[esc].view(np.uint32), x[esc].view(np.uint32))
    fin = np.isfinite(x)
    assert np.all(np.abs(x[fin].astype(np.float64) - out[fin].astype(np.float64)) <= np.float32(eb) * (1 + 1e-6))
    # compressing the reconstruction gives the same bytes back
    c2 = oracle.compress(out, eb, R, S, 12)
    assert np.array_equal(c2.data, c.data)


def test_f16_round_trip():
    x = _payload(2, 200, 32, 9, sigma=0.05, dtype=np.float16)
    eb = 2.0 ** -10 * float(x.max() - x.min())
    c = oracle.compress(x, eb, R, 32, 12)
    cont = cr.parse(c.data)
    cr.check_layout(cont)
    assert cont.dtype == 1
    sym = cr.decode_symbols(cont)
    want, rec = oracle.quantize(x, eb, R)
    assert np.array_equal(sym, want.reshape(2, -1))
    rc, out = oracle.decompress(c.data, x.shape, np.float16)
    assert rc == oracle.OK and np.array_equal(out.view(np.uint16), rec.view(np.uint16))
    assert np.all(np.abs(x.astype(np.float64) - out.astype(np.float64)) <= np.float32(eb) * (1 + 1e-6))
    for t, o in enumerate(cr.outliers(cont)):
        where = np.nonzero(want[t].reshape(-1) == 0)[0]
        assert len(where) > 0
        assert np.array_equal(o[:, 0], where)
        assert np.array_equal(o[:, 1], x[t].reshape(-1).view(np.uint16)[where].astype(np.uint32))


def test_per_table_bounds_and_workload1():
    w = W.workload1()
    c = oracle.compress(w.payload, 1e-3)
    cont = cr.parse(c.data)
    cr.check_layout(cont)
    sym = cr.decode_symbols(cont)
    want, _ = oracle.quantize(w.payload, 1e-3)
    assert np.array_equal(sym, want.reshape(1, -1))
    # mean code length within one bit of the entropy (Huffman), container overhead on top
    h = np.bincount(want.reshape(-1)).astype(np.float64)
    p = h[h > 0] / h.sum()
    H = -(p * np.log2(p)).sum()
    bits = sum(int(l) * int(h[cont.tables[0].sym_lo + i]) for i, l in enumerate(cont.tables[0].lengths))
    assert H * want.size <= bits < (H + 1) * want.size
    # different bounds per table
    x = _payload(3, 64, 16, 1)
    ebs = np.array([1e-3, 4e-3, 0.02], np.float32)
    c = oracle.compress(x, ebs, R, 16, 12)
    rc, out = oracle.decompress(c.data, x.shape, np.float32)
    for t in range(3):
        assert np.all(np.abs(x[t].astype(np.float64) - out[t]) <= ebs[t] * (1 + 1e-6))
        assert cr.parse(c.data).tables[t].eb == ebs[t]


def test_long_codes_fill_a_chunk_to_its_limit():
    """A skewed alphabet drives code lengths to LMAX; the u8 word count of a chunk must still fit."""
    fib = [1, 1]
    while len(fib) < 26:
        fib.append(fib[-1] + fib[-2])
    vals = np.repeat(np.arange(26), fib).astype(np.float32) * np.float32(0.02)
    rng = np.random.default_rng(0)
    rng.shuffle(vals)
    x = vals[: (vals.size // 16) * 16].reshape(1, -1, 16)
    c = oracle.compress(x, 0.01, R, 256, 12)
    cont = cr.parse(c.data)
    assert cont.tables[0].lengths.max() == 12
    rc, out = oracle.decompress(c.data, x.shape, np.float32)
    assert rc == oracle.OK and np.all(np.abs(out - x) <= 0.01 * (1 + 1e-6))


def test_errors():
    x = _payload(2, 32, 8, 5)
    c = oracle.compress(x, 1e-3, R, 8, 12)
    n = c.data.size
    assert oracle.compress(x, 1e-3, R, 8, 12, capacity=n - 1).rc == oracle.ECAPACITY
    assert oracle.compress(x, 1e-3, R, 8, 12, capacity=n).rc == oracle.OK
    assert oracle.compress(x, 0.0, R, 8, 12).rc == oracle.EINVAL
    assert oracle.compress(x, float("nan"), R, 8, 12).rc == oracle.EINVAL
    assert oracle.compress(x, 1e-3, 500, 8, 12, capacity=1 << 20).rc == oracle.EINVAL       # R not a power of two
    assert oracle.compress(x, 1e-3, R, 6, 12, capacity=1 << 20).rc == oracle.EINVAL         # S not a multiple of V
    assert oracle.compress(x, 1e-3, R, 8, 9, capacity=1 << 20).rc == oracle.EINVAL          # 2^LMAX < alphabet
    bad = c.data.copy()
    bad[0] ^= 1
    assert oracle.decompress(bad, x.shape, np.float32)[0] == oracle.ECORRUPT                # magic
    assert oracle.decompress(c.data[:-4], x.shape, np.float32)[0] == oracle.ECORRUPT        # truncated
    assert oracle.decompress(c.data[:64], x.shape, np.float32)[0] == oracle.ECORRUPT
    bad = c.data.copy()
    cont = cr.parse(c.data)
    bad[cont.tables[0].codebook_off] = 13                                                    # length beyond LMAX
    assert oracle.decompress(bad, x.shape, np.float32)[0] == oracle.ECORRUPT
    bad = c.data.copy()
    bad[cont.tables[0].codebook_off] += 1                                                    # Kraft sum broken
    assert oracle.decompress(bad, x.shape, np.float32)[0] == oracle.ECORRUPT


def test_directory_offsets_near_2_to_64_are_refused():
    """A damaged directory whose byte offsets sit just under 2^64 must fail the range test, not wrap past it."""
    x = _payload(2, 32, 8, 5)
    c = oracle.compress(x, 1e-3, R, 8, 12)
    for t in (0, 1):
        entry = 128 + 56 * t
        for off in (2 ** 64 - 1, 2 ** 64 - 4, 2 ** 64 - 1024):
            bad = c.data.copy()
            bad[entry + 24:entry + 32] = np.frombuffer(np.uint64(off).tobytes(), np.uint8)   # code-length block
            assert oracle.decompress(bad, x.shape, np.float32)[0] == oracle.ECORRUPT
            bad = c.data.copy()
            bad[entry + 32:entry + 40] = np.frombuffer(np.uint64(off).tobytes(), np.uint8)   # row references
            assert oracle.decompress(bad, x.shape, np.float32)[0] == oracle.ECORRUPT


def test_compress_bound_is_an_upper_bound():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 50, 24)).astype(np.float32)       # wide alphabet
    x[0, :10] = np.inf                                            # and escapes
    for S in (4, 16, 256):
        c = oracle.compress(x, 1e-3, R, S, 12)
        assert c.rc == oracle.OK
        assert c.data.size <= oracle.compress_bound(oracle.F32, 2, 50, 24, R, S, 12)
