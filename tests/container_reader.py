"""A third reading of the container, in plain Python, for the tests only.

It shares nothing with the oracle's C or the HIP library: it walks the bytes as the format
description says and decodes each chunk on its own, starting from that chunk's word offset.
Slow by design; use on small inputs.
"""
from __future__ import annotations

import struct
from dataclasses import dataclass

import numpy as np

W, V = 64, 4
HEADER, DIRENT = 128, 56


def _a16(x):
    return (x + 15) // 16 * 16


@dataclass
class Table:
    eb: float
    n_used: int
    sym_lo: int
    sym_hi: int
    n_outliers: int
    n_groups: int
    codebook_off: int
    ref_off: int               # row matching: byte offset of u32 ref[B]; 0 = the table does not use it
    payload_word_off: int
    payload_words: int
    lengths: np.ndarray
    ref: np.ndarray | None = None


@dataclass
class Container:
    dtype: int
    T: int
    B: int
    D: int
    R: int
    S: int
    LMAX: int
    n_groups_total: int
    n_outliers_total: int
    payload_words_total: int
    off_group: int
    off_chunk: int
    off_payload: int
    off_codebook: int
    total_bytes: int
    tables: list
    group_off: np.ndarray
    chunk_words: np.ndarray
    words: np.ndarray
    raw: bytes


def parse(buf) -> Container:
    raw = bytes(buf)
    f = struct.unpack_from("<12I", raw, 0)
    q = struct.unpack_from("<7Q", raw, 48)
    assert f[0] == 0x32434C44 and f[1] == 2, "magic/version"
    assert raw[104:128] == b"\0" * 24
    dtype, T, B, D, R, S, LMAX, w, v, NG = f[2:12]
    assert (w, v) == (W, V)
    n_out, n_words, off_g, off_c, off_p, off_cb, total = q
    assert total == len(raw), (total, len(raw))
    tables = []
    for t in range(T):
        e = struct.unpack_from("<6I4Q", raw, HEADER + DIRENT * t)
        eb = struct.unpack("<f", struct.pack("<I", e[0]))[0]
        ln = np.frombuffer(raw, np.uint8, e[3] - e[2] + 1, e[6])
        ref = np.frombuffer(raw, np.uint32, B, e[7]) if e[7] else None
        tables.append(Table(eb, e[1], e[2], e[3], e[4], e[5], e[6], e[7], e[8], e[9], ln, ref))
    group_off = np.frombuffer(raw, np.uint32, NG, off_g)
    chunk_words = np.frombuffer(raw, np.uint8, W * NG, off_c)
    words = np.frombuffer(raw, np.uint32, n_words, off_p)
    return Container(dtype, T, B, D, R, S, LMAX, NG, n_out, n_words, off_g, off_c, off_p, off_cb, total,
                     tables, group_off, chunk_words, words, raw)


def group_extent(c: Container, gi: int):
    """(first word, number of chunk words, number of escape records) of global group gi."""
    start = int(c.group_off[gi])
    end = int(c.group_off[gi + 1]) if gi + 1 < c.n_groups_total else c.payload_words_total
    cw = int(c.chunk_words[gi * W:(gi + 1) * W].astype(np.int64).sum())
    assert end >= start + cw and (end - start - cw) % 2 == 0
    return start, cw, (end - start - cw) // 2


def check_layout(c: Container):
    """Sizes add up; every section sits where the format says; padding is zero."""
    n = c.B * c.D
    G = -(-n // (W * c.S))
    NG = G * c.T
    assert c.n_groups_total == NG
    e = HEADER + DIRENT * c.T
    assert c.off_group == _a16(e) and c.raw[e:c.off_group] == b"\0" * (c.off_group - e)
    e = c.off_group + 4 * NG
    assert c.off_chunk == _a16(e) and c.raw[e:c.off_chunk] == b"\0" * (c.off_chunk - e)
    assert c.off_payload == c.off_chunk + W * NG and c.off_payload % 16 == 0
    e = c.off_payload + 4 * c.payload_words_total
    assert c.off_codebook == _a16(e) and c.raw[e:c.off_codebook] == b"\0" * (c.off_codebook - e)
    cur = c.off_codebook
    words = 0
    outl = 0
    for t, tb in enumerate(c.tables):
        assert tb.n_groups == G
        assert tb.codebook_off == cur
        nlen = tb.sym_hi - tb.sym_lo + 1
        pad = (nlen + 3) // 4 * 4
        assert c.raw[cur + nlen:cur + pad] == b"\0" * (pad - nlen)
        cur += pad
        assert tb.payload_word_off == words
        assert tb.payload_word_off == int(c.group_off[t * G])
        words += tb.payload_words
        n_esc = sum(group_extent(c, t * G + g)[2] for g in range(G))
        assert n_esc == tb.n_outliers
        outl += tb.n_outliers
        if tb.n_used == 1:
            assert tb.sym_lo == tb.sym_hi and tb.lengths[0] == 0 and tb.payload_words == 2 * tb.n_outliers
        else:
            assert np.count_nonzero(tb.lengths) == tb.n_used and tb.lengths[0] and tb.lengths[-1]
    # row references of the tables that have them: behind the code-length blocks, each 16-byte aligned, zero padding
    for tb in c.tables:
        if tb.ref_off:
            assert tb.ref_off == _a16(cur) and c.raw[cur:tb.ref_off] == b"\0" * (tb.ref_off - cur)
            cur = tb.ref_off + 4 * c.B
            rows = np.arange(c.B, dtype=np.uint32)
            assert np.all(tb.ref <= rows) and np.array_equal(tb.ref[tb.ref], tb.ref)   # points back, at a coded row
    assert cur == c.total_bytes
    assert outl == c.n_outliers_total and words == c.payload_words_total
    # group offsets are the exclusive prefix sum of (chunk words + two words per escape)
    pos = 0
    for gi in range(NG):
        start, cw, ne = group_extent(c, gi)
        assert start == pos
        pos += cw + 2 * ne
    assert pos == c.payload_words_total


def _canonical(lengths, sym_lo, LMAX):
    """symbol and length for each codeword, as a dict from (length, value) -> symbol."""
    order = sorted((int(l), sym_lo + i) for i, l in enumerate(lengths) if l)
    book = {}
    code, prev = 0, None
    for l, s in order:
        if prev is not None:
            code = (code + 1) << (l - prev)
        prev = l
        book[(l, code)] = s
    return book


def decode_symbols(c: Container) -> np.ndarray:
    """Symbols [T, B*D], every chunk decoded independently from its own offset."""
    n = c.B * c.D
    G = -(-n // (W * c.S))
    out = np.full((c.T, n), 0xFFFF, np.uint16)
    for t, tb in enumerate(c.tables):
        book = _canonical(tb.lengths, tb.sym_lo, c.LMAX) if tb.n_used > 1 else None
        for g in range(G):
            gi = t * G + g
            cw = c.chunk_words[gi * W:(gi + 1) * W].astype(np.int64)
            starts = int(c.group_off[gi]) + np.concatenate([[0], np.cumsum(cw)[:-1]])
            for l in range(W):
                idx = [g * W * c.S + (k // V) * (W * V) + l * V + (k % V) for k in range(c.S)]
                idx = [i for i in idx if i < n]
                if tb.ref is not None:      # a referencing row has nothing in the stream; its symbols stay 0xFFFF
                    idx = [i for i in idx if tb.ref[i // c.D] == i // c.D]
                if not idx:
                    assert cw[l] == 0
                    continue
                if book is None:
                    out[t, idx] = tb.sym_lo
                    assert cw[l] == 0
                    continue
                ws = c.words[int(starts[l]):int(starts[l]) + int(cw[l])]
                bits = "".join(format(int(w), "032b") for w in ws)
                pos = 0
                for i in idx:
                    L, val = 0, 0
                    while True:
                        val = (val << 1) | int(bits[pos])
                        pos += 1
                        L += 1
                        if (L, val) in book:
                            out[t, i] = book[(L, val)]
                            break
                        assert L < c.LMAX, "no codeword"
                assert (pos + 31) // 32 == cw[l], "chunk word count"
                assert set(bits[pos:]) <= {"0"}, "padding bits must be zero"
    return out


def outliers(c: Container):
    """Per table: array of (index in table, raw bits), gathered from the groups' records in order."""
    n = c.B * c.D
    G = -(-n // (W * c.S))
    res = []
    for t in range(c.T):
        recs = []
        for g in range(G):
            start, cw, ne = group_extent(c, t * G + g)
            r = c.words[start + cw:start + cw + 2 * ne].reshape(-1, 2)
            lo, hi = g * W * c.S, min(n, (g + 1) * W * c.S)
            assert np.all((r[:, 0] >= lo) & (r[:, 0] < hi))
            recs.append(r)
        res.append(np.concatenate(recs) if recs else np.zeros((0, 2), np.uint32))
    return res
