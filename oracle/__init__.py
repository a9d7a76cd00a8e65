"""CPU oracle of the error-bounded embedding-payload compressor -- TEST INFRASTRUCTURE.

Thin ctypes access to ``dlc_oracle.c`` (plain single-threaded C, built with gcc).
Only tests, the smoke check and the CPU-baseline leg of the bench may import this
package.  It shares nothing with the HIP library and never imports it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dlc_oracle.c")
_LIB = os.path.join(_HERE, "libdlc_oracle.so")

F32, F16 = 0, 1
OK, EINVAL, ENOMEM, ECAPACITY, ECORRUPT = 0, -1, -2, -3, -4
CLASS_SMALL, CLASS_MEDIUM, CLASS_LARGE = 0, 1, 2
W, V = 64, 4
HEADER_BYTES, DIR_BYTES = 128, 56


def build(force: bool = False) -> str:
    """Compile the oracle (gcc, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fno-strict-aliasing",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class TableStats(C.Structure):
    _fields_ = [("min", C.c_float), ("max", C.c_float), ("count", C.c_uint64), ("n_rows", C.c_uint32),
                ("n_unique_raw", C.c_uint32), ("n_unique_quant", C.c_uint32), ("probe_eb", C.c_float)]


class ControllerParams(C.Structure):
    _fields_ = [("mode", C.c_int32), ("decay_kind", C.c_int32), ("global_eb", C.c_double), ("alpha", C.c_double),
                ("beta", C.c_double), ("h_large", C.c_double), ("h_small", C.c_double),
                ("decay_start", C.c_int64), ("decay_len", C.c_int64), ("decay_steps", C.c_int32),
                ("reserved", C.c_int32), ("decay_mult0", C.c_double), ("eb_min", C.c_double),
                ("eb_max", C.c_double), ("rel_floor", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_half_to_float.restype = C.c_float
        L.orc_half_to_float.argtypes = [C.c_uint16]
        L.orc_float_to_half.restype = C.c_uint16
        L.orc_float_to_half.argtypes = [C.c_float]
        L.orc_quantize.argtypes = [C.c_void_p, C.c_int, C.c_size_t, C.c_float, C.c_int, C.c_void_p, C.c_void_p]
        L.orc_histogram.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        L.orc_codebook.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.POINTER(C.c_int),
                                   C.POINTER(C.c_int)]
        L.orc_stats.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_void_p,
                                C.POINTER(TableStats)]
        L.orc_homo_index.restype = C.c_double
        L.orc_homo_index.argtypes = [C.c_uint32, C.c_uint32]
        L.orc_classify.argtypes = [C.c_double, C.c_double, C.c_double]
        L.orc_decay_multiplier.restype = C.c_double
        L.orc_decay_multiplier.argtypes = [C.POINTER(ControllerParams), C.c_int64]
        L.orc_controller.argtypes = [C.POINTER(TableStats), C.c_int, C.POINTER(ControllerParams), C.c_void_p,
                                     C.c_int64, C.c_void_p, C.c_void_p]
        L.orc_compress_bound.restype = C.c_size_t
        L.orc_compress_bound.argtypes = [C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int]
        L.orc_compress.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                   C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.orc_compress_carried.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                           C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_compress_rows.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                        C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
        L.orc_decompress.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t, C.c_void_p]
        L.orc_speedup.restype = C.c_double
        L.orc_speedup.argtypes = [C.c_double, C.c_double, C.c_double, C.c_double]
        L.orc_select.argtypes = [C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_double, C.c_void_p, C.c_void_p]
        L.orc_select_compressors.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int,
                                             C.c_void_p, C.c_double, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise TypeError("payload must be float32 or float16")


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def half_to_float(h: int) -> float:
    return float(lib().orc_half_to_float(int(h)))


def float_to_half(f: float) -> int:
    return int(lib().orc_float_to_half(C.c_float(f)))


def quantize(x: np.ndarray, eb: float, R: int = 512):
    """-> (symbols u16, reconstruction in x's dtype)."""
    x = np.ascontiguousarray(x)
    sym = np.empty(x.size, np.uint16)
    rec = np.empty_like(x)
    rc = lib().orc_quantize(_ptr(x), _dtype_code(x), x.size, C.c_float(eb), R, _ptr(sym), _ptr(rec))
    if rc != OK:
        raise ValueError(f"orc_quantize rc={rc}")
    return sym.reshape(x.shape), rec


def histogram(sym: np.ndarray, K: int) -> np.ndarray:
    sym = np.ascontiguousarray(sym, np.uint16)
    h = np.zeros(K, np.uint64)
    rc = lib().orc_histogram(_ptr(sym), sym.size, K, _ptr(h))
    if rc != OK:
        raise ValueError(f"orc_histogram rc={rc}")
    return h


def codebook(hist: np.ndarray, LMAX: int = 12):
    """-> (len u8[K], code u32[K], n_used, n_repairs)."""
    hist = np.ascontiguousarray(hist, np.uint64)
    K = hist.size
    ln = np.zeros(K, np.uint8)
    code = np.zeros(K, np.uint32)
    nu, nh = C.c_int(0), C.c_int(0)
    rc = lib().orc_codebook(_ptr(hist), K, LMAX, _ptr(ln), _ptr(code), C.byref(nu), C.byref(nh))
    if rc != OK:
        raise ValueError(f"orc_codebook rc={rc}")
    return ln, code, nu.value, nh.value


def stats(payload: np.ndarray, probe_eb, R: int = 512):
    """payload [T,B,D] -> list of TableStats."""
    payload = np.ascontiguousarray(payload)
    T, B, D = payload.shape
    pe = np.ascontiguousarray(np.broadcast_to(np.asarray(probe_eb, np.float32), (T,)))
    out = (TableStats * T)()
    rc = lib().orc_stats(_ptr(payload), _dtype_code(payload), T, B, D, R, _ptr(pe), out)
    if rc != OK:
        raise ValueError(f"orc_stats rc={rc}")
    return out


def homo_index(n_original: int, n_compressed: int) -> float:
    return float(lib().orc_homo_index(n_original, n_compressed))


def classify(eta: float, h_large: float, h_small: float) -> int:
    return int(lib().orc_classify(eta, h_large, h_small))


def decay_multiplier(params: ControllerParams, iteration: int) -> float:
    return float(lib().orc_decay_multiplier(C.byref(params), iteration))


def controller(st, params: ControllerParams, iteration: int = 0, class_override=None):
    """-> (eb float32[T], class int32[T])."""
    T = len(st)
    eb = np.zeros(T, np.float32)
    cls = np.zeros(T, np.int32)
    ov = None
    if class_override is not None:
        ov = np.ascontiguousarray(class_override, np.int32)
    rc = lib().orc_controller(st, T, C.byref(params), _ptr(ov) if ov is not None else None, iteration, _ptr(eb),
                              _ptr(cls))
    if rc != OK:
        raise ValueError(f"orc_controller rc={rc}")
    return eb, cls


def compress_bound(dtype: int, T: int, B: int, D: int, R: int = 512, S: int = 256, LMAX: int = 12) -> int:
    return int(lib().orc_compress_bound(dtype, T, B, D, R, S, LMAX))


@dataclass
class Compressed:
    data: np.ndarray      # u8, exactly total_bytes long
    sizes: np.ndarray     # u64[1+T]: total, then bytes attributable to each table
    rc: int
    hist: np.ndarray | None = None   # u64[T, K] symbol counts of this payload (compress(..., want_hist=True))


SAMPLE_ELEMS = 65536  # a table's codebook sample: at least this many elements where the table has them


def sample_groups(n: int, S: int = 256) -> list[int]:
    """The groups (64 * S consecutive elements each) of a table of n elements whose symbols are counted when the
    codebook is built from a sample of the payload (a reading of ours: Section III-D builds the Huffman code from the
    data it codes and does not speak of sampling).  ns groups, evenly spread from group 0 on (0, stride, 2 stride, ...
    with stride = floor(G / ns)): as many as hold SAMPLE_ELEMS elements, ceil(SAMPLE_ELEMS / (64 S)), but no more than
    a quarter of the table's G groups, rounded up."""
    gs = 64 * S
    G = (n + gs - 1) // gs
    ns = min((SAMPLE_ELEMS + gs - 1) // gs, (G + 3) // 4)
    stride = G // ns
    return list(range(0, G, stride))[:ns]


def sample_histogram(payload: np.ndarray, eb, R: int = 512, S: int = 256) -> np.ndarray:
    """u64[T, 2R]: per table, the symbol counts of the elements of its sampled groups."""
    payload = np.ascontiguousarray(payload)
    T = payload.shape[0]
    n = payload[0].size
    ebs = np.broadcast_to(np.asarray(eb, np.float32), (T,))
    gs = 64 * S
    h = np.zeros((T, 2 * R), np.uint64)
    for t in range(T):
        flat = payload[t].reshape(-1)
        for g in sample_groups(n, S):
            sym, _ = quantize(flat[g * gs:min(n, (g + 1) * gs)], float(ebs[t]), R)
            h[t] += histogram(sym, 2 * R)
    return h


def compress(payload: np.ndarray, eb, R: int = 512, S: int = 256, LMAX: int = 12, capacity: int | None = None,
             carry_hist: np.ndarray | None = None, want_hist: bool = False, row_match=None,
             sample_codebook: bool = False):
    """carry_hist (u64[T, 2R]): code with the codebook of these counts (an earlier payload's) instead of the payload's
    own; want_hist: also return this payload's counts, which is what the next call is given.
    row_match (bool or T flags): rows equal to an earlier row of their table are stored as references (not together
    with carry_hist / want_hist).
    sample_codebook: code with the codebook of the counts of the payload's own sampled groups (sample_histogram),
    under the rules of a carried codebook: the escape always has a code, a symbol the sample has not seen is stored as
    an escape."""
    payload = np.ascontiguousarray(payload)
    if sample_codebook:
        if carry_hist is not None or row_match is not None:
            raise ValueError("sample_codebook cannot be combined with carry_hist / row_match")
        carry_hist = sample_histogram(payload, eb, R, S)
    T, B, D = payload.shape
    dt = _dtype_code(payload)
    ebs = np.ascontiguousarray(np.broadcast_to(np.asarray(eb, np.float32), (T,)))
    cap = compress_bound(dt, T, B, D, R, S, LMAX) if capacity is None else capacity
    if cap == 0 and capacity is None:
        raise ValueError("bad geometry")
    out = np.zeros(max(cap, 1), np.uint8)
    sizes = np.zeros(1 + T, np.uint64)
    if row_match is not None:
        if carry_hist is not None or want_hist:
            raise ValueError("row_match cannot be combined with carry_hist / want_hist")
        rm = np.ascontiguousarray(np.broadcast_to(np.asarray(row_match, np.uint8), (T,)))
        cap = cap + 16 * T + 4 * B * T if capacity is None else cap
        out = np.zeros(max(cap, 1), np.uint8)
        rc = lib().orc_compress_rows(_ptr(payload), dt, T, B, D, R, S, LMAX, _ptr(ebs), _ptr(out), cap, _ptr(sizes), _ptr(rm))
        hist = None
    elif carry_hist is None and not want_hist:
        rc = lib().orc_compress(_ptr(payload), dt, T, B, D, R, S, LMAX, _ptr(ebs), _ptr(out), cap, _ptr(sizes))
        hist = None
    else:
        ch = None
        if carry_hist is not None:
            ch = np.ascontiguousarray(carry_hist, np.uint64)
            if ch.shape != (T, 2 * R):
                raise ValueError("carry_hist must be [T, 2R]")
        hist = np.zeros((T, 2 * R), np.uint64) if want_hist else None
        rc = lib().orc_compress_carried(_ptr(payload), dt, T, B, D, R, S, LMAX, _ptr(ebs), _ptr(out), cap, _ptr(sizes),
                                        _ptr(ch) if ch is not None else None, _ptr(hist) if hist is not None else None)
    n = int(sizes[0]) if rc == OK else 0
    return Compressed(out[:n].copy(), sizes, rc, hist)


def decompress(data: np.ndarray, shape, dtype, want_symbols: bool = False):
    data = np.ascontiguousarray(data, np.uint8)
    out = np.zeros(shape, dtype)
    sym = np.zeros(int(np.prod(shape)), np.uint16) if want_symbols else None
    rc = lib().orc_decompress(_ptr(data), data.size, _ptr(out), out.nbytes, _ptr(sym) if want_symbols else None)
    if want_symbols:
        return rc, out, sym.reshape(shape)
    return rc, out


def speedup(cr: float, net: float, tc: float, td: float) -> float:
    """Eq. 2."""
    return float(lib().orc_speedup(cr, net, tc, td))


def select(cr, tc, td, net: float):
    """cr [n_comp, T], tc / td [n_comp] -> (choice int32[T], estimate float64[T]); ties go to the compressor listed first."""
    cr = np.ascontiguousarray(cr, np.float64)
    n_comp, T = cr.shape
    tc = np.ascontiguousarray(tc, np.float64)
    td = np.ascontiguousarray(td, np.float64)
    assert tc.shape == (n_comp,) and td.shape == (n_comp,)
    choice = np.zeros(T, np.int32)
    best = np.zeros(T, np.float64)
    rc = lib().orc_select(T, n_comp, _ptr(cr), _ptr(tc), _ptr(td), net, _ptr(choice), _ptr(best))
    if rc != OK:
        raise ValueError(f"orc_select: {rc}")
    return choice, best


def select_compressors(payload: np.ndarray, eb, net: float, tc, td, R: int = 512, S: int = 256, LMAX: int = 12):
    """The offline procedure on a sampled payload: 0 = entropy coder alone, 1 = row matching in front of it."""
    payload = np.ascontiguousarray(payload)
    T, B, D = payload.shape
    ebs = np.ascontiguousarray(np.broadcast_to(np.asarray(eb, np.float32), (T,)))
    tc = np.ascontiguousarray(tc, np.float64)
    td = np.ascontiguousarray(td, np.float64)
    assert tc.shape == (2,) and td.shape == (2,)
    choice = np.zeros(T, np.int32)
    best = np.zeros(T, np.float64)
    rc = lib().orc_select_compressors(_ptr(payload), _dtype_code(payload), T, B, D, R, S, LMAX, _ptr(ebs), net, _ptr(tc),
                                      _ptr(td), _ptr(choice), _ptr(best))
    if rc != OK:
        raise ValueError(f"orc_select_compressors: {rc}")
    return choice, best
