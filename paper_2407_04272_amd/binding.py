"""ctypes binding of libdlc.so: argument marshalling only -- every step runs in the HIP kernels.

PyTorch is used for device memory and streams.  There is no CPU fallback: if the library is missing
or cannot be loaded, importing names from here raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdlc.so")

F32, F16 = 0, 1
OK, EINVAL, ENOMEM, ECAPACITY, ECORRUPT, EHIP, ESTATE, ELIMIT = 0, -1, -2, -3, -4, -5, -6, -7
STATIC_MAX_TABLES = 4096
CLASS_SMALL, CLASS_MEDIUM, CLASS_LARGE = 0, 1, 2
DECAY_NONE, DECAY_STEPWISE, DECAY_DROP, DECAY_LINEAR, DECAY_LOG = 0, 1, 2, 3, 4


class Config(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("num_tables", C.c_int32), ("batch", C.c_int64), ("dim", C.c_int64),
                ("radius", C.c_int32), ("chunk_symbols", C.c_int32), ("max_code_len", C.c_int32),
                ("flags", C.c_int32), ("num_dest", C.c_int32)]


class TableStats(C.Structure):
    _fields_ = [("min", C.c_float), ("max", C.c_float), ("count", C.c_uint64), ("n_rows", C.c_uint32),
                ("n_unique_raw", C.c_uint32), ("n_unique_quant", C.c_uint32), ("probe_eb", C.c_float)]


class ControllerParams(C.Structure):
    _fields_ = [("mode", C.c_int32), ("decay_kind", C.c_int32), ("global_eb", C.c_double), ("alpha", C.c_double),
                ("beta", C.c_double), ("h_large", C.c_double), ("h_small", C.c_double),
                ("decay_start", C.c_int64), ("decay_len", C.c_int64), ("decay_steps", C.c_int32),
                ("reserved", C.c_int32), ("decay_mult0", C.c_double), ("eb_min", C.c_double),
                ("eb_max", C.c_double), ("rel_floor", C.c_double)]


EXPORTS = ["dlc_create", "dlc_destroy", "dlc_compress_bound", "dlc_workspace_bytes", "dlc_stats",
           "dlc_set_error_bounds", "dlc_compress", "dlc_decompress", "dlc_sync_status", "dlc_quantize",
           "dlc_read_histogram", "dlc_read_codebook", "dlc_read_row_refs", "dlc_set_row_match", "dlc_speedup_estimate",
           "dlc_select_compressors", "dlc_set_row_hash_multipliers", "dlc_decompress_static",
           "dlc_profile_enable", "dlc_profile_read", "dlc_strerror"]

_lib = None


def lib():
    """Loads libdlc.so (built beforehand by ``paper_2407_04272_amd.build`` / ``__graft_entry__.build``)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python -m paper_2407_04272_amd.build` "
                               "(there is no fallback path)")
        # PyTorch brings its own HIP runtime.  It has to be the one that initialises the GPU: if this library's first
        # HIP call came before torch's, torch would find no device afterwards.
        import torch
        if torch.cuda.is_available():
            torch.cuda.init()
        L = C.CDLL(_LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
        L.dlc_create.argtypes = [C.POINTER(vp), C.POINTER(Config)]
        L.dlc_destroy.argtypes = [vp]
        L.dlc_destroy.restype = None
        L.dlc_compress_bound.argtypes = [C.POINTER(Config)]
        L.dlc_compress_bound.restype = sz
        L.dlc_workspace_bytes.argtypes = [C.POINTER(Config)]
        L.dlc_workspace_bytes.restype = sz
        L.dlc_stats.argtypes = [vp, vp, vp, C.POINTER(TableStats), vp]
        L.dlc_set_error_bounds.argtypes = [vp, C.POINTER(TableStats), C.POINTER(ControllerParams), vp, i64, vp, vp, vp]
        L.dlc_compress.argtypes = [vp, vp, vp, sz, vp, vp]
        L.dlc_decompress.argtypes = [vp, vp, sz, vp, sz, vp]
        L.dlc_sync_status.argtypes = [vp, vp]
        L.dlc_quantize.argtypes = [vp, vp, vp, vp]
        L.dlc_read_histogram.argtypes = [vp, vp, vp]
        L.dlc_read_codebook.argtypes = [vp, vp, vp, vp]
        L.dlc_read_row_refs.argtypes = [vp, vp, vp]
        L.dlc_set_row_match.argtypes = [vp, vp, vp]
        L.dlc_set_row_hash_multipliers.argtypes = [vp, vp, vp]
        L.dlc_decompress_static.argtypes = [C.POINTER(Config), vp, C.c_size_t, vp, C.c_size_t, vp, vp]
        L.dlc_speedup_estimate.argtypes = [C.c_double] * 4
        L.dlc_speedup_estimate.restype = C.c_double
        L.dlc_select_compressors.argtypes = [vp, vp, vp, C.c_size_t, vp, vp, C.c_size_t, C.c_double, vp, vp, vp, vp, vp]
        L.dlc_profile_enable.argtypes = [vp, i32]
        L.dlc_profile_read.argtypes = [vp, i32, vp, vp, vp]
        L.dlc_strerror.argtypes = [i32]
        L.dlc_strerror.restype = C.c_char_p
        _lib = L
    return _lib


def dlc_strerror(status: int) -> str:
    return lib().dlc_strerror(status).decode()


class DlcError(RuntimeError):
    def __init__(self, status, where):
        super().__init__(f"{where}: {dlc_strerror(status)} ({status})")
        self.status = status


def _check(status, where):
    if status != OK:
        raise DlcError(status, where)


FLAG_CARRY_CODEBOOK = 2
FLAG_ROW_MATCH = 4
FLAG_STATS_WORKSPACE = 8
FLAG_SAMPLE_CODEBOOK = 16


def make_config(dtype, T, B, D, radius=512, chunk_symbols=256, max_code_len=12, flags=0, num_dest=1) -> Config:
    """num_dest > 1: B is the batch of ONE destination's piece, the payload is [num_dest][T][B][D]."""
    return Config(dtype, T, B, D, radius, chunk_symbols, max_code_len, flags, num_dest)


def dlc_speedup_estimate(cr: float, net_gbps: float, tc_gbps: float, td_gbps: float) -> float:
    return float(lib().dlc_speedup_estimate(cr, net_gbps, tc_gbps, td_gbps))


def dlc_compress_bound(cfg: Config) -> int:
    return int(lib().dlc_compress_bound(C.byref(cfg)))


def dlc_workspace_bytes(cfg: Config) -> int:
    return int(lib().dlc_workspace_bytes(C.byref(cfg)))


def dlc_decompress_static(cfg: Config, d_comp, comp_bytes, d_payload_out, d_status, stream=None) -> int:
    """dlc_decompress without a context and without any allocation; the status goes to the int32 tensor d_status."""
    cap = d_payload_out.numel() * d_payload_out.element_size()
    return lib().dlc_decompress_static(C.byref(cfg), C.c_void_p(d_comp.data_ptr()), comp_bytes,
                                       C.c_void_p(d_payload_out.data_ptr()), cap, C.c_void_p(d_status.data_ptr()),
                                       _stream_ptr(stream))


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(int(stream.cuda_stream))


def _np_ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


class Context:
    """One geometry; owns the library context.  Methods carry the C entry points' names without the prefix."""

    def __init__(self, cfg: Config):
        self.cfg = cfg
        self._h = C.c_void_p()
        _check(lib().dlc_create(C.byref(self._h), C.byref(cfg)), "dlc_create")
        self.T, self.B, self.D = cfg.num_tables, cfg.batch, cfg.dim
        self.ND = max(1, cfg.num_dest)
        self.K = 2 * cfg.radius

    def close(self):
        if self._h:
            lib().dlc_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- statistics and controller ----
    def stats(self, d_payload, probe_eb, stream=None):
        pe = np.ascontiguousarray(np.broadcast_to(np.asarray(probe_eb, np.float32), (self.T,)))
        out = (TableStats * self.T)()
        _check(lib().dlc_stats(self._h, C.c_void_p(d_payload.data_ptr()), _np_ptr(pe), out, _stream_ptr(stream)),
               "dlc_stats")
        return out

    def set_error_bounds(self, eb=None, stats=None, params: ControllerParams | None = None, class_override=None,
                         iteration: int = 0, stream=None):
        """explicit: set_error_bounds(eb=...);  derived: set_error_bounds(stats=..., params=...).
        -> (eb float32[T], class int32[T] or None)"""
        if stats is None:
            ebs = np.ascontiguousarray(np.broadcast_to(np.asarray(eb, np.float32), (self.T,))).copy()
            st = lib().dlc_set_error_bounds(self._h, None, None, None, iteration, _np_ptr(ebs), None,
                                            _stream_ptr(stream))
            _check(st, "dlc_set_error_bounds")
            return ebs, None
        ebs = np.zeros(self.T, np.float32)
        cls = np.zeros(self.T, np.int32)
        ov = np.ascontiguousarray(class_override, np.int32) if class_override is not None else None
        st = lib().dlc_set_error_bounds(self._h, stats, C.byref(params), _np_ptr(ov), iteration, _np_ptr(ebs),
                                        _np_ptr(cls), _stream_ptr(stream))
        _check(st, "dlc_set_error_bounds")
        return ebs, cls

    # ---- compress / decompress ----
    def compress(self, d_payload, d_out, d_out_bytes, stream=None, capacity=None):
        cap = d_out.numel() * d_out.element_size() if capacity is None else capacity
        return lib().dlc_compress(self._h, C.c_void_p(d_payload.data_ptr()), C.c_void_p(d_out.data_ptr()), cap,
                                  C.c_void_p(d_out_bytes.data_ptr()), _stream_ptr(stream))

    def decompress(self, d_comp, comp_bytes, d_payload_out, stream=None):
        cap = d_payload_out.numel() * d_payload_out.element_size()
        return lib().dlc_decompress(self._h, C.c_void_p(d_comp.data_ptr()), comp_bytes,
                                    C.c_void_p(d_payload_out.data_ptr()), cap, _stream_ptr(stream))

    def sync_status(self, stream=None) -> int:
        return lib().dlc_sync_status(self._h, _stream_ptr(stream))

    # ---- inspection ----
    def quantize(self, d_payload, d_symbols, stream=None):
        _check(lib().dlc_quantize(self._h, C.c_void_p(d_payload.data_ptr()), C.c_void_p(d_symbols.data_ptr()),
                                  _stream_ptr(stream)), "dlc_quantize")

    def read_histogram(self, stream=None) -> np.ndarray:
        h = np.zeros((self.ND * self.T, self.K), np.uint32)
        _check(lib().dlc_read_histogram(self._h, _np_ptr(h), _stream_ptr(stream)), "dlc_read_histogram")
        return h

    def read_codebook(self, stream=None):
        ln = np.zeros((self.ND * self.T, self.K), np.uint8)
        code = np.zeros((self.ND * self.T, self.K), np.uint16)
        _check(lib().dlc_read_codebook(self._h, _np_ptr(ln), _np_ptr(code), _stream_ptr(stream)), "dlc_read_codebook")
        return ln, code

    def set_row_match(self, flags=None, stream=None):
        f = None if flags is None else np.ascontiguousarray(np.broadcast_to(np.asarray(flags, np.uint8), (self.T,)))
        _check(lib().dlc_set_row_match(self._h, _np_ptr(f), _stream_ptr(stream)), "dlc_set_row_match")

    def select_compressors(self, sample, out, out_bytes, net_gbps, tc_gbps=None, td_gbps=None, rec=None, capacity=None,
                           stream=None):
        """Per table: entropy coder alone (0) or row matching in front of it (1), by the Eq. 2 estimate on `sample`.
        tc_gbps / td_gbps: the two compressors' rates, or None to have them measured (then `rec` takes the decoded
        sample).  Returns (choice uint8[T], estimate float64[T]); the choice is installed in the context."""
        tc = None if tc_gbps is None else np.ascontiguousarray(tc_gbps, np.float64)
        td = None if td_gbps is None else np.ascontiguousarray(td_gbps, np.float64)
        choice = np.zeros(self.T, np.uint8)
        est = np.zeros(self.T, np.float64)
        cap = out.numel() * out.element_size() if capacity is None else capacity
        rec_ptr = None if rec is None else C.c_void_p(rec.data_ptr())
        rec_cap = 0 if rec is None else rec.numel() * rec.element_size()
        _check(lib().dlc_select_compressors(self._h, C.c_void_p(sample.data_ptr()), C.c_void_p(out.data_ptr()), cap, C.c_void_p(out_bytes.data_ptr()), rec_ptr,
                                            rec_cap, float(net_gbps), _np_ptr(tc), _np_ptr(td), _np_ptr(choice),
                                            _np_ptr(est), _stream_ptr(stream)), "dlc_select_compressors")
        return choice, est

    def set_row_hash_multipliers(self, mult, stream=None):
        m = np.ascontiguousarray(mult, np.uint32)
        assert m.size == 8 * (self.D // 4)
        _check(lib().dlc_set_row_hash_multipliers(self._h, _np_ptr(m), _stream_ptr(stream)), "dlc_set_row_hash_multipliers")

    def read_row_refs(self, stream=None) -> np.ndarray:
        r = np.zeros((self.ND * self.T, self.B), np.uint32)
        _check(lib().dlc_read_row_refs(self._h, _np_ptr(r), _stream_ptr(stream)), "dlc_read_row_refs")
        return r

    def profile_enable(self, level: int):
        _check(lib().dlc_profile_enable(self._h, level), "dlc_profile_enable")

    def profile_read(self) -> dict:
        n = 16
        names = (C.c_char_p * n)()
        ms = (C.c_float * n)()
        cnt = (C.c_int32 * n)()
        k = lib().dlc_profile_read(self._h, n, names, ms, cnt)
        if k < 0:
            raise DlcError(k, "dlc_profile_read")
        return {names[i].decode(): (float(ms[i]), int(cnt[i])) for i in range(min(k, n))}
