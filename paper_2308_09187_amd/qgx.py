"""Thin ctypes binding over libqgx.so (include/qgx.h): argument marshalling only.

Every step of the path runs in the library's gfx950 kernels; torch is used for device memory and
streams.  Loading fails loudly when the library has not been built
(``python -m paper_2308_09187_amd.build``); there is no fallback of any kind.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqgx.so")

OK = 0
ERR_ARG, ERR_LEVELS, ERR_CAPACITY, ERR_STREAM, ERR_NONFINITE, ERR_HIP, ERR_STATE = -1, -2, -3, -4, -5, -6, -7
EBIT_CAPACITY, EBIT_STREAM, EBIT_NONFINITE, EBIT_STATE = 1, 2, 4, 8
CALL_FIRST_HALF, CALL_SECOND_HALF = 0xFFFFFFFE, 0xFFFFFFFF   # call numbers taken from the iteration counter on the device
NORM_LINF, NORM_L2 = 0, 2
CODE_ELIAS_OMEGA, CODE_TABLE = 0, 1
CHUNK, SUB, SUBS, MAX_SYM, MAX_BINS = 4096, 32, 128, 127, 4096
STATIC_MAX_CHUNKS = 65536

EXPORTS = [
    "qgx_create", "qgx_destroy", "qgx_stream_sizes", "qgx_slot_words", "qgx_compact", "qgx_select_table", "qgx_set_levels", "qgx_get_levels", "qgx_set_code_table",
    "qgx_quantize", "qgx_encode", "qgx_quantize_encode", "qgx_decode", "qgx_decode_average", "qgx_fit_levels", "qgx_fit_code",
    "qgx_state_init", "qgx_eg_step", "qgx_eg_step_static", "qgx_average_reset", "qgx_average_export", "qgx_get_scalars", "qgx_stream_bits", "qgx_debug_set_waves_per_position", "qgx_state_export", "qgx_state_import",
    "qgx_poll_error", "qgx_last_error",
    "qgx_game_operator", "qgx_game_dual_vectors", "qgx_quantize_encode_game", "qgx_norm2", "qgx_game_gap", "qgx_quantization_metrics",
]


class QgxError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__("qgx status %d: %s" % (status, text))
        self.status = status


class _Config(C.Structure):
    _fields_ = [("d", C.c_uint64), ("K", C.c_uint32), ("bucket", C.c_uint32), ("n_segments", C.c_uint32),
                ("segment_len", C.POINTER(C.c_uint64)), ("norm", C.c_int32), ("code", C.c_int32),
                ("seed", C.c_uint64)]


class _Game(C.Structure):
    _fields_ = [("z", C.c_void_p), ("a", C.c_void_p), ("b", C.c_void_p), ("mu", C.c_float), ("sigma", C.c_float),
                ("noise_seed", C.c_uint64)]


class _Stream(C.Structure):
    _fields_ = [("norms", C.c_void_p), ("chunk_off", C.c_void_p), ("sub_end", C.c_void_p),
                ("payload", C.c_void_p), ("payload_words_per_worker", C.c_uint64), ("slot_words", C.c_uint64)]


_lib = None


def load():
    """Loads libqgx.so; raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libqgx.so is not built: run `python -m paper_2308_09187_amd.build` "
                              "(hipcc, gfx950); there is no fallback path")
        lib = C.CDLL(LIB_PATH)
        for name in EXPORTS:
            getattr(lib, name)
        lib.qgx_destroy.restype = None
        lib.qgx_poll_error.restype = C.c_uint32
        lib.qgx_last_error.restype = C.c_char_p
        _lib = lib
    return _lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_handle(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class Stream:
    """Device buffers of one CODE o Q result for K workers."""

    def __init__(self, K, NB, NC, cap_words, device="cuda", slot_words=0):
        cap_words = (int(cap_words) + 3) // 4 * 4
        self.slot_words = int(slot_words)
        self.norms = torch.zeros((K, NB), dtype=torch.float32, device=device)
        self.chunk_off = torch.zeros((K, NC + 1), dtype=torch.int32, device=device)
        self.sub_end = torch.zeros((K, NC, SUBS), dtype=torch.int16, device=device)
        self.payload = torch.zeros((K, cap_words), dtype=torch.int32, device=device)
        self.cap_words = cap_words

    def c_struct(self):
        return _Stream(self.norms.data_ptr(), self.chunk_off.data_ptr(), self.sub_end.data_ptr(),
                       self.payload.data_ptr(), self.cap_words, self.slot_words)

    def to_host(self):
        """numpy views in the container's unsigned types."""
        return dict(norms=self.norms.cpu().numpy(),
                    chunk_off=self.chunk_off.cpu().numpy().view(np.uint32),
                    sub_end=self.sub_end.cpu().numpy().view(np.uint16),
                    payload=self.payload.cpu().numpy().view(np.uint32))


class Context:
    def __init__(self, d, K, bucket, norm=NORM_L2, code=CODE_ELIAS_OMEGA, seed=0, segment_len=None, device="cuda"):
        self.lib = load()
        self.d, self.K, self.bucket, self.device = int(d), int(K), int(bucket), device
        seg = None
        nseg = 0
        if segment_len is not None:
            seg = (C.c_uint64 * len(segment_len))(*[int(x) for x in segment_len])
            nseg = len(segment_len)
        cfg = _Config(self.d, self.K, self.bucket, nseg, seg, norm, code, seed)
        self._h = C.c_void_p()
        with torch.cuda.device(device):
            st = self.lib.qgx_create(C.byref(self._h), C.byref(cfg))
        if st != OK:
            raise QgxError(st, "qgx_create rejected the configuration")
        nb, nc, ww = C.c_uint64(), C.c_uint64(), C.c_uint64()
        self._check(self.lib.qgx_stream_sizes(self._h, C.byref(nb), C.byref(nc), C.byref(ww)))
        self.NB, self.NC, self.worst_words = nb.value, nc.value, ww.value

    def _check(self, st):
        if st != OK:
            raise QgxError(st, self.lib.qgx_last_error(self._h).decode())

    def close(self):
        if self._h:
            self.lib.qgx_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def slot_words(self):
        sw = C.c_uint64()
        self._check(self.lib.qgx_slot_words(self._h, C.byref(sw)))
        return sw.value

    def new_stream(self, cap_words=None, slotted=False):
        """Compact stream (worst-case capacity unless cap_words is given), or a slotted one."""
        if slotted:
            sw = self.slot_words()
            return Stream(self.K, self.NB, self.NC, sw * self.NC, self.device, slot_words=sw)
        return Stream(self.K, self.NB, self.NC, self.worst_words if cap_words is None else cap_words, self.device)

    def compact(self, src: Stream, dst: Stream, stream=None):
        a, b = src.c_struct(), dst.c_struct()
        self._check(self.lib.qgx_compact(self._h, C.byref(a), C.byref(b), _stream_handle(stream)))
        return dst

    # -- tables ---------------------------------------------------------------------------------
    def set_levels(self, levels, stream=None):
        lv = np.ascontiguousarray(levels, dtype=np.float32)
        self._check(self.lib.qgx_set_levels(self._h, lv.ctypes.data_as(C.c_void_p), C.c_uint32(len(lv)),
                                            _stream_handle(stream)))

    def get_levels(self, stream=None):
        lv = np.zeros(MAX_SYM, np.float32)
        n = C.c_uint32()
        self._check(self.lib.qgx_get_levels(self._h, lv.ctypes.data_as(C.c_void_p), C.byref(n), _stream_handle(stream)))
        return lv[: n.value].copy()

    def set_code_table(self, code_len, code_bits, stream=None):
        cl = np.ascontiguousarray(code_len, dtype=np.uint8)
        cb = np.ascontiguousarray(code_bits, dtype=np.uint32)
        self._check(self.lib.qgx_set_code_table(self._h, cl.ctypes.data_as(C.c_void_p), cb.ctypes.data_as(C.c_void_p),
                                                C.c_uint32(len(cl)), _stream_handle(stream)))

    # -- CODE o Q -------------------------------------------------------------------------------
    def quantize(self, V, call_id, norms_in=None, stream=None):
        norms = torch.empty((self.K, self.NB), dtype=torch.float32, device=V.device)
        sym = torch.empty((self.K, self.d), dtype=torch.uint8, device=V.device)
        self._check(self.lib.qgx_quantize(self._h, _ptr(V), C.c_uint32(call_id), _ptr(norms_in), _ptr(norms),
                                          _ptr(sym), _stream_handle(stream)))
        return norms, sym

    def encode(self, norms, sym, out: Stream, stream=None):
        s = out.c_struct()
        self._check(self.lib.qgx_encode(self._h, _ptr(norms), _ptr(sym), C.byref(s), _stream_handle(stream)))
        return out

    def quantize_encode(self, V, call_id, out: Stream, norms_in=None, stream=None):
        s = out.c_struct()
        self._check(self.lib.qgx_quantize_encode(self._h, _ptr(V), C.c_uint32(call_id), _ptr(norms_in), C.byref(s),
                                                 _stream_handle(stream)))
        return out

    # -- the large quadratic game's operator, dual vectors and residual norm on the device -------------
    @staticmethod
    def _game(z, a, b, mu, sigma, noise_seed):
        return _Game(z.data_ptr(), a.data_ptr(), b.data_ptr(), mu, sigma, noise_seed)

    def game_operator(self, z, a, b, mu, out=None, stream=None):
        if out is None:
            out = torch.empty(self.d, dtype=torch.float32, device=z.device)
        g = self._game(z, a, b, mu, 0.0, 0)
        self._check(self.lib.qgx_game_operator(self._h, C.byref(g), _ptr(out), _stream_handle(stream)))
        return out

    def game_gap(self, z, a, b, mu, centre, radius, stream=None):
        r = C.c_double()
        g = self._game(z, a, b, mu, 0.0, 0)
        self._check(self.lib.qgx_game_gap(self._h, C.byref(g), _ptr(centre), C.c_double(radius), C.byref(r), _stream_handle(stream)))
        return r.value

    def game_dual_vectors(self, z, a, b, mu, sigma, noise_seed, call_id, out=None, stream=None):
        if out is None:
            out = torch.empty((self.K, self.d), dtype=torch.float32, device=z.device)
        g = self._game(z, a, b, mu, sigma, noise_seed)
        self._check(self.lib.qgx_game_dual_vectors(self._h, C.byref(g), C.c_uint32(call_id), _ptr(out), _stream_handle(stream)))
        return out

    def quantize_encode_game(self, z, a, b, mu, sigma, noise_seed, call_id, out: Stream, V_out=None, stream=None):
        g, s = self._game(z, a, b, mu, sigma, noise_seed), out.c_struct()
        self._check(self.lib.qgx_quantize_encode_game(self._h, C.byref(g), C.c_uint32(call_id), C.byref(s), _ptr(V_out),
                                                      _stream_handle(stream)))
        return out

    def norm2(self, x, stream=None):
        r = C.c_double()
        self._check(self.lib.qgx_norm2(self._h, _ptr(x), C.c_uint64(x.numel()), C.byref(r), _stream_handle(stream)))
        return r.value

    def quantization_metrics(self, V, Vhat, stream=None):
        """Per worker: (number of nonzeros of Q(v), ||Q(v) - v||^2, ||v||^2) as three numpy arrays of K."""
        import numpy as np
        nnz = np.zeros(self.K, np.uint64)
        err = np.zeros(self.K, np.float64)
        nrm = np.zeros(self.K, np.float64)
        self._check(self.lib.qgx_quantization_metrics(self._h, _ptr(V), _ptr(Vhat), C.c_void_p(nnz.ctypes.data),
                                                      C.c_void_p(err.ctypes.data), C.c_void_p(nrm.ctypes.data),
                                                      _stream_handle(stream)))
        return nnz, err, nrm

    # -- DEQ o CODE and the fused updates ---------------------------------------------------------
    def decode(self, st: Stream, out=None, stream=None):
        if out is None:
            out = torch.empty((self.K, self.d), dtype=torch.float32, device=st.payload.device)
        s = st.c_struct()
        self._check(self.lib.qgx_decode(self._h, C.byref(s), _ptr(out), _stream_handle(stream)))
        return out

    def decode_average(self, st: Stream, out=None, stream=None):
        if out is None:
            out = torch.empty(self.d, dtype=torch.float32, device=st.payload.device)
        s = st.c_struct()
        self._check(self.lib.qgx_decode_average(self._h, C.byref(s), _ptr(out), _stream_handle(stream)))
        return out

    def fit_levels(self, V, n_sym, n_bins=4096, sweeps=10, hist_out=None, stream=None):
        self._check(self.lib.qgx_fit_levels(self._h, _ptr(V), C.c_uint32(n_sym), C.c_uint32(n_bins),
                                            C.c_uint32(sweeps), _ptr(hist_out), _stream_handle(stream)))

    def fit_code(self, stream=None):
        """Returns (p, code_len, code_bits) of the code the context now uses."""
        n = len(self.get_levels(stream))
        p = np.zeros(n, np.float64); cl = np.zeros(n, np.uint8); cb = np.zeros(n, np.uint32)
        self._check(self.lib.qgx_fit_code(self._h, p.ctypes.data_as(C.c_void_p), cl.ctypes.data_as(C.c_void_p),
                                          cb.ctypes.data_as(C.c_void_p), _stream_handle(stream)))
        return p, cl, cb

    def state_init(self, X1=None, stream=None):
        self._check(self.lib.qgx_state_init(self._h, _ptr(X1), _stream_handle(stream)))

    def eg_step(self, half, cur: Stream, prev: Stream = None, X_out=None, stream=None, static=False):
        """static: through qgx_eg_step_static (scratch in the library's device image, nothing allocated)."""
        c = cur.c_struct()
        p = prev.c_struct() if prev is not None else None
        fn = self.lib.qgx_eg_step_static if static else self.lib.qgx_eg_step
        self._check(fn(self._h, C.c_int(half), C.byref(c), C.byref(p) if p is not None else None,
                       _ptr(X_out), _stream_handle(stream)))
        return X_out

    def select_table(self, table, prev_table=None):
        self._check(self.lib.qgx_select_table(self._h, C.c_uint32(table),
                                              C.c_uint32(table if prev_table is None else prev_table)))

    def average_reset(self, on=True, stream=None):
        self._check(self.lib.qgx_average_reset(self._h, C.c_int(1 if on else 0), _stream_handle(stream)))

    def average_export(self, out=None, stream=None):
        """(X_bar [d], number of half-steps averaged)."""
        if out is None:
            out = torch.empty(self.d, dtype=torch.float32, device=self.device)
        n = C.c_uint64()
        self._check(self.lib.qgx_average_export(self._h, _ptr(out), C.byref(n), _stream_handle(stream)))
        return out, n.value

    def scalars(self, stream=None):
        S, g, t = C.c_double(), C.c_double(), C.c_uint64()
        self._check(self.lib.qgx_get_scalars(self._h, C.byref(S), C.byref(g), C.byref(t), _stream_handle(stream)))
        return dict(S=S.value, gamma=g.value, t=t.value)

    def stream_bits(self, coded: Stream, stream=None):
        """Code-word and sign bits of a coded stream over all workers (no padding, no norms)."""
        c, b = coded.c_struct(), C.c_uint64()
        self._check(self.lib.qgx_stream_bits(self._h, C.byref(c), C.byref(b), _stream_handle(stream)))
        return b.value

    def debug_set_waves_per_position(self, waves):
        self._check(self.lib.qgx_debug_set_waves_per_position(self._h, C.c_int(waves)))

    def state_export(self, stream=None):
        Y = torch.empty(self.d, dtype=torch.float32, device=self.device)
        A = torch.empty(self.d, dtype=torch.float32, device=self.device)
        self._check(self.lib.qgx_state_export(self._h, _ptr(Y), _ptr(A), _stream_handle(stream)))
        return Y, A

    def state_import(self, Y, anchor, S, t, stream=None):
        self._check(self.lib.qgx_state_import(self._h, _ptr(Y), _ptr(anchor), C.c_double(S), C.c_uint64(t),
                                              _stream_handle(stream)))

    def poll_error(self, stream=None):
        return int(self.lib.qgx_poll_error(self._h, _stream_handle(stream)))
