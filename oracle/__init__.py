"""CPU oracle of the Q-GenX hot path -- TEST INFRASTRUCTURE, not the product.

Thin ctypes access to ``qgx_oracle.c`` (compiled with gcc on first use) plus
the few lines of glue that string its functions together.  Only ``tests/``,
the smoke check and the ``cpu_baseline`` leg of the benchmark may import this
package; it imports nothing from the HIP library's package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# QGX_ORACLE_SRC names another C source to build (next to itself) and load instead: the test that plants
# mistakes in a copy of the oracle, to see that the pins catch them, runs the pins that way.
_SRC = os.environ.get("QGX_ORACLE_SRC") or os.path.join(_HERE, "qgx_oracle.c")
_LIB = os.path.join(os.path.dirname(os.path.abspath(_SRC)), "libqgx_oracle.so")

NORM_LINF = 0
NORM_L2 = 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, no contraction of a*b+c)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        # QGX_ORACLE_CFLAGS: extra compiler flags for a build named by QGX_ORACLE_SRC (the sanitizer test)
        extra = os.environ.get("QGX_ORACLE_CFLAGS", "").split() if os.environ.get("QGX_ORACLE_SRC") else []
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", *extra,
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_uniform24.restype = C.c_float
        _lib.orc_uniform24.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
        _lib.orc_bucket_norm.restype = C.c_float
        _lib.orc_quantize.restype = C.c_uint64
        _lib.orc_elias_omega.restype = C.c_uint32
        _lib.orc_encode.restype = C.c_int
        _lib.orc_decode.restype = C.c_int
        _lib.orc_bin_of.restype = C.c_uint32
        _lib.orc_bin_of.argtypes = [C.c_float, C.c_uint32]
        _lib.orc_bin_edge.restype = C.c_double
        _lib.orc_bin_edge.argtypes = [C.c_uint32, C.c_uint32]
        _lib.orc_qada_objective.restype = C.c_double
        _lib.orc_stationary_point.restype = C.c_double
        _lib.orc_normal.restype = C.c_double
        _lib.orc_normal.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
        _lib.orc_norm2.restype = C.c_double
        _lib.orc_game_gap.restype = C.c_double
        for f in ("orc_chunk_coords", "orc_sub_coords", "orc_align_words"):
            getattr(_lib, f).restype = C.c_uint32
    return _lib


def _p(a, ty):
    return None if a is None else a.ctypes.data_as(C.POINTER(ty))


def _c(a, dt):
    return None if a is None else np.ascontiguousarray(a, dtype=dt)


def CH():
    return int(lib().orc_chunk_coords())


def SUB():
    return int(lib().orc_sub_coords())


def SUBS():
    """Sub-chunk table entries per chunk."""
    return CH() // SUB()


def philox4x32_10(ctr, key):
    ctr = _c(ctr, np.uint32); key = _c(key, np.uint32)
    out = np.zeros(4, np.uint32)
    lib().orc_philox4x32_10(_p(ctr, C.c_uint32), _p(key, C.c_uint32), _p(out, C.c_uint32))
    return out


def uniform24(seed, k, call_id, i):
    return float(lib().orc_uniform24(seed, k, call_id, i))


def elias_omega(n: int):
    bits = np.zeros(64, np.uint8)
    ln = lib().orc_elias_omega(C.c_uint32(n), _p(bits, C.c_uint8))
    return [int(b) for b in bits[:ln]]


@dataclass
class Layout:
    """Buckets and chunks of one worker's vector of d coordinates."""
    d: int
    bucket: int
    bucket_start: np.ndarray   # uint64 [NB+1]
    chunk_start: np.ndarray    # uint64 [NC+1]
    chunk_bucket: np.ndarray   # uint64 [NC]: bucket of the chunk's first coordinate

    @property
    def NB(self):
        return len(self.bucket_start) - 1

    @property
    def NC(self):
        return len(self.chunk_start) - 1


def layout(d: int, bucket: int, segment_len=None) -> Layout:
    seg = None if segment_len is None else _c(segment_len, np.uint64)
    nseg = 0 if seg is None else len(seg)
    nb = C.c_uint64(); nc = C.c_uint64()
    lib().orc_layout_counts(C.c_uint64(d), C.c_uint32(bucket), C.c_uint32(nseg), _p(seg, C.c_uint64),
                            C.byref(nb), C.byref(nc))
    bs = np.zeros(nb.value + 1, np.uint64)
    cs = np.zeros(nc.value + 1, np.uint64)
    cb = np.zeros(max(nc.value, 1), np.uint64)[:nc.value]
    lib().orc_layout_fill(C.c_uint64(d), C.c_uint32(bucket), C.c_uint32(nseg), _p(seg, C.c_uint64),
                          _p(bs, C.c_uint64), _p(cs, C.c_uint64), _p(cb, C.c_uint64))
    return Layout(d, bucket, bs, cs, cb)


def bucket_norm(v, norm_kind):
    v = _c(v, np.float32)
    fin = C.c_int(1)
    n = lib().orc_bucket_norm(_p(v, C.c_float), C.c_uint64(v.size), C.c_int(norm_kind), C.byref(fin))
    return np.float32(n), bool(fin.value)


def quantize(V, lay: Layout, norm_kind, levels, seed, call_id, norms_in=None, k0=0, i0=0):
    """Q_l of Definition 1 per bucket.  V is [K][d] float32.
    Returns (norms [K][NB] f32, idx [K][d] u8, neg [K][d] u8, n_nonfinite_buckets)."""
    V = _c(V, np.float32)
    K, d = V.shape
    assert d == lay.d
    levels = _c(levels, np.float32)
    norms_in = _c(norms_in, np.float32)
    norms = np.zeros((K, lay.NB), np.float32)
    idx = np.zeros((K, d), np.uint8)
    neg = np.zeros((K, d), np.uint8)
    bad = lib().orc_quantize(_p(V, C.c_float), C.c_uint32(K), C.c_uint64(d),
                             _p(lay.bucket_start, C.c_uint64), C.c_uint64(lay.NB), C.c_int(norm_kind),
                             _p(levels, C.c_float), C.c_uint32(len(levels)),
                             C.c_uint64(seed), C.c_uint32(call_id),
                             _p(norms_in, C.c_float), _p(norms, C.c_float),
                             _p(idx, C.c_uint8), _p(neg, C.c_uint8), C.c_uint32(k0), C.c_uint64(i0))
    return norms, idx, neg, int(bad)


@dataclass
class Stream:
    """CODE o Q output of K workers (the norms travel beside it)."""
    payload: np.ndarray     # uint32 [K][cap_words]
    chunk_off: np.ndarray   # uint32 [K][NC+1]
    sub_end: np.ndarray     # uint16 [K][NC][SUBS()]
    total_bits: np.ndarray  # uint64 [K]   symbols + signs, no padding
    norms: np.ndarray = None


def encode(idx, neg, lay: Layout, cap_words: int, code_len=None, code_bits=None) -> Stream:
    idx = _c(idx, np.uint8); neg = _c(neg, np.uint8)
    K, d = idx.shape
    code_len = _c(code_len, np.uint8); code_bits = _c(code_bits, np.uint32)
    payload = np.zeros((K, cap_words), np.uint32)
    chunk_off = np.zeros((K, lay.NC + 1), np.uint32)
    sub_end = np.zeros((K, lay.NC, SUBS()), np.uint16)
    total = np.zeros(K, np.uint64)
    rc = lib().orc_encode(_p(idx, C.c_uint8), _p(neg, C.c_uint8), C.c_uint32(K), C.c_uint64(d),
                          _p(lay.chunk_start, C.c_uint64), C.c_uint64(lay.NC),
                          _p(code_len, C.c_uint8), _p(code_bits, C.c_uint32),
                          _p(payload, C.c_uint32), C.c_uint64(cap_words),
                          _p(chunk_off, C.c_uint32), _p(sub_end, C.c_uint16), _p(total, C.c_uint64))
    if rc != 0:
        raise OverflowError("oracle encode: stream does not fit cap_words (rc=%d)" % rc)
    return Stream(payload, chunk_off, sub_end, total)


def decode(st: Stream, norms, lay: Layout, levels, code_len=None, code_bits=None):
    """DEQ o CODE.  Returns (Vhat [K][d] f32, idx, neg).  Raises on a malformed stream."""
    payload = _c(st.payload, np.uint32)
    K, cap = payload.shape
    chunk_off = _c(st.chunk_off, np.uint32); sub_end = _c(st.sub_end, np.uint16)
    norms = _c(norms, np.float32); levels = _c(levels, np.float32)
    code_len = _c(code_len, np.uint8); code_bits = _c(code_bits, np.uint32)
    Vhat = np.zeros((K, lay.d), np.float32)
    idx = np.zeros((K, lay.d), np.uint8); neg = np.zeros((K, lay.d), np.uint8)
    rc = lib().orc_decode(_p(payload, C.c_uint32), C.c_uint64(cap), _p(chunk_off, C.c_uint32),
                          _p(sub_end, C.c_uint16), _p(norms, C.c_float),
                          C.c_uint32(K), C.c_uint64(lay.d), _p(lay.chunk_start, C.c_uint64),
                          _p(lay.chunk_bucket, C.c_uint64), _p(lay.bucket_start, C.c_uint64),
                          C.c_uint64(lay.NC), C.c_uint64(lay.NB),
                          _p(levels, C.c_float), C.c_uint32(len(levels)),
                          _p(code_len, C.c_uint8), _p(code_bits, C.c_uint32),
                          _p(Vhat, C.c_float), _p(idx, C.c_uint8), _p(neg, C.c_uint8))
    if rc != 0:
        raise ValueError("oracle decode: malformed stream (rc=%d)" % rc)
    return Vhat, idx, neg


def mean(Vhat):
    Vhat = _c(Vhat, np.float32)
    K, d = Vhat.shape
    m = np.zeros(d, np.float64)
    lib().orc_mean(_p(Vhat, C.c_float), C.c_uint32(K), C.c_uint64(d), _p(m, C.c_double))
    return m


class EGState:
    """(Y_t, anchor = X_1, S, gamma_t) of eq. (Q-GenX); gamma_1 = K."""

    def __init__(self, d: int, K: int, X1=None):
        self.d, self.K = d, K
        self.Y = np.zeros(d, np.float64)
        self.anchor = None if X1 is None else np.array(X1, np.float64)
        self.S = 0.0
        self.gamma = float(K)
        self.t = 1

    def X(self):
        a = 0.0 if self.anchor is None else self.anchor
        return a + self.gamma * self.Y

    def half0(self, Vhat):
        Vhat = _c(Vhat, np.float32)
        out = np.zeros(self.d, np.float64)
        lib().orc_eg_half0(_p(Vhat, C.c_float), C.c_uint32(self.K), C.c_uint64(self.d),
                           _p(self.Y, C.c_double), _p(self.anchor, C.c_double),
                           C.c_double(self.gamma), _p(out, C.c_double))
        return out

    def half1(self, Vhat_cur, Vhat_prev=None):
        Vhat_cur = _c(Vhat_cur, np.float32); Vhat_prev = _c(Vhat_prev, np.float32)
        S = C.c_double(self.S); g = C.c_double(self.gamma)
        out = np.zeros(self.d, np.float64)
        lib().orc_eg_half1(_p(Vhat_cur, C.c_float), _p(Vhat_prev, C.c_float), C.c_uint32(self.K),
                           C.c_uint64(self.d), _p(self.Y, C.c_double), _p(self.anchor, C.c_double),
                           C.byref(S), C.byref(g), _p(out, C.c_double))
        self.S, self.gamma = S.value, g.value
        self.t += 1
        return out


def bin_of(u, n_bins):
    return int(lib().orc_bin_of(C.c_float(u), C.c_uint32(n_bins)))


def bin_edges(n_bins):
    return np.array([lib().orc_bin_edge(C.c_uint32(b), C.c_uint32(n_bins)) for b in range(n_bins + 1)])


def histogram(V, lay: Layout, norm_kind, n_bins=4096, norms_in=None):
    V = _c(V, np.float32)
    K, d = V.shape
    norms_in = _c(norms_in, np.float32)
    H = np.zeros(n_bins, np.float64)
    lib().orc_histogram(_p(V, C.c_float), C.c_uint32(K), C.c_uint64(d),
                        _p(lay.bucket_start, C.c_uint64), C.c_uint64(lay.NB), C.c_int(norm_kind),
                        _p(norms_in, C.c_float), C.c_uint32(n_bins), _p(H, C.c_double))
    return H


def fit_levels(H, levels, sweeps):
    H = _c(H, np.float64)
    lv = np.array(levels, np.float32)
    lib().orc_fit_levels(_p(H, C.c_double), C.c_uint32(len(H)), _p(lv, C.c_float),
                         C.c_uint32(len(lv)), C.c_uint32(sweeps))
    return lv


def stationary_point(H, a, c):
    """One level update: the smallest root of the stationarity condition between the neighbours a < c."""
    H = _c(H, np.float64)
    return float(lib().orc_stationary_point(_p(H, C.c_double), C.c_uint32(len(H)), C.c_double(a), C.c_double(c)))


def symbol_probabilities(H, levels):
    """p_j of Proposition 1 on the histogram's piecewise-uniform density."""
    H = _c(H, np.float64); lv = _c(levels, np.float32)
    p = np.zeros(len(lv), np.float64)
    lib().orc_symbol_probabilities(_p(H, C.c_double), C.c_uint32(len(H)), _p(lv, C.c_float), C.c_uint32(len(lv)),
                                   _p(p, C.c_double))
    return p


def code_weights(p):
    p = _c(p, np.float64)
    w = np.zeros(len(p), np.uint64)
    lib().orc_code_weights(_p(p, C.c_double), C.c_uint32(len(p)), _p(w, C.c_uint64))
    return w


def limited_prefix_lengths(w, max_len):
    """Lengths of an optimal prefix code for integer weights w with no word longer than max_len."""
    w = _c(w, np.uint64)
    ln = np.zeros(len(w), np.uint8)
    rc = lib().orc_limited_prefix_lengths(_p(w, C.c_uint64), C.c_uint32(len(w)), C.c_uint32(max_len), _p(ln, C.c_uint8))
    if rc != 0:
        raise ValueError("no prefix code with these limits")
    return ln


def canonical_code(lengths):
    ln = _c(lengths, np.uint8)
    bits = np.zeros(len(ln), np.uint32)
    rc = lib().orc_canonical_code(_p(ln, C.c_uint8), C.c_uint32(len(ln)), _p(bits, C.c_uint32))
    if rc != 0:
        raise ValueError("lengths overfill the code space")
    return bits


def huffman_table(H, levels, max_len=13):
    """(p, code_len, code_bits): Proposition 1's probabilities and the optimal prefix code on them."""
    p = symbol_probabilities(H, levels)
    ln = limited_prefix_lengths(code_weights(p), max_len)
    return p, ln, canonical_code(ln)


def qada_objective(H, levels):
    H = _c(H, np.float64); lv = _c(levels, np.float32)
    return float(lib().orc_qada_objective(_p(H, C.c_double), C.c_uint32(len(H)),
                                          _p(lv, C.c_float), C.c_uint32(len(lv))))


def game_operator(z, a, b, mu):
    """F(z) = M z + b for the block-diagonal M of the large quadratic game, binary64."""
    z = _c(z, np.float32); a = _c(a, np.float32); b = _c(b, np.float32)
    F = np.zeros(len(z), np.float64)
    lib().orc_game_operator(_p(z, C.c_float), _p(a, C.c_float), _p(b, C.c_float), C.c_double(mu), C.c_uint64(len(z)), _p(F, C.c_double))
    return F


def normal(noise_seed, k, call_id, i):
    return float(lib().orc_normal(noise_seed, k, call_id, i))


def game_dual_vectors(z, a, b, mu, sigma, noise_seed, call_id, K):
    """[K][d] float32: F(z) + sigma N(0, 1), the reproducible draws of the game's stochastic oracle."""
    z = _c(z, np.float32); a = _c(a, np.float32); b = _c(b, np.float32)
    V = np.zeros((K, len(z)), np.float32)
    lib().orc_game_dual_vectors(_p(z, C.c_float), _p(a, C.c_float), _p(b, C.c_float), C.c_double(mu), C.c_double(sigma),
                                C.c_uint64(noise_seed), C.c_uint32(call_id), C.c_uint32(K), C.c_uint64(len(z)), _p(V, C.c_float))
    return V


def game_gap(xhat, a, b, mu, center, R, want_maximiser=False):
    """Restricted gap sup_{x in C} <A(x), xhat - x> over the ball C of radius R around center (None = origin)."""
    xhat = _c(xhat, np.float32); a = _c(a, np.float32); b = _c(b, np.float32)
    c = None if center is None else _c(center, np.float32)
    x = np.zeros(len(xhat), np.float64)
    g = lib().orc_game_gap(_p(xhat, C.c_float), _p(a, C.c_float), _p(b, C.c_float), C.c_double(mu), None if c is None else _p(c, C.c_float),
          C.c_double(R), C.c_uint64(len(xhat)), _p(x, C.c_double))
    return (float(g), x) if want_maximiser else float(g)


def norm2(x):
    x = _c(x, np.float32)
    return float(lib().orc_norm2(_p(x, C.c_float), C.c_uint64(x.size)))
