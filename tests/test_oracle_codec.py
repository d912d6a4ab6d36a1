"""Pins for the oracle's CODE / DEQ (Section 3.2, Appendix J): Elias' recursive code against its
published table, prefix-freeness, lossless round trip, the stream rebuilt independently from the
golden code words, expected length, and the error paths."""
import os

import numpy as np
import pytest

import oracle
from paper_2308_09187_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_codes():
    out = {}
    for line in open(os.path.join(GOLDEN, "elias_omega.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n, w = line.split()
        out[int(n)] = w
    return out


def _omega_str(n):
    return "".join(str(b) for b in oracle.elias_omega(n))


def test_elias_omega_golden_table_and_lengths():
    for n, w in _golden_codes().items():
        assert _omega_str(n) == w
    ranges = {1: 1, 2: 3, 3: 3, 4: 6, 7: 6, 8: 7, 15: 7, 16: 11, 31: 11, 32: 12, 63: 12, 64: 13, 127: 13, 128: 14, 255: 14}
    for n, ln in ranges.items():
        assert len(oracle.elias_omega(n)) == ln
    # shorter words for smaller values (what Appendix J asks of the universal code)
    lens = [len(oracle.elias_omega(n)) for n in range(1, 257)]
    assert lens == sorted(lens)


def test_elias_omega_prefix_free_and_kraft():
    words = [_omega_str(n) for n in range(1, 257)]
    assert len(set(words)) == len(words)
    for i, a in enumerate(words):
        for j, b in enumerate(words):
            if i != j:
                assert not b.startswith(a)
    assert sum(2.0 ** -len(w) for w in words) <= 1.0


def _plain_stream(idx_row, neg_row):
    """The paper's bit string for one run of coordinates: Psi(idx) then a sign bit iff idx != 0,
    built from string concatenation of the golden-checked code words."""
    return "".join(_omega_str(int(s) + 1) + (str(int(g)) if s else "") for s, g in zip(idx_row, neg_row))


def _container_bits(st, k, c):
    base = int(st.chunk_off[k, c]) * 32
    nbits = int(st.sub_end[k, c, -1])
    w = st.payload[k]
    return "".join(str((int(w[(base + p) >> 5]) >> ((base + p) & 31)) & 1) for p in range(nbits))


@pytest.mark.parametrize("kind,bucket", [("random", 8192), ("zeros", 8192), ("max", 8192), ("alternating", 8192), ("ramp", 8192),
                                         ("random", 1024), ("ramp", 256)])
def test_round_trip_and_strip_padding_invariant(kind, bucket):
    K, n_sym = 3, 33
    # chunks of 4096, 4096 and 777 coordinates (ragged tail); with small buckets a chunk holds several of them
    lay = oracle.layout(2 * 4096 + 777, bucket)
    assert lay.NC == 3 and lay.NB == -(-lay.d // bucket)
    d = lay.d
    rng = np.random.default_rng(5)
    if kind == "random":
        idx = rng.integers(0, n_sym, (K, d)).astype(np.uint8)
    elif kind == "zeros":
        idx = np.zeros((K, d), np.uint8)
    elif kind == "max":
        idx = np.full((K, d), n_sym - 1, np.uint8)
    elif kind == "alternating":
        idx = np.tile(np.array([0, n_sym - 1], np.uint8), (K, d // 2 + 1))[:, :d].copy()
    else:
        idx = (np.arange(K * d).reshape(K, d) % n_sym).astype(np.uint8)
    neg = rng.integers(0, 2, (K, d)).astype(np.uint8)
    levels = np.linspace(0, 1, n_sym).astype(np.float32)
    norms = rng.uniform(0.5, 2.0, (K, lay.NB)).astype(np.float32)
    st = oracle.encode(idx, neg, lay, cap_words=d)
    Vhat, idx2, neg2 = oracle.decode(st, norms, lay, levels)
    np.testing.assert_array_equal(idx2, idx)
    np.testing.assert_array_equal(neg2[idx != 0], neg[idx != 0])
    assert not neg2[idx == 0].any()
    # vhat = +-(norm * level), one binary32 product
    per_coord_norm = np.repeat(norms, np.diff(lay.bucket_start).astype(int), axis=1)
    want = per_coord_norm * levels[idx] * np.where((neg == 1) & (idx != 0), np.float32(-1), np.float32(1))
    np.testing.assert_array_equal(Vhat, want.astype(np.float32))
    # container minus padding == the paper's plain symbol stream, chunk by chunk
    for k in range(K):
        total = 0
        for c in range(lay.NC):
            lo, hi = int(lay.chunk_start[c]), int(lay.chunk_start[c + 1])
            plain = _plain_stream(idx[k, lo:hi], neg[k, lo:hi])
            assert _container_bits(st, k, c) == plain
            total += len(plain)
            # chunk starts are 128-bit aligned, pad bits are zero, offsets are an exclusive scan
            assert int(st.chunk_off[k, c]) % 4 == 0
            words = -(-len(plain) // 32)
            words = -(-words // 4) * 4
            assert int(st.chunk_off[k, c + 1]) - int(st.chunk_off[k, c]) == words
            # sub-chunk table: ends of runs of SUB coordinates
            pos, S = 0, oracle.SUB()
            assert st.sub_end.shape[2] == oracle.CH() // S
            for j in range(oracle.CH() // S):
                a, b = lo + S * j, min(lo + S * (j + 1), hi)
                if a < hi:
                    pos += len(_plain_stream(idx[k, a:b], neg[k, a:b]))
                assert int(st.sub_end[k, c, j]) == pos
        assert int(st.total_bits[k]) == total
        used = int(st.chunk_off[k, lay.NC])
        assert not st.payload[k, used:].any()


def test_expected_code_length_exact_formula():
    """Mean stream length over many draws equals sum_i [(1-xi) L(tau) + xi L(tau+1)],
    L(j) = |omega(j+1)| + [j != 0]; plus 32 bits per bucket for the norm (C_b = 32)."""
    d, R = 4096, 64
    v = synth.gaussian_vector(d, seed=21)
    levels = synth.levels_exponential(16)
    lv = levels.astype(np.float64)
    n = np.sqrt((v.astype(np.float64) ** 2).sum())
    u = np.abs(v) / n
    tau = np.minimum(np.searchsorted(lv, u, side="right") - 1, len(lv) - 2)
    xi = (u - lv[tau]) / (lv[tau + 1] - lv[tau])
    L = np.array([len(oracle.elias_omega(j + 1)) + (j != 0) for j in range(len(lv))], np.float64)
    exp_bits = ((1 - xi) * L[tau] + xi * L[tau + 1]).sum()
    sd = np.sqrt((xi * (1 - xi) * (L[tau + 1] - L[tau]) ** 2).sum() / R)
    lay = oracle.layout(d, d)
    V = np.tile(v[None, :], (R, 1))
    norms, idx, neg, _ = oracle.quantize(V, lay, oracle.NORM_L2, levels, 3, 0)
    st = oracle.encode(idx, neg, lay, cap_words=d)
    assert abs(st.total_bits.astype(np.float64).mean() - exp_bits) < 5 * sd
    # Theorem 2's proof bounds an *optimal* prefix code by C_b + (1-p0) d + (H+1) d; the universal
    # code is not optimal, so only the sign-bit count (1 - p0) d of Lemma 2 is compared here.
    nnz = (idx != 0).sum(1).mean()
    p0 = np.where(tau == 0, 1 - xi, 0.0).mean()
    assert abs(nnz - (1 - p0) * d) < 5 * np.sqrt(np.where(tau == 0, xi * (1 - xi), 0).sum() / R) + 1e-9


def test_table_code_round_trip():
    """A caller-supplied prefix code table (here a fixed-length 3-bit code) goes through the same
    container."""
    n_sym = 8
    code_len = np.full(n_sym, 3, np.uint8)
    # first-written bit in bit 0: write the 3-bit binary MSB first => reverse the bits
    code_bits = np.array([int(format(j, "03b")[::-1], 2) for j in range(n_sym)], np.uint32)
    lay = oracle.layout(5000, 4096)
    rng = np.random.default_rng(8)
    idx = rng.integers(0, n_sym, (2, lay.d)).astype(np.uint8)
    neg = rng.integers(0, 2, (2, lay.d)).astype(np.uint8)
    st = oracle.encode(idx, neg, lay, cap_words=2048, code_len=code_len, code_bits=code_bits)
    assert int(st.total_bits[0]) == 3 * lay.d + int((idx[0] != 0).sum())
    _, idx2, _ = oracle.decode(st, np.ones((2, lay.NB), np.float32), lay, np.linspace(0, 1, n_sym),
                               code_len=code_len, code_bits=code_bits)
    np.testing.assert_array_equal(idx2, idx)


def test_capacity_overflow_and_malformed_stream():
    lay = oracle.layout(4096, 4096)
    idx = np.full((1, 4096), 32, np.uint8)                 # 12 + 1 bits each = 1664 words
    neg = np.zeros((1, 4096), np.uint8)
    with pytest.raises(OverflowError):
        oracle.encode(idx, neg, lay, cap_words=1663)
    st = oracle.encode(idx, neg, lay, cap_words=1664)
    levels = np.linspace(0, 1, 33).astype(np.float32)
    norms = np.ones((1, 1), np.float32)
    oracle.decode(st, norms, lay, levels)
    # a symbol outside the table
    with pytest.raises(ValueError):
        oracle.decode(st, norms, lay, levels[:20])
    # a flipped bit breaks the parse or the sub-chunk table check
    bad = oracle.Stream(st.payload.copy(), st.chunk_off, st.sub_end, st.total_bits)
    bad.payload[0, 10] ^= 1 << 3
    with pytest.raises(ValueError):
        oracle.decode(bad, norms, lay, levels)
    # a truncated chunk
    cut = oracle.Stream(st.payload, st.chunk_off.copy(), st.sub_end, st.total_bits)
    cut.chunk_off[0, 1] = 100
    with pytest.raises(ValueError):
        oracle.decode(cut, norms, lay, levels)
