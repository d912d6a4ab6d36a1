"""Pins for the oracle's symbol probabilities (Proposition 1) and its optimal prefix code Psi
(Appendix J: Huffman coding on estimated symbol probabilities; Theorem (Huffman): H <= E[L] <= H + 1),
including the limit on the word length that the GPU decoder's table needs."""
import heapq
import itertools

import numpy as np
import pytest

import oracle
from paper_2308_09187_amd import synth


def _huffman_expected_length(w):
    """Textbook Huffman by repeated merging of the two lightest nodes: the cost is the sum of all
    merged weights.  Independent of the oracle's construction."""
    h = [int(x) for x in w]
    heapq.heapify(h)
    cost = 0
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        cost += a + b
        heapq.heappush(h, a + b)
    return cost


def _huffman_depth(w):
    h = [(int(x), 0, i) for i, x in enumerate(w)]        # (weight, depth of subtree, tiebreak)
    heapq.heapify(h)
    n = len(h)
    while len(h) > 1:
        a, b = heapq.heappop(h), heapq.heappop(h)
        n += 1
        heapq.heappush(h, (a[0] + b[0], max(a[1], b[1]) + 1, n))
    return h[0][1]


def test_probabilities_closed_form_on_uniform_density():
    """Uniform density and uniform levels: every interior level collects 1/s, the two ends half of it."""
    nb = 4096
    H = np.diff(oracle.bin_edges(nb))
    for s in (2, 4, 16):
        lv = synth.levels_uniform(s)
        p = oracle.symbol_probabilities(H, lv)
        want = np.full(s + 1, 1.0 / s); want[0] = want[-1] = 0.5 / s
        np.testing.assert_allclose(p, want, rtol=0, atol=1e-12)
    # a point mass inside one narrow bin: the hat functions of its two neighbours split it
    H = np.zeros(nb); b = oracle.bin_of(0.3, nb); H[b] = 7.0
    e = oracle.bin_edges(nb)
    mid = 0.5 * (e[b] + e[b + 1])
    p = oracle.symbol_probabilities(H, np.array([0, 0.25, 0.5, 1], np.float32))
    np.testing.assert_allclose(p, [0, (0.5 - mid) / 0.25, (mid - 0.25) / 0.25, 0], atol=1e-12)


def test_probabilities_sum_to_one_and_match_emitted_symbols():
    """p_j against the frequency with which Q_l emits l_j (one bucket, so the weights of F~ play no
    role), and Lemma 2: the expected number of non-zeros is (1 - p_0) d."""
    d = 1 << 17
    V = synth.student_t3(1, d, seed=23)
    lay = oracle.layout(d, d)
    lv = synth.levels_exponential(8)
    H = oracle.histogram(V, lay, oracle.NORM_L2, 4096)
    p = oracle.symbol_probabilities(H, lv)
    assert abs(p.sum() - 1) < 1e-12 and (p >= 0).all()
    R = 8
    cnt = np.zeros(len(lv))
    for call in range(R):
        _, idx, _, _ = oracle.quantize(V, lay, oracle.NORM_L2, lv, 3, call)
        cnt += np.bincount(idx[0], minlength=len(lv))
    freq = cnt / (R * d)
    # sampling error of R*d draws plus the binning error of the density (64 bins per octave)
    np.testing.assert_allclose(freq, p, atol=4 * np.sqrt(p.max() / (R * d)) + 2e-4)
    assert abs((cnt[1:].sum() / R) - (1 - p[0]) * d) < 4 * np.sqrt(d) + 2e-4 * d


def test_proposition_1_typo_reading():
    """The printed p_0 integrates (1 - u)/l_1; read as (l_1 - u)/l_1 (what Definition 1 gives).  With
    all mass just above 0 the symbol 0 must then be (almost) certain, not 1/l_1 times too likely."""
    nb = 4096
    H = np.zeros(nb); H[0] = 1.0
    p = oracle.symbol_probabilities(H, np.array([0, 0.25, 1], np.float32))
    assert 0.999 < p[0] <= 1.0 and abs(p.sum() - 1) < 1e-12


@pytest.mark.parametrize("seed", range(6))
def test_code_is_huffman_optimal_when_the_limit_is_slack(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(2, 60))
    w = rng.integers(1, 1 << 20, n).astype(np.uint64)
    if _huffman_depth(w) > 13:
        pytest.skip("limit active")
    ln = oracle.limited_prefix_lengths(w, 13)
    assert (ln >= 1).all() and (ln <= 13).all()
    assert sum(2.0 ** -int(x) for x in ln) == 1.0 if n > 1 else True           # complete code
    assert int((w * ln.astype(np.uint64)).sum()) == _huffman_expected_length(w)
    # Theorem (Huffman): H <= E[L] <= H + 1
    p = w / w.sum()
    Hent = -(p * np.log2(p)).sum()
    EL = (p * ln).sum()
    assert Hent - 1e-12 <= EL <= Hent + 1 + 1e-12


def test_limited_code_is_optimal_by_brute_force():
    """Geometric weights force Huffman deeper than the limit; every length assignment that satisfies
    Kraft's inequality is tried."""
    for n, L in ((5, 3), (6, 3), (7, 4), (8, 3)):
        w = np.array([1 << (2 * (n - 1 - i)) for i in range(n)], np.uint64)
        assert _huffman_depth(w) > L or n <= L
        ln = oracle.limited_prefix_lengths(w, L)
        assert (ln >= 1).all() and (ln <= L).all()
        assert sum(2.0 ** -int(x) for x in ln) <= 1.0
        best = min(sum(int(a) * b for a, b in zip(w, cand))
                   for cand in itertools.product(range(1, L + 1), repeat=n)
                   if sum(2.0 ** -c for c in cand) <= 1.0)
        assert int((w * ln.astype(np.uint64)).sum()) == best
    with pytest.raises(ValueError):
        oracle.limited_prefix_lengths(np.ones(9, np.uint64), 3)          # 9 words do not fit 3 bits


def test_geometric_weights_with_127_symbols_respect_the_limit():
    w = np.array([max(1, 1 << max(0, 40 - i)) for i in range(127)], np.uint64)
    ln = oracle.limited_prefix_lengths(w, 13)
    assert ln.max() <= 13 and sum(2.0 ** -int(x) for x in ln) <= 1.0
    assert (np.diff(ln.astype(int)) >= 0).all()                           # heavier symbols: never longer words


def test_canonical_words_are_prefix_free_in_stream_bit_order():
    ln = np.array([2, 1, 3, 3], np.uint8)
    bits = oracle.canonical_code(ln)
    # canonical numbering, most significant bit first: 1 -> "0", 0 -> "10", 2 -> "110", 3 -> "111"
    words = ["".join(str((int(b) >> q) & 1) for q in range(int(l))) for b, l in zip(bits, ln)]
    assert words == ["10", "0", "110", "111"]
    with pytest.raises(ValueError):
        oracle.canonical_code(np.array([1, 1, 2], np.uint8))
    rng = np.random.default_rng(1)
    w = rng.integers(1, 1000, 40).astype(np.uint64)
    ln = oracle.limited_prefix_lengths(w, 13)
    bits = oracle.canonical_code(ln)
    words = ["".join(str((int(b) >> q) & 1) for q in range(int(l))) for b, l in zip(bits, ln)]
    for i, a in enumerate(words):
        for j, b in enumerate(words):
            assert i == j or not b.startswith(a)


def test_fitted_code_round_trip_and_length_bound():
    """The whole chain on heavy-tailed data: fit levels, estimate p_j, build the code, encode and
    decode with it; the bits spent respect C_b + (1 - p_0) d + (H + 1) d (Section 3.2) and undercut
    the universal code on the same symbols."""
    K, d, bucket = 2, 1 << 15, 8192
    V = synth.student_t3(K, d, seed=24)
    lay = oracle.layout(d, bucket)
    H = oracle.histogram(V, lay, oracle.NORM_L2, 4096)
    lv = oracle.fit_levels(H, synth.levels_exponential(32), sweeps=10)
    p, ln, bits = oracle.huffman_table(H, lv, max_len=13)
    assert ln.max() <= 13 and abs(p.sum() - 1) < 1e-12
    norms, idx, neg, _ = oracle.quantize(V, lay, oracle.NORM_L2, lv, 9, 0)
    st_h = oracle.encode(idx, neg, lay, cap_words=d, code_len=ln, code_bits=bits)
    st_e = oracle.encode(idx, neg, lay, cap_words=d)
    Vh, idx2, neg2 = oracle.decode(st_h, norms, lay, lv, code_len=ln, code_bits=bits)
    np.testing.assert_array_equal(idx2, idx)
    Ve, _, _ = oracle.decode(st_e, norms, lay, lv)
    np.testing.assert_array_equal(Vh, Ve)
    pe = np.where(p > 0, p, 1.0)
    Hent = -(p * np.log2(pe)).sum()
    for k in range(K):
        assert int(st_h.total_bits[k]) + 32 * lay.NB <= 32 * lay.NB + (1 - p[0]) * d * 1.05 + (Hent + 1) * d
        assert int(st_h.total_bits[k]) < int(st_e.total_bits[k])
