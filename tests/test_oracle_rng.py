"""Pins for the oracle's counter-based generator (Philox4x32-10, Salmon et al. SC'11)."""
import os

import numpy as np

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat():
    rows = []
    for line in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        rows.append([int(x, 16) for x in line.split()])
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for r in rows:
        out = oracle.philox4x32_10(r[0:4], r[4:6])
        assert [int(x) for x in out] == r[6:10]


def test_uniform24_takes_word_i_mod_4_top_24_bits():
    seed = 0x0123456789ABCDEF
    for i in [0, 1, 2, 3, 4, 5, 1023, (1 << 34) + 7]:
        for k, call in [(0, 0), (3, 9)]:
            blk = i >> 2
            w = oracle.philox4x32_10([blk & 0xFFFFFFFF, blk >> 32, k, call],
                                     [seed & 0xFFFFFFFF, seed >> 32])
            want = (int(w[i & 3]) >> 8) / float(1 << 24)
            assert oracle.uniform24(seed, k, call, i) == want
            assert 0.0 <= want < 1.0


def test_uniform24_is_uniform_chi_square():
    n, bins = 200_000, 64
    r = np.array([oracle.uniform24(7, 0, 0, i) for i in range(n)])
    cnt = np.bincount((r * bins).astype(int), minlength=bins)
    chi2 = ((cnt - n / bins) ** 2 / (n / bins)).sum()
    # 63 degrees of freedom: mean 63, sd ~11.2; 5 sd above the mean
    assert chi2 < 63 + 5 * 11.3
    assert abs(r.mean() - 0.5) < 5 * np.sqrt(1 / 12 / n)
    # neighbouring draws are uncorrelated
    c = np.corrcoef(r[:-1], r[1:])[0, 1]
    assert abs(c) < 5 / np.sqrt(n)


def test_streams_differ_by_worker_call_and_seed():
    base = [oracle.uniform24(1, 0, 0, i) for i in range(64)]
    assert base != [oracle.uniform24(1, 1, 0, i) for i in range(64)]
    assert base != [oracle.uniform24(1, 0, 1, i) for i in range(64)]
    assert base != [oracle.uniform24(2, 0, 0, i) for i in range(64)]
    assert base == [oracle.uniform24(1, 0, 0, i) for i in range(64)]
