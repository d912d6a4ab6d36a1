"""Pins for the oracle's Q_l (Definition 1): unbiasedness, the exact variance of eq. (var),
the bound of Theorem 1, Lemma 2, and the special cases the definition fixes."""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2308_09187_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _xi_table(v, levels, q):
    """tau, xi and u of Definition 1 in binary64, straight from the definition."""
    v = np.asarray(v, np.float64)
    lv = np.asarray(levels, np.float64)
    n = np.sqrt((v * v).sum()) if q == 2 else np.abs(v).max()
    u = np.abs(v) / n
    tau = np.minimum(np.searchsorted(lv, u, side="right") - 1, len(lv) - 2)
    xi = (u - lv[tau]) / (lv[tau + 1] - lv[tau])
    return n, u, tau, xi


def _replicas(v, R):
    """R copies of v as R 'workers': one oracle call gives R independent draws."""
    return np.tile(np.asarray(v, np.float32)[None, :], (R, 1))


def _dequant(norms, idx, neg, levels):
    lv = np.asarray(levels, np.float64)
    return norms.astype(np.float64) * lv[idx] * np.where(neg == 1, -1.0, 1.0)


@pytest.mark.parametrize("q", [oracle.NORM_L2, oracle.NORM_LINF])
def test_enumeration_d8_mean_variance_and_joint_law(q):
    """All 2^d up/down outcomes, weighted by prod xi / (1 - xi): the mean is v, the variance is
    eq. (var); and the oracle's empirical law over outcomes matches those weights (chi-square),
    so coordinates are rounded independently with the stated probabilities."""
    d, R = 8, 1 << 16
    v = np.array([0.31, -0.12, 0.05, 0.77, -0.4, 0.013, 0.22, -0.09], np.float32)
    levels = np.array([0, 0.05, 0.15, 0.3, 0.6, 1.0], np.float32)
    n, u, tau, xi = _xi_table(v, levels, 2 if q == oracle.NORM_L2 else 0)
    lv = levels.astype(np.float64)
    outcomes = list(itertools.product([0, 1], repeat=d))
    prob = np.array([np.prod(np.where(np.array(o) == 1, xi, 1 - xi)) for o in outcomes])
    vals = np.array([n * lv[tau + np.array(o)] * np.sign(v) for o in outcomes])
    assert abs(prob.sum() - 1) < 1e-12
    mean = (prob[:, None] * vals).sum(0)
    np.testing.assert_allclose(mean, v.astype(np.float64), rtol=0, atol=1e-7)
    var_enum = (prob * ((vals - v.astype(np.float64)) ** 2).sum(1)).sum()
    var_closed = n * n * ((lv[tau + 1] - u) * (u - lv[tau])).sum()          # eq. (var)
    assert abs(var_enum - var_closed) < 1e-12

    lay = oracle.layout(d, d)
    norms, idx, neg, bad = oracle.quantize(_replicas(v, R), lay, q, levels, seed=11, call_id=0)
    assert bad == 0
    up = idx.astype(int) - tau[None, :]
    assert up.min() >= 0 and up.max() <= 1                 # only the two neighbouring levels occur
    code = (up * (1 << np.arange(d - 1, -1, -1))[None, :]).sum(1)
    cnt = np.bincount(code, minlength=1 << d).astype(np.float64)
    exp = prob * R
    big = exp >= 5
    chi2 = ((cnt[big] - exp[big]) ** 2 / exp[big]).sum() + (cnt[~big].sum() - exp[~big].sum()) ** 2 / max(exp[~big].sum(), 1)
    dof = big.sum()
    assert chi2 < dof + 5 * np.sqrt(2 * dof)
    np.testing.assert_array_equal(neg, np.tile((v < 0).astype(np.uint8), (R, 1)))
    np.testing.assert_allclose(norms[:, 0], n, rtol=1e-7)


def test_rounding_is_a_threshold_on_the_draw_at_xi():
    """Up iff r < xi: every draw that rounded up lies below every draw that rounded down, and the
    split sits at xi to within the 24-bit grid."""
    d, R, seed, call = 8, 20000, 5, 3
    v = np.array([0.3, -0.2, 0.11, 0.5, -0.07, 0.4, 0.01, 0.6], np.float32)
    levels = synth.levels_uniform(4)
    n, u, tau, xi = _xi_table(v, levels, 2)
    lay = oracle.layout(d, d)
    _, idx, _, _ = oracle.quantize(_replicas(v, R), lay, oracle.NORM_L2, levels, seed, call)
    up = idx.astype(int) - tau[None, :]
    for i in range(d):
        r = np.array([oracle.uniform24(seed, k, call, i) for k in range(R)])
        ups, downs = r[up[:, i] == 1], r[up[:, i] == 0]
        assert len(ups) and len(downs)
        assert ups.max() < downs.min()
        assert ups.max() < xi[i] + 1e-6 and downs.min() > xi[i] - 1e-6


@pytest.mark.parametrize("table,q", [("exponential", oracle.NORM_L2), ("uniform", oracle.NORM_L2),
                                     ("exponential", oracle.NORM_LINF)])
def test_monte_carlo_unbiased_variance_closed_form_and_theorem1_bound(table, q):
    d, R = 2048, 256
    v = synth.gaussian_vector(d, seed=10)
    levels = synth.levels_exponential(16) if table == "exponential" else synth.levels_uniform(16)
    n, u, tau, xi = _xi_table(v, levels, 2 if q == oracle.NORM_L2 else 0)
    lv = levels.astype(np.float64)
    var_closed = n * n * ((lv[tau + 1] - u) * (u - lv[tau])).sum()
    lay = oracle.layout(d, d)
    norms, idx, neg, _ = oracle.quantize(_replicas(v, R), lay, q, levels, seed=1, call_id=0)
    Qv = _dequant(norms, idx, neg, levels)
    # unbiasedness, Theorem 1: ||mean - v||^2 ~ Var / R, coordinate-wise within 5 sigma
    sd = n * np.sqrt((lv[tau + 1] - u) * (u - lv[tau]) / R)
    err = np.abs(Qv.mean(0) - v.astype(np.float64))
    assert (err <= 5.5 * sd + 1e-7 * n).all()
    assert abs(((Qv.mean(0) - v) ** 2).sum() - var_closed / R) < 0.25 * var_closed / R
    # exact variance, eq. (var)
    var_mc = ((Qv - v.astype(np.float64)[None, :]) ** 2).sum(1).mean()
    assert abs(var_mc - var_closed) < 0.01 * var_closed
    # Theorem 1 bound with eps_Q from the printed formula (d = bucket length)
    l1 = lv[1]
    lbar = (lv[2:] / lv[1:-1]).max()
    mq = 2.0
    dth = (2 / l1) ** mq
    eps = (lbar + 1 / lbar) / 4 - 0.5 + (0.25 * l1 * l1 * d ** (2 / mq) if d < dth else (l1 * d ** (1 / mq) - 1))
    assert var_closed <= eps * (v.astype(np.float64) ** 2).sum()
    assert var_mc <= eps * (v.astype(np.float64) ** 2).sum()


def test_theorem1_eps_q_golden_values():
    """The three worked values of eps_Q (bucket lengths of the workloads) against the formula."""
    for line in open(os.path.join(GOLDEN, "theorem1_eps_q.txt")):
        if line.startswith("#") or not line.strip():
            continue
        table, s, q, d, want = line.split()
        s, q, d, want = int(s), int(q), int(d), float(want)
        lv = (synth.levels_exponential(s) if table == "exponential" else synth.levels_uniform(s)).astype(np.float64)
        lbar = (lv[2:] / lv[1:-1]).max()
        l1, mq = lv[1], min(q, 2)
        dth = (2 / l1) ** mq
        eps = (lbar + 1 / lbar) / 4 - 0.5 + (0.25 * l1 * l1 * d ** (2 / mq) if d < dth else l1 * d ** (1 / mq) - 1)
        assert abs(eps - want) < 1e-7
        # and the oracle's variance on a Gaussian bucket of that length respects it
        v = synth.gaussian_vector(d, seed=12)
        n, u, tau, xi = _xi_table(v, lv, q)
        var_closed = n * n * ((lv[tau + 1] - u) * (u - lv[tau])).sum()
        lay = oracle.layout(d, d)
        norms, idx, neg, _ = oracle.quantize(_replicas(v, 64), lay, oracle.NORM_L2, lv, 2, 0)
        var_mc = ((_dequant(norms, idx, neg, lv) - v) ** 2).sum(1).mean()
        assert var_mc <= want * (v.astype(np.float64) ** 2).sum()
        assert abs(var_mc - var_closed) < 0.05 * var_closed


def test_lemma2_expected_nonzeros():
    """E ||Q(v)||_0 = (1 - p_0) d with p_0 the mean over coordinates of P(symbol 0)."""
    d, R = 4096, 128
    v = synth.gaussian_vector(d, seed=13)
    levels = synth.levels_exponential(6)       # l_1 = 2^-5 > typical u => many zeros
    n, u, tau, xi = _xi_table(v, levels, 2)
    p0 = np.where(tau == 0, 1 - xi, 0.0).mean()
    lay = oracle.layout(d, d)
    _, idx, _, _ = oracle.quantize(_replicas(v, R), lay, oracle.NORM_L2, levels, 4, 1)
    nnz = (idx != 0).sum(1)
    sd = np.sqrt(np.where(tau == 0, xi * (1 - xi), 0.0).sum() / R)
    assert abs(nnz.mean() - (1 - p0) * d) < 5 * sd + 1e-9


def test_exact_cases():
    levels = synth.levels_uniform(4)           # 0, .25, .5, .75, 1
    lay = oracle.layout(4, 4)
    # L-inf: u = 1 for the largest coordinate => last symbol, always; u on a level never moves
    v = np.array([[2.0, -1.0, 0.5, 0.0]], np.float32)
    for call in range(50):
        norms, idx, neg, bad = oracle.quantize(v, lay, oracle.NORM_LINF, levels, 9, call)
        assert norms[0, 0] == 2.0 and bad == 0
        assert idx[0].tolist() == [4, 2, 1, 0]
        assert neg[0].tolist() == [0, 1, 0, 0]
    # the zero vector: norm 0, every symbol 0
    norms, idx, neg, bad = oracle.quantize(np.zeros((1, 4), np.float32), lay, oracle.NORM_L2, levels, 9, 0)
    assert norms[0, 0] == 0.0 and not idx.any() and bad == 0
    # a non-finite coordinate poisons its bucket: symbols 0, stored norm 0, counted
    for q in (oracle.NORM_L2, oracle.NORM_LINF):
        for poison in (np.nan, np.inf):
            w = np.array([[1.0, poison, 3.0, 4.0]], np.float32)
            norms, idx, neg, bad = oracle.quantize(w, lay, q, levels, 9, 0)
            assert bad == 1 and norms[0, 0] == 0.0 and not idx.any()
    # sign of -0.0 is kept in neg (and is irrelevant to the stream since the symbol is 0)
    norms, idx, neg, _ = oracle.quantize(np.array([[1.0, -0.0, 0, 0]], np.float32), lay, oracle.NORM_L2, levels, 9, 0)
    assert neg[0, 1] == 1 and idx[0, 1] == 0


def test_norms_closed_forms_and_buckets():
    # 3-4-5, all-ones of length 16384 -> 128, L-inf is the exact maximum
    assert oracle.bucket_norm([3, 4], oracle.NORM_L2)[0] == 5.0
    assert oracle.bucket_norm(np.ones(16384), oracle.NORM_L2)[0] == 128.0
    v = synth.gaussian_vector(5000, seed=14)
    assert oracle.bucket_norm(v, oracle.NORM_LINF)[0] == np.abs(v).max()
    # per-bucket norms with a short last bucket per segment
    lay = oracle.layout(5000, 1024, [3000, 2000])
    assert lay.NB == 5 and lay.bucket_start.tolist() == [0, 1024, 2048, 3000, 4024, 5000]
    norms, idx, neg, _ = oracle.quantize(v[None, :], lay, oracle.NORM_L2, synth.levels_uniform(8), 1, 0)
    for b in range(lay.NB):
        lo, hi = int(lay.bucket_start[b]), int(lay.bucket_start[b + 1])
        want = np.sqrt((v[lo:hi].astype(np.float64) ** 2).sum())
        assert abs(norms[0, b] - want) <= 1e-7 * want
    # norms_in overrides: doubling the norm halves u, so no symbol above the middle of the table
    n2 = norms * 2
    norms_b, idx_b, _, _ = oracle.quantize(v[None, :], lay, oracle.NORM_LINF, synth.levels_uniform(8), 1, 0,
                                           norms_in=np.abs(v).max() * 2 * np.ones_like(norms))
    assert idx_b.max() <= 4
    np.testing.assert_array_equal(norms_b, np.float32(np.abs(v).max() * 2) * np.ones_like(norms))


def test_layout_chunks():
    CH = oracle.CH()
    lay = oracle.layout(3 * CH + 100, 2 * CH)          # buckets: 2CH, CH+100
    assert lay.NB == 2 and lay.NC == 4
    assert lay.chunk_start.tolist() == [0, CH, 2 * CH, 3 * CH, 3 * CH + 100]
    assert lay.chunk_bucket.tolist() == [0, 0, 1, 1]
    # buckets of 256..2048 share chunks: a segment is cut into runs of CH coordinates holding whole buckets
    lay = oracle.layout(2 * CH + 1500, 1024, [CH + 1024, CH + 476])
    assert lay.bucket_start.tolist() == [0, 1024, 2048, 3072, 4096, 5120, 6144, 7168, 8192, 9216, 9692]
    assert lay.chunk_start.tolist() == [0, CH, CH + 1024, 2 * CH + 1024, 2 * CH + 1500]
    assert lay.chunk_bucket.tolist() == [0, 4, 5, 9]
    lay = oracle.layout(3000, 1000)                    # other small sizes keep a chunk per bucket
    assert lay.chunk_start.tolist() == [0, 1000, 2000, 3000] and lay.chunk_bucket.tolist() == [0, 1, 2]
    lay = oracle.layout(int(synth.GAN_SEGMENTS.sum()), 8192, synth.GAN_SEGMENTS)
    assert lay.d == 9855936 and lay.NB == 1207
    short = np.diff(lay.bucket_start.astype(np.int64))
    assert sorted(short[short < 8192].tolist()) == [64, 128, 256, 512]


def test_general_q_norm_against_the_library_norm():
    """||v||_q of Definition 1 for q in Z_+ other than 2: numpy's vector norm in binary64 is the
    reference; q = 2 agrees with the dedicated route, a large q approaches the maximum, tiny and huge
    magnitudes neither underflow nor overflow, and u = |v| / ||v||_q stays in [0, 1]."""
    rng = np.random.default_rng(12)
    v = (rng.standard_t(3, 3000) * 1e-2).astype(np.float32)
    for q in (1, 3, 4, 7, 16):
        n, fin = oracle.bucket_norm(v, q)
        assert fin
        want = np.linalg.norm(v.astype(np.float64), ord=q)
        assert abs(float(n) - want) <= 1e-7 * want
        assert (np.abs(v) / n <= 1.0).all()
    n2, _ = oracle.bucket_norm(v, 2)
    assert abs(float(n2) - np.linalg.norm(v.astype(np.float64))) <= 1e-7 * float(n2)
    n64, _ = oracle.bucket_norm(v, 64)
    ninf, _ = oracle.bucket_norm(v, oracle.NORM_LINF)
    assert ninf <= n64 <= ninf * 3000 ** (1 / 64)
    for scale in (1e-30, 1e30):
        w = (v.astype(np.float64) * scale).astype(np.float32)
        n, fin = oracle.bucket_norm(w, 8)
        want = np.linalg.norm(w.astype(np.float64) / scale, ord=8) * scale
        assert fin and abs(float(n) - want) <= 1e-6 * want
    assert oracle.bucket_norm(np.zeros(10, np.float32), 3) == (0.0, True)
    assert not oracle.bucket_norm(np.array([1, np.inf], np.float32), 3)[1]
    # Q_l with q = 3: symbols follow u = |v| / ||v||_3
    lay = oracle.layout(3000, 1024)
    lv = synth.levels_uniform(8)
    norms, idx, neg, bad = oracle.quantize(v[None, :], lay, 3, lv, 1, 0)
    assert bad == 0
    for b in range(lay.NB):
        lo, hi = int(lay.bucket_start[b]), int(lay.bucket_start[b + 1])
        assert norms[0, b] == oracle.bucket_norm(v[lo:hi], 3)[0]
        u = np.abs(v[lo:hi]) * (np.float32(1) / norms[0, b])
        j = np.minimum(np.floor(np.minimum(u, 1) * 8).astype(int), 7)
        assert ((idx[0, lo:hi] == j) | (idx[0, lo:hi] == j + 1)).all()
