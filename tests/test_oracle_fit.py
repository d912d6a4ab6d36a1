"""Pins for the oracle's adaptive levels (Section 3.3, eq. (QAda))."""
import numpy as np

import oracle
from paper_2308_09187_amd import synth


def test_bins_follow_the_binary32_grid():
    nb = 4096
    e = oracle.bin_edges(nb)
    assert e[0] == 0.0 and e[-1] == 1.0 and (np.diff(e) > 0).all()
    for b in [1, 2, 63, 64, 65, 1000, 4095]:
        assert oracle.bin_of(np.float32(e[b]), nb) == b                       # an edge opens its bin
        assert oracle.bin_of(np.nextafter(np.float32(e[b]), np.float32(0)), nb) == b - 1
    assert oracle.bin_of(0.0, nb) == 0 and oracle.bin_of(1e-30, nb) == 0
    assert oracle.bin_of(1.0, nb) == nb - 1
    # 64 equal-width bins per octave
    w = np.diff(e[nb - 64:])
    np.testing.assert_allclose(w, 0.5 / 64, rtol=0, atol=0)
    # fewer octaves
    e2 = oracle.bin_edges(256)
    assert e2[1] == 2.0 ** -4 * (1 + 1 / 64) and oracle.bin_of(0.3, 256) == 256 - 128 + int((0.3 / 0.25 - 1) * 64)


def test_histogram_weights_are_squared_bucket_norms():
    lay = oracle.layout(3000, 1024)
    V = synth.student_t3(2, 3000, seed=3)
    H = oracle.histogram(V, lay, oracle.NORM_L2, 4096)
    norms, _, _, _ = oracle.quantize(V, lay, oracle.NORM_L2, synth.levels_uniform(2), 0, 0)
    lens = np.diff(lay.bucket_start).astype(np.float64)
    want_total = (norms.astype(np.float64) ** 2 * lens[None, :]).sum()
    assert abs(H.sum() - want_total) < 1e-9 * want_total
    # brute force: place every coordinate by comparing u with the edges
    e = oracle.bin_edges(4096)
    H2 = np.zeros(4096)
    for k in range(2):
        for b in range(lay.NB):
            lo, hi = int(lay.bucket_start[b]), int(lay.bucket_start[b + 1])
            n = norms[k, b]
            u = np.minimum(np.abs(V[k, lo:hi]) * (np.float32(1) / n), np.float32(1)).astype(np.float64)
            bins = np.minimum(np.searchsorted(e, u, side="right") - 1, 4095)
            np.add.at(H2, bins, float(n) ** 2)
    np.testing.assert_allclose(H, H2, rtol=1e-12, atol=0)


def _objective_riemann(H, edges, levels, m=64):
    """(QAda) objective by a midpoint Riemann sum over a fine subdivision of every bin."""
    lv = np.asarray(levels, np.float64)
    tot = 0.0
    for b in np.nonzero(H)[0]:
        x = edges[b] + (np.arange(m) + 0.5) * (edges[b + 1] - edges[b]) / m
        j = np.minimum(np.searchsorted(lv, x, side="right") - 1, len(lv) - 2)
        tot += H[b] / m * ((lv[j + 1] - x) * (x - lv[j])).sum()
    return tot


def test_uniform_density_gives_uniform_levels():
    nb = 4096
    e = oracle.bin_edges(nb)
    H = np.diff(e)                                  # mass proportional to width: uniform density on [0,1]
    for n_sym in (3, 5, 9, 17):
        start = np.sort(np.concatenate([[0, 1], np.random.default_rng(n_sym).uniform(0.05, 0.95, n_sym - 2)])).astype(np.float32)
        lv = oracle.fit_levels(H, start, sweeps=400)
        np.testing.assert_allclose(lv, np.arange(n_sym) / (n_sym - 1), atol=2e-6)


def test_objective_never_increases_and_matches_riemann_sum():
    nb = 4096
    lay = oracle.layout(1 << 15, 4096)
    V = synth.student_t3(2, lay.d, seed=4)
    H = oracle.histogram(V, lay, oracle.NORM_L2, nb)
    e = oracle.bin_edges(nb)
    lv = synth.levels_exponential(16)
    obj = [oracle.qada_objective(H, lv)]
    assert abs(obj[0] - _objective_riemann(H, e, lv, m=256)) < 2e-4 * obj[0]
    for _ in range(12):
        lv = oracle.fit_levels(H, lv, sweeps=1)
        assert (np.diff(lv) > 0).all() and lv[0] == 0 and lv[-1] == 1
        obj.append(oracle.qada_objective(H, lv))
    assert all(b <= a * (1 + 1e-6) for a, b in zip(obj, obj[1:]))
    assert obj[-1] < 0.5 * obj[0]


def test_single_free_level_against_grid_search():
    nb = 1024
    lay = oracle.layout(1 << 14, 1 << 14)
    V = synth.gaussian_vector(lay.d, seed=6)[None, :]
    H = oracle.histogram(V, lay, oracle.NORM_LINF, nb)
    e = oracle.bin_edges(nb)
    lv = oracle.fit_levels(H, np.array([0, 0.5, 1], np.float32), sweeps=1)
    grid = np.linspace(0.01, 0.99, 393)
    vals = [_objective_riemann(H, e, [0, g, 1], m=16) for g in grid]
    g_best = grid[int(np.argmin(vals))]
    assert abs(lv[1] - g_best) <= 1.5 * (grid[1] - grid[0])
    assert oracle.qada_objective(H, lv) <= min(vals) * (1 + 1e-3)


def test_fitted_levels_beat_exponential_levels_in_realised_variance():
    """What (MinVar) is for: the realised quantisation error with the fitted table is below the
    error with the heuristic exponential table on the same dual vectors, and the histogram
    objective predicts it."""
    lay = oracle.layout(1 << 16, 16384)
    V = synth.student_t3(2, lay.d, seed=7)
    H = oracle.histogram(V, lay, oracle.NORM_L2, 4096)
    lv_exp = synth.levels_exponential(32)
    lv_fit = oracle.fit_levels(H, lv_exp, sweeps=30)

    def realised(lv):
        tot = 0.0
        for call in range(4):
            norms, idx, neg, _ = oracle.quantize(V, lay, oracle.NORM_L2, lv, 9, call)
            nb = np.repeat(norms, np.diff(lay.bucket_start).astype(int), axis=1).astype(np.float64)
            q = nb * lv.astype(np.float64)[idx] * np.where(neg == 1, -1.0, 1.0)
            tot += ((q - V) ** 2).sum() / 4
        return tot

    r_fit, r_exp = realised(lv_fit), realised(lv_exp)
    assert r_fit < r_exp
    assert abs(r_fit - oracle.qada_objective(H, lv_fit)) < 0.15 * r_fit
    assert abs(r_exp - oracle.qada_objective(H, lv_exp)) < 0.15 * r_exp


def test_empty_histogram_and_collapsed_levels_stay_valid():
    lv0 = synth.levels_uniform(8)
    lv = oracle.fit_levels(np.zeros(4096), lv0, sweeps=3)
    np.testing.assert_array_equal(lv, lv0)
    # all mass in one bin: interior levels crowd into it but stay strictly increasing
    H = np.zeros(4096); H[3000] = 1.0
    lv = oracle.fit_levels(H, lv0, sweeps=50)
    assert lv[0] == 0 and lv[-1] == 1 and (np.diff(lv) >= 2.0 ** -24).all()


def test_flat_stationarity_takes_the_smallest_root():
    """Histograms with empty bins, answers by hand (64 bins: one octave, bins of width 1/128 above 0.5).
    (i) One free level between 0 and 1, mass m1 in bin 16 and m2 in bin 48 with m1 * mid1 = m2 * (1 - mid2):
    the stationarity condition holds on the whole empty stretch between the two bins, and the level goes
    to its left end, the top edge of bin 16.  (ii) No mass between the neighbours: the level goes to the
    lower neighbour; the first level with mass above it goes where the mass below it reaches
    int (1 - u) dF: a fraction (1 - mid) of the bin's mass, that far into the bin."""
    e = oracle.bin_edges(64)
    assert e[16] == 0.625 and e[17] == 0.6328125 and e[48] == 0.875
    mid1, mid2 = 0.5 * (e[16] + e[17]), 0.5 * (e[48] + e[49])
    H = np.zeros(64); H[16] = 1.0 - mid2; H[48] = mid1                    # both products are exact in binary64
    for start in (0.55, 0.7, 0.95):
        lv = oracle.fit_levels(H, np.array([0, start, 1], np.float32), sweeps=1)
        assert lv[1] == np.float32(e[17])
    # a little more mass on the right moves the root into bin 48, a little less into bin 16
    H2 = H.copy(); H2[48] *= 1.01
    assert e[48] < oracle.fit_levels(H2, np.array([0, 0.7, 1], np.float32), sweeps=1)[1] < e[49]
    H2[48] = H[48] * 0.99
    assert e[16] < oracle.fit_levels(H2, np.array([0, 0.7, 1], np.float32), sweeps=1)[1] < e[17]
    # (ii)
    H = np.zeros(64); H[60] = 3.0
    lv = oracle.fit_levels(H, np.array([0, 0.6, 0.7, 0.9, 1], np.float32), sweeps=1)
    mid = 0.5 * (e[60] + e[61])
    want3 = e[60] + (1.0 - mid) * (e[61] - e[60])
    assert want3 == 0.968963623046875
    np.testing.assert_array_equal(lv, np.array([0, 2.0 ** -24, 2.0 ** -23, want3, 1], np.float32))


def _exact_G(H, edges, a, x, c):
    """The stationarity function of a level update in exact rational arithmetic, from its definition:
    int_a^x (u - a) dF - int_x^c (c - u) dF for the piecewise-uniform density of the histogram."""
    from fractions import Fraction as Fr
    a, x, c = Fr(float(a)), Fr(float(x)), Fr(float(c))
    tot = Fr(0)
    for b in np.nonzero(H)[0]:
        e0, e1 = Fr(float(edges[b])), Fr(float(edges[b + 1]))
        dens = Fr(float(H[b])) / (e1 - e0)
        lo, hi = max(a, e0), min(x, e1)
        if hi > lo:                                    # int (u - a) du = [(u - a)^2 / 2]
            tot += dens * ((hi - a) ** 2 - (lo - a) ** 2) / 2
        lo, hi = max(x, e0), min(c, e1)
        if hi > lo:                                    # int (c - u) du = [-(c - u)^2 / 2]
            tot -= dens * ((c - lo) ** 2 - (c - hi) ** 2) / 2
    return tot


def test_every_update_is_the_smallest_root_in_exact_arithmetic():
    """Single updates on histograms with many empty bins and masses of very different sizes: the level must
    be, to a few roundings of binary64, the smallest root of its stationarity function, evaluated here from
    the definition in rational arithmetic: negative just below the level (unless that is the lower
    neighbour), not negative just above.  In a third of the cases the lower neighbour sits a hair below
    the top edge of a bin that ends a run of mass: the sliver of mass above it decides the sign against a
    total mass up to 10^15 times larger (a difference of cumulative sums taken from 0 loses it, and the
    level then lands at the far end of the empty stretch, which is no root)."""
    rng = np.random.default_rng(11)
    inside = at_a = slivers = 0
    for case in range(120):
        n_bins = int(rng.choice([64, 256]))
        edges = oracle.bin_edges(n_bins)
        H = rng.random(n_bins) * 10.0 ** rng.integers(-12, 3, n_bins)
        H[rng.random(n_bins) < 0.6] = 0.0
        H[n_bins - 1 - int(rng.integers(0, 8))] = 1.0
        a, c = np.sort(rng.uniform(0.0, 1.0, 2))
        if case % 3 == 0:
            ends = [i for i in range(8, n_bins - 9) if H[i] > 0 and H[i + 1] == 0]
            if not ends:
                continue
            b = int(rng.choice(ends))
            a = float(np.nextafter(np.float32(edges[b + 1]), np.float32(0)))
            nxt = [i for i in range(b + 1, n_bins) if H[i] > 0]
            c = float(edges[nxt[0]]) if nxt and case % 2 == 0 else float(rng.uniform(edges[b + 2], 1.0))
            slivers += 1
        if not c - a > 1e-6:
            continue
        x = oracle.stationary_point(H, a, c)
        assert a <= x <= c
        step = 8 * np.spacing(max(x, 1e-3))
        assert _exact_G(H, edges, a, min(x + step, c), c) >= 0, case
        if x - step > a:
            assert _exact_G(H, edges, a, x - step, c) < 0, case
            inside += 1
        else:
            at_a += 1
    assert inside > 60 and slivers > 20 and at_a > 5
