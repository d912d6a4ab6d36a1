"""Pins for the oracle's synthetic stochastic oracle of the large quadratic game (Section 2: g = A + U with
E U = 0 and bounded variance; A strongly monotone): the operator against a dense matrix and its closed-form
solution, the noise against the normal law."""
import numpy as np
from scipy import stats

import oracle
from paper_2308_09187_amd import synth


def test_operator_against_a_dense_matrix_and_the_closed_form_solution():
    game = synth.QuadraticGame(d=64, K=2)
    rng = np.random.default_rng(0)
    z = rng.standard_normal(64).astype(np.float32)
    M = np.zeros((64, 64))
    for j in range(32):
        M[2 * j, 2 * j] = M[2 * j + 1, 2 * j + 1] = game.mu
        M[2 * j, 2 * j + 1] = game.a[j]
        M[2 * j + 1, 2 * j] = -float(game.a[j])
    want = M @ z.astype(np.float64) + game.b
    np.testing.assert_allclose(oracle.game_operator(z, game.a, game.b, game.mu), want, rtol=0, atol=1e-12)
    # the solution of F(z) = 0, and strong monotonicity <F(x) - F(y), x - y> = mu |x - y|^2 (the skew part drops out)
    zs = game.solution().astype(np.float32)
    assert np.abs(oracle.game_operator(zs, game.a, game.b, game.mu)).max() < 1e-5
    y = rng.standard_normal(64).astype(np.float32)
    lhs = (oracle.game_operator(z, game.a, game.b, game.mu) - oracle.game_operator(y, game.a, game.b, game.mu)) @ (z.astype(np.float64) - y)
    assert abs(lhs - game.mu * ((z.astype(np.float64) - y) ** 2).sum()) < 1e-9
    assert abs(oracle.norm2(np.array([3, 4], np.float32)) - 5.0) == 0.0


def test_noise_is_standard_normal_and_independent():
    n = 1 << 16
    x = np.array([oracle.normal(99, 0, 0, i) for i in range(n)])
    assert abs(x.mean()) < 5 / np.sqrt(n) and abs(x.var() - 1) < 5 * np.sqrt(2.0 / n)
    assert abs(stats.skew(x)) < 5 * np.sqrt(6.0 / n) and abs(stats.kurtosis(x)) < 5 * np.sqrt(24.0 / n)
    assert stats.kstest(x, "norm").pvalue > 1e-3
    assert np.abs(x).max() < 5.78                       # sqrt(-2 ln 2^-24): the 24-bit uniform bounds the tail
    # the two halves of a Box-Muller pair, neighbouring pairs, other workers, calls and seeds: uncorrelated
    other = {"pair": x[1::2][: n // 2 - 1], "worker": [oracle.normal(99, 1, 0, i) for i in range(0, n, 2)][: n // 2 - 1],
             "call": [oracle.normal(99, 0, 1, i) for i in range(0, n, 2)][: n // 2 - 1],
             "seed": [oracle.normal(98, 0, 0, i) for i in range(0, n, 2)][: n // 2 - 1], "next": x[2::2][: n // 2 - 1]}
    base = x[0::2][: n // 2 - 1]
    for name, y in other.items():
        r = np.corrcoef(base, np.asarray(y))[0, 1]
        assert abs(r) < 5 / np.sqrt(n / 2), name
    # squares too (a shared radius would show there)
    assert abs(np.corrcoef(base ** 2, other["pair"] ** 2)[0, 1]) < 5 / np.sqrt(n / 2)
    assert oracle.normal(99, 0, 0, 5) == x[5]


def test_dual_vectors_are_unbiased_with_the_stated_variance():
    game = synth.QuadraticGame(d=4096, K=64)
    z = np.random.default_rng(1).standard_normal(4096).astype(np.float32)
    F = oracle.game_operator(z, game.a, game.b, game.mu)
    V = oracle.game_dual_vectors(z, game.a, game.b, game.mu, game.noise, noise_seed=7, call_id=3, K=64).astype(np.float64)
    assert V.shape == (64, 4096)
    dev = V - F[None, :]
    assert np.abs(dev.mean(0)).max() < 5.5 * game.noise / np.sqrt(64)
    assert abs(dev.var() - game.noise ** 2) < 5 * game.noise ** 2 * np.sqrt(2.0 / dev.size)
    # reproducible, and a dual vector is the operator plus sigma times the draw of its (worker, call, coordinate)
    assert V[5, 77] == np.float32(F[77] + game.noise * oracle.normal(7, 5, 3, 77))


def _dense(game, d):
    M = np.zeros((d, d))
    for j in range(d // 2):
        M[2 * j, 2 * j] = M[2 * j + 1, 2 * j + 1] = game.mu
        M[2 * j, 2 * j + 1] = game.a[j]
        M[2 * j + 1, 2 * j] = -float(game.a[j])
    return M


def test_restricted_gap_is_the_supremum_over_the_ball():
    """eq. (Gap) over a ball, from the definition with a dense matrix: no point of the ball does better than the
    oracle's value, its maximiser lies in the ball and attains it, and projected gradient ascent ends there;
    with the ball large enough the gap is the free maximum, and at the solution it is zero."""
    d = 16
    game = synth.QuadraticGame(d=d, K=1)
    M, b = _dense(game, d), game.b.astype(np.float64)
    rng = np.random.default_rng(3)
    g_of = lambda x, h: (M @ x + b) @ (h - x)
    for trial in range(12):
        xhat = (rng.standard_normal(d) * (0.2 + trial)).astype(np.float32)
        centre = None if trial % 3 == 0 else rng.standard_normal(d).astype(np.float32)
        c = np.zeros(d) if centre is None else centre.astype(np.float64)
        R = [0.3, 2.0, 50.0, 1e4][trial % 4]
        gap, x_star = oracle.game_gap(xhat, game.a, game.b, game.mu, centre, R, want_maximiser=True)
        h = xhat.astype(np.float64)
        assert np.linalg.norm(x_star - c) <= R * (1 + 1e-12)
        assert abs(g_of(x_star, h) - gap) <= 1e-9 * max(1.0, abs(gap))
        # random points of the ball (surface and inside) never do better
        pts = rng.standard_normal((4000, d))
        pts = c + pts / np.linalg.norm(pts, axis=1, keepdims=True) * R * rng.random((4000, 1)) ** (1.0 / d)
        pts[:2000] = c + (pts[:2000] - c) / np.linalg.norm(pts[:2000] - c, axis=1, keepdims=True) * R
        vals = np.array([g_of(x, h) for x in pts])
        assert vals.max() <= gap + 1e-9 * max(1.0, abs(gap))
        # projected gradient ascent on the concave objective from the centre
        x = c.copy()
        step = 0.25 / game.mu
        for _ in range(4000):
            grad = M.T @ (h - x) - (M @ x + b)
            x = x + step * grad
            r = np.linalg.norm(x - c)
            if r > R:
                x = c + (x - c) * (R / r)
        assert abs(g_of(x, h) - gap) <= 1e-7 * max(1.0, abs(gap))
        if R == 1e4:                      # the ball holds the free maximiser: a closed form
            w = M.T @ h - b
            assert abs(gap - (w @ w / (4 * game.mu) + b @ h)) <= 1e-9 * max(1.0, abs(gap))
    # at the solution the gap vanishes when the ball holds it, and it is non-negative for any candidate then
    zs = game.solution()
    assert abs(oracle.game_gap(zs.astype(np.float32), game.a, game.b, game.mu, zs.astype(np.float32), 1.0)) < 1e-6
    for _ in range(5):
        xhat = (zs + rng.standard_normal(d) * 0.1).astype(np.float32)
        assert oracle.game_gap(xhat, game.a, game.b, game.mu, zs.astype(np.float32), 1.0) >= 0.0
    # without coupling and offset: sup -mu |x|^2 + mu <xhat, x> = mu |xhat|^2 / 4
    e = np.zeros(d, np.float32); e[0] = 2.0
    assert abs(oracle.game_gap(e, np.zeros(d // 2, np.float32), np.zeros(d, np.float32), 0.5, None, 10.0) - 0.5) < 1e-12
    # ... and on a ball too small for the free maximiser x0 = xhat / 2 the best point is on the sphere towards it
    assert abs(oracle.game_gap(e, np.zeros(d // 2, np.float32), np.zeros(d, np.float32), 0.5, None, 0.5)
               - (-0.5 * 0.25 + 0.5 * 2.0 * 0.5)) < 1e-12
