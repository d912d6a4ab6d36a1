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
