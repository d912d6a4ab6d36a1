"""Pins for the oracle's aggregate / half-steps / step size (Algorithm 1, eq. (Q-GenX), Theorem 3)."""
import numpy as np

import oracle
from paper_2308_09187_amd import synth


def test_mean_and_half_steps_closed_forms():
    K, d = 4, 6
    # worker k holds the constant vector (k+1) * e, so the mean is 2.5 * e
    e = np.arange(1, d + 1, dtype=np.float32)
    Vhat = np.stack([(k + 1) * e for k in range(K)])
    np.testing.assert_allclose(oracle.mean(Vhat), 2.5 * e, rtol=0, atol=0)
    st = oracle.EGState(d, K, X1=np.ones(d))
    assert st.gamma == K and st.S == 0.0                      # gamma_1 = K
    Xh = st.half0(Vhat)                                       # X_1 - gamma_1 * mean
    np.testing.assert_allclose(Xh, 1.0 - K * 2.5 * e, rtol=1e-15)
    # second half-step with Vhat_{t+1/2} = 2 * Vhat_t : differences are -(k+1) e
    Xn = st.half1(2 * Vhat, Vhat)
    np.testing.assert_allclose(st.Y, -5.0 * e, rtol=1e-15)
    S = sum((k + 1) ** 2 for k in range(K)) * float((e.astype(np.float64) ** 2).sum())
    assert abs(st.S - S) < 1e-9 * S
    assert abs(st.gamma - K / np.sqrt(1 + S)) < 1e-15
    np.testing.assert_allclose(Xn, 1.0 + st.gamma * st.Y, rtol=1e-15)
    assert st.t == 2


def test_gamma_non_increasing_and_dual_averaging_case():
    K, d = 3, 50
    rng = np.random.default_rng(0)
    st = oracle.EGState(d, K)
    g = [st.gamma]
    for t in range(20):
        a = rng.standard_normal((K, d)).astype(np.float32)
        b = rng.standard_normal((K, d)).astype(np.float32)
        st.half0(a)
        st.half1(b, a)
        g.append(st.gamma)
    assert g[0] == K and all(x >= y for x, y in zip(g, g[1:]))
    # dual averaging (Example 1): Vhat_t = 0 gives X_{t+1/2} = X_t, and S accumulates ||Vhat_{t+1/2}||^2
    st = oracle.EGState(d, K, X1=rng.standard_normal(d))
    X_before = st.X()
    Xh = st.half0(np.zeros((K, d), np.float32))
    np.testing.assert_array_equal(Xh, X_before)
    b = rng.standard_normal((K, d)).astype(np.float32)
    st.half1(b, None)
    assert abs(st.S - float((b.astype(np.float64) ** 2).sum())) < 1e-9


def _textbook_dual_extrapolation(game, T, X1, noise_fn):
    """Nesterov's dual extrapolation with the adaptive step of Theorem 3, written directly in
    numpy/binary64 with exact (unquantised) dual vectors: the limit of Q-GenX for fine levels."""
    K = game.K
    Y = np.zeros(game.d)
    S, gamma = 0.0, float(K)
    X = X1.astype(np.float64).copy()
    hist = []
    for t in range(T):
        Vt = noise_fn(X, 2 * t)
        Xh = X - gamma * Vt.mean(0)
        Vh = noise_fn(Xh, 2 * t + 1)
        Y = Y - Vh.mean(0)
        S += ((Vt - Vh) ** 2).sum()
        gamma = K / np.sqrt(1 + S)
        X = X1 + gamma * Y
        hist.append(Xh)
    return X, np.mean(hist, axis=0)


def test_fine_levels_limit_reproduces_textbook_extragradient():
    game = synth.BilinearGame(n=16, K=4, noise=0.1)
    X1 = game.x1()
    T = 30
    fine = np.linspace(0, 1, 250).astype(np.float32)          # a fine uniform table: Q -> identity
    lay = oracle.layout(game.d, game.d)

    def draw(z, call):
        return game.dual_vectors(z, call).astype(np.float64)

    X_ref, Xbar_ref = _textbook_dual_extrapolation(game, T, X1, draw)

    st = oracle.EGState(game.d, game.K, X1=X1)
    hist = []
    for t in range(T):
        Vt = game.dual_vectors(st.X(), 2 * t)
        n0, i0, s0, _ = oracle.quantize(Vt, lay, oracle.NORM_LINF, fine, 77, 2 * t)
        c0 = oracle.encode(i0, s0, lay, cap_words=game.d)
        Vhat0, _, _ = oracle.decode(c0, n0, lay, fine)
        Xh = st.half0(Vhat0)
        Vh = game.dual_vectors(Xh, 2 * t + 1)
        n1, i1, s1, _ = oracle.quantize(Vh, lay, oracle.NORM_LINF, fine, 77, 2 * t + 1)
        c1 = oracle.encode(i1, s1, lay, cap_words=game.d)
        Vhat1, _, _ = oracle.decode(c1, n1, lay, fine)
        st.half1(Vhat1, Vhat0)
        hist.append(Xh)
    X_q = st.X()
    # quantisation noise at 249 levels is ~1e-3 of the vector scale; the runs must agree to that
    scale = np.linalg.norm(X_ref)
    assert np.linalg.norm(X_q - X_ref) < 5e-3 * scale
    assert np.linalg.norm(np.mean(hist, 0) - Xbar_ref) < 5e-3 * np.linalg.norm(Xbar_ref)
    # and with exactly representable dual vectors (on-level values) the two coincide to rounding
    # (every u lands on a level, so Q is the identity): checked in the step below
    lv = synth.levels_uniform(4)
    V = np.array([[1.0, -0.5, 0.25, 0.0, 0.75, -1.0]] * 2, np.float32)
    lay6 = oracle.layout(6, 6)
    n, i, s, _ = oracle.quantize(V, lay6, oracle.NORM_LINF, lv, 1, 0)
    Vhat, _, _ = oracle.decode(oracle.encode(i, s, lay6, 64), n, lay6, lv)
    np.testing.assert_array_equal(Vhat, V)


def test_residual_decreases_on_the_bilinear_game():
    """Trend only (Theorem 3): the operator residual at the ergodic average shrinks with T."""
    game = synth.BilinearGame(n=64, K=4, noise=0.1)
    levels = synth.levels_exponential(8)
    lay = oracle.layout(game.d, game.d)
    st = oracle.EGState(game.d, game.K, X1=game.x1())
    hist, res = [], {}
    for t in range(100):
        Vt = game.dual_vectors(st.X(), 2 * t)
        n0, i0, s0, _ = oracle.quantize(Vt, lay, oracle.NORM_L2, levels, 5, 2 * t)
        Vhat0, _, _ = oracle.decode(oracle.encode(i0, s0, lay, game.d), n0, lay, levels)
        Xh = st.half0(Vhat0)
        Vh = game.dual_vectors(Xh, 2 * t + 1)
        n1, i1, s1, _ = oracle.quantize(Vh, lay, oracle.NORM_L2, levels, 5, 2 * t + 1)
        Vhat1, _, _ = oracle.decode(oracle.encode(i1, s1, lay, game.d), n1, lay, levels)
        st.half1(Vhat1, Vhat0)
        hist.append(Xh)
        if t + 1 in (10, 100):
            res[t + 1] = np.linalg.norm(game.operator(np.mean(hist, 0)))
    assert res[100] < 0.5 * res[10]
