"""Parity at full size and in the benchmark's launch configurations: the headline workload (K = 8
vectors of d = 2^24 coordinates, buckets of 16384, L2, 33-symbol fitted table; slotted chunk placement
as timed, and compact) and the shape of the large quadratic game (K = 16 vectors of d = 2^26, buckets of
65536, 65 fitted levels), the latter also as 50 iterations with refits.  Properties that hold at any
size are checked over the whole output; sampled buckets and chunks are recomputed one by one by the oracle."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2308_09187_amd import synth

pytestmark = pytest.mark.gpu

REL = 1e-6


def chunk_words(h, k, c):
    """The words of chunk c of worker k, whatever the placement: its size follows from its bit length."""
    bits = int(h["sub_end"][k, c, -1])
    n = ((bits + 31) // 32 + 3) // 4 * 4
    off = int(h["chunk_off"][k, c])
    return h["payload"][k, off:off + n]


def mini_stream(h, k, c0, c1):
    """The chunks c0..c1-1 of worker k as a stand-alone compact oracle Stream."""
    parts = [chunk_words(h, k, c) for c in range(c0, c1)]
    off = np.concatenate([[0], np.cumsum([len(p) for p in parts])]).astype(np.uint32)
    return oracle.Stream(np.concatenate(parts)[None, :], off[None, :], h["sub_end"][k:k + 1, c0:c1], np.zeros(1, np.uint64))


@pytest.mark.parametrize("K,logd,bucket,n_sym,slotted,fitted_code",
                         [(8, 24, 16384, 33, True, False), (8, 24, 16384, 33, False, False), (8, 24, 16384, 33, True, True),
                          (16, 26, 65536, 65, True, False), (16, 24, 65536, 65, False, False)])
def test_full_size_sampled_against_oracle(K, logd, bucket, n_sym, slotted, fitted_code):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2308_09187_amd import qgx
    qgx.load()
    d, seed, call = 1 << logd, 2308, 6
    print("generating", K, logd, bucket, n_sym, slotted, fitted_code, flush=True)
    V = synth.student_t3_device(K, d, seed=20)
    ctx = qgx.Context(d, K, bucket, norm=qgx.NORM_L2, seed=seed, code=qgx.CODE_TABLE if fitted_code else qgx.CODE_ELIAS_OMEGA)
    ctx.set_levels(synth.levels_exponential(n_sym - 1))
    ctx.fit_levels(V, n_sym, 4096, sweeps=10)
    levels = ctx.get_levels()
    assert (np.diff(levels) > 0).all()
    # the fitted prefix code, if any, is taken from the library (its parity is checked elsewhere)
    code_len, code_bits = ctx.fit_code()[1:] if fitted_code else (None, None)
    longest = int(code_len.max()) if fitted_code else len(oracle.elias_omega(n_sym))
    x1 = torch.randn(d, device="cuda", generator=torch.Generator(device="cuda").manual_seed(3))
    ctx.state_init(x1)
    a = ctx.new_stream(slotted=slotted)
    Xh = torch.empty(d, device="cuda")
    print("encode + half-step", flush=True)
    ctx.quantize_encode(V, call, a)
    ctx.eg_step(0, a, None, Xh)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    h = a.to_host()
    NC, NB, CPB = ctx.NC, ctx.NB, bucket // 4096

    # -- whole-output properties ---------------------------------------------------------------
    off = h["chunk_off"].astype(np.int64)
    bits = h["sub_end"][:, :, -1].astype(np.int64)
    assert (off[:, 0] == 0).all()
    words = (bits + 31) // 32
    words = (words + 3) // 4 * 4
    if slotted:
        assert (np.diff(off, axis=1) == ctx.slot_words()).all() and (words <= ctx.slot_words()).all()
    else:
        np.testing.assert_array_equal(np.diff(off, axis=1), words)        # exclusive scan of chunk sizes
    assert (np.diff(h["sub_end"].astype(np.int64), axis=2) >= oracle.SUB()).all()    # >= 1 bit per coordinate
    assert (h["sub_end"][:, :, 0] >= oracle.SUB()).all()
    assert (bits <= 4096 * (longest + 1)).all()                            # longest word plus sign
    assert ctx.stream_bits(a) == int(bits.sum())
    assert np.isfinite(h["norms"]).all() and (h["norms"] > 0).all()

    # -- sampled buckets: norm, symbols -> stream bits, exactly --------------------------------
    rng = np.random.default_rng(0)
    picks = [(0, 0), (K - 1, NB - 1)] + [(int(rng.integers(K)), int(rng.integers(NB))) for _ in range(6)]
    lay_b = oracle.layout(bucket, bucket)
    for k, b in picks:
        print("bucket", k, b, flush=True)
        vb = V[k, b * bucket:(b + 1) * bucket].cpu().numpy()[None, :]
        n_o, _, _, _ = oracle.quantize(vb, lay_b, oracle.NORM_L2, levels, seed, call, k0=k, i0=b * bucket)
        assert abs(h["norms"][k, b] - n_o[0, 0]) <= REL * n_o[0, 0]
        _, idx, neg, _ = oracle.quantize(vb, lay_b, oracle.NORM_L2, levels, seed, call,
                                         norms_in=h["norms"][k:k + 1, b:b + 1], k0=k, i0=b * bucket)
        so = oracle.encode(idx, neg, lay_b, cap_words=bucket, code_len=code_len, code_bits=code_bits)
        ms = mini_stream(h, k, b * CPB, (b + 1) * CPB)
        np.testing.assert_array_equal(ms.chunk_off, so.chunk_off)
        np.testing.assert_array_equal(ms.sub_end, so.sub_end)
        np.testing.assert_array_equal(ms.payload[0], so.payload[0, :ms.payload.shape[1]])
        assert not so.payload[0, ms.payload.shape[1]:].any()

    # -- sampled chunks: decode all K workers, mean and first half-step --------------------------
    lay_c = oracle.layout(4096, 4096)
    gamma = ctx.scalars()["gamma"]
    assert gamma == K
    for c in [0, NC - 1] + [int(rng.integers(NC)) for _ in range(4)]:
        print("chunk", c, flush=True)
        dec = []
        for k in range(K):
            ms = mini_stream(h, k, c, c + 1)
            dec.append(oracle.decode(ms, h["norms"][k:k + 1, c // CPB:c // CPB + 1], lay_c, levels,
                                     code_len=code_len, code_bits=code_bits)[0][0])
        st = oracle.EGState(4096, K, X1=x1[c * 4096:(c + 1) * 4096].cpu().numpy())
        want = st.half0(np.stack(dec))
        got = Xh[c * 4096:(c + 1) * 4096].cpu().numpy()
        assert np.linalg.norm(got - want) <= REL * np.linalg.norm(want)
    ctx.close()


def test_large_quadratic_game_50_iterations_on_device():
    """The large strongly monotone game at its real shape: z in R^(2^26), F(z) = Mz + b with 2x2 blocks
    [[mu, a], [-a, mu]], K = 16 workers with N(0, 0.05^2) noise, buckets of 65536, L2, 65 levels refitted
    every 10 iterations, 50 iterations of eq. (Q-GenX) with X_1 = 0.  The operator and the noise are
    torch device code outside the library (the caller's part); every iterate stays on the device.
    Whole-run properties (S grows, gamma shrinks, t counts, no error bit, the refits move the table),
    and at iteration 11, right after a refit, sampled buckets of the coded stream and a sampled chunk of
    the second half-step are recomputed by the oracle."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2308_09187_amd import qgx
    qgx.load()
    K, d, bucket, n_sym, seed, T = 16, 1 << 26, 65536, 65, 77, 50
    game = synth.QuadraticGame(d, K)
    a_d, b_d = torch.from_numpy(game.a).cuda(), torch.from_numpy(game.b).cuda()
    mu, noise = game.mu, game.noise

    def operator(z):
        z2 = z.view(-1, 2)
        f = torch.empty_like(z2)
        f[:, 0] = mu * z2[:, 0] + a_d * z2[:, 1]
        f[:, 1] = mu * z2[:, 1] - a_d * z2[:, 0]
        return f.view(-1) + b_d

    V = torch.empty(K, d, device="cuda")
    gen = torch.Generator(device="cuda")

    def dual_vectors(z, call):
        gen.manual_seed(4200 + call)
        V.normal_(0.0, noise, generator=gen)
        V.add_(operator(z))
        return V

    ctx = qgx.Context(d, K, bucket, norm=qgx.NORM_L2, seed=seed)
    ctx.set_levels(synth.levels_exponential(n_sym - 1))
    ctx.state_init(None)
    prev, cur = ctx.new_stream(slotted=True), ctx.new_stream(slotted=True)
    X = torch.zeros(d, device="cuda")
    Xh, Xn = torch.empty(d, device="cuda"), torch.empty(d, device="cuda")
    res0 = float(torch.linalg.vector_norm(operator(X).double()))
    S_last, gamma_last, tables = 0.0, float(K), []
    lay_b, lay_c, CPB = oracle.layout(bucket, bucket), oracle.layout(4096, 4096), bucket // 4096
    rng = np.random.default_rng(1)
    for t in range(T):
        V0 = dual_vectors(X, 2 * t)
        if t % 10 == 0:
            ctx.fit_levels(V0, n_sym, 4096, sweeps=8)
            tables.append(ctx.get_levels())
            assert (np.diff(tables[-1]) > 0).all() and tables[-1][0] == 0 and tables[-1][-1] == 1
        ctx.quantize_encode(V0, 2 * t, prev)
        if t == 10:                                  # sampled buckets of the stream, bit for bit
            levels = tables[-1]
            h = prev.to_host()
            for k, b in [(0, 0), (K - 1, ctx.NB - 1), (int(rng.integers(K)), int(rng.integers(ctx.NB)))]:
                print("bucket", k, b, flush=True)
                vb = V0[k, b * bucket:(b + 1) * bucket].cpu().numpy()[None, :]
                n_o, _, _, _ = oracle.quantize(vb, lay_b, oracle.NORM_L2, levels, seed, 2 * t, k0=k, i0=b * bucket)
                assert abs(h["norms"][k, b] - n_o[0, 0]) <= REL * n_o[0, 0]
                _, idx, neg, _ = oracle.quantize(vb, lay_b, oracle.NORM_L2, levels, seed, 2 * t,
                                                 norms_in=h["norms"][k:k + 1, b:b + 1], k0=k, i0=b * bucket)
                so = oracle.encode(idx, neg, lay_b, cap_words=bucket)
                ms = mini_stream(h, k, b * CPB, (b + 1) * CPB)
                np.testing.assert_array_equal(ms.sub_end, so.sub_end)
                np.testing.assert_array_equal(ms.payload[0], so.payload[0, :ms.payload.shape[1]])
        ctx.eg_step(0, prev, None, Xh)
        V1 = dual_vectors(Xh, 2 * t + 1)
        ctx.quantize_encode(V1, 2 * t + 1, cur)
        if t == 10:
            Y_before, _ = ctx.state_export()
        ctx.eg_step(1, cur, prev, Xn)
        if t == 10:                                  # a sampled chunk of the second half-step
            Y_after, _ = ctx.state_export()
            hc = cur.to_host()
            c = int(rng.integers(ctx.NC))
            print("chunk", c, flush=True)
            dec_c, dec_p = [], []
            for k in range(K):
                nb = slice(c // CPB, c // CPB + 1)
                dec_c.append(oracle.decode(mini_stream(hc, k, c, c + 1), hc["norms"][k:k + 1, nb], lay_c, levels)[0][0])
                dec_p.append(oracle.decode(mini_stream(h, k, c, c + 1), h["norms"][k:k + 1, nb], lay_c, levels)[0][0])
            sl = slice(c * 4096, (c + 1) * 4096)
            want = Y_before[sl].cpu().numpy().astype(np.float64) - np.mean(np.stack(dec_c), axis=0)
            got = Y_after[sl].cpu().numpy()
            assert np.linalg.norm(got - want) <= REL * np.linalg.norm(want)
            del Y_before, Y_after
        sc = ctx.scalars()
        assert sc["S"] > S_last and sc["gamma"] < gamma_last and sc["t"] == t + 2
        assert abs(sc["gamma"] - K / np.sqrt(1.0 + sc["S"])) <= 1e-12 * sc["gamma"]
        S_last, gamma_last = sc["S"], sc["gamma"]
        X, Xn = Xn, X
    assert ctx.poll_error() == 0
    assert len(tables) == 5 and all(np.abs(tables[i] - tables[0]).max() > 0 for i in range(1, 5))
    res = float(torch.linalg.vector_norm(operator(X).double()))
    print("residual |F(X)|: %.6e at X_1, %.6e after %d iterations; gamma_T = %.3e" % (res0, res, T, gamma_last), flush=True)
    # the drift of the iterates is along -b and lowers |F| by about gamma_T T mu (the noise is orthogonal to it to first order)
    assert np.isfinite(res) and res < res0
    ctx.close()


def test_longest_vector():
    """The largest d the boundary takes (2^31 - 4 coordinates, here with K = 1, buckets of 65536, the last
    one short and ending in a chunk of 4092): coordinate indices, Philox counters and byte offsets near the
    top of their ranges.  Sampled buckets of the stream (the first, one in the middle, the last two) and the
    chunks of the first half-step under them are recomputed by the oracle; sizes and totals over the whole."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2308_09187_amd import qgx
    qgx.load()
    K, d, bucket, seed, call = 1, (1 << 31) - 4, 65536, 99, 3
    V = torch.empty(K, d, device="cuda")
    V.normal_(0.0, 1e-3, generator=torch.Generator(device="cuda").manual_seed(5))
    levels = synth.levels_exponential(16)
    ctx = qgx.Context(d, K, bucket, norm=qgx.NORM_L2, seed=seed)
    ctx.set_levels(levels)
    NB, NC, CPB = ctx.NB, ctx.NC, bucket // 4096
    assert NB == 32768 and NC == 524288
    x1 = torch.empty(d, device="cuda")
    x1.normal_(0.0, 1.0, generator=torch.Generator(device="cuda").manual_seed(6))
    ctx.state_init(x1)
    a = ctx.new_stream(slotted=True)
    Xh = torch.empty(d, device="cuda")
    print("encode + half-step", flush=True)
    ctx.quantize_encode(V, call, a)
    ctx.eg_step(0, a, None, Xh)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    h = a.to_host()
    bits = h["sub_end"][:, :, -1].astype(np.int64)
    assert ctx.stream_bits(a) == int(bits.sum())
    assert (np.diff(h["chunk_off"].astype(np.int64), axis=1) == ctx.slot_words()).all()
    assert np.isfinite(h["norms"]).all() and (h["norms"] > 0).all()
    lay_c = oracle.layout(4096, 4096)
    for b in [0, NB // 2 + 1, NB - 2, NB - 1]:
        print("bucket", b, flush=True)
        lo, hi = b * bucket, min((b + 1) * bucket, d)
        vb = V[0, lo:hi].cpu().numpy()[None, :]
        lay_b = oracle.layout(hi - lo, bucket)
        n_o, _, _, _ = oracle.quantize(vb, lay_b, oracle.NORM_L2, levels, seed, call, k0=0, i0=lo)
        assert abs(h["norms"][0, b] - n_o[0, 0]) <= REL * n_o[0, 0]
        _, idx, neg, _ = oracle.quantize(vb, lay_b, oracle.NORM_L2, levels, seed, call,
                                         norms_in=h["norms"][0:1, b:b + 1], k0=0, i0=lo)
        so = oracle.encode(idx, neg, lay_b, cap_words=bucket)
        ms = mini_stream(h, 0, b * CPB, b * CPB + lay_b.NC)
        np.testing.assert_array_equal(ms.sub_end, so.sub_end)
        np.testing.assert_array_equal(ms.payload[0], so.payload[0, :ms.payload.shape[1]])
        Vhat, _, _ = oracle.decode(so, h["norms"][0:1, b:b + 1], lay_b, levels)
        st = oracle.EGState(hi - lo, K, X1=x1[lo:hi].cpu().numpy())
        want = st.half0(Vhat)
        got = Xh[lo:hi].cpu().numpy()
        assert np.linalg.norm(got - want) <= REL * np.linalg.norm(want)
    ctx.close()
