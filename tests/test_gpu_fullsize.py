"""Parity at full size and in the benchmark's launch configurations: the headline workload (K = 8
vectors of d = 2^24 coordinates, buckets of 16384, L2, 33-symbol fitted table; slotted chunk placement
as timed, and compact) and the shape of the large quadratic game (K = 16 vectors of d = 2^26, buckets of
65536, 65 fitted levels).  Properties that hold at any size are checked over the whole output; sampled
buckets and chunks are recomputed one by one by the oracle."""
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
    assert ctx.scalars(want_bits=True)["total_bits"] == int(bits.sum())
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
