"""qgx_eg_step_static, the variant of qgx_eg_step whose scratch (the per-chunk partial sums of the
step-size accumulator) lives in a fixed array of the library's device image: two iterations in a row
through the C ABI, the second on a smaller problem, each against qgx_eg_step on a twin context: same
kernels, so every output must agree bit for bit."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2308_09187_amd import synth

pytestmark = pytest.mark.gpu


def _iteration(qgx, d, K, bucket, segs, static, prev_stream=True):
    seg_arr = None if segs is None else np.array(segs, np.uint64)
    ctx = qgx.Context(d, K, bucket, norm=qgx.NORM_L2, seed=77, segment_len=seg_arr)
    ctx.set_levels(synth.levels_exponential(16))
    V0 = torch.from_numpy(synth.student_t3(K, d, seed=5)).cuda()
    V1 = torch.from_numpy(synth.student_t3(K, d, seed=6)).cuda()
    ctx.state_init(torch.from_numpy(synth.gaussian_vector(d, seed=3)).cuda())
    a, b = ctx.new_stream(), ctx.new_stream(slotted=False)
    Xh = torch.empty(d, device="cuda"); Xn = torch.empty(d, device="cuda")
    out = []
    for t in range(2):                                   # two iterations: S carries over
        ctx.quantize_encode(V0, 2 * t, a)
        ctx.eg_step(0, a, None, Xh, static=static)
        ctx.quantize_encode(V1, 2 * t + 1, b)
        ctx.eg_step(1, b, a if prev_stream else None, Xn, static=static)
        sc = ctx.scalars()
        Y, _ = ctx.state_export()
        out.append((Xh.cpu().numpy().copy(), Xn.cpu().numpy().copy(), Y.cpu().numpy().copy(), sc["S"], sc["gamma"], sc["t"]))
    assert ctx.poll_error() == 0
    ctx.close()
    return out


def test_static_scratch_variant_matches_the_allocating_one():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2308_09187_amd import qgx
    qgx.load()
    # the first layout has full and ragged chunk positions (one launch for both) and many chunks; the second is smaller,
    # so the static array still holds the first call's partial sums beyond the entries the second one uses
    cases = [((1 << 17) + 4096 + 520, 5, 8192, [1 << 16, 4096 + 520, 1 << 16], True),
             (3 * 4096 + 300, 3, 4096, None, True),
             (2 * 4096, 2, 4096, None, False)]           # dual-averaging form: no previous streams
    for d, K, bucket, segs, prev in cases:
        want = _iteration(qgx, d, K, bucket, segs, static=False, prev_stream=prev)
        got = _iteration(qgx, d, K, bucket, segs, static=True, prev_stream=prev)
        for w, g in zip(want, got):
            for x, y in zip(w[:3], g[:3]):
                np.testing.assert_array_equal(x, y)
            assert w[3:] == g[3:] and w[3] > 0


def test_static_scratch_variant_rejects_layouts_beyond_its_array():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2308_09187_amd import qgx
    qgx.load()
    d = (qgx.STATIC_MAX_CHUNKS + 1) * 64                 # buckets of 64: a chunk per bucket
    ctx = qgx.Context(d, 1, 64, norm=qgx.NORM_LINF, seed=1)
    assert ctx.NC == qgx.STATIC_MAX_CHUNKS + 1
    ctx.set_levels(synth.levels_uniform(4))
    ctx.state_init(None)
    a = ctx.new_stream()
    with pytest.raises(qgx.QgxError) as e:
        ctx.eg_step(1, a, None, None, static=True)
    assert e.value.status == qgx.ERR_CAPACITY and "65536" in str(e.value)
    ctx.close()
