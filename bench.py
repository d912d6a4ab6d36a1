#!/usr/bin/env python3
"""Benchmark of the Q-GenX hot path on one MI355X.

A step is one pass of the path over one batch of K synthetic dual vectors already resident in HBM:
CODE o Q of all K vectors (fused quantise + encode), then the fused decode + average + first
extra-gradient half-step.  The level table is fitted once from a histogram of the same batch before
timing (it is refitted only at the update steps of Algorithm 1).  Default workload: K = 8 vectors of
d = 2^24 Student-t(3) * 1e-2 coordinates, buckets of 16384, L2 norm, 33-symbol fitted table.

Before the W warm-up steps the same step runs untimed for --preroll-ms (default 150 ms): the steps
take a fraction of a millisecond, and a few of them are over before the GPU has left its idle clocks.

Prints one JSON line: whole-job GB/s of fp32 dual vectors, the roofline of the dominant kernel
(the encoder) from event timings on the launch stream, and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--preroll-ms", type=float, default=150.0,
                    help="untimed steps run for this long before the warm-up, so that the GPU has left its idle "
                         "clocks (a handful of sub-millisecond steps is over before they have risen)")
    ap.add_argument("--logd", type=int, default=24, help="log2 of coordinates per worker")
    ap.add_argument("--K", type=int, default=8)
    ap.add_argument("--bucket", type=int, default=16384)
    ap.add_argument("--n-sym", type=int, default=33)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-logd", type=int, default=24, help="log2 of coordinates per worker in the oracle sample")
    ap.add_argument("--full-iteration", action="store_true", help="also time encode + second half-step")
    ap.add_argument("--rotate", action="store_true",
                    help="alternate between two input batches and two stream buffers from step to step")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain device copy of the input (known size) to calibrate rocprofv3 HBM counters")
    ap.add_argument("--workload", choices=["t3", "gan", "game"], default="t3",
                    help="t3: the headline batch of heavy-tailed vectors; gan: K vectors in a GAN-shaped layout of 14 "
                         "tensors with per-tensor scale, buckets of 8192 per tensor, L-infinity norm, 16 exponential "
                         "levels, full iteration (ignores --logd, --bucket, --n-sym); game: the large quadratic game, "
                         "K = 16 workers, z in R^(2^26), buckets of 65536, 65 levels, whole iterations on the device with "
                         "the dual vectors formed inside the coding kernel and, for comparison, written out and coded from memory")
    ap.add_argument("--code", choices=["omega", "huffman", "fixed"], default="omega",
                    help="Psi: Elias' recursive code of the level index (default), the optimal prefix code "
                         "fitted to the estimated symbol probabilities, or words of one width (with uniform levels: "
                         "the fixed-width setting of the paper's experiment, e.g. --workload gan --bucket 1024 "
                         "--n-sym 8 --code fixed for 3 bits + sign)")
    ap.add_argument("--graph", action="store_true",
                    help="with --full-iteration: also capture the iteration as one HIP graph and time its replays "
                         "(reported as an extra object; matters for small vectors, where launches dominate)")
    ap.add_argument("--no-huffman", action="store_true",
                    help="skip the second leg of the default run (the same step with Psi fitted to the symbol probabilities)")
    ap.add_argument("--placement", choices=["slotted", "compact"], default="slotted",
                    help="chunk placement of the coded streams handed from the encoder to the update kernel")
    return ap.parse_args()


def _profile_number(key):
    """A figure from the committed rocprofv3 counter summary of the encoder, if there is one."""
    path = os.path.join(ROOT, "profiles", "encode_t3_K8_d2p24_pmc.txt")
    try:
        m = re.search(r"^%s:\s*([0-9.eE+]+)" % key, open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def measured_traffic():
    """HBM bytes per encoder launch (FETCH_SIZE + WRITE_SIZE, calibrated against a plain copy)."""
    return _profile_number("traffic_bytes_per_launch")


def cpu_baseline(args, levels, seed, V, code=(None, None)):
    """The oracle as it stands on a bounded sample of the same workload: CODE o Q, DEQ, mean, half-step."""
    import numpy as np

    import oracle
    K, d = V.shape
    lay = oracle.layout(d, args.bucket)
    st = oracle.EGState(d, K)
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    t0 = time.perf_counter()
    norms, idx, neg, _ = oracle.quantize(V, lay, oracle.NORM_L2, levels, seed, 0)
    s = oracle.encode(idx, neg, lay, cap_words=d // 2, code_len=code[0], code_bits=code[1])
    Vhat, _, _ = oracle.decode(s, norms, lay, levels, code_len=code[0], code_bits=code[1])
    st.half0(Vhat)
    dt = time.perf_counter() - t0
    out = {"value": 4.0 * K * d / dt / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
           "sample": "first 2^%d coordinates of each of the %d workers, one pass quantise+encode+decode+half-step, %.2f s"
                     % (args.cpu_sample_logd, K, dt)}
    # the same on one thread, on an eighth of the sample (the oracle's loops are OpenMP over workers and buckets)
    try:
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        d1 = max(d // 8, args.bucket)
        lay1 = oracle.layout(d1, args.bucket)
        V1 = np.ascontiguousarray(V[:, :d1])
        gomp.omp_set_num_threads(1)
        t0 = time.perf_counter()
        norms, idx, neg, _ = oracle.quantize(V1, lay1, oracle.NORM_L2, levels, seed, 0)
        s = oracle.encode(idx, neg, lay1, cap_words=d1 // 2, code_len=code[0], code_bits=code[1])
        Vhat, _, _ = oracle.decode(s, norms, lay1, levels, code_len=code[0], code_bits=code[1])
        oracle.EGState(d1, K).half0(Vhat)
        dt1 = time.perf_counter() - t0
        gomp.omp_set_num_threads(threads)
        out["single_thread"] = {"value": 4.0 * K * d1 / dt1 / 1e9, "unit": "GB/s",
                                "sample": "first %d coordinates of each worker, %.2f s" % (d1, dt1)}
    except OSError:
        pass
    return out


def fitted_code_leg(args, V, seed, Xh):
    """The default step once more with the paper's other choice of Psi (Appendix J: Huffman coding once the
    symbol probabilities can be estimated, which a fitted level table implies): the optimal prefix code on the
    p_j of Proposition 1.  Fewer bytes move (about 4.5 instead of 11.9 bits per coordinate) in nearly the same
    time, so the fraction of the HBM peak is lower: it is on record beside the headline."""
    import numpy as np
    import torch

    from paper_2308_09187_amd import qgx, synth
    K, d = V.shape
    ctx = qgx.Context(d, K, args.bucket, norm=qgx.NORM_L2, seed=seed, code=qgx.CODE_TABLE)
    ctx.set_levels(synth.levels_exponential(args.n_sym - 1))
    ctx.fit_levels(V, args.n_sym, 4096, sweeps=10)
    ctx.fit_code()
    ctx.state_init(None)
    a = ctx.new_stream(slotted=True)
    for i in range(args.warmup):
        ctx.quantize_encode(V, 2 * i, a); ctx.eg_step(0, a, None, Xh)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    for i in range(args.steps):
        ev[i][0].record(); ctx.quantize_encode(V, 2 * i, a)
        ev[i][1].record(); ctx.eg_step(0, a, None, Xh)
        ev[i][2].record()
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    enc_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    upd_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
    h_bits = a.sub_end.cpu().numpy().view(np.uint16)[:, :, -1].astype(np.int64)
    words = int((((h_bits + 31) // 32 + 3) // 4 * 4).sum())
    stream_bytes = words * 4 + K * ((ctx.NC + 1) * 4 + ctx.NC * qgx.SUBS * 2 + ctx.NB * 4)
    enc_bytes, upd_bytes = 4 * K * d + stream_bytes, stream_bytes + 8 * d
    bits = ctx.stream_bits(a)
    ctx.close()
    return {"config": {"workload": "the same batch and level table, Psi = optimal prefix code fitted to the symbol probabilities",
                       "bits_per_coordinate": bits / float(K * d), "stream_bytes": stream_bytes},
            "value": 4.0 * K * d / ((enc_ms + upd_ms) * 1e-3) / 1e9, "unit": "GB/s",
            "kernels_ms": {"encode": enc_ms, "decode_avg_half0": upd_ms},
            "hbm_frac_step": (enc_bytes + upd_bytes) / ((enc_ms + upd_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "roofline": {"kernel": "k_encode<Fused, false, 4>", "bound": "hbm", "achieved": enc_bytes / (enc_ms * 1e-3) / 1e9,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": enc_bytes / (enc_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "traffic": None, "algorithmic_bytes": enc_bytes}}


def game_bench(args):
    """Whole iterations of eq. (Q-GenX) on the large strongly monotone quadratic game with nothing but scalars
    leaving the device: per iteration two rounds of (K dual vectors at the current point -> CODE o Q -> fused
    half-step).  Timed twice: with the dual vectors formed inside the coding kernel (qgx_quantize_encode_game),
    and with them written to memory by qgx_game_dual_vectors and coded from there (generator included)."""
    import numpy as np
    import torch

    from paper_2308_09187_amd import qgx, synth
    qgx.load()
    torch.cuda.set_device(0)
    K = 16 if args.K == 8 else args.K
    logd = 26 if args.logd == 24 else args.logd
    bucket = 65536 if args.bucket == 16384 else args.bucket
    n_sym = 65 if args.n_sym == 33 else args.n_sym
    d, seed = 1 << logd, 2308
    game = synth.QuadraticGame(d, K)
    a_d, b_d = torch.from_numpy(game.a).cuda(), torch.from_numpy(game.b).cuda()
    ctx = qgx.Context(d, K, bucket, norm=qgx.NORM_L2, seed=seed)
    ctx.set_levels(synth.levels_exponential(n_sym - 1))
    X = torch.zeros(d, device="cuda")
    Xh, Xn = torch.empty(d, device="cuda"), torch.empty(d, device="cuda")
    V = torch.empty((K, d), device="cuda")
    ctx.game_dual_vectors(X, a_d, b_d, game.mu, game.noise, 42, 0, out=V)
    ctx.fit_levels(V, n_sym, 4096, sweeps=8)
    sa, sb = ctx.new_stream(slotted=True), ctx.new_stream(slotted=True)
    names = ["generate", "encode", "decode_avg_half0", "generate_2", "encode_2", "decode_avg_half1"]

    def iteration(fused, ev=None):
        nonlocal X, Xn
        def mark(j):
            if ev: ev[j].record()
        mark(0)
        if not fused: ctx.game_dual_vectors(X, a_d, b_d, game.mu, game.noise, 42, qgx.CALL_FIRST_HALF, out=V)
        mark(1)
        if fused: ctx.quantize_encode_game(X, a_d, b_d, game.mu, game.noise, 42, qgx.CALL_FIRST_HALF, sa)
        else: ctx.quantize_encode(V, qgx.CALL_FIRST_HALF, sa)
        mark(2)
        ctx.eg_step(0, sa, None, Xh)
        mark(3)
        if not fused: ctx.game_dual_vectors(Xh, a_d, b_d, game.mu, game.noise, 42, qgx.CALL_SECOND_HALF, out=V)
        mark(4)
        if fused: ctx.quantize_encode_game(Xh, a_d, b_d, game.mu, game.noise, 42, qgx.CALL_SECOND_HALF, sb)
        else: ctx.quantize_encode(V, qgx.CALL_SECOND_HALF, sb)
        mark(5)
        ctx.eg_step(1, sb, sa, Xn)
        mark(6)
        X, Xn = Xn, X

    def timed(fused):
        nonlocal X
        X.zero_()
        ctx.state_init(None)
        for _ in range(args.warmup):
            iteration(fused)
        torch.cuda.synchronize()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
        t0 = time.perf_counter()
        for i in range(args.steps):
            iteration(fused, events[i])
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / args.steps
        assert ctx.poll_error() == 0
        per = {n: float(np.mean([e[j].elapsed_time(e[j + 1]) for e in events])) for j, n in enumerate(names)}
        return wall, per

    wall_f, per_f = timed(True)
    wall_m, per_m = timed(False)
    res = ctx.norm2(ctx.game_operator(X, a_d, b_d, game.mu))
    bits = ctx.stream_bits(sa)
    h_bits = sa.sub_end.cpu().numpy().view(np.uint16)[:, :, -1].astype(np.int64)
    stream_bytes = int((((h_bits + 31) // 32 + 3) // 4 * 4).sum()) * 4 + K * ((ctx.NC + 1) * 4 + ctx.NC * qgx.SUBS * 2 + ctx.NB * 4)
    # The coding kernel that forms its own input is bound by vector-ALU issue, not by memory (it reads z, a and b
    # once, 10 bytes per coordinate, and writes the streams: 13 % of the memory roof).  Its row loop holds 256
    # vector instructions per four coordinates in the compiled kernel (140 of the plain coding kernel, of which
    # Philox4x32-10 is 56, plus a second Philox block, two Box-Muller pairs and the operator): 64 per coordinate.
    # Roof: one vector instruction per SIMD every four clocks, 256 CUs x 4 SIMDs x 64 lanes x 2.4 GHz / 4.
    VALU_PER_COORD, ALU_PEAK = 64.0, 256 * 4 * 64 * 2.4e9 / 4 / 1e12
    alu_rate = VALU_PER_COORD * K * d / (per_f["encode"] * 1e-3) / 1e12
    enc_bytes_f = d * 10 + stream_bytes
    gap = ctx.game_gap(X, a_d, b_d, game.mu, torch.from_numpy(game.solution().astype(np.float32)).cuda(), 1.0)
    out = {
        "metric": "GB/s of fp32 dual vectors through quantize->encode->decode->avg->EG step; % HBM peak",
        "value": 2 * 4.0 * K * d / wall_f / 1e9, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_f * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "large quadratic game, K=%d x d=2^%d, F(z) = Mz + b with 2x2 blocks, N(0, %.2f^2) noise, bucket %d, L2, "
                               "%d-symbol fitted table, Elias-omega, slotted; step = one whole iteration on the device, dual vectors "
                               "formed inside the coding kernel" % (K, logd, game.noise, bucket, n_sym),
                   "K": K, "d": d, "bucket": bucket, "n_sym": n_sym, "bits_per_coordinate": bits / float(K * d), "stream_bytes": stream_bytes},
        "kernels_ms": per_f,
        "materialised": {"what": "the same iterations with the dual vectors written to memory by qgx_game_dual_vectors and coded from there",
                         "ms_per_step": wall_m * 1e3, "value": 2 * 4.0 * K * d / wall_m / 1e9, "unit": "GB/s", "kernels_ms": per_m},
        "roofline": {"kernel": "k_encode<Generate, false, %d>" % (4 if n_sym <= 33 else 5 if n_sym <= 65 else 6), "bound": "alu",
                     "achieved": alu_rate, "peak": ALU_PEAK, "unit": "T lane-instructions/s", "frac": alu_rate / ALU_PEAK, "traffic": None,
                     "valu_instructions_per_coordinate": VALU_PER_COORD, "algorithmic_bytes": enc_bytes_f,
                     "hbm_frac": enc_bytes_f / (per_f["encode"] * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "residual_norm_at_the_last_iterate": res,
        "restricted_gap_at_the_last_iterate_unit_ball_around_the_solution": gap,
    }
    ctx.close()
    print(json.dumps(out))


def main():
    args = parse_args()
    if args.gpus == 1 and args.workload == "game":
        return game_bench(args)
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the K workers are a batch on it); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_2308_09187_amd import qgx, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    qgx.load()
    torch.cuda.set_device(0)
    K, seed = args.K, 2308
    huffman, fixed = args.code == "huffman", args.code == "fixed"
    code_kind = qgx.CODE_TABLE if (huffman or fixed) else qgx.CODE_ELIAS_OMEGA
    if args.workload == "gan":
        args.full_iteration = True
        if not fixed:
            args.n_sym = 17
        if args.bucket == 16384:                                   # the option's default: this workload's own
            args.bucket = 8192
        seg = [int(x) for x in synth.GAN_SEGMENTS]
        d = sum(seg)
        V = torch.from_numpy(synth.gan_dual_vectors(K, 0)).cuda()
        V1 = torch.from_numpy(synth.gan_dual_vectors(K, 1)).cuda()
        ctx = qgx.Context(d, K, args.bucket, norm=qgx.NORM_LINF, seed=seed, code=code_kind, segment_len=seg)
        ctx.set_levels(synth.levels_uniform(args.n_sym - 1) if fixed else synth.levels_exponential(16))
        if huffman:
            ctx.fit_levels(V, args.n_sym, 4096, sweeps=0)          # only measures: the table stays
        what = "K=%d x d=%d in 14 tensors (GAN-shaped), N(0, sigma_t^2) with sigma_t log-uniform in [1e-5, 1e-2], " \
               "buckets of %d per tensor, L-infinity, %s levels" % (K, d, args.bucket, "%d uniform" % (args.n_sym - 1) if fixed
                                                                    else "16 exponential")
    else:
        d = 1 << args.logd
        V = synth.student_t3_device(K, d, seed=20)
        V1 = synth.student_t3_device(K, d, seed=21) if args.full_iteration else None
        Vr = synth.student_t3_device(K, d, seed=21) if args.rotate and not args.full_iteration else None
        ctx = qgx.Context(d, K, args.bucket, norm=qgx.NORM_L2, seed=seed, code=code_kind)
        if fixed:
            ctx.set_levels(synth.levels_uniform(args.n_sym - 1))
            what = "K=%d x d=2^%d Student-t(3)*1e-2, bucket %d, L2, %d uniform levels" % (K, args.logd, args.bucket, args.n_sym - 1)
        else:
            ctx.set_levels(synth.levels_exponential(args.n_sym - 1))
            ctx.fit_levels(V, args.n_sym, 4096, sweeps=10)
            # what an update step of Algorithm 1 adds to its iteration (the fit is not part of the timed step):
            # histogram, reduction, 10 sweeps from the table just fitted and the rebuild of the device tables
            fitted = ctx.get_levels()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                ctx.fit_levels(V, args.n_sym, 4096, sweeps=10)
            torch.cuda.synchronize()
            level_fit_ms = (time.perf_counter() - t0) * 1e3 / 5
            ctx.set_levels(fitted)                                 # the workload's table is the one of the first fit
            what = "K=%d x d=2^%d Student-t(3)*1e-2, bucket %d, L2, %d-symbol fitted table" % (K, args.logd, args.bucket, args.n_sym)
    if "level_fit_ms" not in locals():
        level_fit_ms = None
    default_workload = (args.workload, args.logd, K, args.bucket, args.n_sym, args.code, args.placement) == \
                       ("t3", 24, 8, 16384, 33, "omega", "slotted")
    levels = ctx.get_levels()
    if fixed:                                                      # words of ceil(log2 n_sym) bits, symbol j as the number j
        width = max(1, (args.n_sym - 1).bit_length())
        code = (np.full(args.n_sym, width, np.uint8), np.arange(args.n_sym, dtype=np.uint32))
        ctx.set_code_table(*code)
    else:
        code = ctx.fit_code()[1:] if huffman else (None, None)
    ctx.state_init(None)
    slotted = args.placement == "slotted"
    a, b = ctx.new_stream(slotted=slotted), ctx.new_stream(slotted=slotted)
    Xh = torch.empty(d, dtype=torch.float32, device="cuda")

    def step(i, ev=None):
        if args.rotate and not args.full_iteration:
            Vi, si = ((V, a), (Vr, b))[i & 1]
            if ev: ev[0].record()
            ctx.quantize_encode(Vi, 2 * i, si)
            if ev: ev[1].record()
            ctx.eg_step(0, si, None, Xh)
            if ev: ev[2].record()
            return
        if ev: ev[0].record()
        ctx.quantize_encode(V, 2 * i, a)
        if ev: ev[1].record()
        ctx.eg_step(0, a, None, Xh)
        if ev: ev[2].record()
        if args.full_iteration:
            ctx.quantize_encode(V1, 2 * i + 1, b)
            if ev: ev[3].record()
            ctx.eg_step(1, b, a, None)
            if ev: ev[4].record()

    if args.copy_probe:
        probe = V.clone()          # plain copy kernel: reads and writes 4*K*d bytes
        torch.cuda.synchronize()
        del probe

    def copy_bandwidth():
        """What a plain device-to-device pass over the input reaches on this machine (read + written bytes per
        second): the practical ceiling next to the published HBM peak.  Two of torch's kernels are timed, the
        copy and an elementwise one (one float4 per thread, which streams faster here); the better one counts."""
        dst = torch.empty_like(V)
        best = {}
        for kind, fn in (("copy", lambda: dst.copy_(V)), ("elementwise", lambda: torch.neg(V, out=dst))):
            for _ in range(30):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                fn()
            e1.record()
            torch.cuda.synchronize()
            best[kind] = 2.0 * V.numel() * 4 * 20 / (e0.elapsed_time(e1) * 1e-3) / 1e9
        return best
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.preroll_ms:
        for i in range(8):
            step(i)
        torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    n_ev = 5 if args.full_iteration else 3
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i, events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert ctx.poll_error() == 0

    # The same two kernels with the half-step reading a stream that is NOT fresh in the 256 MB infinity cache:
    # the encoder fills one of two stream buffers while the half-step decodes the other, coded one step (and
    # about 1 GB of traffic) earlier.  On one GPU the default loop's flow (decode what was just coded) is the
    # method's own; over a network the streams arrive from elsewhere, which is what this loop stands for.
    cold = None
    if not args.full_iteration and not args.rotate:
        b_cold = ctx.new_stream(slotted=slotted)
        ctx.quantize_encode(V, 1, b_cold)
        bufs = (a, b_cold)
        ev_c = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
        for i in range(args.warmup + args.steps):
            e = ev_c[i - args.warmup] if i >= args.warmup else None
            if e: e[0].record()
            ctx.quantize_encode(V, 2 * i, bufs[i & 1])
            if e: e[1].record()
            ctx.eg_step(0, bufs[(i + 1) & 1], None, Xh)
            if e: e[2].record()
        torch.cuda.synchronize()
        assert ctx.poll_error() == 0
        cold = (float(np.mean([e[0].elapsed_time(e[1]) for e in ev_c])), float(np.mean([e[1].elapsed_time(e[2]) for e in ev_c])))
        del b_cold

    graph_ms = None
    if args.graph and args.full_iteration:
        # every kernel of the iteration takes what changes from device memory, the call numbers included
        def iteration():
            ctx.quantize_encode(V, qgx.CALL_FIRST_HALF, a)
            ctx.eg_step(0, a, None, Xh)
            ctx.quantize_encode(V1, qgx.CALL_SECOND_HALF, b)
            ctx.eg_step(1, b, a, None)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            iteration()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        assert ctx.poll_error() == 0

    copy_gbs = copy_bandwidth()
    ms_step = wall * 1e3 / args.steps
    enc_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in events]))
    upd_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in events]))
    h_bits = a.sub_end.cpu().numpy().view(np.uint16)[:, :, -1].astype(np.int64)
    words = int((((h_bits + 31) // 32 + 3) // 4 * 4).sum())
    bits = ctx.stream_bits(a)
    side_bytes = K * ((ctx.NC + 1) * 4 + ctx.NC * qgx.SUBS * 2 + ctx.NB * 4)
    stream_bytes = words * 4 + side_bytes
    enc_bytes = 4 * K * d + stream_bytes                 # read V once, write the coded streams
    upd_bytes = stream_bytes + 4 * d + 4 * d             # read streams and Y, write X_{t+1/2}
    passes = 2 if args.full_iteration else 1
    value = 4.0 * K * d * passes / (wall / args.steps) / 1e9
    achieved = enc_bytes / (enc_ms * 1e-3) / 1e9

    out = {
        "metric": "GB/s of fp32 dual vectors through quantize->encode->decode->avg->EG step; % HBM peak",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "preroll_ms": args.preroll_ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s, %s; %s chunk placement; step = fused CODE.Q + fused decode/average/half-step%s"
                               % (what, "fitted optimal prefix code" if huffman else "fixed-width code" if fixed else "Elias-omega", args.placement,
                                  " + CODE.Q + second half-step" if args.full_iteration else ""),
                   "K": K, "d": d, "bucket": args.bucket, "n_sym": args.n_sym,
                   "bits_per_coordinate": bits / float(K * d), "stream_bytes": stream_bytes},
        "hbm_frac_step": (enc_bytes + upd_bytes) / ((enc_ms + upd_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "kernels_ms": {"encode": enc_ms, "decode_avg_half0": upd_ms},
        "level_fit_ms": level_fit_ms,      # per update step of Algorithm 1, outside the timed step (histogram, reduction, 10 sweeps, tables)
        "roofline": {"kernel": "k_encode<Fused, %s, %d>" % ("true" if args.bucket in (256, 512, 1024, 2048) else "false",
                                                            4 if args.n_sym <= 33 else 5 if args.n_sym <= 65 else 6),
                     "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     # HBM bytes per launch from the committed rocprofv3 counter run of this command (FETCH_SIZE and
                     # WRITE_SIZE, calibrated on a plain copy), not measured in this run; default workload only
                     "traffic": measured_traffic() if default_workload else None,
                     "traffic_source": "profiles/encode_t3_K8_d2p24_pmc.txt" if default_workload else None,
                     "algorithmic_bytes": enc_bytes,
                     # a plain copy of the same input on this machine, and the encoder's rate relative to it
                     "copy_gbs": max(copy_gbs.values()), "copy_gbs_by_kernel": copy_gbs,
                     "frac_of_copy": achieved / max(copy_gbs.values()),
                     # upper bound on the vector-ALU time of a launch from the counter run: instructions issued
                     # per SIMD x 4 clocks (simple instructions take fewer: the ALUs are the second ceiling)
                     # (from the same committed counter run)
                     "valu_busy_us": _profile_number("valu_busy_us") if default_workload else None},
    }
    if cold is not None:
        out["kernels_ms_cold_stream"] = {"encode": cold[0], "decode_avg_half0": cold[1],
                                         "what": "the half-step decodes a stream coded one step earlier (not fresh in the infinity cache)"}
        out["hbm_frac_step_cold_stream"] = (enc_bytes + upd_bytes) / ((cold[0] + cold[1]) * 1e-3) / 1e9 / HBM_PEAK_GBS
    if out["roofline"]["valu_busy_us"]:
        # the same bound as a share of this run's launch time: near 1 means the ALUs, not HBM, are the nearer ceiling
        out["roofline"]["valu_busy_frac"] = out["roofline"]["valu_busy_us"] / (enc_ms * 1e3)
    if graph_ms is not None:
        out["graph"] = {"ms_per_step": graph_ms, "value": 4.0 * K * d * passes / (graph_ms * 1e-3) / 1e9, "unit": "GB/s",
                        "what": "the same iteration captured once as a HIP graph and replayed"}
    names = ["encode", "decode_avg_half0", "encode_2", "decode_avg_half1"][:n_ev - 1]
    per_step = {n: np.array([e[j].elapsed_time(e[j + 1]) for e in events]) for j, n in enumerate(names)}
    if args.full_iteration:
        out["kernels_ms"]["encode_2"] = float(per_step["encode_2"].mean())
        out["kernels_ms"]["decode_avg_half1"] = float(per_step["decode_avg_half1"].mean())
    out["kernels_ms_median"] = {n: float(np.median(v)) for n, v in per_step.items()}
    out["kernels_ms_min"] = {n: float(v.min()) for n, v in per_step.items()}
    ctx.close()
    if default_workload and not args.full_iteration and not args.no_huffman:
        out["fitted_code"] = fitted_code_leg(args, V, seed, Xh)
    if not args.no_cpu_baseline and args.workload == "t3":
        ds = min(d, 1 << args.cpu_sample_logd)
        args.cpu_sample_logd = ds.bit_length() - 1
        V_host = V[:, :ds].contiguous().cpu().numpy()
        del V, V1, a, b
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(args, levels, seed, V_host, code)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
