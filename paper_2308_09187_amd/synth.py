"""Seeded synthetic inputs: dual vectors, operators and level tables.

This module serves both the HIP library's tests/benchmark and the CPU oracle's
tests.  It holds none of the method's arithmetic (no norms, no rounding, no
coding, no updates) and imports neither of them.

Host generators use numpy's PCG64 keyed by a tuple of integers; the two large
workloads can also be drawn on the device with torch's seeded generator.
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------
# Level tables l = (0 = l_0 < l_1 < ... < l_last = 1), Definition 1.
# `s` counts the non-zero symbols, so a table has s + 1 entries.
# ---------------------------------------------------------------------------


def levels_uniform(s: int) -> np.ndarray:
    return (np.arange(s + 1, dtype=np.float64) / s).astype(np.float32)


def levels_exponential(s: int) -> np.ndarray:
    lv = np.zeros(s + 1, np.float64)
    lv[1:] = 2.0 ** (-(s - np.arange(1, s + 1)))
    return lv.astype(np.float32)


def _rng(*key) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(list(key)))


# ---------------------------------------------------------------------------
# Workload 1: stochastic bilinear game  min_x max_y x^T A y,  z = (x, y).
# ---------------------------------------------------------------------------


class BilinearGame:
    def __init__(self, n: int = 512, K: int = 4, noise: float = 0.1):
        self.n, self.K, self.noise, self.d = n, K, noise, 2 * n
        self.A = (_rng(1).standard_normal((n, n)) / np.sqrt(n)).astype(np.float32)

    def x1(self) -> np.ndarray:
        return _rng(3).standard_normal(self.d).astype(np.float32)

    def operator(self, z: np.ndarray) -> np.ndarray:
        z = np.asarray(z, np.float64)
        x, y = z[: self.n], z[self.n:]
        A = self.A.astype(np.float64)
        return np.concatenate([A @ y, -(A.T @ x)])

    def dual_vectors(self, z: np.ndarray, call: int) -> np.ndarray:
        """[K][d] float32: F(z) + N(0, noise^2) independently per worker."""
        f = self.operator(z)
        out = np.empty((self.K, self.d), np.float32)
        for k in range(self.K):
            out[k] = (f + self.noise * _rng(2, k, call).standard_normal(self.d)).astype(np.float32)
        return out


# ---------------------------------------------------------------------------
# Workload 2: one vector of iid N(0,1).
# ---------------------------------------------------------------------------


def gaussian_vector(d: int = 1 << 20, seed: int = 10) -> np.ndarray:
    return _rng(seed).standard_normal(d).astype(np.float32)


# ---------------------------------------------------------------------------
# Workload 3: K heavy-tailed vectors, Student-t with nu = 3, scaled by 1e-2.
# ---------------------------------------------------------------------------


def uniform_vectors(K: int, d: int, seed: int = 50) -> np.ndarray:
    """[K][d] float32, iid U(-1, 1): with the L-infinity norm the normalised magnitudes fill (0, 1]
    densely, so that a level fit on them has a unique answer."""
    out = np.empty((K, d), np.float32)
    for k in range(K):
        out[k] = _rng(seed, k).uniform(-1.0, 1.0, d).astype(np.float32)
    return out


def vectors_on_intervals(K: int, d: int, bucket: int, lo, hi, seed: int = 60) -> np.ndarray:
    """[K][d] float32 with random signs whose magnitudes lie in the union of the intervals
    [lo_i, hi_i) of (0, 1): an interval at random, weighted by its index to give masses of unequal size,
    then a uniform point of it, and one coordinate of magnitude exactly 1 in every bucket of `bucket`
    coordinates.  Under the L-infinity norm the normalised magnitudes are then the magnitudes
    themselves, so the caller decides which stretches of (0, 1) stay empty."""
    lo, hi = np.asarray(lo, np.float64), np.asarray(hi, np.float64)
    w = 1.0 + np.arange(len(lo)) % 7
    out = np.empty((K, d), np.float32)
    for k in range(K):
        g = _rng(seed, k)
        which = g.choice(len(lo), size=d, p=w / w.sum())
        mag = (lo[which] + g.random(d) * (hi[which] - lo[which])).astype(np.float32)
        mag = np.minimum(np.maximum(mag, lo[which].astype(np.float32)), np.nextafter(hi[which].astype(np.float32), np.float32(0)))
        mag[::bucket] = 1.0
        out[k] = mag * np.where(g.random(d) < 0.5, np.float32(-1), np.float32(1))
    return out


def student_t3(K: int, d: int, seed: int = 20, scale: float = 1e-2) -> np.ndarray:
    out = np.empty((K, d), np.float32)
    for k in range(K):
        g = _rng(seed, k)
        z = g.standard_normal(d)
        w = g.standard_normal((3, d))
        out[k] = (scale * z / np.sqrt((w * w).sum(0) / 3.0)).astype(np.float32)
    return out


def student_t3_device(K: int, d: int, seed: int = 20, scale: float = 1e-2, device="cuda"):
    import torch
    g = torch.Generator(device=device)
    out = torch.empty((K, d), dtype=torch.float32, device=device)
    for k in range(K):
        g.manual_seed(seed * 1000003 + k)
        z = torch.randn(d, generator=g, device=device)
        w = torch.zeros(d, device=device)
        for _ in range(3):
            t = torch.randn(d, generator=g, device=device)
            w.addcmul_(t, t)
        out[k] = scale * z / torch.sqrt(w / 3.0)
    return out


# ---------------------------------------------------------------------------
# Workload 4: GAN-shaped layout, 14 tensors, per-tensor scale.
# ---------------------------------------------------------------------------

GAN_SEGMENTS = np.array([
    1048576, 8192,      # linear 128 -> 8192: weight, bias
    2097152, 256,       # 4x4 conv 512 <-> 256: weight, bias
    524288, 128,        # 4x4 conv 256 <-> 128: weight, bias
    73728, 64,          # 3x3 conv 128 <-> 64: weight, bias
    73728,              # 3x3 conv 64 -> 128: weight
    524288,             # 4x4 conv 128 -> 256: weight
    2097152,            # 4x4 conv 256 -> 512: weight
    2359296, 512,       # 3x3 conv 512 -> 512: weight, bias
    1048576,            # linear 8192 -> 128: weight
], dtype=np.uint64)


def gan_sigmas(segments=GAN_SEGMENTS, seed: int = 30) -> np.ndarray:
    u = _rng(seed).random(len(segments))
    return 10.0 ** (-5.0 + 3.0 * u)


def gan_dual_vectors(K: int, call: int, segments=GAN_SEGMENTS, seed: int = 31) -> np.ndarray:
    sig = gan_sigmas(segments)
    d = int(np.sum(segments))
    out = np.empty((K, d), np.float32)
    for k in range(K):
        g = _rng(seed, k, call)
        pos = 0
        for s, n in zip(sig, segments):
            n = int(n)
            out[k, pos:pos + n] = (s * g.standard_normal(n)).astype(np.float32)
            pos += n
    return out


# ---------------------------------------------------------------------------
# Workload 5: strongly monotone quadratic game F(z) = M z + b,
# M block-diagonal with 2x2 blocks [[mu, a], [-a, mu]].
# ---------------------------------------------------------------------------


class QuadraticGame:
    def __init__(self, d: int = 1 << 26, K: int = 16, mu: float = 0.1, noise: float = 0.05):
        assert d % 2 == 0
        self.d, self.K, self.mu, self.noise = d, K, mu, noise
        self.a = _rng(40).uniform(-1.0, 1.0, d // 2).astype(np.float32)
        self.b = _rng(41).standard_normal(d).astype(np.float32)

    def operator(self, z: np.ndarray) -> np.ndarray:
        z = np.asarray(z, np.float64)
        z0, z1 = z[0::2], z[1::2]
        a = self.a.astype(np.float64)
        f = np.empty(self.d, np.float64)
        f[0::2] = self.mu * z0 + a * z1
        f[1::2] = -a * z0 + self.mu * z1
        return f + self.b

    def solution(self) -> np.ndarray:
        a = self.a.astype(np.float64)
        det = self.mu * self.mu + a * a
        b0, b1 = self.b[0::2].astype(np.float64), self.b[1::2].astype(np.float64)
        z = np.empty(self.d, np.float64)
        z[0::2] = -(self.mu * b0 - a * b1) / det
        z[1::2] = -(a * b0 + self.mu * b1) / det
        return z

    def dual_vectors(self, z: np.ndarray, call: int) -> np.ndarray:
        f = self.operator(z)
        out = np.empty((self.K, self.d), np.float32)
        for k in range(self.K):
            out[k] = (f + self.noise * _rng(42, k, call).standard_normal(self.d)).astype(np.float32)
        return out
