"""Do the pins have teeth?  Each case plants one plausible mistake (a dropped term, a wrong sign or index,
a swapped operand, a missing root) in a copy of the oracle's C source, builds it, and runs the pin tests
of that part against the copy in a child process: at least one of them has to fail.  The mistakes live
on the CPU and in a temporary directory only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "qgx_oracle.c")

Q, C, E, F, H, R = ("tests/test_oracle_quantize.py", "tests/test_oracle_codec.py", "tests/test_oracle_eg.py",
                    "tests/test_oracle_fit.py", "tests/test_oracle_huffman.py", "tests/test_oracle_rng.py")
G = "tests/test_oracle_game.py"

MUTANTS = [
    ("nine Philox rounds", "round < 10; ++round", "round < 9; ++round", [R]),
    ("23 random bits instead of 24", "(out[i & 3] >> 8) * 0x1p-24f", "(out[i & 3] >> 9) * 0x1p-24f", [Q]),
    ("rounds down where it should round up", "sym = j + ((r * g < t) ? 1u : 0u);", "sym = j + ((r * g < t) ? 0u : 1u);", [Q]),
    ("signs dropped", "neg[(uint64_t)k * d + i] = (uint8_t)(signbit(x) ? 1 : 0);", "neg[(uint64_t)k * d + i] = 0;", [Q]),
    ("L2 norm without the root", "n = (float)sqrt(acc);", "n = (float)acc;", [Q]),
    ("level index one too high", "while (j + 2 < n_sym && levels[j + 1] <= u) ++j;",
     "while (j + 2 < n_sym && levels[j] <= u) ++j;", [Q]),
    ("gap without its lower end", "const float g = levels[j + 1] - levels[j];", "const float g = levels[j + 1];", [Q]),
    ("Elias groups least significant bit first", "tmp[len++] = (uint8_t)((N >> i) & 1u);",
     "tmp[len++] = (uint8_t)((N >> (nb - 1 - i)) & 1u);", [C]),
    ("a sign bit for zeros too", "if (sym != 0) put_bit(words, word_pos * 32 + p++,", "put_bit(words, word_pos * 32 + p++,", [C]),
    ("decoded sign inverted", "Vhat[(uint64_t)k * d + i] = sg ? -mag : mag;", "Vhat[(uint64_t)k * d + i] = sg ? mag : -mag;", [C]),
    ("half-step towards the dual vector", "X_half[i] = x_t - gamma * (acc / (double)K);",
     "X_half[i] = x_t + gamma * (acc / (double)K);", [E]),
    ("mean not divided by K", "Y[i] = Y[i] - acc / (double)K;", "Y[i] = Y[i] - acc;", [E]),
    ("step size without the root", "*gamma = (double)K / sqrt(1.0 + *S);", "*gamma = (double)K / (1.0 + *S);", [E]),
    ("S from sums instead of differences", "s_add += (prev - cur) * (prev - cur);", "s_add += (prev + cur) * (prev + cur);", [E]),
    ("histogram weighted by the norm, not its square", "const double w = (double)n * (double)n;", "const double w = (double)n;", [F]),
    ("stationarity with a wrong sign", "left[p + 1] = left[p] + mass[p] * (piece_mid - a);",
     "left[p + 1] = left[p] + mass[p] * (piece_mid + a);", [F]),
    ("the largest root where the condition holds on an interval", "if (G_lo < 0.0 && G_hi >= 0.0) {",
     "if (G_lo <= 0.0 && G_hi > 0.0) {", [F]),
    ("slope of the stationarity function without the distance between the neighbours",
     "const double slope = (c - a) * mass[p] / (hi[p] - lo[p]);", "const double slope = mass[p] / (hi[p] - lo[p]);", [F]),
    ("symbol probabilities mirrored", "p[j] += mass * (1.0 - up);\n            p[j + 1] += mass * up;",
     "p[j] += mass * up;\n            p[j + 1] += mass * (1.0 - up);", [H]),
    ("a word charged the code space of one a bit longer", "const uint32_t space = 1u << (max_len - l);\n                if (space > k || BEST(i + 1, k - space) == none) continue;\n                const uint64_t cost",
     "const uint32_t space = (1u << (max_len - l)) >> 1;\n                if (space > k || BEST(i + 1, k - space) == none) continue;\n                const uint64_t cost", [H]),
    ("canonical words not advanced", "if (r > 0) word = (word + 1) << (order[r].len - order[r - 1].len);",
     "if (r > 0) word = word << (order[r].len - order[r - 1].len);", [H]),
    ("largest magnitude taken as the smallest", "if (a > n) n = a;", "if (a < n || n == 0.0f) n = a;", [Q]),
    ("q-norm raised to q instead of 1/q", "n = (float)(m * pow(acc, 1.0 / q));", "n = (float)(m * pow(acc, q));", [Q]),
    ("mean over K - 1", "mean[i] = acc / (double)K;", "mean[i] = acc / (double)(K - 1);", [E, C]),
    ("bins half an octave off", "const int64_t key = (int64_t)(bits >> 17) - ((int64_t)127 * 64 - (int64_t)n_bins);",
     "const int64_t key = (int64_t)(bits >> 17) - ((int64_t)127 * 64 - (int64_t)n_bins) - 32;", [F]),
    ("the next word of the Philox block", "out[i & 3]", "out[(i + 1) & 3]", [Q, R]),
    ("draws that ignore the call", "ctr[1] = (uint32_t)(blk >> 32); ctr[2] = k; ctr[3] = call_id;",
     "ctr[1] = (uint32_t)(blk >> 32); ctr[2] = k; ctr[3] = 0;", [Q, R]),
    ("draws that ignore the worker", "ctr[1] = (uint32_t)(blk >> 32); ctr[2] = k; ctr[3] = call_id;",
     "ctr[1] = (uint32_t)(blk >> 32); ctr[2] = 0; ctr[3] = call_id;", [Q, R]),
    ("moment of a piece taken at its lower end", "const double piece_mid = 0.5 * (lo[p] + hi[p]);",
     "const double piece_mid = lo[p];", [F]),
    ("stationarity without its right-hand term", "const double G_lo = left[p] - right[p], G_hi = left[p + 1] - right[p + 1];",
     "const double G_lo = left[p], G_hi = left[p + 1];", [F]),
    ("every bucket decoded with the first norm", "const float n = norms[(uint64_t)k * NB + b];",
     "const float n = norms[(uint64_t)k * NB];", [C]),
    ("symbol probabilities not normalised", "for (uint32_t j = 0; j < n_sym; ++j) p[j] /= total;", "", [H]),
    ("next iterate without the anchor", "X_next[i] = (anchor ? anchor[i] : 0.0) + (*gamma) * Y[i];",
     "X_next[i] = (*gamma) * Y[i];", [E]),
    ("current iterate without the step size", "const double x_t = (anchor ? anchor[i] : 0.0) + gamma * Y[i];",
     "const double x_t = (anchor ? anchor[i] : 0.0) + Y[i];", [E]),
    ("objective without the cubic term", "const double P_hi = -hi * hi * hi / 3.0 + (a + c) * hi * hi / 2.0 - a * c * hi;",
     "const double P_hi = (a + c) * hi * hi / 2.0 - a * c * hi;", [F]),
    ("noise radius without the root", "const double r = sqrt(-2.0 * log(u1));", "const double r = -2.0 * log(u1);", [G]),
    ("both halves of a noise pair from the cosine", "return (i & 1) ? r * sin(two_pi * u2) : r * cos(two_pi * u2);",
     "return r * cos(two_pi * u2);", [G]),
    ("noise that ignores the worker", "ctr[0] = (uint32_t)g; ctr[1] = 1u; ctr[2] = k; ctr[3] = call_id;",
     "ctr[0] = (uint32_t)g; ctr[1] = 1u; ctr[2] = 0; ctr[3] = call_id;", [G]),
    ("operator with a symmetric coupling", "F[j + 1] = -aj * z0 + mu * z1 + (double)b[j + 1];",
     "F[j + 1] = aj * z0 + mu * z1 + (double)b[j + 1];", [G]),
    ("free maximiser of the gap without the factor two", "x[j] = (mu * h0 - aj * h1 - (double)b[j]) / (2.0 * mu);",
     "x[j] = (mu * h0 - aj * h1 - (double)b[j]) / mu;", [G]),
    ("gap's maximiser from the operator instead of its transpose", "x[j + 1] = (aj * h0 + mu * h1 - (double)b[j + 1]) / (2.0 * mu);",
     "x[j + 1] = (-aj * h0 + mu * h1 - (double)b[j + 1]) / (2.0 * mu);", [G]),
    ("gap's ball taken around the origin", "x[i] = c + (R / dist) * (x[i] - c);", "x[i] = (R / dist) * x[i];", [G]),
    ("cost of a word without its weight", "const uint64_t cost = w[i] * l + BEST(i + 1, k - space);",
     "const uint64_t cost = l + BEST(i + 1, k - space);", [H]),
]


@pytest.mark.parametrize("name,old,new,files", MUTANTS, ids=[m[0].replace(" ", "_") for m in MUTANTS])
def test_a_pin_fails_for_the_planted_mistake(tmp_path, name, old, new, files):
    src = open(SRC).read()
    assert src.count(old) == 1, "the text to change must occur exactly once"
    mutant = tmp_path / "qgx_oracle.c"
    mutant.write_text(src.replace(old, new))
    env = dict(os.environ, QGX_ORACLE_SRC=str(mutant))
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 1 and " failed" in r.stdout, "no pin caught: %s\n%s" % (name, r.stdout[-2000:] + r.stderr[-2000:])
