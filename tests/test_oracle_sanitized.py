"""The oracle's pins once more against a build of its C source with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only: nothing here touches a GPU): an out-of-bounds access, a
use after free, a signed overflow or a misaligned access in the checker would stop the child process."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_rng.py", "tests/test_oracle_quantize.py", "tests/test_oracle_codec.py", "tests/test_oracle_game.py",
        "tests/test_oracle_eg.py", "tests/test_oracle_fit.py", "tests/test_oracle_huffman.py"]


def test_pins_pass_on_a_sanitized_build_of_the_oracle(tmp_path):
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime next to gcc")
    src = tmp_path / "qgx_oracle.c"
    shutil.copy(os.path.join(ROOT, "oracle", "qgx_oracle.c"), src)
    preload = " ".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x)     # the interpreter is not instrumented
    env = dict(os.environ, QGX_ORACLE_SRC=str(src),
               QGX_ORACLE_CFLAGS="-fsanitize=address,undefined -fno-sanitize-recover=undefined -fno-omit-frame-pointer -g",
               LD_PRELOAD=preload, ASAN_OPTIONS="detect_leaks=0:verify_asan_link_order=0:abort_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PINS],
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=1500)
    tail = r.stdout[-3000:] + r.stderr[-3000:]
    assert r.returncode == 0, tail
    assert "runtime error" not in tail and "AddressSanitizer" not in tail, tail
    assert " passed" in r.stdout
