"""The C-ABI library: it loads, exports every function include/qgx.h declares, and rejects bad
configurations on the host before anything touches a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2308_09187_amd", "libqgx.so")
HEADER = os.path.join(ROOT, "include", "qgx.h")


def _lib():
    if not os.path.exists(LIB):
        from paper_2308_09187_amd import build
        build.build()
    return C.CDLL(LIB)


def _declared():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qgx_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_function_is_exported():
    lib = _lib()
    names = _declared()
    assert len(names) >= 19
    for n in names:
        assert hasattr(lib, n), n


def test_binding_lists_the_same_functions():
    from paper_2308_09187_amd import qgx
    assert sorted(qgx.EXPORTS) == _declared()


def test_create_rejects_bad_configurations_on_the_host():
    from paper_2308_09187_amd.qgx import _Config
    lib = _lib()
    h = C.c_void_p()

    def create(**kw):
        base = dict(d=1024, K=2, bucket=256, n_segments=0, segment_len=None, norm=2, code=0, seed=1)
        base.update(kw)
        cfg = _Config(**base)
        return lib.qgx_create(C.byref(h), C.byref(cfg))

    assert create(d=0) == -1
    assert create(d=1 << 31) == -1
    assert create(K=0) == -1
    assert create(bucket=0) == -1
    assert create(bucket=250) == -1            # not a multiple of 4
    assert create(bucket=1 << 17) == -1        # above the largest bucket
    assert create(norm=65) == -1               # q of the norm: 0 (maximum) or 1..64
    assert create(norm=-1) == -1
    assert create(code=7) == -1
    seg = (C.c_uint64 * 2)(1000, 25)           # does not sum to d
    assert create(n_segments=2, segment_len=seg) == -1
    seg = (C.c_uint64 * 2)(1022, 2)            # inner segment not a multiple of 4
    assert create(n_segments=2, segment_len=seg) == -1
    assert lib.qgx_create(None, None) == -1
    lib.qgx_last_error.restype = C.c_char_p
    assert lib.qgx_last_error(None) == b"null context"


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_binding_constants_match_the_header():
    """The numbers the binding repeats (status codes, error bits, limits, the call numbers that stand for
    'from the iteration counter') are the header's."""
    from paper_2308_09187_amd import qgx
    text = open(HEADER).read()
    defs = {m.group(1): int(m.group(2).rstrip("uU"), 0) for m in re.finditer(r"#define\s+(QGX_[A-Z0-9_]+)\s+(0x[0-9A-Fa-f]+[uU]?|\d+[uU]?)\s", text)}
    assert defs["QGX_CALL_FIRST_HALF"] == qgx.CALL_FIRST_HALF and defs["QGX_CALL_SECOND_HALF"] == qgx.CALL_SECOND_HALF
    assert defs["QGX_CHUNK"] == qgx.CHUNK and defs["QGX_SUB"] == qgx.SUB and defs["QGX_SUBS"] == qgx.SUBS
    assert defs["QGX_MAX_BINS"] == qgx.MAX_BINS
    for bit in ("CAPACITY", "STREAM", "NONFINITE", "STATE"):
        assert defs["QGX_EBIT_" + bit] == getattr(qgx, "EBIT_" + bit)
