"""Host-side checks that need no GPU: the library loads, exports what the header declares,
and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2505_09326_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        pkg.build_library()
    return pkg.load_library()


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(sphattn_\w+)\s*\(", text)
    return sorted(set(names))


def test_header_symbols_are_exported(lib):
    import paper_2505_09326_amd as pkg
    declared = _declared_functions()
    assert declared, "no functions found in include/*.h"
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in include/ but not exported"
    assert sorted(pkg.EXPORTED_SYMBOLS) == declared


def test_version_and_strerror(lib):
    assert lib.sphattn_version() >= 100
    assert lib.sphattn_strerror(0) == b"success"
    for code in range(-8, 0):
        assert b"unknown" not in lib.sphattn_strerror(code)
    assert b"unknown" in lib.sphattn_strerror(-99)


def _call(lib, fn="sphattn_fwd", Q=0x1000, K=0x2000000, V=0x4000000, O=0x6000000,
          B=1, H=1, N=128, d=128, dtype=1):
    return getattr(lib, fn)(ctypes.c_void_p(Q), ctypes.c_void_p(K), ctypes.c_void_p(V),
                            ctypes.c_void_p(O), B, H, N, d, dtype, None)


@pytest.mark.parametrize("fn", ["sphattn_fwd", "sphattn_softmax_fwd"])
def test_argument_errors_are_reported_before_any_launch(lib, fn):
    """Fake (never dereferenced) addresses: every call must fail in validation."""
    assert _call(lib, fn, Q=0) == -1
    assert _call(lib, fn, O=0) == -1
    assert _call(lib, fn, B=0) == -2
    assert _call(lib, fn, N=-5) == -2
    assert _call(lib, fn, B=2 ** 20, H=2 ** 20, N=2 ** 20) == -2
    assert _call(lib, fn, d=96) == -3
    assert _call(lib, fn, dtype=9) == -4
    assert _call(lib, fn, K=0x2000008) == -5
    assert _call(lib, fn, O=0x1000) == -7                       # O is Q
    assert _call(lib, fn, O=0x2000000 + 128 * 128 * 2 - 16) == -7  # O overlaps the end of K


def test_grn_entry_argument_errors(lib):
    def call(Q=0x1000, K=0x2000000, V=0x4000000, mult=0x8000000, O=0x6000000,
             B=1, H=4, H_kv=2, N=128, d=128, dtype=1):
        return lib.sphattn_grn_fwd(ctypes.c_void_p(Q), ctypes.c_void_p(K), ctypes.c_void_p(V),
                                   ctypes.c_void_p(mult), ctypes.c_void_p(O), B, H, H_kv, N, d, dtype, None)
    assert call(K=0) == -1
    assert call(H_kv=3) == -2
    assert call(H_kv=0) == -2
    assert call(d=32) == -3
    assert call(dtype=7) == -4
    assert call(mult=0x8000002) == -5
    assert call(O=0x8000000) == -7            # O is mult


def test_normalized_entry_argument_errors(lib):
    def call(normalizer=0, dtype=1, d=128):
        return lib.sphattn_normalized_fwd(ctypes.c_void_p(0x1000), ctypes.c_void_p(0x2000000),
                                          ctypes.c_void_p(0x4000000), ctypes.c_void_p(0x6000000),
                                          1, 1, 128, d, dtype, normalizer, None)
    assert call(normalizer=4) == -8
    assert call(normalizer=-1) == -8
    assert call(normalizer=2, dtype=2) == -4       # fp8 Q/K only with the L2 normalizer
    assert call(normalizer=3, dtype=0) == -4
    assert call(normalizer=1, dtype=3) == -4       # fp16 storage only with the L2 normalizer
    assert call(d=100) == -3


def test_shape_limits_are_rejected_not_truncated(lib):
    """One head of one tensor must fit a 32-bit buffer range: larger N is an error code."""
    rc = lib.sphattn_fwd(ctypes.c_void_p(0x1000), ctypes.c_void_p(0x100000000), ctypes.c_void_p(0x200000000),
                         ctypes.c_void_p(0x300000000), 1, 1, 5_000_000, 128, 1, None)
    assert rc == -2


def test_softmax_twin_is_bf16_only(lib):
    assert _call(lib, "sphattn_softmax_fwd", dtype=0) == -4
    assert _call(lib, "sphattn_softmax_fwd", dtype=2) == -4
    assert _call(lib, "sphattn_softmax_fwd", dtype=3) == -4


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
