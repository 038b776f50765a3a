"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved).

  * oracle/sphattn_oracle.c: built with gcc -fsanitize=address,undefined together with a driver
    (tests/sanitizers/oracle_driver.c) that calls every entry point on exactly sized heap
    buffers; the outputs must equal the ordinary build's on the same inputs, and the run must
    end without a sanitizer report.
  * the host half of the C ABI (paper_2505_09326_amd/csrc/sphattn_api.hip: argument checks,
    slice planning, workspace arithmetic, overlap logic): built with hipcc, host code under the
    same sanitizers, and driven by tests/sanitizers/abi_driver.cpp through calls that return
    before any launch.
"""
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitizers")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")

KINDS = {0: np.float64, 1: np.float32, 2: np.uint16, 3: np.uint8, 4: np.uint16}
KIND_NAMES = {0: "f64", 1: "f32", 2: "bf16", 3: "e4m3fn", 4: "f16"}


@pytest.fixture(scope="module")
def oracle_driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "oracle_driver")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-o", exe, os.path.join(ROOT, "oracle", "sphattn_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return exe


def _records(path):
    raw = open(path, "rb").read()
    out, pos = [], 0
    while pos < len(raw):
        n = int(np.frombuffer(raw, dtype=np.uint64, count=1, offset=pos)[0])
        out.append(raw[pos + 8: pos + 8 + n])
        pos += 8 + n
    return out


CASES = [  # B, H, H_kv, N_q, N_k, d, kind
    (1, 1, 1, 1, 1, 1, 0), (2, 4, 2, 37, 37, 8, 2), (1, 3, 3, 65, 65, 16, 1), (1, 2, 2, 33, 33, 5, 0),
    (2, 2, 1, 20, 20, 64, 3), (1, 2, 2, 19, 19, 128, 4), (1, 2, 1, 5, 19, 16, 3), (2, 6, 3, 40, 7, 4, 2),
]


@pytest.mark.parametrize("B,H,H_kv,Nq,Nk,d,kind", CASES)
def test_oracle_under_asan_ubsan_matches_the_ordinary_build(oracle, oracle_driver, tmp_path, B, H, H_kv, Nq, Nk, d, kind):
    out = str(tmp_path / "case.bin")
    r = subprocess.run([oracle_driver, *map(str, (B, H, H_kv, Nq, Nk, d, kind, 1000 + Nq * 7 + d)), out],
                       capture_output=True, text=True, env=ENV)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
    rec = _records(out)
    dt, name = KINDS[kind], KIND_NAMES[kind]
    Q = np.frombuffer(rec[0], dtype=dt).reshape(B, H, Nq, d)
    K = np.frombuffer(rec[1], dtype=dt).reshape(B, H_kv, Nk, d)
    V = np.frombuffer(rec[2], dtype=dt).reshape(B, H_kv, Nk, d)
    G = np.frombuffer(rec[3], dtype=dt).reshape(B, H, Nq, d)
    mult = np.frombuffer(rec[4], dtype=np.float64).reshape(B, Nk)
    kinds = (name,) * 3
    f64 = lambda b, *shape: np.frombuffer(b, dtype=np.float64).reshape(shape)   # noqa: E731
    o_raw, z = oracle.spherical_accumulate(Q, K, V, mult, kinds=kinds)
    assert np.array_equal(f64(rec[5], B, H, Nq, d), o_raw) and np.array_equal(f64(rec[6], B, H, Nq), z)
    if Nq != Nk:
        assert len(rec) == 7
        return
    N = Nq
    assert np.array_equal(f64(rec[7], B, H, N, d), oracle.grn_attention(Q, K, V, mult, kinds=kinds), equal_nan=True)
    W = f64(rec[8], B, H, N, N)
    Z = f64(rec[9], B, H, N)
    assert np.array_equal(Z, z)
    live = Z > 0
    assert np.allclose((W * W).sum(-1)[live], 1.0, rtol=1e-12)                 # unit-norm weight rows
    rows = [0, N - 1, N // 2]
    assert np.array_equal(f64(rec[10], 3, d), oracle.grn_attention_rows(Q, K, V, mult, B * H - 1, rows, kinds=kinds))
    dQ, dK, dV = oracle.grn_attention_bwd(Q, K, V, G, mult, kinds=(name,) * 4)
    assert np.array_equal(f64(rec[11], B, H, N, d), dQ, equal_nan=True)
    assert np.array_equal(f64(rec[12], B, H_kv, N, d), dK, equal_nan=True)
    assert np.array_equal(f64(rec[13], B, H_kv, N, d), dV, equal_nan=True)
    if H_kv != H:
        assert len(rec) == 14
        return
    pos = 14
    for norm in ("softmax", "l1", "sqrelu"):
        assert np.array_equal(f64(rec[pos], B, H, N, d), oracle.normalized_attention(Q, K, V, norm, kinds=kinds), equal_nan=True)
        assert np.array_equal(f64(rec[pos + 1], 3, d), oracle.normalized_attention_rows(Q, K, V, norm, 0, rows, kinds=kinds),
                              equal_nan=True)
        pos += 2
    Qd, Kd, Vd = (oracle.widen(x, name) for x in (Q, K, V))
    for chunk in (1, 7, N + 3):
        assert np.array_equal(f64(rec[pos], B, H, N, d), oracle.spherical_attention_streamed(Qd, Kd, Vd, chunk), equal_nan=True)
        pos += 1
    assert pos == len(rec)


def test_abi_host_code_under_asan_ubsan(tmp_path):
    from paper_2505_09326_amd._build import HIPCC_FLAGS, SOURCES
    exe = str(tmp_path / "abi_driver")
    flags = [f for f in HIPCC_FLAGS if f not in ("-O3", "-shared", "-fPIC")]
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=all"]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), *flags, "-O1", "-g", "-Wno-inline-asm", *san, "-o", exe,
           *SOURCES, os.path.join(SAN, "abi_driver.cpp")]
    b = subprocess.run(cmd, capture_output=True, text=True)
    assert b.returncode == 0, b.stderr[-4000:]
    r = subprocess.run([exe], capture_output=True, text=True, env=ENV)
    assert r.returncode == 0 and r.stdout.strip() == "ok", (r.stdout + r.stderr)[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr
