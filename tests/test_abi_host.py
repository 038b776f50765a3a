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
    for code in range(-10, 0):
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
    assert call(normalizer=2, dtype=2) == -4       # fp8 Q/K only with the L2 normalizer and the SoftMax twin
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


def test_partial_and_combine_argument_errors(lib):
    P = ctypes.c_void_p

    def partial(Q=0x1000, K=0x2000000, V=0x4000000, mult=0, o=0x10000000, z=0x20000000,
                B=1, H=2, H_kv=1, Nq=100, Nk=300, d=64, dtype=1):
        return lib.sphattn_partial_fwd(P(Q), P(K), P(V), P(mult), P(o), P(z), B, H, H_kv, Nq, Nk, d, dtype, None)
    assert partial(z=0) == -1
    assert partial(o=0) == -1
    assert partial(Nq=0) == -2
    assert partial(Nk=-1) == -2
    assert partial(H_kv=3) == -2
    assert partial(d=80) == -3
    assert partial(dtype=5) == -4
    assert partial(o=0x10000004) == -5
    assert partial(z=0x20000002) == -5
    assert partial(o=0x1000) == -7                           # o_part is Q
    assert partial(z=0x10000000 + 16) == -7                  # z_part inside o_part

    def combine(o=0x10000000, z=0x20000000, n=3, O=0x30000000, Z=0, B=1, H=2, N=100, d=64, dtype=1):
        return lib.sphattn_combine(P(o), P(z), n, P(O), P(Z), B, H, N, d, dtype, None)
    assert combine(o=0) == -1
    assert combine(O=0) == -1
    assert combine(n=0) == -2
    assert combine(n=10 ** 6) == -2
    assert combine(N=0) == -2
    assert combine(d=32) == -3
    assert combine(dtype=-1) == -4
    assert combine(O=0x30000008) == -5
    assert combine(O=0x10000000 + 3 * 200 * 64 * 4 - 16) == -7     # O overlaps the last part
    assert combine(Z=0x20000000) == -7                             # Z is z_parts


def test_splitkv_argument_errors_and_workspace_size(lib):
    P = ctypes.c_void_p
    need = lib.sphattn_splitkv_workspace_bytes(1, 2, 1000, 128, 4)
    assert need >= 4 * 2 * 1000 * 129 * 4 and need % 256 == 0 and need < 4 * 2 * 1000 * 129 * 4 + 256
    assert lib.sphattn_splitkv_workspace_bytes(1, 2, 1000, 100, 4) == 0
    assert lib.sphattn_splitkv_workspace_bytes(0, 2, 1000, 128, 4) == 0
    assert lib.sphattn_splitkv_workspace_bytes(1, 2, 1000, 128, 0) == 0

    def call(ws=0x40000000, size=need, n_splits=4, O=0x6000000, Z=0, N=1000, dtype=1):
        return lib.sphattn_splitkv_fwd(P(0x1000), P(0x2000000), P(0x4000000), P(0), P(O), P(Z),
                                       1, 2, 2, N, 128, dtype, n_splits, P(ws), size, None)
    assert call(ws=0) == -9
    assert call(size=need - 256) == -9
    assert call(ws=0x40000004) == -9
    assert call(n_splits=-1) == -2
    assert call(N=0) == -2
    assert call(dtype=8) == -4
    assert call(ws=0x6000000) == -7                          # workspace is O
    assert call(Z=0x40000000 + 64) == -7                     # Z inside the workspace


def test_splitkv_heuristic_splits_only_underfilled_launches(lib):
    h = lib.sphattn_splitkv_heuristic
    assert h(2, 16, 8192, 128, 1) == 1                # 1024 workgroups already
    assert h(1, 1, 65536, 128, 1) == 1                # 256 workgroups
    assert h(1, 1, 8192, 128, 1) == 8                 # 32 workgroups -> 8 slices of 16 tiles
    assert h(1, 2, 4096, 64, 1) in (7, 8)             # 32 workgroups; 64 tiles in slices of 8 to 10
    assert h(1, 1, 40000, 128, 1) == 3                # 157 workgroups: 471 items = two rounds of 236, not 2 x 157
    assert h(1, 3, 16384, 128, 1) == 4                # 192 workgroups: 768 items = three full rounds
    assert h(1, 5, 16384, 64, 1) == 3                 # d = 64: 512 resident workgroups; 960 items = two rounds
    assert h(1, 8, 20000, 128, 1) == 2                # 632 workgroups = 2.47 rounds: 1264 half-length items = 5 rounds
    assert h(1, 8, 40960, 128, 1) == 1                # 1280 workgroups = five full rounds
    assert h(1, 8, 4096, 128, 1) == 1                 # 128 workgroups: 128-row tiles fill the CUs instead
    assert h(1, 1, 32768, 128, 1) == 2                # 128 workgroups, long: two slices of 256-row tiles
    assert h(1, 1, 300, 128, 1) == 1                  # 5 tiles: too short to cut
    assert h(1, 1, 2048, 64, 0) == 4                  # fp32: 32-row workgroups, 64 of them
    assert h(0, 1, 8192, 128, 1) == 1                 # nonsense in, 1 out


def test_backward_argument_errors(lib):
    P = ctypes.c_void_p
    base = dict(Q=0x1000000, K=0x2000000, V=0x3000000, O=0x4000000, dO=0x5000000, Z=0x6000000,
                dQ=0x7000000, dK=0x8000000, dV=0x9000000, delta=0xA000000)

    def call(B=1, H=2, N=300, d=64, dtype=1, **over):
        a = dict(base, **over)
        return lib.sphattn_bwd(P(a["Q"]), P(a["K"]), P(a["V"]), P(a["O"]), P(a["dO"]), P(a["Z"]),
                               P(a["dQ"]), P(a["dK"]), P(a["dV"]), P(a["delta"]), B, H, N, d, dtype, None)
    for name in base:
        assert call(**{name: 0}) == -1
    assert call(N=0) == -2
    assert call(d=96) == -3
    assert call(dtype=0) == -4                 # fp32 and fp8 storage have no backward
    assert call(dtype=2) == -4
    assert call(dtype=9) == -4
    assert call(dK=0x8000008) == -5
    assert call(delta=0xA000002) == -5
    assert call(dQ=0x1000000) == -7            # dQ is Q
    assert call(dV=0x8000000) == -7            # dV is dK
    assert call(delta=0x6000000) == -7         # delta is Z
    assert call(delta=0x6000000 - 2400) == -7  # [2,B,H,N]: the second plane of delta lies over Z

    def grn(mult=0xB000000, H_kv=1, **over):
        a = dict(base, **over)
        return lib.sphattn_grn_bwd(P(a["Q"]), P(a["K"]), P(a["V"]), P(mult), P(a["O"]), P(a["dO"]), P(a["Z"]),
                                   P(a["dQ"]), P(a["dK"]), P(a["dV"]), P(a["delta"]), 1, 2, H_kv, 300, 64, 1, None)
    assert grn(H_kv=3) == -2
    assert grn(H_kv=0) == -2
    assert grn(mult=0xB000002) == -5
    assert grn(dK=0xB000000) == -7             # dK is mult
    assert grn(Q=0) == -1


def test_cross_argument_errors(lib):
    P = ctypes.c_void_p

    def call(Q=0x1000000, K=0x2000000, V=0x3000000, mult=0, O=0x4000000, Z=0, B=1, H=4, H_kv=2, Nq=100, Nk=300,
             d=64, dtype=1):
        return lib.sphattn_cross_fwd(P(Q), P(K), P(V), P(mult), P(O), P(Z), B, H, H_kv, Nq, Nk, d, dtype, None)
    assert call(Q=0) == -1 and call(O=0) == -1
    assert call(Nq=0) == -2 and call(Nk=0) == -2 and call(H_kv=3) == -2
    assert call(d=32) == -3 and call(dtype=7) == -4
    assert call(K=0x2000004) == -5 and call(Z=0x5000002) == -5
    assert call(O=0x1000000) == -7
    assert call(O=0x2000000 + 300 * 64 * 2) == -7          # O inside K (N_k rows of it)
    assert call(Z=0x4000000) == -7                         # Z is O
    assert call(mult=0x4000000 + 64) == -7                 # mult inside O


def test_fp8_argument_errors_and_workspace_size(lib):
    P = ctypes.c_void_p
    wsb = lib.sphattn_fp8_workspace_bytes
    # V^T padded to whole 128-key tiles (one byte per element) + one float per head, rounded up
    assert wsb(2, 3, 300, 128) == 2 * 3 * 128 * 384 + 256
    assert wsb(1, 1, 128, 128) == 128 * 128 + 256
    assert wsb(1, 1, 130, 64) == 64 * 256 + 256
    assert wsb(1, 1, 128, 96) == 0 and wsb(0, 1, 128, 128) == 0 and wsb(1, 1, 0, 128) == 0
    need = wsb(1, 2, 1000, 128)

    def call(Q=0x1000000, K=0x2000000, V=0x3000000, O=0x4000000, ws=0x40000000, size=need, B=1, H=2, H_kv=2,
             N=1000, d=128):
        return lib.sphattn_fp8_fwd(P(Q), P(K), P(V), P(O), P(ws), size, B, H, H_kv, N, d, None)
    assert call(Q=0) == -1 and call(K=0) == -1 and call(V=0) == -1 and call(O=0) == -1
    assert call(N=0) == -2 and call(H=0) == -2 and call(H=3, H_kv=2) == -2
    assert call(H=4, H_kv=2, size=wsb(1, 2, 1000, 128) - 1) == -9   # the workspace is sized by H_kv
    assert call(d=96) == -3 and call(d=32) == -3           # d = 64 or 128
    assert call(d=64, size=wsb(1, 2, 1000, 64) - 1) == -9
    assert call(V=0x3000008) == -5
    assert call(O=0x1000000) == -7                         # O is Q
    assert call(O=0x3000000 - 256) == -7                   # O runs into V
    assert call(ws=0) == -9 and call(ws=0x40000004) == -9 and call(size=need - 1) == -9
    assert call(ws=0x2000000) == -7                        # workspace is K
    assert call(ws=0x4000000 + 4096) == -7                 # workspace inside O
    # the SoftMax twin shares the checks
    twin = lib.sphattn_fp8_softmax_fwd
    assert twin(P(0x1000000), P(0x2000000), P(0x3000000), P(0x4000000), P(0x40000000), need - 1, 1, 2, 2, 1000, 128, None) == -9
    assert twin(P(0x1000000), P(0x2000000), P(0x3000000), P(0x4000000), P(0x40000000), need, 1, 2, 2, 1000, 96, None) == -3
    # multiplicities: alignment and overlap with what the call writes
    grn = lib.sphattn_fp8_grn_fwd

    def g(mult, O=0x4000000, ws=0x40000000):
        return grn(P(0x1000000), P(0x2000000), P(0x3000000), P(mult), P(O), P(ws), need, 1, 2, 2, 1000, 128, None)
    assert g(0x5000002) == -5 and g(0x4000000 + 64) == -7 and g(0x40000000 + 1024) == -7


def test_bench_probe_library_argument_errors():
    """The matrix-instruction probe is the benchmark's own library, not part of the ABI."""
    path = os.path.join(ROOT, "libbench_mfma_probe.so")
    if not os.path.exists(path):
        import __graft_entry__ as g
        g.build_bench_probe()
    probe = ctypes.CDLL(path).bench_mfma_probe
    probe.restype = ctypes.c_int
    probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    P = ctypes.c_void_p
    assert probe(P(0), P(0x2000), 0, 10, None) == -1
    assert probe(P(0x1000), P(0), 0, 10, None) == -1
    assert probe(P(0x1000), P(0x2000), 5, 10, None) == -2
    assert probe(P(0x1000), P(0x2000), 0, 0, None) == -2
    assert probe(P(0x1008), P(0x2000), 0, 10, None) == -5
    assert probe(P(0x1000), P(0x2004), 0, 10, None) == -5


def test_no_measurement_probe_in_the_attention_library(lib):
    assert not hasattr(lib, "sphattn_mfma_probe")


def test_tile_rows_argument(lib):
    P = ctypes.c_void_p

    def call(tile_rows, Z=0):
        return lib.sphattn_fwd_tile_rows(P(0x1000), P(0x2000000), P(0x4000000), P(0x6000000), P(Z),
                                         1, 1, 128, 128, 1, tile_rows, None)
    for bad in (-1, 1, 64, 129, 512):
        assert call(bad) == -2
    assert call(128, Z=0x6000000) == -7        # checks of sphattn_fwd_z apply: Z is O


def test_splitkv_slice_counts_never_divide_by_zero(lib):
    """Any n_splits >= 0 is accepted: more slices than 64-key tiles means one tile per slice.
    (INT_MAX used to overflow the ceiling division and end the process with SIGFPE.)"""
    P = ctypes.c_void_p
    wsb = lib.sphattn_splitkv_workspace_bytes
    N, d = 1024, 128                            # 16 tiles
    for n_splits in (17, 1000, 2 ** 31 - 1):
        rc = lib.sphattn_splitkv_fwd(P(0x1000), P(0x2000000), P(0x4000000), P(0), P(0x6000000), P(0),
                                     1, 1, 1, N, d, 1, n_splits, P(0x10000000), wsb(1, 1, N, d, 16) - 1, None)
        assert rc == -9                          # 16 slices planned: one byte short of their workspace
    assert lib.sphattn_splitkv_heuristic(1, 1, 2 ** 31 - 1, 128, 1) >= 1


def test_noalloc_entry_point_checks_before_it_needs_a_device(lib):
    P = ctypes.c_void_p

    def call(Q=0x1000000, O=0x4000000, B=1, H=1, N=1024, d=128, dtype=1, n_splits=4, H_kv=1):
        return lib.sphattn_splitkv_fwd_noalloc(P(Q), P(0x2000000), P(0x3000000), P(0), P(O), P(0),
                                               B, H, H_kv, N, d, dtype, n_splits, None)
    assert call(Q=0) == -1 and call(N=0) == -2 and call(d=100) == -3 and call(dtype=8) == -4
    assert call(O=0x4000008) == -5 and call(O=0x1000000) == -7 and call(n_splits=-1) == -2
    # 8 heads of 32768 rows in 2 slices: 270 MB of partial pairs, more than the library's array
    assert lib.sphattn_splitkv_workspace_bytes(1, 8, 32768, 128, 2) > (64 << 20)
    assert call(H=8, H_kv=8, N=32768, n_splits=2, O=0x40000000) == -10
    assert b"scratch" in lib.sphattn_strerror(-10)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
