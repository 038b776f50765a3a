"""CPU oracle for spherical attention -- TEST INFRASTRUCTURE, not the product.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It shares no code with the HIP library and never imports it.

The arithmetic lives in ``sphattn_oracle.c`` (plain fp64 C, two passes per query
row, straight from the paper's definition of a normalized contraction in
Appendix A.1 with a1 = id, a2 = square, b = sqrt; Section 3).  This module only
compiles that file with gcc and marshals numpy arrays into it.

Stored formats understood for the inputs ("kind"):
    "f64", "f32"  -- numpy float64 / float32 arrays
    "bf16"        -- numpy uint16 arrays holding bfloat16 bit patterns
    "e4m3fn"      -- numpy uint8 arrays holding OCP E4M3 (finite-only) bytes
    "f16"         -- numpy uint16 arrays holding IEEE binary16 bit patterns
All are widened exactly to fp64 inside the C code.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sphattn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_sphattn.so")

_KINDS = {"f64": 0, "f32": 1, "bf16": 2, "e4m3fn": 3, "f16": 4}
_KIND_DTYPES = {"f64": np.float64, "f32": np.float32, "bf16": np.uint16, "e4m3fn": np.uint8,
                "f16": np.uint16}

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP, no fast-math). Returns the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, ip, dp = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_double)
        lib.oracle_attention_fwd.restype = ip
        lib.oracle_attention_fwd.argtypes = [ip, vp, ip, vp, ip, vp, ip, dp, dp, dp, ip, ip, ip, ip]
        lib.oracle_attention_rows.restype = ip
        lib.oracle_attention_rows.argtypes = [ip, vp, ip, vp, ip, vp, ip, dp, ip, ip, ip, ip, ip,
                                              ctypes.POINTER(ctypes.c_int), ip]
        lib.oracle_attention_fwd_grn.restype = ip
        lib.oracle_attention_fwd_grn.argtypes = [ip, vp, ip, vp, ip, vp, ip, dp, dp, dp, dp, ip, ip, ip, ip, ip]
        lib.oracle_attention_rows_grn.restype = ip
        lib.oracle_attention_rows_grn.argtypes = [ip, vp, ip, vp, ip, vp, ip, dp, dp, ip, ip, ip, ip, ip, ip,
                                                  ctypes.POINTER(ctypes.c_int), ip]
        lib.oracle_spherical_streamed.restype = ip
        lib.oracle_spherical_streamed.argtypes = [dp, dp, dp, dp, ip, ip, ip, ip, ip]
        lib.oracle_spherical_accumulate.restype = ip
        lib.oracle_spherical_accumulate.argtypes = [vp, ip, vp, ip, vp, ip, dp, dp, dp, ip, ip, ip, ip, ip, ip]
        lib.oracle_spherical_bwd.restype = ip
        lib.oracle_spherical_bwd.argtypes = [vp, ip, vp, ip, vp, ip, vp, ip, dp, dp, dp, ip, ip, ip, ip]
        lib.oracle_spherical_bwd_grn.restype = ip
        lib.oracle_spherical_bwd_grn.argtypes = [vp, ip, vp, ip, vp, ip, vp, ip, dp, dp, dp, dp, ip, ip, ip, ip, ip]
        lib.oracle_widen.restype = None
        lib.oracle_widen.argtypes = [vp, ip, ctypes.c_size_t, ctypes.c_size_t, dp]
        lib.oracle_num_threads.restype = ip
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _kind_of(a: np.ndarray, kind: str | None) -> str:
    if kind is None:
        if a.dtype == np.float64:
            kind = "f64"
        elif a.dtype == np.float32:
            kind = "f32"
        else:
            raise TypeError("kind must be given for arrays that are not float32/float64")
    if kind not in _KINDS:
        raise ValueError(f"unknown kind {kind!r}")
    if a.dtype != _KIND_DTYPES[kind]:
        raise TypeError(f"kind {kind!r} needs dtype {_KIND_DTYPES[kind]}, got {a.dtype}")
    return kind


def _prep(a, kind):
    a = np.ascontiguousarray(a)
    kind = _kind_of(a, kind)
    if a.ndim != 4:
        raise ValueError("expected a [B,H,N,d] array")
    return a, kind


def _dptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def num_threads() -> int:
    """Threads the OpenMP loops will use."""
    return int(_load().oracle_num_threads())


def widen(a: np.ndarray, kind: str | None = None) -> np.ndarray:
    """Exact fp64 values of a stored array (any shape)."""
    a = np.ascontiguousarray(a)
    kind = _kind_of(a, kind)
    out = np.empty(a.shape, dtype=np.float64)
    _load().oracle_widen(a.ctypes.data_as(ctypes.c_void_p), _KINDS[kind], 0, a.size, _dptr(out))
    return out


def _fwd(mode, Q, K, V, kinds, want_weights, want_z):
    kq, kk, kv = kinds if kinds is not None else (None, None, None)
    Q, kq = _prep(Q, kq)
    K, kk = _prep(K, kk)
    V, kv = _prep(V, kv)
    if not (Q.shape == K.shape == V.shape):
        raise ValueError("Q, K, V must share the shape [B,H,N,d]")
    B, H, N, d = Q.shape
    O = np.empty((B, H, N, d), dtype=np.float64)
    W = np.empty((B, H, N, N), dtype=np.float64) if want_weights else None
    Z = np.empty((B, H, N), dtype=np.float64) if want_z else None
    rc = _load().oracle_attention_fwd(
        mode, Q.ctypes.data_as(ctypes.c_void_p), _KINDS[kq],
        K.ctypes.data_as(ctypes.c_void_p), _KINDS[kk],
        V.ctypes.data_as(ctypes.c_void_p), _KINDS[kv],
        _dptr(O), _dptr(W) if W is not None else None, _dptr(Z) if Z is not None else None,
        B, H, N, d)
    if rc != 0:
        raise RuntimeError(f"oracle_attention_fwd failed with {rc}")
    return O, W, Z


def spherical_attention(Q, K, V, kinds=None) -> np.ndarray:
    """O = (S V) / ||S row||_2 with S = Q K^T, fp64, [B,H,N,d]."""
    return _fwd(0, Q, K, V, kinds, False, False)[0]


def spherical_attention_full(Q, K, V, kinds=None):
    """(O, W, Z): output, normalized weights [B,H,N,N], squared row norms [B,H,N]."""
    return _fwd(0, Q, K, V, kinds, True, True)


def softmax_attention(Q, K, V, kinds=None) -> np.ndarray:
    """Comparison twin: softmax(Q K^T / sqrt(d)) V, fp64."""
    return _fwd(1, Q, K, V, kinds, False, False)[0]


NORMALIZERS = {"l2": 0, "softmax": 1, "l1": 2, "sqrelu": 3}


def normalized_attention(Q, K, V, normalizer: str, kinds=None) -> np.ndarray:
    """Attention with the normalizer of Definition 2 named by `normalizer`:
    "l2" (spherical), "softmax" (with 1/sqrt(d)), "l1" (x / sum|x|), "sqrelu" (relu(x)^2 / sum relu(x)^2)."""
    return _fwd(NORMALIZERS[normalizer], Q, K, V, kinds, False, False)[0]


def normalized_attention_rows(Q, K, V, normalizer: str, bh: int, rows, kinds=None) -> np.ndarray:
    return _rows(NORMALIZERS[normalizer], Q, K, V, bh, rows, kinds)


def _rows(mode, Q, K, V, bh, rows, kinds):
    kq, kk, kv = kinds if kinds is not None else (None, None, None)
    Q, kq = _prep(Q, kq)
    K, kk = _prep(K, kk)
    V, kv = _prep(V, kv)
    B, H, N, d = Q.shape
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty((rows.size, d), dtype=np.float64)
    rc = _load().oracle_attention_rows(
        mode, Q.ctypes.data_as(ctypes.c_void_p), _KINDS[kq],
        K.ctypes.data_as(ctypes.c_void_p), _KINDS[kk],
        V.ctypes.data_as(ctypes.c_void_p), _KINDS[kv],
        _dptr(out), B, H, N, d, int(bh),
        rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), int(rows.size))
    if rc != 0:
        raise RuntimeError(f"oracle_attention_rows failed with {rc}")
    return out


def spherical_attention_rows(Q, K, V, bh: int, rows, kinds=None) -> np.ndarray:
    """Output rows `rows` of flattened head index `bh` (= b*H + h): [len(rows), d]."""
    return _rows(0, Q, K, V, bh, rows, kinds)


def softmax_attention_rows(Q, K, V, bh: int, rows, kinds=None) -> np.ndarray:
    return _rows(1, Q, K, V, bh, rows, kinds)


def spherical_attention_streamed(Q, K, V, chunk: int) -> np.ndarray:
    """Lemma 1's loop: carry (o, z) over key chunks of size `chunk`, then o/sqrt(z)."""
    Q = np.ascontiguousarray(Q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    B, H, N, d = Q.shape
    O = np.empty_like(Q)
    rc = _load().oracle_spherical_streamed(_dptr(Q), _dptr(K), _dptr(V), _dptr(O),
                                           B, H, N, d, int(chunk))
    if rc != 0:
        raise RuntimeError(f"oracle_spherical_streamed failed with {rc}")
    return O


def _prep_mult(mult, B, N):
    if mult is None:
        return None
    m = np.ascontiguousarray(mult, dtype=np.float64)
    if m.shape != (B, N):
        raise ValueError("mult must have shape [B, N]")
    return m


def grn_attention(Q, K, V, mult=None, kinds=None) -> np.ndarray:
    """Gene-regulatory-network variant: s_ij = q_i . (m_j k_j) with per-cell multiplicities
    mult[B,N] (None = all ones) and grouped K/V heads (K, V are [B,H_kv,N,d], H % H_kv == 0)."""
    kq, kk, kv = kinds if kinds is not None else (None, None, None)
    Q, kq = _prep(Q, kq)
    K, kk = _prep(K, kk)
    V, kv = _prep(V, kv)
    B, H, N, d = Q.shape
    if K.shape != V.shape or K.shape[0] != B or K.shape[2:] != (N, d):
        raise ValueError("K, V must be [B,H_kv,N,d]")
    H_kv = K.shape[1]
    m = _prep_mult(mult, B, N)
    O = np.empty((B, H, N, d), dtype=np.float64)
    rc = _load().oracle_attention_fwd_grn(
        0, Q.ctypes.data_as(ctypes.c_void_p), _KINDS[kq], K.ctypes.data_as(ctypes.c_void_p), _KINDS[kk],
        V.ctypes.data_as(ctypes.c_void_p), _KINDS[kv], _dptr(m) if m is not None else None,
        _dptr(O), None, None, B, H, H_kv, N, d)
    if rc != 0:
        raise RuntimeError(f"oracle_attention_fwd_grn failed with {rc}")
    return O


def grn_attention_rows(Q, K, V, mult, bh: int, rows, kinds=None) -> np.ndarray:
    """Rows `rows` of query head `bh` (= b*H + h) of the GRN variant: [len(rows), d]."""
    kq, kk, kv = kinds if kinds is not None else (None, None, None)
    Q, kq = _prep(Q, kq)
    K, kk = _prep(K, kk)
    V, kv = _prep(V, kv)
    B, H, N, d = Q.shape
    H_kv = K.shape[1]
    m = _prep_mult(mult, B, N)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    out = np.empty((rows.size, d), dtype=np.float64)
    rc = _load().oracle_attention_rows_grn(
        0, Q.ctypes.data_as(ctypes.c_void_p), _KINDS[kq], K.ctypes.data_as(ctypes.c_void_p), _KINDS[kk],
        V.ctypes.data_as(ctypes.c_void_p), _KINDS[kv], _dptr(m) if m is not None else None,
        _dptr(out), B, H, H_kv, N, d, int(bh),
        rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int)), int(rows.size))
    if rc != 0:
        raise RuntimeError(f"oracle_attention_rows_grn failed with {rc}")
    return out


def spherical_accumulate(Q, K, V, mult=None, kinds=None):
    """The accumulator of Lemma 1 without its tail: (o_raw [B,H,N_q,d], z [B,H,N_q]) of the
    query rows Q [B,H,N_q,d] over the keys/values K, V [B,H_kv,N_k,d] (mult [B,N_k] or None)."""
    kq, kk, kv = kinds if kinds is not None else (None, None, None)
    Q, kq = _prep(Q, kq)
    K, kk = _prep(K, kk)
    V, kv = _prep(V, kv)
    B, H, Nq, d = Q.shape
    if K.shape != V.shape or K.shape[0] != B or K.shape[3] != d:
        raise ValueError("K, V must be [B,H_kv,N_k,d]")
    H_kv, Nk = K.shape[1], K.shape[2]
    m = _prep_mult(mult, B, Nk)
    o_raw = np.empty((B, H, Nq, d), dtype=np.float64)
    z = np.empty((B, H, Nq), dtype=np.float64)
    rc = _load().oracle_spherical_accumulate(
        Q.ctypes.data_as(ctypes.c_void_p), _KINDS[kq], K.ctypes.data_as(ctypes.c_void_p), _KINDS[kk],
        V.ctypes.data_as(ctypes.c_void_p), _KINDS[kv], _dptr(m) if m is not None else None,
        _dptr(o_raw), _dptr(z), B, H, H_kv, Nq, Nk, d)
    if rc != 0:
        raise RuntimeError(f"oracle_spherical_accumulate failed with {rc}")
    return o_raw, z


def spherical_tail(o_parts, z_parts) -> np.ndarray:
    """Lemma 1's tail on a sum of accumulators: t(sum_p o_p, sum_p z_p) = o / sqrt(z), 0 where
    z = 0.  o_parts [P,B,H,N,d], z_parts [P,B,H,N] (fp64)."""
    o = np.asarray(o_parts, dtype=np.float64).sum(axis=0)
    z = np.asarray(z_parts, dtype=np.float64).sum(axis=0)
    out = np.zeros_like(o)
    nz = z > 0.0
    out[nz] = o[nz] / np.sqrt(z[nz])[:, None]
    return out


def spherical_attention_bwd(Q, K, V, dO, kinds=None):
    """Gradients (dQ, dK, dV), fp64 [B,H,N,d], of sum(O * dO) for spherical attention O(Q, K, V);
    kinds = (q, k, v, dO) stored formats."""
    kq, kk, kv, kg = kinds if kinds is not None else (None, None, None, None)
    Q, kq = _prep(Q, kq)
    K, kk = _prep(K, kk)
    V, kv = _prep(V, kv)
    dO, kg = _prep(dO, kg)
    if not (Q.shape == K.shape == V.shape == dO.shape):
        raise ValueError("Q, K, V, dO must share the shape [B,H,N,d]")
    B, H, N, d = Q.shape
    dQ, dK, dV = (np.empty((B, H, N, d), dtype=np.float64) for _ in range(3))
    rc = _load().oracle_spherical_bwd(
        Q.ctypes.data_as(ctypes.c_void_p), _KINDS[kq], K.ctypes.data_as(ctypes.c_void_p), _KINDS[kk],
        V.ctypes.data_as(ctypes.c_void_p), _KINDS[kv], dO.ctypes.data_as(ctypes.c_void_p), _KINDS[kg],
        _dptr(dQ), _dptr(dK), _dptr(dV), B, H, N, d)
    if rc != 0:
        raise RuntimeError(f"oracle_spherical_bwd failed with {rc}")
    return dQ, dK, dV


def grn_attention_bwd(Q, K, V, dO, mult=None, kinds=None):
    """Gradients (dQ [B,H,N,d], dK, dV [B,H_kv,N,d]) of sum(O * dO) for the gene-regulatory-network
    variant O = grn_attention(Q, K, V, mult); kinds = (q, k, v, dO) stored formats."""
    kq, kk, kv, kg = kinds if kinds is not None else (None, None, None, None)
    Q, kq = _prep(Q, kq)
    K, kk = _prep(K, kk)
    V, kv = _prep(V, kv)
    dO, kg = _prep(dO, kg)
    B, H, N, d = Q.shape
    if K.shape != V.shape or K.shape[0] != B or K.shape[2:] != (N, d) or dO.shape != Q.shape:
        raise ValueError("K, V must be [B,H_kv,N,d] and dO like Q")
    H_kv = K.shape[1]
    m = _prep_mult(mult, B, N)
    dQ = np.empty((B, H, N, d), dtype=np.float64)
    dK, dV = (np.empty((B, H_kv, N, d), dtype=np.float64) for _ in range(2))
    rc = _load().oracle_spherical_bwd_grn(
        Q.ctypes.data_as(ctypes.c_void_p), _KINDS[kq], K.ctypes.data_as(ctypes.c_void_p), _KINDS[kk],
        V.ctypes.data_as(ctypes.c_void_p), _KINDS[kv], dO.ctypes.data_as(ctypes.c_void_p), _KINDS[kg],
        _dptr(m) if m is not None else None, _dptr(dQ), _dptr(dK), _dptr(dV), B, H, H_kv, N, d)
    if rc != 0:
        raise RuntimeError(f"oracle_spherical_bwd_grn failed with {rc}")
    return dQ, dK, dV
