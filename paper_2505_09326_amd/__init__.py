"""Spherical attention forward for AMD MI355X: thin binding over libsphattn.so.

Every step of the computation runs in the HIP kernels behind the C ABI of
include/sphattn.h; this module only marshals torch tensors (device memory and
streams) into that ABI.  There is no fallback: if the library has not been
built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
import os

from ._build import LIB_PATH, build_library

SPHATTN_F32 = 0
SPHATTN_BF16 = 1
SPHATTN_FP8QK_BF16V = 2
SPHATTN_F16 = 3

_DTYPE_NAMES = {"f32": SPHATTN_F32, "bf16": SPHATTN_BF16, "fp8qk_bf16v": SPHATTN_FP8QK_BF16V,
                "f16": SPHATTN_F16}

EXPORTED_SYMBOLS = ("sphattn_fwd", "sphattn_fwd_z", "sphattn_grn_fwd", "sphattn_normalized_fwd",
                    "sphattn_softmax_fwd", "sphattn_cross_fwd", "sphattn_partial_fwd", "sphattn_combine", "sphattn_splitkv_fwd",
                    "sphattn_splitkv_workspace_bytes", "sphattn_splitkv_heuristic", "sphattn_bwd", "sphattn_grn_bwd",
                    "sphattn_fp8_workspace_bytes", "sphattn_fp8_fwd", "sphattn_fp8_softmax_fwd", "sphattn_mfma_probe",
                    "sphattn_strerror", "sphattn_version")

NORMALIZERS = {"l2": 0, "softmax": 1, "l1": 2, "sqrelu": 3}

_lib = None


class SphattnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"sphattn error {code}: {text}")
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load the built library; raise if it is missing (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        path = os.environ.get("SPHATTN_LIBRARY", LIB_PATH)   # another build of the same library
        if not os.path.exists(path):
            raise ImportError(
                f"{path} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = ctypes.CDLL(path)
        vp, ip = ctypes.c_void_p, ctypes.c_int
        for name in ("sphattn_fwd", "sphattn_softmax_fwd"):
            fn = getattr(lib, name)
            fn.restype = ip
            fn.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, ip, vp]
        lib.sphattn_grn_fwd.restype = ip
        lib.sphattn_grn_fwd.argtypes = [vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_normalized_fwd.restype = ip
        lib.sphattn_normalized_fwd.argtypes = [vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_fwd_z.restype = ip
        lib.sphattn_fwd_z.argtypes = [vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, vp]
        lib.sphattn_cross_fwd.restype = ip
        lib.sphattn_cross_fwd.argtypes = [vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_partial_fwd.restype = ip
        lib.sphattn_partial_fwd.argtypes = [vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_combine.restype = ip
        lib.sphattn_combine.argtypes = [vp, vp, ip, vp, vp, ip, ip, ip, ip, ip, vp]
        lib.sphattn_splitkv_fwd.restype = ip
        lib.sphattn_splitkv_fwd.argtypes = [vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip,
                                            vp, ctypes.c_size_t, vp]
        lib.sphattn_splitkv_workspace_bytes.restype = ctypes.c_size_t
        lib.sphattn_splitkv_workspace_bytes.argtypes = [ip, ip, ip, ip, ip]
        lib.sphattn_splitkv_heuristic.restype = ip
        lib.sphattn_splitkv_heuristic.argtypes = [ip, ip, ip, ip, ip]
        lib.sphattn_bwd.restype = ip
        lib.sphattn_bwd.argtypes = [vp] * 10 + [ip, ip, ip, ip, ip, vp]
        lib.sphattn_grn_bwd.restype = ip
        lib.sphattn_grn_bwd.argtypes = [vp] * 11 + [ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_fp8_workspace_bytes.restype = ctypes.c_size_t
        lib.sphattn_fp8_workspace_bytes.argtypes = [ip, ip, ip, ip]
        for name in ("sphattn_fp8_fwd", "sphattn_fp8_softmax_fwd"):
            fn = getattr(lib, name)
            fn.restype = ip
            fn.argtypes = [vp, vp, vp, vp, vp, ctypes.c_size_t, ip, ip, ip, ip, ip, vp]
        lib.sphattn_mfma_probe.restype = ip
        lib.sphattn_mfma_probe.argtypes = [vp, vp, ip, ip, vp]
        lib.sphattn_strerror.restype = ctypes.c_char_p
        lib.sphattn_strerror.argtypes = [ip]
        lib.sphattn_version.restype = ip
        lib.sphattn_version.argtypes = []
        _lib = lib
    return _lib


def sphattn_strerror(code: int) -> str:
    return load_library().sphattn_strerror(int(code)).decode()


def sphattn_version() -> int:
    return int(load_library().sphattn_version())


def _dtype_code(dtype) -> int:
    if isinstance(dtype, str):
        return _DTYPE_NAMES[dtype]
    return int(dtype)


def _call(fn_name, Q, K, V, O, dtype, stream):
    import torch
    lib = load_library()
    code = _dtype_code(dtype)
    for t in (Q, K, V, O):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("Q, K, V, O must be contiguous device tensors")
    B, H, N, d = Q.shape
    if stream is None:
        stream = torch.cuda.current_stream(Q.device).cuda_stream
    rc = getattr(lib, fn_name)(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                               B, H, N, d, code, ctypes.c_void_p(stream))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O


def _alloc_out(Q, V, dtype):
    import torch
    code = _dtype_code(dtype)
    dt = {SPHATTN_F32: torch.float32, SPHATTN_F16: torch.float16}.get(code, torch.bfloat16)
    return torch.empty(Q.shape, dtype=dt, device=Q.device)


def sphattn_fwd(Q, K, V, O=None, dtype="bf16", stream=None):
    """O = (Q K^T) V with each score row divided by its L2 norm; tensors are [B,H,N,d]."""
    if O is None:
        O = _alloc_out(Q, V, dtype)
    return _call("sphattn_fwd", Q, K, V, O, dtype, stream)


def sphattn_grn_fwd(Q, K, V, mult=None, O=None, dtype="bf16", stream=None):
    """Gene-regulatory-network variant: keys scaled by per-gene multiplicity mult[B,N] (fp32 or
    None) and K, V of shape [B,H_kv,N,d] shared by groups of H/H_kv query heads."""
    import torch
    lib = load_library()
    if O is None:
        O = _alloc_out(Q, V, dtype)
    tensors = (Q, K, V, O) + ((mult,) if mult is not None else ())
    for t in tensors:
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("Q, K, V, O, mult must be contiguous device tensors")
    if mult is not None and mult.dtype != torch.float32:
        raise ValueError("mult must be float32")
    B, H, N, d = Q.shape
    if stream is None:
        stream = torch.cuda.current_stream(Q.device).cuda_stream
    rc = lib.sphattn_grn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(),
                             mult.data_ptr() if mult is not None else None, O.data_ptr(),
                             B, H, K.shape[1], N, d, _dtype_code(dtype), ctypes.c_void_p(stream))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O


def sphattn_normalized_fwd(Q, K, V, O=None, dtype="bf16", normalizer="l2", stream=None):
    """Attention with the normalizer "l2", "softmax", "l1" or "sqrelu" in place of the SoftMax."""
    import torch
    lib = load_library()
    if O is None:
        O = _alloc_out(Q, V, dtype)
    for t in (Q, K, V, O):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("Q, K, V, O must be contiguous device tensors")
    B, H, N, d = Q.shape
    if stream is None:
        stream = torch.cuda.current_stream(Q.device).cuda_stream
    code = NORMALIZERS[normalizer] if isinstance(normalizer, str) else int(normalizer)
    rc = lib.sphattn_normalized_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                    B, H, N, d, _dtype_code(dtype), code, ctypes.c_void_p(stream))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O


def sphattn_softmax_fwd(Q, K, V, O=None, dtype="bf16", stream=None):
    """Comparison twin: softmax(Q K^T / sqrt(d)) V on the same tiling."""
    if O is None:
        O = _alloc_out(Q, V, dtype)
    return _call("sphattn_softmax_fwd", Q, K, V, O, dtype, stream)


def _check_device(names, *tensors):
    for t in tensors:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError(f"{names} must be contiguous device tensors")


def _stream_of(t, stream):
    import torch
    return torch.cuda.current_stream(t.device).cuda_stream if stream is None else stream


def _ptr(t):
    return t.data_ptr() if t is not None else None


def sphattn_fwd_z(Q, K, V, O=None, Z=None, dtype="bf16", stream=None):
    """sphattn_fwd that also returns the row aggregates z_i = sum_j s_ij^2: (O, Z [B,H,N] fp32)."""
    import torch
    lib = load_library()
    if O is None:
        O = _alloc_out(Q, V, dtype)
    if Z is None:
        Z = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    _check_device("Q, K, V, O, Z", Q, K, V, O, Z)
    B, H, N, d = Q.shape
    rc = lib.sphattn_fwd_z(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), Z.data_ptr(),
                           B, H, N, d, _dtype_code(dtype), ctypes.c_void_p(_stream_of(Q, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O, Z


def sphattn_cross_fwd(Q, K, V, mult=None, O=None, Z=None, dtype="bf16", stream=None):
    """Spherical attention of Q [B,H,N_q,d] over the keys K, V [B,H_kv,N_k,d] (optional
    multiplicities mult [B,N_k], optional row aggregates Z [B,H,N_q]); returns O [B,H,N_q,d]."""
    import torch
    lib = load_library()
    if O is None:
        O = torch.empty(Q.shape, dtype=V.dtype, device=Q.device)
    _check_device("Q, K, V, mult, O, Z", Q, K, V, mult, O, Z)
    B, H, Nq, d = Q.shape
    rc = lib.sphattn_cross_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(), _ptr(Z),
                               B, H, K.shape[1], Nq, K.shape[2], d, _dtype_code(dtype),
                               ctypes.c_void_p(_stream_of(Q, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O


def sphattn_partial_fwd(Q, K, V, mult=None, o_part=None, z_part=None, dtype="bf16", stream=None):
    """Unnormalised accumulator pair of Q [B,H,N_q,d] over the keys K, V [B,H_kv,N_k,d]:
    (o_part [B,H,N_q,d] fp32, z_part [B,H,N_q] fp32)."""
    import torch
    lib = load_library()
    if o_part is None:
        o_part = torch.empty(Q.shape, dtype=torch.float32, device=Q.device)
    if z_part is None:
        z_part = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    _check_device("Q, K, V, mult, o_part, z_part", Q, K, V, mult, o_part, z_part)
    B, H, Nq, d = Q.shape
    rc = lib.sphattn_partial_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult),
                                 o_part.data_ptr(), z_part.data_ptr(), B, H, K.shape[1], Nq, K.shape[2], d,
                                 _dtype_code(dtype), ctypes.c_void_p(_stream_of(Q, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return o_part, z_part


def sphattn_combine(o_parts, z_parts, O=None, Z=None, dtype="bf16", stream=None):
    """Tail of the summed accumulators: o_parts [P,B,H,N,d], z_parts [P,B,H,N] (fp32) -> O."""
    import torch
    lib = load_library()
    P, B, H, N, d = o_parts.shape
    if O is None:
        code = _dtype_code(dtype)
        dt = {SPHATTN_F32: torch.float32, SPHATTN_F16: torch.float16}.get(code, torch.bfloat16)
        O = torch.empty((B, H, N, d), dtype=dt, device=o_parts.device)
    _check_device("o_parts, z_parts, O, Z", o_parts, z_parts, O, Z)
    rc = lib.sphattn_combine(o_parts.data_ptr(), z_parts.data_ptr(), P, O.data_ptr(), _ptr(Z),
                             B, H, N, d, _dtype_code(dtype), ctypes.c_void_p(_stream_of(o_parts, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O


def sphattn_splitkv_workspace_bytes(B, H, N, d, n_splits) -> int:
    return int(load_library().sphattn_splitkv_workspace_bytes(B, H, N, d, n_splits))


def sphattn_splitkv_heuristic(B, H, N, d, dtype="bf16") -> int:
    return int(load_library().sphattn_splitkv_heuristic(B, H, N, d, _dtype_code(dtype)))


def sphattn_splitkv_fwd(Q, K, V, workspace, mult=None, O=None, Z=None, n_splits=0, dtype="bf16", stream=None):
    """sphattn_grn_fwd with the key axis cut into n_splits slices (0: the library's choice);
    `workspace` is a device byte tensor of at least sphattn_splitkv_workspace_bytes(...)."""
    lib = load_library()
    if O is None:
        O = _alloc_out(Q, V, dtype)
    _check_device("Q, K, V, mult, O, Z, workspace", Q, K, V, mult, O, Z, workspace)
    B, H, N, d = Q.shape
    rc = lib.sphattn_splitkv_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(), _ptr(Z),
                                 B, H, K.shape[1], N, d, _dtype_code(dtype), int(n_splits),
                                 workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                 ctypes.c_void_p(_stream_of(Q, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O


def sphattn_fp8_workspace_bytes(B, H_kv, N, d) -> int:
    """Workspace of sphattn_fp8_fwd for K, V of shape [B,H_kv,N,d]."""
    return int(load_library().sphattn_fp8_workspace_bytes(B, H_kv, N, d))


def sphattn_fp8_softmax_fwd(Q, K, V, workspace, O=None, stream=None):
    """SoftMax comparison twin of sphattn_fp8_fwd (same arguments): for timing, on inputs of
    moderate size."""
    return sphattn_fp8_fwd(Q, K, V, workspace, O=O, stream=stream, _entry="sphattn_fp8_softmax_fwd")


def sphattn_fp8_fwd(Q, K, V, workspace, O=None, stream=None, _entry="sphattn_fp8_fwd"):
    """Spherical attention with Q [B,H,N,128], K and V [B,H_kv,N,128] all stored in E4M3
    (float8_e4m3fn tensors) and both contractions on the fp8 matrix instructions; O is bfloat16.
    `workspace` is a device byte tensor of at least sphattn_fp8_workspace_bytes(B, H_kv, N, 128)."""
    import torch
    lib = load_library()
    if O is None:
        O = torch.empty(Q.shape, dtype=torch.bfloat16, device=Q.device)
    _check_device("Q, K, V, O, workspace", Q, K, V, O, workspace)
    B, H, N, d = Q.shape
    rc = getattr(lib, _entry)(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), workspace.data_ptr(),
                              workspace.numel() * workspace.element_size(), B, H, K.shape[1], N, d,
                              ctypes.c_void_p(_stream_of(Q, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return O


def sphattn_bwd(Q, K, V, O, dO, Z, dQ=None, dK=None, dV=None, delta=None, dtype="bf16", stream=None):
    """Gradients (dQ, dK, dV) of sum(O * dO) for O, Z = sphattn_fwd_z(Q, K, V); 16-bit storage."""
    import torch
    lib = load_library()
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if delta is None:
        delta = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    _check_device("all arguments", Q, K, V, O, dO, Z, dQ, dK, dV, delta)
    B, H, N, d = Q.shape
    rc = lib.sphattn_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), Z.data_ptr(),
                         dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), delta.data_ptr(),
                         B, H, N, d, _dtype_code(dtype), ctypes.c_void_p(_stream_of(Q, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return dQ, dK, dV


def sphattn_grn_bwd(Q, K, V, mult, O, dO, Z, dQ=None, dK=None, dV=None, delta=None, dtype="bf16", stream=None):
    """Gradients (dQ, dK, dV) of sum(O * dO) for O = sphattn_grn_fwd(Q, K, V, mult): per-gene
    multiplicities mult[B,N] (or None) and K, V of shape [B,H_kv,N,d]."""
    import torch
    lib = load_library()
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if delta is None:
        delta = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    _check_device("all arguments", Q, K, V, mult, O, dO, Z, dQ, dK, dV, delta)
    B, H, N, d = Q.shape
    rc = lib.sphattn_grn_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(), dO.data_ptr(),
                             Z.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), delta.data_ptr(),
                             B, H, K.shape[1], N, d, _dtype_code(dtype), ctypes.c_void_p(_stream_of(Q, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return dQ, dK, dV


def sphattn_mfma_probe(operands, clocks, form: int, iters: int, stream=None):
    """Measurement aid: one launch of a loop of matrix instructions only (form 0: bf16 32x32x16,
    1: bf16 16x16x32, 2: E4M3 16x16x128; 3, 4: form 2 with an L2 / a SoftMax kernel's other
    instructions pinned behind every matrix instruction) on `operands` (64 KB device tensor); `clocks` (3 int64 on the device) receives
    shader clocks and 100 MHz ticks of workgroup 0.  Returns the flop count of the launch."""
    lib = load_library()
    _check_device("operands, clocks", operands, clocks)
    rc = lib.sphattn_mfma_probe(operands.data_ptr(), clocks.data_ptr(), int(form), int(iters),
                                ctypes.c_void_p(_stream_of(operands, stream)))
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))
    return 256.0 * 4 * iters * 16 * 32768.0
