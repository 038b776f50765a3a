"""Spherical attention forward for AMD MI355X: thin binding over libsphattn.so.

Every step of the computation runs in the HIP kernels behind the C ABI of
include/sphattn.h; this module only marshals torch tensors (device memory and
streams) into that ABI.  There is no fallback: if the library has not been
built, importing the entry points raises.

The C ABI cannot see how large a buffer behind a pointer is, so the binding checks what it
can see before any launch: every tensor's shape against the shapes the entry point's header
states, its torch dtype against the `dtype` code, contiguity and device.  A mismatch raises
ValueError; nothing is enqueued.
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

EXPORTED_SYMBOLS = ("sphattn_fwd", "sphattn_fwd_z", "sphattn_fwd_tile_rows", "sphattn_grn_fwd",
                    "sphattn_normalized_fwd", "sphattn_softmax_fwd", "sphattn_cross_fwd", "sphattn_partial_fwd",
                    "sphattn_combine", "sphattn_splitkv_fwd", "sphattn_splitkv_workspace_bytes",
                    "sphattn_splitkv_heuristic", "sphattn_splitkv_fwd_noalloc",
                    "sphattn_bwd", "sphattn_grn_bwd",
                    "sphattn_fp8_workspace_bytes", "sphattn_fp8_fwd", "sphattn_fp8_grn_fwd", "sphattn_fp8_softmax_fwd",
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
        vp, ip, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
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
        lib.sphattn_fwd_tile_rows.restype = ip
        lib.sphattn_fwd_tile_rows.argtypes = [vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_cross_fwd.restype = ip
        lib.sphattn_cross_fwd.argtypes = [vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_partial_fwd.restype = ip
        lib.sphattn_partial_fwd.argtypes = [vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_combine.restype = ip
        lib.sphattn_combine.argtypes = [vp, vp, ip, vp, vp, ip, ip, ip, ip, ip, vp]
        lib.sphattn_splitkv_fwd.restype = ip
        lib.sphattn_splitkv_fwd.argtypes = [vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, vp, sz, vp]
        lib.sphattn_splitkv_fwd_noalloc.restype = ip
        lib.sphattn_splitkv_fwd_noalloc.argtypes = [vp, vp, vp, vp, vp, vp, ip, ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_splitkv_workspace_bytes.restype = sz
        lib.sphattn_splitkv_workspace_bytes.argtypes = [ip, ip, ip, ip, ip]
        lib.sphattn_splitkv_heuristic.restype = ip
        lib.sphattn_splitkv_heuristic.argtypes = [ip, ip, ip, ip, ip]
        lib.sphattn_bwd.restype = ip
        lib.sphattn_bwd.argtypes = [vp] * 10 + [ip, ip, ip, ip, ip, vp]
        lib.sphattn_grn_bwd.restype = ip
        lib.sphattn_grn_bwd.argtypes = [vp] * 11 + [ip, ip, ip, ip, ip, ip, vp]
        lib.sphattn_fp8_workspace_bytes.restype = sz
        lib.sphattn_fp8_workspace_bytes.argtypes = [ip, ip, ip, ip]
        for name in ("sphattn_fp8_fwd", "sphattn_fp8_softmax_fwd"):
            fn = getattr(lib, name)
            fn.restype = ip
            fn.argtypes = [vp, vp, vp, vp, vp, sz, ip, ip, ip, ip, ip, vp]
        lib.sphattn_fp8_grn_fwd.restype = ip
        lib.sphattn_fp8_grn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, sz, ip, ip, ip, ip, ip, vp]
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


# ---- what the binding can check and the C ABI cannot: shapes and element types -------------

def _qk_types(code):
    import torch
    return {SPHATTN_F32: (torch.float32,), SPHATTN_BF16: (torch.bfloat16,), SPHATTN_F16: (torch.float16,),
            SPHATTN_FP8QK_BF16V: (torch.float8_e4m3fn, torch.uint8)}[code]


def _vo_types(code):
    import torch
    return {SPHATTN_F32: (torch.float32,), SPHATTN_F16: (torch.float16,)}.get(code, (torch.bfloat16,))


def _e4m3_types():
    import torch
    return (torch.float8_e4m3fn, torch.uint8)


def _f32_types():
    import torch
    return (torch.float32,)


def _need(name, t, shape, types, optional=False):
    """Shape, element type and contiguity of one argument (its device: _on_device, once the
    shapes of all arguments have been checked)."""
    if t is None:
        if optional:
            return
        raise ValueError(f"{name} is required")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    if t.dtype not in types:
        raise ValueError(f"{name} must have dtype {' or '.join(str(x) for x in types)}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def _on_device(**tensors):
    """All the (non-None) arguments of a call must live on one GPU."""
    first = None
    for name, t in tensors.items():
        if t is None:
            continue
        if not t.is_cuda:
            raise ValueError(f"{name} must be a device tensor")
        if first is None:
            first = (name, t.device)
        elif t.device != first[1]:
            raise ValueError(f"{name} is on {t.device}, {first[0]} on {first[1]}")


def _shape4(name, t):
    if t is None or t.dim() != 4:
        raise ValueError(f"{name} must be a [B,H,N,d] tensor")
    return tuple(int(x) for x in t.shape)


def _kv_shape(Q, K, same_n):
    """(B, H, N_q, d, H_kv, N_k) from Q [B,H,N_q,d] and K [B,H_kv,N_k,d]."""
    B, H, Nq, d = _shape4("Q", Q)
    Bk, H_kv, Nk, dk = _shape4("K", K)
    if Bk != B or dk != d:
        raise ValueError(f"K must be [B,H_kv,N_k,d] with Q's B and d, got {tuple(K.shape)} for Q {tuple(Q.shape)}")
    if H_kv <= 0 or H % H_kv != 0:
        raise ValueError(f"the number of K/V heads ({H_kv}) must divide the number of query heads ({H})")
    if same_n and Nk != Nq:
        raise ValueError(f"K must have Q's N ({Nq}), got {Nk}: this entry point is self-attention")
    return B, H, Nq, d, H_kv, Nk


def _check_forward(Q, K, V, O, mult, Z, code, same_n=True, same_h=False):
    B, H, Nq, d, H_kv, Nk = _kv_shape(Q, K, same_n)
    if same_h and H_kv != H:
        raise ValueError(f"K must have Q's {H} heads, got {H_kv}")
    _need("Q", Q, (B, H, Nq, d), _qk_types(code))
    _need("K", K, (B, H_kv, Nk, d), _qk_types(code))
    _need("V", V, (B, H_kv, Nk, d), _vo_types(code))
    _need("O", O, (B, H, Nq, d), _vo_types(code))
    _need("mult", mult, (B, Nk), _f32_types(), optional=True)
    _need("Z", Z, (B, H, Nq), _f32_types(), optional=True)
    _on_device(Q=Q, K=K, V=V, O=O, mult=mult, Z=Z)
    return B, H, Nq, d, H_kv, Nk


def _alloc_out(Q, dtype):
    import torch
    return torch.empty(Q.shape, dtype=_vo_types(_dtype_code(dtype))[0], device=Q.device)


def _stream_of(t, stream):
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream(t.device).cuda_stream if stream is None else stream)


def _ptr(t):
    return t.data_ptr() if t is not None else None


def _raise_on(rc):
    if rc != 0:
        raise SphattnError(rc, sphattn_strerror(rc))


# ---- entry points, same names as the C ABI ----------------------------------------------------

def sphattn_fwd(Q, K, V, O=None, dtype="bf16", stream=None):
    """O = (Q K^T) V with each score row divided by its L2 norm; tensors are [B,H,N,d]."""
    lib, code = load_library(), _dtype_code(dtype)
    if O is None:
        O = _alloc_out(Q, dtype)
    B, H, N, d, _, _ = _check_forward(Q, K, V, O, None, None, code, same_h=True)
    _raise_on(lib.sphattn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                              B, H, N, d, code, _stream_of(Q, stream)))
    return O


def sphattn_softmax_fwd(Q, K, V, O=None, dtype="bf16", stream=None):
    """Comparison twin: softmax(Q K^T / sqrt(d)) V on the same tiling."""
    lib, code = load_library(), _dtype_code(dtype)
    if O is None:
        O = _alloc_out(Q, dtype)
    B, H, N, d, _, _ = _check_forward(Q, K, V, O, None, None, code, same_h=True)
    _raise_on(lib.sphattn_softmax_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                      B, H, N, d, code, _stream_of(Q, stream)))
    return O


def sphattn_fwd_z(Q, K, V, O=None, Z=None, dtype="bf16", stream=None):
    """sphattn_fwd that also returns the row aggregates z_i = sum_j s_ij^2: (O, Z [B,H,N] fp32)."""
    return sphattn_fwd_tile_rows(Q, K, V, O=O, Z=Z, dtype=dtype, tile_rows=0, stream=stream, _want_z=True)


def sphattn_fwd_tile_rows(Q, K, V, O=None, Z=None, dtype="bf16", tile_rows=0, stream=None, _want_z=False):
    """sphattn_fwd_z with the workgroup shape forced to 128 or 256 query rows (0: the library's
    choice); returns (O, Z), Z being None unless given."""
    import torch
    lib, code = load_library(), _dtype_code(dtype)
    if O is None:
        O = _alloc_out(Q, dtype)
    if Z is None and _want_z:
        Z = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    B, H, N, d, _, _ = _check_forward(Q, K, V, O, None, Z, code, same_h=True)
    _raise_on(lib.sphattn_fwd_tile_rows(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), _ptr(Z),
                                        B, H, N, d, code, int(tile_rows), _stream_of(Q, stream)))
    return O, Z


def sphattn_grn_fwd(Q, K, V, mult=None, O=None, dtype="bf16", stream=None):
    """Gene-regulatory-network variant: keys scaled by per-gene multiplicity mult[B,N] (fp32 or
    None) and K, V of shape [B,H_kv,N,d] shared by groups of H/H_kv query heads."""
    lib, code = load_library(), _dtype_code(dtype)
    if O is None:
        O = _alloc_out(Q, dtype)
    B, H, N, d, H_kv, _ = _check_forward(Q, K, V, O, mult, None, code)
    _raise_on(lib.sphattn_grn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(),
                                  B, H, H_kv, N, d, code, _stream_of(Q, stream)))
    return O


def sphattn_normalized_fwd(Q, K, V, O=None, dtype="bf16", normalizer="l2", stream=None):
    """Attention with the normalizer "l2", "softmax", "l1" or "sqrelu" in place of the SoftMax."""
    lib, code = load_library(), _dtype_code(dtype)
    if O is None:
        O = _alloc_out(Q, dtype)
    B, H, N, d, _, _ = _check_forward(Q, K, V, O, None, None, code, same_h=True)
    norm = NORMALIZERS[normalizer] if isinstance(normalizer, str) else int(normalizer)
    _raise_on(lib.sphattn_normalized_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                         B, H, N, d, code, norm, _stream_of(Q, stream)))
    return O


def sphattn_cross_fwd(Q, K, V, mult=None, O=None, Z=None, dtype="bf16", stream=None):
    """Spherical attention of Q [B,H,N_q,d] over the keys K, V [B,H_kv,N_k,d] (optional
    multiplicities mult [B,N_k], optional row aggregates Z [B,H,N_q]); returns O [B,H,N_q,d]."""
    lib, code = load_library(), _dtype_code(dtype)
    if O is None:
        O = _alloc_out(Q, dtype)
    B, H, Nq, d, H_kv, Nk = _check_forward(Q, K, V, O, mult, Z, code, same_n=False)
    _raise_on(lib.sphattn_cross_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(), _ptr(Z),
                                    B, H, H_kv, Nq, Nk, d, code, _stream_of(Q, stream)))
    return O


def sphattn_partial_fwd(Q, K, V, mult=None, o_part=None, z_part=None, dtype="bf16", stream=None):
    """Unnormalised accumulator pair of Q [B,H,N_q,d] over the keys K, V [B,H_kv,N_k,d]:
    (o_part [B,H,N_q,d] fp32, z_part [B,H,N_q] fp32)."""
    import torch
    lib, code = load_library(), _dtype_code(dtype)
    if o_part is None:
        o_part = torch.empty(Q.shape, dtype=torch.float32, device=Q.device)
    if z_part is None:
        z_part = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    B, H, Nq, d, H_kv, Nk = _kv_shape(Q, K, same_n=False)
    _need("Q", Q, (B, H, Nq, d), _qk_types(code))
    _need("K", K, (B, H_kv, Nk, d), _qk_types(code))
    _need("V", V, (B, H_kv, Nk, d), _vo_types(code))
    _need("mult", mult, (B, Nk), _f32_types(), optional=True)
    _need("o_part", o_part, (B, H, Nq, d), _f32_types())
    _need("z_part", z_part, (B, H, Nq), _f32_types())
    _on_device(Q=Q, K=K, V=V, mult=mult, o_part=o_part, z_part=z_part)
    _raise_on(lib.sphattn_partial_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult),
                                      o_part.data_ptr(), z_part.data_ptr(), B, H, H_kv, Nq, Nk, d,
                                      code, _stream_of(Q, stream)))
    return o_part, z_part


def sphattn_combine(o_parts, z_parts, O=None, Z=None, dtype="bf16", stream=None):
    """Tail of the summed accumulators: o_parts [P,B,H,N,d], z_parts [P,B,H,N] (fp32) -> O."""
    import torch
    lib, code = load_library(), _dtype_code(dtype)
    if o_parts is None or o_parts.dim() != 5:
        raise ValueError("o_parts must be a [P,B,H,N,d] tensor")
    P, B, H, N, d = (int(x) for x in o_parts.shape)
    if O is None:
        O = torch.empty((B, H, N, d), dtype=_vo_types(code)[0], device=o_parts.device)
    _need("o_parts", o_parts, (P, B, H, N, d), _f32_types())
    _need("z_parts", z_parts, (P, B, H, N), _f32_types())
    _need("O", O, (B, H, N, d), _vo_types(code))
    _need("Z", Z, (B, H, N), _f32_types(), optional=True)
    _on_device(o_parts=o_parts, z_parts=z_parts, O=O, Z=Z)
    _raise_on(lib.sphattn_combine(o_parts.data_ptr(), z_parts.data_ptr(), P, O.data_ptr(), _ptr(Z),
                                  B, H, N, d, code, _stream_of(o_parts, stream)))
    return O


def sphattn_splitkv_workspace_bytes(B, H, N, d, n_splits) -> int:
    return int(load_library().sphattn_splitkv_workspace_bytes(B, H, N, d, n_splits))


def sphattn_splitkv_heuristic(B, H, N, d, dtype="bf16") -> int:
    return int(load_library().sphattn_splitkv_heuristic(B, H, N, d, _dtype_code(dtype)))


def _need_workspace(workspace):
    """Size in bytes of a workspace argument (its device is checked with the other arguments')."""
    if workspace is None or workspace.dim() != 1:
        raise ValueError("workspace must be a one-dimensional device byte tensor")
    _need("workspace", workspace, workspace.shape, (workspace.dtype,))
    return workspace.numel() * workspace.element_size()


def sphattn_splitkv_fwd(Q, K, V, workspace, mult=None, O=None, Z=None, n_splits=0, dtype="bf16", stream=None):
    """sphattn_grn_fwd with the key axis cut into n_splits slices (0: the library's choice);
    `workspace` is a device byte tensor of at least sphattn_splitkv_workspace_bytes(...)."""
    lib, code = load_library(), _dtype_code(dtype)
    if O is None:
        O = _alloc_out(Q, dtype)
    ws_bytes = _need_workspace(workspace)
    B, H, N, d, H_kv, _ = _check_forward(Q, K, V, O, mult, Z, code)
    _on_device(Q=Q, workspace=workspace)
    _raise_on(lib.sphattn_splitkv_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(), _ptr(Z),
                                      B, H, H_kv, N, d, code, int(n_splits),
                                      workspace.data_ptr(), ws_bytes, _stream_of(Q, stream)))
    return O


NOALLOC_SCRATCH_BYTES = 64 << 20   # SPHATTN_NOALLOC_SCRATCH_BYTES of include/sphattn.h


def sphattn_splitkv_fwd_noalloc(Q, K, V, O, mult=None, Z=None, n_splits=0, dtype="bf16", stream=None):
    """sphattn_splitkv_fwd on the library's own scratch array (NOALLOC_SCRATCH_BYTES): no
    workspace argument and no allocation anywhere in the call, so O must be given."""
    lib, code = load_library(), _dtype_code(dtype)
    B, H, N, d, H_kv, _ = _check_forward(Q, K, V, O, mult, Z, code)
    _raise_on(lib.sphattn_splitkv_fwd_noalloc(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(),
                                              _ptr(Z), B, H, H_kv, N, d, code, int(n_splits), _stream_of(Q, stream)))
    return O


def sphattn_fp8_workspace_bytes(B, H_kv, N, d) -> int:
    """Workspace of sphattn_fp8_fwd for K, V of shape [B,H_kv,N,d]."""
    return int(load_library().sphattn_fp8_workspace_bytes(B, H_kv, N, d))


def _check_fp8(Q, K, V, O, mult):
    import torch
    B, H, N, d, H_kv, _ = _kv_shape(Q, K, same_n=True)
    _need("Q", Q, (B, H, N, d), _e4m3_types())
    _need("K", K, (B, H_kv, N, d), _e4m3_types())
    _need("V", V, (B, H_kv, N, d), _e4m3_types())
    _need("O", O, (B, H, N, d), (torch.bfloat16,))
    _need("mult", mult, (B, N), _f32_types(), optional=True)
    _on_device(Q=Q, K=K, V=V, O=O, mult=mult)
    return B, H, N, d, H_kv


def sphattn_fp8_fwd(Q, K, V, workspace, O=None, stream=None, _entry="sphattn_fp8_fwd"):
    """Spherical attention with Q [B,H,N,d], K and V [B,H_kv,N,d] all stored in E4M3
    (float8_e4m3fn tensors) and both contractions on the fp8 matrix instructions; O is bfloat16.
    `workspace` is a device byte tensor of at least sphattn_fp8_workspace_bytes(B, H_kv, N, d)."""
    import torch
    lib = load_library()
    if O is None:
        O = torch.empty(Q.shape, dtype=torch.bfloat16, device=Q.device)
    ws_bytes = _need_workspace(workspace)
    B, H, N, d, H_kv = _check_fp8(Q, K, V, O, None)
    _on_device(Q=Q, workspace=workspace)
    _raise_on(getattr(lib, _entry)(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), workspace.data_ptr(),
                                   ws_bytes, B, H, H_kv, N, d, _stream_of(Q, stream)))
    return O


def sphattn_fp8_softmax_fwd(Q, K, V, workspace, O=None, stream=None):
    """SoftMax comparison twin of sphattn_fp8_fwd (same arguments): for timing, on inputs of
    moderate size."""
    return sphattn_fp8_fwd(Q, K, V, workspace, O=O, stream=stream, _entry="sphattn_fp8_softmax_fwd")


def sphattn_fp8_grn_fwd(Q, K, V, mult, workspace, O=None, stream=None):
    """sphattn_fp8_fwd with per-gene multiplicities mult [B,N] (fp32, or None) on the scores."""
    import torch
    lib = load_library()
    if O is None:
        O = torch.empty(Q.shape, dtype=torch.bfloat16, device=Q.device)
    ws_bytes = _need_workspace(workspace)
    B, H, N, d, H_kv = _check_fp8(Q, K, V, O, mult)
    _on_device(Q=Q, workspace=workspace)
    _raise_on(lib.sphattn_fp8_grn_fwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(),
                                      workspace.data_ptr(), ws_bytes, B, H, H_kv, N, d, _stream_of(Q, stream)))
    return O


def _check_backward(Q, K, V, mult, O, dO, Z, dQ, dK, dV, delta, code):
    import torch
    if code not in (SPHATTN_BF16, SPHATTN_F16):
        raise ValueError("the backward pass takes 16-bit storage (bf16 or f16)")
    B, H, N, d, H_kv, _ = _kv_shape(Q, K, same_n=True)
    t = _vo_types(code)
    for name, x in (("Q", Q), ("O", O), ("dO", dO), ("dQ", dQ)):
        _need(name, x, (B, H, N, d), t)
    for name, x in (("K", K), ("V", V), ("dK", dK), ("dV", dV)):
        _need(name, x, (B, H_kv, N, d), t)
    _need("Z", Z, (B, H, N), _f32_types())
    _need("delta", delta, (2, B, H, N), _f32_types())
    _need("mult", mult, (B, N), _f32_types(), optional=True)
    _on_device(Q=Q, K=K, V=V, mult=mult, O=O, dO=dO, Z=Z, dQ=dQ, dK=dK, dV=dV, delta=delta)
    return B, H, N, d, H_kv


def sphattn_grn_bwd(Q, K, V, mult, O, dO, Z, dQ=None, dK=None, dV=None, delta=None, dtype="bf16", stream=None):
    """Gradients (dQ, dK, dV) of sum(O * dO) for O = sphattn_grn_fwd(Q, K, V, mult): per-gene
    multiplicities mult[B,N] (or None) and K, V of shape [B,H_kv,N,d]."""
    import torch
    lib, code = load_library(), _dtype_code(dtype)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if delta is None:
        delta = torch.empty((2, *Q.shape[:3]), dtype=torch.float32, device=Q.device)
    B, H, N, d, H_kv = _check_backward(Q, K, V, mult, O, dO, Z, dQ, dK, dV, delta, code)
    _raise_on(lib.sphattn_grn_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), _ptr(mult), O.data_ptr(), dO.data_ptr(),
                                  Z.data_ptr(), dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), delta.data_ptr(),
                                  B, H, H_kv, N, d, code, _stream_of(Q, stream)))
    return dQ, dK, dV


def sphattn_bwd(Q, K, V, O, dO, Z, dQ=None, dK=None, dV=None, delta=None, dtype="bf16", stream=None):
    """Gradients (dQ, dK, dV) of sum(O * dO) for O, Z = sphattn_fwd_z(Q, K, V); 16-bit storage."""
    import torch
    lib, code = load_library(), _dtype_code(dtype)
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if delta is None:
        delta = torch.empty((2, *Q.shape[:3]), dtype=torch.float32, device=Q.device)
    if Q.dim() == 4 and K.dim() == 4 and K.shape[1] != Q.shape[1]:
        raise ValueError(f"K must have Q's {Q.shape[1]} heads, got {K.shape[1]} (sphattn_grn_bwd takes shared heads)")
    B, H, N, d, H_kv = _check_backward(Q, K, V, None, O, dO, Z, dQ, dK, dV, delta, code)
    _raise_on(lib.sphattn_bwd(Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), Z.data_ptr(),
                              dQ.data_ptr(), dK.data_ptr(), dV.data_ptr(), delta.data_ptr(),
                              B, H, N, d, code, _stream_of(Q, stream)))
    return dQ, dK, dV
