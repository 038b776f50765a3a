"""The Python binding checks shapes and element types before it hands pointers to the C ABI
(which cannot see buffer sizes): a mismatch must raise ValueError and touch no device.  These
run without a GPU: all tensors are CPU tensors, so a call that passed every shape and dtype
check ends with "must be a device tensor" -- also a ValueError, also before any launch."""
import pytest
import torch

import paper_2505_09326_amd as pkg
from paper_2505_09326_amd import autograd as sph_autograd


def _t(*shape, dtype=torch.bfloat16):
    return torch.zeros(shape, dtype=dtype)


def test_forward_rejects_shapes_that_would_read_past_the_buffers():
    q, k, v = _t(1, 2, 64, 128), _t(1, 2, 64, 128), _t(1, 2, 64, 128)
    with pytest.raises(ValueError, match="device tensor"):        # everything matches: only the device is wrong
        pkg.sphattn_fwd(q, k, v, dtype="bf16")
    with pytest.raises(ValueError, match="K must have Q's N"):
        pkg.sphattn_fwd(q, _t(1, 2, 32, 128), _t(1, 2, 32, 128), dtype="bf16")
    with pytest.raises(ValueError, match="V must have shape"):
        pkg.sphattn_fwd(q, k, _t(1, 2, 32, 128), dtype="bf16")
    with pytest.raises(ValueError, match="K must have Q's 2 heads"):
        pkg.sphattn_fwd(q, _t(1, 1, 64, 128), _t(1, 1, 64, 128), dtype="bf16")
    with pytest.raises(ValueError, match="with Q's B and d"):
        pkg.sphattn_fwd(q, _t(1, 2, 64, 64), _t(1, 2, 64, 64), dtype="bf16")
    with pytest.raises(ValueError, match="O must have shape"):
        pkg.sphattn_fwd(q, k, v, O=_t(1, 2, 63, 128), dtype="bf16")
    with pytest.raises(ValueError, match=r"\[B,H,N,d\]"):
        pkg.sphattn_fwd(_t(64, 128), k, v, dtype="bf16")


def test_forward_rejects_element_types_that_do_not_match_the_dtype_code():
    q, k, v = _t(1, 1, 64, 64), _t(1, 1, 64, 64), _t(1, 1, 64, 64)
    with pytest.raises(ValueError, match="Q must have dtype torch.float32"):
        pkg.sphattn_fwd(q, k, v, dtype="f32")                      # 4-byte reads of 2-byte buffers
    with pytest.raises(ValueError, match="Q must have dtype torch.float16"):
        pkg.sphattn_fwd(q, k, v, dtype="f16")
    with pytest.raises(ValueError, match="O must have dtype torch.bfloat16"):
        pkg.sphattn_fwd(q, k, v, O=_t(1, 1, 64, 64, dtype=torch.float32), dtype="bf16")
    q8 = _t(1, 1, 64, 64, dtype=torch.float8_e4m3fn)
    with pytest.raises(ValueError, match="device tensor"):
        pkg.sphattn_fwd(q8, q8, v, dtype="fp8qk_bf16v")
    with pytest.raises(ValueError, match="V must have dtype torch.bfloat16"):
        pkg.sphattn_fwd(q8, q8, q8, dtype="fp8qk_bf16v")
    with pytest.raises(ValueError, match="contiguous"):
        pkg.sphattn_fwd(_t(1, 1, 64, 128)[..., ::2], k, v, dtype="bf16")


def test_grn_cross_partial_and_split_shapes():
    q, k, v = _t(2, 4, 100, 64), _t(2, 2, 100, 64), _t(2, 2, 100, 64)
    with pytest.raises(ValueError, match="device tensor"):
        pkg.sphattn_grn_fwd(q, k, v, mult=_t(2, 100, dtype=torch.float32))
    with pytest.raises(ValueError, match="mult must have shape"):
        pkg.sphattn_grn_fwd(q, k, v, mult=_t(2, 99, dtype=torch.float32))
    with pytest.raises(ValueError, match="mult must have dtype"):
        pkg.sphattn_grn_fwd(q, k, v, mult=_t(2, 100))
    with pytest.raises(ValueError, match="must divide"):
        pkg.sphattn_grn_fwd(q, _t(2, 3, 100, 64), _t(2, 3, 100, 64))
    k2, v2 = _t(2, 2, 300, 64), _t(2, 2, 300, 64)
    with pytest.raises(ValueError, match="self-attention"):
        pkg.sphattn_grn_fwd(q, k2, v2)
    with pytest.raises(ValueError, match="device tensor"):        # rectangular is what cross is for
        pkg.sphattn_cross_fwd(q, k2, v2, mult=_t(2, 300, dtype=torch.float32))
    with pytest.raises(ValueError, match="mult must have shape"):  # ... with N_k multiplicities
        pkg.sphattn_cross_fwd(q, k2, v2, mult=_t(2, 100, dtype=torch.float32))
    with pytest.raises(ValueError, match="Z must have shape"):
        pkg.sphattn_cross_fwd(q, k2, v2, Z=_t(2, 4, 300, dtype=torch.float32))
    with pytest.raises(ValueError, match="o_part must have dtype"):
        pkg.sphattn_partial_fwd(q, k2, v2, o_part=_t(2, 4, 100, 64))
    with pytest.raises(ValueError, match="z_parts must have shape"):
        pkg.sphattn_combine(_t(3, 1, 2, 50, 64, dtype=torch.float32), _t(3, 1, 2, 49, dtype=torch.float32))
    with pytest.raises(ValueError, match="workspace"):
        pkg.sphattn_splitkv_fwd(q, k, v, workspace=_t(4, 4, dtype=torch.uint8))


def test_backward_shapes_and_autograd_rejects_cross_attention():
    q, k, v = _t(1, 4, 128, 64), _t(1, 2, 128, 64), _t(1, 2, 128, 64)
    o, do = _t(1, 4, 128, 64), _t(1, 4, 128, 64)
    z = _t(1, 4, 128, dtype=torch.float32)
    with pytest.raises(ValueError, match="device tensor"):
        pkg.sphattn_grn_bwd(q, k, v, None, o, do, z)
    with pytest.raises(ValueError, match="self-attention"):        # would write dK/dV past K-sized buffers
        pkg.sphattn_grn_bwd(q, _t(1, 2, 64, 64), _t(1, 2, 64, 64), None, o, do, z)
    with pytest.raises(ValueError, match="dO must have shape"):
        pkg.sphattn_grn_bwd(q, k, v, None, o, _t(1, 4, 127, 64), z)
    with pytest.raises(ValueError, match="Z must have shape"):
        pkg.sphattn_grn_bwd(q, k, v, None, o, do, _t(1, 4, 127, dtype=torch.float32))
    with pytest.raises(ValueError, match="dK must have shape"):
        pkg.sphattn_grn_bwd(q, k, v, None, o, do, z, dK=_t(1, 4, 128, 64))
    with pytest.raises(ValueError, match="16-bit"):
        pkg.sphattn_grn_bwd(q, k, v, None, o, do, z, dtype="f32")
    with pytest.raises(ValueError, match="heads"):
        pkg.sphattn_bwd(q, k, v, o, do, z)
    with pytest.raises(ValueError, match="Q's N"):
        sph_autograd.spherical_attention(q, _t(1, 2, 64, 64), _t(1, 2, 64, 64))
    with pytest.raises(TypeError):
        sph_autograd.spherical_attention(q.float(), k.float(), v.float())


def test_fp8_entry_points():
    q = _t(1, 2, 256, 128, dtype=torch.float8_e4m3fn)
    ws = _t(1 << 16, dtype=torch.uint8)
    with pytest.raises(ValueError, match="device tensor"):
        pkg.sphattn_fp8_fwd(q, q, q, ws)
    with pytest.raises(ValueError, match="V must have dtype"):
        pkg.sphattn_fp8_fwd(q, q, _t(1, 2, 256, 128), ws)
    with pytest.raises(ValueError, match="self-attention"):
        pkg.sphattn_fp8_fwd(q, q[:, :, :128].contiguous(), q[:, :, :128].contiguous(), ws)
    with pytest.raises(ValueError, match="O must have dtype"):
        pkg.sphattn_fp8_softmax_fwd(q, q, q, ws, O=_t(1, 2, 256, 128, dtype=torch.float16))
