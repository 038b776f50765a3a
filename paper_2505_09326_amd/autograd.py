"""torch.autograd wrapper around the C ABI: argument marshalling only.

    from paper_2505_09326_amd.autograd import spherical_attention
    O = spherical_attention(Q, K, V)          # [B,H,N,d] bf16 or fp16 CUDA tensors
    O.sum().backward()                        # dQ, dK, dV from sphattn_bwd / sphattn_grn_bwd

Forward = sphattn_fwd_z (O and the row aggregates z, which the backward needs), or
sphattn_cross_fwd when multiplicities or shared K/V heads are given; backward = the library's
two backward kernels.  Nothing is computed here.
"""
import torch

from . import sphattn_bwd, sphattn_cross_fwd, sphattn_fwd_z, sphattn_grn_bwd

_DTYPES = {torch.bfloat16: "bf16", torch.float16: "f16"}


class _SphericalAttention(torch.autograd.Function):
    @staticmethod
    def forward(ctx, Q, K, V, mult):
        if Q.dtype not in _DTYPES or K.dtype != Q.dtype or V.dtype != Q.dtype:
            raise TypeError("spherical_attention differentiates bf16 or fp16 tensors of one dtype")
        if Q.dim() != 4 or K.dim() != 4 or K.shape[2] != Q.shape[2]:
            # the backward kernels are self-attention only; catch it before anything is launched
            raise ValueError(f"spherical_attention needs K, V with Q's N: Q {tuple(Q.shape)}, K {tuple(K.shape)}")
        dtype = _DTYPES[Q.dtype]
        Q, K, V = Q.contiguous(), K.contiguous(), V.contiguous()
        plain = mult is None and K.shape[1] == Q.shape[1]
        if plain:
            O, Z = sphattn_fwd_z(Q, K, V, dtype=dtype)
        else:
            Z = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
            O = sphattn_cross_fwd(Q, K, V, mult, Z=Z, dtype=dtype)
        ctx.save_for_backward(Q, K, V, O, Z)
        ctx.mult, ctx.plain, ctx.dtype = mult, plain, dtype
        return O

    @staticmethod
    def backward(ctx, dO):
        Q, K, V, O, Z = ctx.saved_tensors
        dO = dO.contiguous()
        if ctx.plain:
            dQ, dK, dV = sphattn_bwd(Q, K, V, O, dO, Z, dtype=ctx.dtype)
        else:
            dQ, dK, dV = sphattn_grn_bwd(Q, K, V, ctx.mult, O, dO, Z, dtype=ctx.dtype)
        return dQ, dK, dV, None


def spherical_attention(Q, K, V, mult=None):
    """Differentiable spherical attention: Q [B,H,N,d]; K, V [B,H_kv,N,d]; optional per-key
    multiplicities mult [B,N] (fp32, no gradient)."""
    return _SphericalAttention.apply(Q, K, V, mult)
