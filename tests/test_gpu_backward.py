"""GPU parity of the backward pass (sphattn_bwd, through the C ABI) against the fp64 CPU oracle.

The backward takes what the forward leaves behind on the GPU (O in the storage type, z in
fp32).  Tolerance: the gradients are sums of products of one operand rounded to the 16-bit
type (W or dS, 2^-9 relative per term for bfloat16) and are stored in the 16-bit type
(half an ulp, 2^-9 relative for bfloat16, of entries that reach about 5 rms, more with
multiplicities, which scale whole rows of dK).  The bound, per gradient tensor, is therefore
the sum of the two: half an ulp of the largest reference entry plus 1.5e-2 (bfloat16) or 3e-3
(half) of the rms of the reference for the inner rounding; measured totals are 1.3e-2 .. 2.0e-2
of the rms for bfloat16 and 1.5e-3 .. 2.3e-3 for half without multiplicities.
"""
import numpy as np
import pytest
import torch

import synthetic_inputs as si

pytestmark = pytest.mark.gpu

INNER = {"bf16": 1.5e-2, "f16": 3e-3}
HALF_ULP = {"bf16": 2.0 ** -9, "f16": 2.0 ** -12}
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    import paper_2505_09326_amd as p
    p.load_library()
    return p


def _rel_err(got, ref):
    return np.abs(got - ref).max() / np.sqrt((ref ** 2).mean())


def _bound(ref, dtype):
    """Allowed max|err| / rms(ref): output rounding of the largest entry + inner rounding."""
    rms = np.sqrt((ref ** 2).mean())
    return HALF_ULP[dtype] * np.abs(ref).max() / rms + INNER[dtype]


def _inputs(B, H, N, d, dtype, seed):
    q, k, v = si.make_qkv(B, H, N, d, dtype, seed=seed)
    g = torch.Generator(device="cpu").manual_seed(seed + 7)
    dO = torch.randn((B, H, N, d), generator=g, dtype=torch.float32).to(q.dtype)
    return q, k, v, dO


def _run(pkg, q, k, v, dO, dtype):
    qd, kd, vd, gd = (t.to(DEV) for t in (q, k, v, dO))
    O, Z = pkg.sphattn_fwd_z(qd, kd, vd, dtype=dtype)
    dQ, dK, dV = pkg.sphattn_bwd(qd, kd, vd, O, gd, Z, dtype=dtype)
    torch.cuda.synchronize()
    return tuple(t.cpu().double().numpy() for t in (dQ, dK, dV))


CASES = [
    (1, 2, 300, 64, "bf16"), (2, 1, 257, 128, "bf16"), (1, 1, 2, 64, "bf16"), (1, 2, 64, 128, "bf16"),
    (1, 1, 1000, 128, "bf16"), (2, 2, 129, 64, "bf16"), (1, 3, 33, 128, "bf16"), (1, 1, 2048, 64, "bf16"),
    (1, 2, 300, 128, "f16"), (1, 1, 515, 64, "f16"),
]


@pytest.mark.parametrize("B,H,N,d,dtype", CASES)
def test_backward_full_compare(pkg, oracle, B, H, N, d, dtype):
    """dQ, dK, dV element by element over several tiles of both kernels and ragged tails."""
    print(f"case bwd B={B} H={H} N={N} d={d} {dtype}", flush=True)
    q, k, v, dO = _inputs(B, H, N, d, dtype, 2000 + N + d)
    got = _run(pkg, q, k, v, dO, dtype)
    bits = [si.storage_bits(t)[0] for t in (q, k, v, dO)]
    kind = si.storage_bits(q)[1]
    ref = oracle.spherical_attention_bwd(*bits, kinds=(kind,) * 4)
    for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
        assert np.all(np.isfinite(a)), name
        err = _rel_err(a, b)
        print(f"  {name}: max|err|/rms = {err:.3e}", flush=True)
        assert err <= _bound(b, dtype), name


def test_backward_single_key(pkg):
    """N = 1: O = sign(s) v does not depend on the size of q or k, so dQ = dK = 0 (two equal
    terms cancel: the result must be small against either of them) and dV = sign(s) dO."""
    B, H, N, d = 1, 3, 1, 128
    q, k, v, dO = _inputs(B, H, N, d, "bf16", 2050)
    dQ, dK, dV = _run(pkg, q, k, v, dO, "bf16")
    qf, kf, vf, gf = (t.double().numpy() for t in (q, k, v, dO))
    s = (qf * kf).sum(-1, keepdims=True)
    term = np.abs((gf * vf).sum(-1, keepdims=True) / s)            # |r (dO.v)|
    assert np.all(np.abs(dQ) <= 2.0 ** -6 * term * np.abs(kf).max())
    assert np.all(np.abs(dK) <= 2.0 ** -6 * term * np.abs(qf).max())
    np.testing.assert_allclose(dV, np.sign(s) * gf, rtol=2.0 ** -7, atol=0)


def test_backward_one_long_head(pkg, oracle):
    """One head of 4096 keys and queries at d = 128: 16 query tiles x 64 key tiles in the dQ
    kernel, 32 key tiles x 64 query tiles in the dK/dV kernel."""
    B, H, N, d = 1, 1, 4096, 128
    q, k, v, dO = _inputs(B, H, N, d, "bf16", 2100)
    got = _run(pkg, q, k, v, dO, "bf16")
    bits = [si.storage_bits(t)[0] for t in (q, k, v, dO)]
    ref = oracle.spherical_attention_bwd(*bits, kinds=("bf16",) * 4)
    for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
        err = _rel_err(a, b)
        print(f"  {name}: max|err|/rms = {err:.3e}", flush=True)
        assert err <= _bound(b, "bf16"), name


def test_backward_zero_query_row_and_determinism(pkg):
    """A query row of zeros has z = 0: its dQ row is 0 and it adds nothing to dK, dV; two runs
    give the same bits (no atomics)."""
    B, H, N, d = 1, 2, 700, 128
    q, k, v, dO = _inputs(B, H, N, d, "bf16", 2200)
    q[0, 1, 5] = 0
    a = _run(pkg, q, k, v, dO, "bf16")
    b = _run(pkg, q, k, v, dO, "bf16")
    assert all(np.all(np.isfinite(x)) for x in a)
    assert np.all(a[0][0, 1, 5] == 0.0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_backward_does_not_write_outside_its_outputs(pkg):
    B, H, N, d = 1, 2, 333, 64
    q, k, v, dO = _inputs(B, H, N, d, "bf16", 2300)
    qd, kd, vd, gd = (t.to(DEV) for t in (q, k, v, dO))
    O, Z = pkg.sphattn_fwd_z(qd, kd, vd, dtype="bf16")
    n = B * H * N * d
    pad = 4096
    bufs = [torch.full((n + 2 * pad,), 7.0, dtype=torch.bfloat16, device=DEV) for _ in range(3)]
    outs = [b[pad:pad + n].view(B, H, N, d) for b in bufs]
    dbuf = torch.full((2 * B * H * N + 2 * pad,), 7.0, dtype=torch.float32, device=DEV)
    pkg.sphattn_bwd(qd, kd, vd, O, gd, Z, dQ=outs[0], dK=outs[1], dV=outs[2],
                    delta=dbuf[pad:pad + 2 * B * H * N].view(2, B, H, N), dtype="bf16")
    torch.cuda.synchronize()
    for b in bufs:
        assert bool((b[:pad] == 7.0).all()) and bool((b[pad + n:] == 7.0).all())
    assert bool((dbuf[:pad] == 7.0).all()) and bool((dbuf[pad + 2 * B * H * N:] == 7.0).all())


GRN_BWD_CASES = [
    # B, H, H_kv, N, d, dtype, with multiplicities
    (1, 4, 2, 300, 64, "bf16", True), (2, 6, 2, 257, 128, "bf16", True), (1, 3, 1, 515, 128, "bf16", False),
    (1, 2, 2, 130, 64, "bf16", True), (1, 4, 1, 200, 128, "f16", True), (2, 2, 1, 64, 64, "bf16", True),
]


@pytest.mark.parametrize("B,H,H_kv,N,d,dtype,with_mult", GRN_BWD_CASES)
def test_grn_backward_parity(pkg, oracle, B, H, H_kv, N, d, dtype, with_mult):
    """Multiplicities (zeros among them) and shared K/V heads: dK and dV sum over a group's heads."""
    print(f"case grn bwd B={B} H={H} H_kv={H_kv} N={N} d={d} {dtype} mult={with_mult}", flush=True)
    q, _, _, dO = _inputs(B, H, N, d, dtype, 2400 + N)
    _, k, v = si.make_qkv(B, H_kv, N, d, dtype, seed=2450 + N)
    mult = None
    if with_mult:
        g = torch.Generator(device="cpu").manual_seed(2470 + N)
        mult = torch.poisson(torch.full((B, N), 1.5), generator=g).to(torch.float32)
        mult[:, 0] = 2.0
    qd, kd, vd, gd = (t.to(DEV) for t in (q, k, v, dO))
    md = mult.to(DEV) if with_mult else None
    O = pkg.sphattn_grn_fwd(qd, kd, vd, md, dtype=dtype)
    # z of the scaled scores: from the partial entry point (the whole key axis as one slice)
    _, Z = pkg.sphattn_partial_fwd(qd, kd, vd, md, dtype=dtype)
    got = pkg.sphattn_grn_bwd(qd, kd, vd, md, O, gd, Z, dtype=dtype)
    torch.cuda.synchronize()
    bits = [si.storage_bits(t)[0] for t in (q, k, v, dO)]
    kind = si.storage_bits(q)[1]
    ref = oracle.grn_attention_bwd(*bits, mult.numpy() if with_mult else None, kinds=(kind,) * 4)
    # rows of dK and dV scale with the gene's multiplicity (and so do their rounding errors):
    # compare them on a common scale, each key row divided by max(m_j, 1)
    row_scale = 1.0 / np.maximum(mult.numpy(), 1.0)[:, None, :, None] if with_mult else 1.0
    for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
        a = a.cpu().double().numpy()
        assert a.shape == b.shape and np.all(np.isfinite(a)), name
        if name != "dQ":
            a, b = a * row_scale, b * row_scale
        err = _rel_err(a, b)
        print(f"  {name}: max|err|/rms = {err:.3e}", flush=True)
        assert err <= _bound(b, dtype), name


def test_grn_backward_without_options_equals_plain_call(pkg):
    B, H, N, d = 1, 2, 400, 128
    q, k, v, dO = _inputs(B, H, N, d, "bf16", 2500)
    qd, kd, vd, gd = (t.to(DEV) for t in (q, k, v, dO))
    O, Z = pkg.sphattn_fwd_z(qd, kd, vd, dtype="bf16")
    a = pkg.sphattn_bwd(qd, kd, vd, O, gd, Z, dtype="bf16")
    b = pkg.sphattn_grn_bwd(qd, kd, vd, None, O, gd, Z, dtype="bf16")
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_autograd_wrapper_routes_to_the_library(pkg):
    """paper_2505_09326_amd.autograd.spherical_attention: forward and backward are the library's
    (bitwise the same as calling the entry points), with and without the GRN options."""
    from paper_2505_09326_amd.autograd import spherical_attention
    print("case autograd wrapper", flush=True)
    B, H, N, d = 1, 4, 300, 64
    q, _, _ = si.make_qkv(B, H, N, d, "bf16", seed=61)
    _, k, v = si.make_qkv(B, 2, N, d, "bf16", seed=62)
    g = torch.Generator(device="cpu").manual_seed(63)
    dO = torch.randn((B, H, N, d), generator=g).to(torch.bfloat16).to(DEV)
    mult = torch.poisson(torch.full((B, N), 1.5), generator=g).to(torch.float32).to(DEV)
    qd, kd, vd = (t.to(DEV).requires_grad_(True) for t in (q, k, v))
    out = spherical_attention(qd, kd, vd, mult)
    out.backward(dO)
    torch.cuda.synchronize()
    Z = torch.empty(B, H, N, dtype=torch.float32, device=DEV)
    O = pkg.sphattn_cross_fwd(qd.detach(), kd.detach(), vd.detach(), mult, Z=Z, dtype="bf16")
    dQ, dK, dV = pkg.sphattn_grn_bwd(qd.detach(), kd.detach(), vd.detach(), mult, O, dO, Z, dtype="bf16")
    torch.cuda.synchronize()
    assert torch.equal(out, O)
    assert torch.equal(qd.grad, dQ) and torch.equal(kd.grad, dK) and torch.equal(vd.grad, dV)
    # plain case
    q2, k2, v2 = (t.to(DEV).requires_grad_(True) for t in si.make_qkv(B, H, N, d, "f16", seed=64))
    dO2 = dO.to(torch.float16)
    out2 = spherical_attention(q2, k2, v2)
    out2.backward(dO2)
    O2, Z2 = pkg.sphattn_fwd_z(q2.detach(), k2.detach(), v2.detach(), dtype="f16")
    g2 = pkg.sphattn_bwd(q2.detach(), k2.detach(), v2.detach(), O2, dO2, Z2, dtype="f16")
    torch.cuda.synchronize()
    assert torch.equal(out2, O2)
    assert all(torch.equal(a.grad, b) for a, b in zip((q2, k2, v2), g2))
