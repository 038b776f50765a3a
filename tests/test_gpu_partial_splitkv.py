"""GPU parity for the accumulator entry points: the row aggregates z, the partial pair (o, z)
of Lemma 1 over a key slice, the combine step (sum of pairs, then the tail) and the split-key
forward built from them -- all through the C ABI, against the fp64 CPU oracle.

Tolerances.  Outputs O: the ones of test_gpu_parity.py.  z: fp32 sums of non-negative fp32
squares of scores that are exact products summed in fp32 -> 2e-4 relative.  o_part: no output
rounding, only the rounding of P to the 16-bit type before the second contraction (2^-9 per
term for bfloat16, 2^-12 for half), compared after division by sqrt(z_ref): 1e-2 of the rms
for bfloat16 P, 2e-3 for half, 1e-4 for fp32.
"""
import numpy as np
import pytest
import torch

import synthetic_inputs as si

pytestmark = pytest.mark.gpu

TOL_O = {"bf16": 2e-2, "fp8qk_bf16v": 6e-2, "f32": 1e-4, "f16": 5e-3}
TOL_PART = {"bf16": 1e-2, "fp8qk_bf16v": 1e-2, "f32": 1e-4, "f16": 2e-3}
Z_RTOL = 2e-4
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    import paper_2505_09326_amd as p
    p.load_library()
    return p


def _bits(*tensors):
    pairs = [si.storage_bits(t) for t in tensors]
    return [p[0] for p in pairs], tuple(p[1] for p in pairs)


def _rel_err(got, ref):
    return np.abs(got - ref).max() / np.sqrt((ref ** 2).mean())


def _mult(B, N, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    m = torch.poisson(torch.full((B, N), 1.5), generator=g).to(torch.float32)
    m[:, 0] = 2.0
    return m


def _rect_inputs(B, H, H_kv, Nq, Nk, d, dtype, seed):
    q, _, _ = si.make_qkv(B, H, Nq, d, dtype, seed=seed)
    _, k, v = si.make_qkv(B, H_kv, Nk, d, dtype, seed=seed + 1)
    return q, k, v


def _workspace(pkg, B, H, N, d, n_splits, guard=4096):
    need = pkg.sphattn_splitkv_workspace_bytes(B, H, N, d, max(n_splits, 1))
    buf = torch.full((need + guard,), 0xFF, dtype=torch.uint8, device=DEV)   # all-ones bytes: fp32 NaN
    return buf, need


# ---------------------------------------------------------------- z beside O
@pytest.mark.parametrize("B,H,N,d,dtype", [
    (1, 2, 300, 64, "bf16"), (2, 1, 1029, 128, "bf16"), (1, 2, 257, 128, "fp8qk_bf16v"),
    (1, 2, 131, 64, "f32"), (1, 1, 700, 128, "f32"), (1, 2, 300, 128, "f16"), (1, 1, 1, 64, "bf16"),
])
def test_fwd_z_emits_the_row_aggregates(pkg, oracle, B, H, N, d, dtype):
    print(f"case fwd_z B={B} H={H} N={N} d={d} {dtype}", flush=True)
    q, k, v = si.make_qkv(B, H, N, d, dtype, seed=800 + N + d)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    O, Z = pkg.sphattn_fwd_z(qd, kd, vd, dtype=dtype)
    O_plain = pkg.sphattn_fwd(qd, kd, vd, dtype=dtype)
    torch.cuda.synchronize()
    assert torch.equal(O, O_plain)                      # the same kernel, one more store
    bits, kinds = _bits(q, k, v)
    ref_O, _, ref_Z = oracle.spherical_attention_full(*bits, kinds=kinds)
    np.testing.assert_allclose(Z.cpu().double().numpy(), ref_Z, rtol=Z_RTOL)
    assert _rel_err(O.cpu().double().numpy(), ref_O) <= TOL_O[dtype]


# ---------------------------------------------------------------- partial accumulator
PARTIAL_CASES = [
    # B, H, H_kv, N_q, N_k, d, dtype, with multiplicities
    (1, 2, 2, 300, 500, 64, "bf16", False), (1, 4, 2, 257, 129, 128, "bf16", True),
    (2, 2, 1, 1, 1000, 128, "bf16", True), (1, 2, 2, 513, 1, 64, "bf16", False),
    (1, 1, 1, 1024, 2048, 128, "bf16", False), (1, 2, 1, 200, 333, 128, "fp8qk_bf16v", True),
    (1, 2, 2, 70, 515, 64, "fp8qk_bf16v", False), (1, 2, 2, 300, 131, 128, "f16", False),
    (1, 2, 1, 100, 77, 64, "f32", True), (1, 1, 1, 33, 700, 128, "f32", False),
    (2, 3, 3, 65, 64, 64, "f32", False),
]


@pytest.mark.parametrize("B,H,H_kv,Nq,Nk,d,dtype,with_mult", PARTIAL_CASES)
def test_partial_accumulator_rectangular(pkg, oracle, B, H, H_kv, Nq, Nk, d, dtype, with_mult):
    """(o, z) without the tail, N_q != N_k, every storage type, element by element."""
    print(f"case partial B={B} H={H} H_kv={H_kv} Nq={Nq} Nk={Nk} d={d} {dtype} mult={with_mult}", flush=True)
    q, k, v = _rect_inputs(B, H, H_kv, Nq, Nk, d, dtype, 900 + Nq + Nk)
    mult = _mult(B, Nk, 950 + Nk) if with_mult else None
    o, z = pkg.sphattn_partial_fwd(q.to(DEV), k.to(DEV), v.to(DEV),
                                   mult.to(DEV) if with_mult else None, dtype=dtype)
    torch.cuda.synchronize()
    bits, kinds = _bits(q, k, v)
    ref_o, ref_z = oracle.spherical_accumulate(*bits, mult.numpy() if with_mult else None, kinds=kinds)
    got_o, got_z = o.cpu().double().numpy(), z.cpu().double().numpy()
    assert np.all(np.isfinite(got_o)) and np.all(np.isfinite(got_z))
    np.testing.assert_allclose(got_z, ref_z, rtol=Z_RTOL)
    nrm = np.sqrt(ref_z)[..., None]
    err = _rel_err(got_o / nrm, ref_o / nrm)
    print(f"partial max|err|/rms={err:.3e}", flush=True)
    assert err <= TOL_PART[dtype]


# ---------------------------------------------------------------- combine
@pytest.mark.parametrize("P", [1, 3, 8])
@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
def test_combine_sums_parts_and_applies_the_tail(pkg, oracle, P, dtype):
    """Parts made on the host (any fp32 values will do), so this isolates the combine kernel.
    Rows 0 and 5 have z = 0 in every part and must give 0."""
    B, H, N, d = 1, 2, 131, 64
    g = torch.Generator(device="cpu").manual_seed(1000 + P)
    o_parts = torch.randn((P, B, H, N, d), generator=g, dtype=torch.float32) * 30.0
    z_parts = torch.rand((P, B, H, N), generator=g, dtype=torch.float32) * 900.0 + 1.0
    for r in (0, 5):
        o_parts[:, 0, 1, r] = 0.0
        z_parts[:, 0, 1, r] = 0.0
    Z = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
    O = pkg.sphattn_combine(o_parts.to(DEV), z_parts.to(DEV), Z=Z, dtype=dtype)
    torch.cuda.synchronize()
    ref = oracle.spherical_tail(o_parts.double().numpy(), z_parts.double().numpy())
    got = O.cpu().double().numpy()
    # one rounding to the output type, on top of fp32 sums whose error scales with the size
    # of the terms (they may cancel), not of the result
    ulp = {"bf16": 2.0 ** -8, "f16": 2.0 ** -11, "f32": 2.0 ** -22}[dtype]
    zsum = z_parts.double().numpy().sum(0)[..., None]
    terms = np.abs(o_parts.double().numpy()).sum(0) / np.sqrt(np.where(zsum > 0, zsum, 1.0))
    assert np.all(np.abs(got - ref) <= ulp * np.abs(ref) + P * 2.0 ** -23 * terms + 1e-30)
    assert np.all(got[0, 1, 0] == 0.0) and np.all(got[0, 1, 5] == 0.0)
    np.testing.assert_allclose(Z.cpu().double().numpy(), z_parts.double().numpy().sum(0), rtol=1e-6)


def test_key_slices_from_separate_calls_combine_to_attention(pkg, oracle):
    """The way the key axis would be sharded over streams or GPUs: one partial call per
    (ragged) slice, the pairs stacked, one combine."""
    B, H, H_kv, N, d = 1, 4, 2, 1100, 128
    q, k, v = _rect_inputs(B, H, H_kv, N, N, d, "bf16", 1100)
    mult = _mult(B, N, 1101)
    cuts = [0, 300, 301, 900, 1100]
    qd = q.to(DEV)
    os_, zs = [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        o, z = pkg.sphattn_partial_fwd(qd, k[:, :, a:b].contiguous().to(DEV), v[:, :, a:b].contiguous().to(DEV),
                                       mult[:, a:b].contiguous().to(DEV), dtype="bf16")
        os_.append(o)
        zs.append(z)
    O = pkg.sphattn_combine(torch.stack(os_), torch.stack(zs), dtype="bf16")
    torch.cuda.synchronize()
    bits, kinds = _bits(q, k, v)
    ref = oracle.grn_attention(*bits, mult.numpy(), kinds=kinds)
    assert _rel_err(O.cpu().double().numpy(), ref) <= TOL_O["bf16"]


# ---------------------------------------------------------------- split-key forward
SPLIT_CASES = [
    # B, H, H_kv, N, d, dtype, with multiplicities
    (1, 2, 2, 1000, 128, "bf16", False), (1, 4, 2, 777, 64, "bf16", True), (2, 1, 1, 2048, 128, "bf16", False),
    (1, 2, 1, 515, 128, "fp8qk_bf16v", True), (1, 2, 2, 640, 64, "f16", False),
    (1, 2, 1, 300, 64, "f32", True), (1, 1, 1, 50, 128, "bf16", False),
]


@pytest.mark.parametrize("n_splits", [1, 2, 3, 7, 0, 40])
@pytest.mark.parametrize("B,H,H_kv,N,d,dtype,with_mult", SPLIT_CASES)
def test_splitkv_parity(pkg, oracle, B, H, H_kv, N, d, dtype, with_mult, n_splits):
    """Any number of slices (more than there are tiles included) gives the attention output;
    the NaN-filled workspace shows that every slot that is read was written, and its guard
    bytes that nothing is written past the stated size."""
    print(f"case splitkv B={B} H={H} H_kv={H_kv} N={N} d={d} {dtype} mult={with_mult} splits={n_splits}", flush=True)
    q, k, v = _rect_inputs(B, H, H_kv, N, N, d, dtype, 1200 + N)
    mult = _mult(B, N, 1250 + N) if with_mult else None
    eff = n_splits if n_splits > 0 else pkg.sphattn_splitkv_heuristic(B, H, N, d, dtype)
    ws, need = _workspace(pkg, B, H, N, d, eff)
    Z = torch.empty((B, H, N), dtype=torch.float32, device=DEV)
    O = pkg.sphattn_splitkv_fwd(q.to(DEV), k.to(DEV), v.to(DEV), ws, mult=mult.to(DEV) if with_mult else None,
                                Z=Z, n_splits=n_splits, dtype=dtype)
    torch.cuda.synchronize()
    assert bool((ws[need:] == 0xFF).all())
    bits, kinds = _bits(q, k, v)
    ref = oracle.grn_attention(*bits, mult.numpy() if with_mult else None, kinds=kinds)
    got = O.cpu().double().numpy()
    assert np.all(np.isfinite(got))
    err = _rel_err(got, ref)
    print(f"splitkv max|err|/rms={err:.3e}", flush=True)
    assert err <= TOL_O[dtype]
    _, ref_z = oracle.spherical_accumulate(*bits, mult.numpy() if with_mult else None, kinds=kinds)
    np.testing.assert_allclose(Z.cpu().double().numpy(), ref_z, rtol=Z_RTOL)


def test_splitkv_single_slice_equals_unsplit_call(pkg):
    """One slice runs the same arithmetic in the same order as the unsplit 256-row kernel."""
    B, H, N, d = 1, 3, 900, 128
    q, k, v = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "bf16", seed=1300))
    ws, _ = _workspace(pkg, B, H, N, d, 1)
    a = pkg.sphattn_splitkv_fwd(q, k, v, ws, n_splits=1, dtype="bf16")
    b, _ = pkg.sphattn_fwd_tile_rows(q, k, v, dtype="bf16", tile_rows=256)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_splitkv_is_deterministic(pkg):
    B, H, N, d = 1, 2, 3000, 128
    q, k, v = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "bf16", seed=1301))
    ws, _ = _workspace(pkg, B, H, N, d, 6)
    a = pkg.sphattn_splitkv_fwd(q, k, v, ws, n_splits=6, dtype="bf16").clone()
    ws.fill_(0xFF)
    b = pkg.sphattn_splitkv_fwd(q, k, v, ws, n_splits=6, dtype="bf16")
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_splitkv_rejects_a_small_workspace(pkg):
    B, H, N, d = 1, 1, 512, 64
    q, k, v = (t.to(DEV) for t in si.make_qkv(B, H, N, d, "bf16", seed=1302))
    need = pkg.sphattn_splitkv_workspace_bytes(B, H, N, d, 4)
    ws = torch.empty(need - 256, dtype=torch.uint8, device=DEV)
    out = torch.full((B, H, N, d), 7.0, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(pkg.SphattnError) as e:
        pkg.sphattn_splitkv_fwd(q, k, v, ws, O=out, n_splits=4, dtype="bf16")
    assert e.value.code == -9
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                     # nothing was enqueued


def test_splitkv_few_heads_at_full_length(pkg, oracle):
    """The case the split is for: two heads of the C3 length (64 unsplit workgroups on 256
    CUs), the library's own choice of slices, sampled rows against the oracle."""
    B, H, N, d = 1, 2, 8192, 128
    q, k, v = si.make_qkv(B, H, N, d, "bf16", seed=1303)
    S = pkg.sphattn_splitkv_heuristic(B, H, N, d, "bf16")
    print(f"case splitkv full length: heuristic slices = {S}", flush=True)
    assert S > 1
    ws, need = _workspace(pkg, B, H, N, d, S)
    O = pkg.sphattn_splitkv_fwd(q.to(DEV), k.to(DEV), v.to(DEV), ws, n_splits=0, dtype="bf16")
    torch.cuda.synchronize()
    assert bool((ws[need:] == 0xFF).all())
    got = O.cpu().double().numpy()
    bits, kinds = _bits(q, k, v)
    rng = np.random.default_rng(11)
    worst = 0.0
    for bh in range(B * H):
        rows = np.sort(rng.choice(N, size=192, replace=False))
        ref = oracle.spherical_attention_rows(*bits, bh, rows, kinds=kinds)
        worst = max(worst, np.abs(got.reshape(B * H, N, d)[bh, rows] - ref).max())
    print(f"splitkv full length: max|err| = {worst:.3e} (outputs have unit variance)", flush=True)
    assert worst <= TOL_O["bf16"]


CROSS_SHAPES = [(1, 2, 2, 1, 700, 128, "bf16", False), (2, 4, 2, 300, 77, 64, "bf16", True),
                (1, 2, 1, 513, 2049, 128, "f16", True), (1, 3, 3, 64, 1000, 64, "fp8qk_bf16v", False),
                (2, 2, 1, 257, 130, 128, "f32", True), (1, 1, 1, 1000, 1, 64, "bf16", False),
                # 528 query tiles of d = 64 for 512 resident workgroups, shared K/V heads: one full
                # round, then the 16 remaining tiles as 128-row halves (the last ones half empty)
                (1, 66, 33, 1900, 300, 64, "f16", False)]


@pytest.mark.parametrize("B,H,H_kv,Nq,Nk,d,dtype,with_mult", CROSS_SHAPES)
def test_cross_forward_parity(pkg, oracle, B, H, H_kv, Nq, Nk, d, dtype, with_mult):
    """N_q query rows against N_k keys (sphattn_cross_fwd), with and without multiplicities and
    shared K/V heads; O and z against the oracle's accumulator followed by its tail."""
    print(f"case cross B={B} H={H} H_kv={H_kv} Nq={Nq} Nk={Nk} d={d} {dtype} mult={with_mult}", flush=True)
    q, _, _ = si.make_qkv(B, H, Nq, d, dtype, seed=700 + Nq)
    _, k, v = si.make_qkv(B, H_kv, Nk, d, dtype, seed=800 + Nk)
    mult = None
    if with_mult:
        g = torch.Generator(device="cpu").manual_seed(900 + Nk)
        mult = torch.poisson(torch.full((B, Nk), 1.5), generator=g).to(torch.float32)
        mult[:, 0] = 2.0
    bits, kinds = _bits(q, k, v)
    o_raw, z_ref = oracle.spherical_accumulate(*bits, mult=None if mult is None else mult.numpy(), kinds=kinds)
    ref = oracle.spherical_tail(o_raw[None], z_ref[None])
    Z = torch.empty(B, H, Nq, dtype=torch.float32, device=DEV)
    O = pkg.sphattn_cross_fwd(q.to(DEV), k.to(DEV), v.to(DEV), None if mult is None else mult.to(DEV), Z=Z, dtype=dtype)
    torch.cuda.synchronize()
    got = O.cpu().to(torch.float64).numpy()
    assert got.shape == (B, H, Nq, d) and np.all(np.isfinite(got))
    assert _rel_err(got, ref) <= TOL_O[dtype]
    # a score that nearly cancels (|s| << |q||k|) carries the fp32 rounding of its d products,
    # about d 2^-24 |q||k|, which a row with a single key does not average out: absolute slack
    # of 1e-7 of the largest z on top of the relative tolerance
    np.testing.assert_allclose(Z.cpu().to(torch.float64).numpy(), z_ref, rtol=Z_RTOL, atol=1e-7 * z_ref.max())
