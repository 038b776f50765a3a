"""Seeded sweep over random small shapes: every entry point against the oracle on shapes nobody
picked by hand (ragged tails of every residue, one to many tiles, both head dimensions)."""
import numpy as np
import pytest
import torch

import synthetic_inputs as si

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "fp8qk_bf16v": 6e-2, "f32": 1e-4, "f16": 5e-3}
BWD_INNER = {"bf16": 1.5e-2, "f16": 3e-3}
BWD_HALF_ULP = {"bf16": 2.0 ** -9, "f16": 2.0 ** -12}
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pkg():
    import paper_2505_09326_amd as p
    p.load_library()
    return p


def _rel_err(got, ref):
    return np.abs(got - ref).max() / np.sqrt((ref ** 2).mean())


def _shapes(seed, count, nmax):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        H_kv = int(rng.integers(1, 4))
        out.append((int(rng.integers(1, 3)), H_kv * int(rng.integers(1, 4)), H_kv,
                    int(rng.integers(1, nmax)), int(rng.choice([64, 128]))))
    return out


@pytest.mark.parametrize("dtype", ["bf16", "f16", "fp8qk_bf16v", "f32"])
def test_forward_family_on_random_shapes(pkg, oracle, dtype):
    """sphattn_fwd_z, sphattn_grn_fwd (multiplicities, shared K/V heads) and sphattn_splitkv_fwd
    on 12 random shapes per storage type."""
    for idx, (B, H, H_kv, N, d) in enumerate(_shapes({"bf16": 1, "f16": 2, "fp8qk_bf16v": 3, "f32": 4}[dtype], 12, 900)):
        print(f"case random fwd {dtype} B={B} H={H} H_kv={H_kv} N={N} d={d}", flush=True)
        q, _, _ = si.make_qkv(B, H, N, d, dtype, seed=3000 + idx)
        _, k, v = si.make_qkv(B, H_kv, N, d, dtype, seed=3100 + idx)
        g = torch.Generator(device="cpu").manual_seed(3200 + idx)
        mult = torch.poisson(torch.full((B, N), 1.5), generator=g).to(torch.float32)
        mult[:, 0] = 1.0
        (qb, qk), (kb, kk), (vb, vk) = (si.storage_bits(t) for t in (q, k, v))
        ref = oracle.grn_attention(qb, kb, vb, mult.numpy(), kinds=(qk, kk, vk))
        qd, kd, vd, md = q.to(DEV), k.to(DEV), v.to(DEV), mult.to(DEV)
        got = pkg.sphattn_grn_fwd(qd, kd, vd, md, dtype=dtype)
        n_splits = 1 + idx % 4
        ws = torch.empty(pkg.sphattn_splitkv_workspace_bytes(B, H, N, d, n_splits), dtype=torch.uint8, device=DEV)
        got_split = pkg.sphattn_splitkv_fwd(qd, kd, vd, ws, mult=md, n_splits=n_splits, dtype=dtype)
        torch.cuda.synchronize()
        assert _rel_err(got.cpu().double().numpy(), ref) <= TOL[dtype]
        assert _rel_err(got_split.cpu().double().numpy(), ref) <= TOL[dtype]
        if H_kv == H:
            kq, kv_ = k.to(DEV), v.to(DEV)
            O, Z = pkg.sphattn_fwd_z(qd, kq, kv_, dtype=dtype)
            torch.cuda.synchronize()
            ref_O, _, ref_Z = oracle.spherical_attention_full(qb, kb, vb, kinds=(qk, kk, vk))
            assert _rel_err(O.cpu().double().numpy(), ref_O) <= TOL[dtype]
            np.testing.assert_allclose(Z.cpu().double().numpy(), ref_Z, rtol=2e-4)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_backward_on_random_shapes(pkg, oracle, dtype):
    for idx, (B, H, _, N, d) in enumerate(_shapes({"bf16": 5, "f16": 6}[dtype], 10, 600)):
        if N < 2:
            N = 2                                   # one key: every gradient but dV is exactly 0
        print(f"case random bwd {dtype} B={B} H={H} N={N} d={d}", flush=True)
        q, k, v = si.make_qkv(B, H, N, d, dtype, seed=3300 + idx)
        g = torch.Generator(device="cpu").manual_seed(3400 + idx)
        dO = torch.randn((B, H, N, d), generator=g, dtype=torch.float32).to(q.dtype)
        qd, kd, vd, gd = (t.to(DEV) for t in (q, k, v, dO))
        O, Z = pkg.sphattn_fwd_z(qd, kd, vd, dtype=dtype)
        got = pkg.sphattn_bwd(qd, kd, vd, O, gd, Z, dtype=dtype)
        torch.cuda.synchronize()
        bits = [si.storage_bits(t)[0] for t in (q, k, v, dO)]
        kind = si.storage_bits(q)[1]
        ref = oracle.spherical_attention_bwd(*bits, kinds=(kind,) * 4)
        for name, a, b in zip(("dQ", "dK", "dV"), got, ref):
            bound = BWD_HALF_ULP[dtype] * np.abs(b).max() / np.sqrt((b ** 2).mean()) + BWD_INNER[dtype]
            assert _rel_err(a.cpu().double().numpy(), b) <= bound, (name, B, H, N, d)
