"""GPU parity for the all-E4M3 forward (sphattn_fp8_fwd): Q, K, V in E4M3, both contractions
on the fp8 matrix instructions, through the C ABI, against the CPU oracle.

Two comparisons.
  * Against the oracle's MODEL of the variant (scores divided by 2^e_i and rounded to E4M3,
    output formed from the rounded scores in fp64).  What is left is the rounding of O to
    bfloat16 (2^-9 relative), fp32 accumulation, and the rare score that rounds to the other
    neighbour because the kernel's fp32 score differs from the fp64 one in the last bits (one
    E4M3 step on one of N terms; the stored values lie on a coarse grid, so scores on or next
    to a rounding boundary are not rare).  Tolerance: the bfloat16 path's, 2e-2 of rms(O), plus,
    per output element, one such step: max_j step(p_ij) * max_j |v_jc| / sqrt(z_i).  At most
    2 % of the rows may need that allowance at all.  Rows whose bound |q_i| max|k_j| / 440 is
    within 1e-5 of a power of two may take the neighbouring exponent in fp32 and are left out
    of this comparison (the test asserts that they are fewer than 1 %).
  * Against the exact oracle: the price of the 3-bit mantissa.  A term's relative rounding
    error is uniform within +-2^-4 .. +-2^-5 across a binade (about 0.026 in the root mean
    square) and independent between terms, so rms(err) is about 0.026 rms(O) and the largest
    of 10^5 .. 10^7 outputs about five times that.  Asserted: rms(err) <= 0.04, max <= 0.25.
"""
import numpy as np
import pytest
import torch

import synthetic_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_MODEL = 2e-2
TOL_EXACT_RMS, TOL_EXACT_MAX = 0.04, 0.25


@pytest.fixture(scope="module")
def pkg():
    import paper_2505_09326_amd as p
    p.load_library()
    return p


@pytest.fixture(scope="module")
def oracle():
    import oracle as o
    o.build()
    return o


def _run(pkg, q, k, v, slack=0):
    B, H, N, d = q.shape
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(B, k.shape[1], N, d) + slack, dtype=torch.uint8, device=DEV)
    out = pkg.sphattn_fp8_fwd(q.to(DEV), k.to(DEV), v.to(DEV), ws)
    torch.cuda.synchronize()
    return out.cpu().to(torch.float64).numpy()


def _bits(*tensors):
    return [si.storage_bits(t)[0] for t in tensors]


def _check(oracle, got, q, k, v):
    bits = _bits(q, k, v)
    kinds = ("e4m3fn",) * 3
    model = oracle.spherical_attention_e4m3_scores(*bits, kinds=kinds)
    exact = oracle.spherical_attention(*bits, kinds=kinds)
    rms = np.sqrt((exact ** 2).mean())
    assert np.all(np.isfinite(got))
    _, m = oracle.e4m3_row_exponents(oracle.widen(bits[0], "e4m3fn"), oracle.widen(bits[1], "e4m3fn"))
    safe = (np.abs(m - 0.5) > 1e-5) & (np.abs(m - 1.0) > 1e-5)
    assert safe.mean() > 0.99
    # one E4M3 step of the largest score of the row, times the largest |v| of the column
    Qw, Kw, Vw = (oracle.widen(b, "e4m3fn") for b in bits)
    e, _ = oracle.e4m3_row_exponents(Qw, Kw)
    P = oracle.round_to_e4m3((Qw @ np.swapaxes(Kw, -1, -2)) * np.ldexp(1.0, -e)[..., None])
    _, ex = np.frexp(np.abs(P).max(-1))
    step = np.ldexp(1.0, np.maximum(ex - 1, -6) - 3)
    z = (P * P).sum(-1)
    flip = (step / np.sqrt(np.where(z > 0, z, 1.0)))[..., None] * np.abs(Vw).max(-2)[..., None, :]
    diff = np.abs(got - model)
    assert np.all(diff[safe] <= (TOL_MODEL * rms + flip)[safe])
    rows_over = (diff > TOL_MODEL * rms).any(-1)[safe]
    assert rows_over.mean() <= 0.02 or rows_over.sum() <= 1
    err_model = diff[safe].max() / rms
    err = got - exact
    err_rms, err_max = np.sqrt((err ** 2).mean()) / rms, np.abs(err).max() / rms
    print(f"vs model {err_model:.3e}; vs exact rms {err_rms:.3e} max {err_max:.3e}", flush=True)
    assert err_rms <= TOL_EXACT_RMS and err_max <= TOL_EXACT_MAX


SHAPES = [(1, 1, 1), (1, 2, 33), (2, 2, 77), (1, 1, 128), (1, 3, 129), (2, 1, 255), (1, 2, 256), (1, 1, 257),
          (1, 2, 300), (1, 1, 1000), (2, 2, 513), (1, 1, 2048), (1, 1, 2176)]


@pytest.mark.parametrize("B,H,N", SHAPES)
def test_fp8_all_small_full_compare(pkg, oracle, B, H, N):
    print(f"case fp8-all B={B} H={H} N={N}", flush=True)
    q, k, v = si.make_qkv(B, H, N, 128, "fp8", seed=900 + N)
    _check(oracle, _run(pkg, q, k, v), q, k, v)


@pytest.mark.parametrize("factor", [2.0 ** -6, 30.0])
def test_fp8_all_input_scale(pkg, oracle, factor):
    """Small inputs (many E4M3 subnormals) and inputs near the top of the E4M3 range: the row
    factor brings the scores into range either way."""
    print(f"case fp8-all factor={factor}", flush=True)
    q, k, v = si.make_qkv(1, 2, 400, 128, "fp8", seed=77, factor=factor)
    _check(oracle, _run(pkg, q, k, v), q, k, v)


def test_fp8_all_rows_of_very_different_norm(pkg, oracle):
    """Query rows spanning 2^-8 .. 2^7 in norm and one long key: every row gets its own
    exponent, and the long key sets the bound for all of them."""
    print("case fp8-all mixed norms", flush=True)
    q, k, v = si.gaussian_qkv(1, 2, 300, 128, seed=5)
    q = q * torch.exp2(torch.arange(300) % 16 - 8.0)[None, None, :, None] * 0.05
    k[:, :, 17] *= 12.0
    q, k, v = si.cast_storage(q, k, v, "fp8")
    _check(oracle, _run(pkg, q, k, v), q, k, v)


@pytest.mark.parametrize("B,H,H_kv,N", [(1, 4, 2, 300), (2, 6, 1, 129), (1, 8, 4, 1000)])
def test_fp8_all_shared_kv_heads(pkg, oracle, B, H, H_kv, N):
    """Query head h reads K/V head h / (H / H_kv): against the oracle on K, V repeated per group."""
    print(f"case fp8-all shared heads B={B} H={H} H_kv={H_kv} N={N}", flush=True)
    q, _, _ = si.make_qkv(B, H, N, 128, "fp8", seed=970 + N)
    _, k, v = si.make_qkv(B, H_kv, N, 128, "fp8", seed=980 + N)
    got = _run(pkg, q, k, v)
    rep = H // H_kv
    k_full = k.view(torch.uint8).repeat_interleave(rep, dim=1).view(torch.float8_e4m3fn)
    v_full = v.view(torch.uint8).repeat_interleave(rep, dim=1).view(torch.float8_e4m3fn)
    _check(oracle, got, q, k_full, v_full)


def test_fp8_all_degenerate_rows(pkg, oracle):
    """A zero query row and all-zero keys give z = 0 and O = 0 (no NaN from the row factor)."""
    print("case fp8-all degenerate", flush=True)
    q, k, v = si.make_qkv(1, 2, 200, 128, "fp8", seed=3)
    qf = q.to(torch.float32)
    qf[0, 0, 5] = 0.0
    q = si.to_e4m3fn(qf)
    kf = k.to(torch.float32)
    kf[0, 1] = 0.0
    k = si.to_e4m3fn(kf)
    got = _run(pkg, q, k, v)
    assert np.all(np.isfinite(got))
    assert np.all(got[0, 0, 5] == 0.0)
    assert np.all(got[0, 1] == 0.0)
    _check(oracle, got, q, k, v)


def test_fp8_all_twice_with_one_workspace(pkg, oracle):
    """The workspace carries nothing from one call to the next (the key-norm maximum is cleared
    by the call itself): a second, smaller problem in the same, larger workspace."""
    print("case fp8-all workspace reuse", flush=True)
    q1, k1, v1 = si.make_qkv(1, 2, 500, 128, "fp8", seed=8, factor=8.0)
    q2, k2, v2 = si.make_qkv(1, 2, 260, 128, "fp8", seed=9, factor=0.1)
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(1, 2, 500, 128), dtype=torch.uint8, device=DEV)
    o1 = pkg.sphattn_fp8_fwd(q1.to(DEV), k1.to(DEV), v1.to(DEV), ws)
    o2 = pkg.sphattn_fp8_fwd(q2.to(DEV), k2.to(DEV), v2.to(DEV), ws)
    torch.cuda.synchronize()
    _check(oracle, o1.cpu().to(torch.float64).numpy(), q1, k1, v1)
    _check(oracle, o2.cpu().to(torch.float64).numpy(), q2, k2, v2)


def test_fp8_all_full_size_sampled_rows(pkg, oracle):
    """The benchmark's shape (B=4, H=16, N=16384, d=128, all E4M3) in the launch configuration
    that bench.py times; sampled rows against both oracles."""
    print("case fp8-all full size", flush=True)
    B, H, N, d = 4, 16, 16384, 128
    q, k, v = si.make_qkv(B, H, N, d, "fp8", seed=4)
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=DEV)
    out = pkg.sphattn_fp8_fwd(q.to(DEV), k.to(DEV), v.to(DEV), ws)
    torch.cuda.synchronize()
    got = out.cpu().to(torch.float64).numpy()
    assert np.all(np.isfinite(got))
    rows = [0, 1, 255, 256, 8191, 12345, N - 1]
    for bh in (0, 17, B * H - 1):
        b, h = divmod(bh, H)
        Q = oracle.widen(si.storage_bits(q[b, h])[0], "e4m3fn")
        K = oracle.widen(si.storage_bits(k[b, h])[0], "e4m3fn")
        V = oracle.widen(si.storage_bits(v[b, h])[0], "e4m3fn")
        Qr = Q[rows]
        exact = oracle.spherical_attention_rows(si.storage_bits(q)[0], si.storage_bits(k)[0], si.storage_bits(v)[0],
                                                bh, rows, kinds=("e4m3fn",) * 3)
        e, m = oracle.e4m3_row_exponents(Q[None, None], K[None, None])
        S = Qr @ K.T
        P = oracle.round_to_e4m3(S * np.ldexp(1.0, -e[0, 0, rows])[:, None])
        model = (P @ V) / np.sqrt((P * P).sum(-1))[:, None]
        rms = np.sqrt((exact ** 2).mean())
        g = got[b, h][rows]
        err_model = np.abs(g - model).max() / rms
        err_exact = np.abs(g - exact).max() / rms
        print(f"bh={bh}: vs model {err_model:.3e} vs exact {err_exact:.3e}", flush=True)
        # N = 16384: one step of one term is far below the tolerance
        assert err_model <= TOL_MODEL and err_exact <= TOL_EXACT_MAX


def test_fp8_all_argument_errors_on_device(pkg):
    q, k, v = (t.to(DEV) for t in si.make_qkv(1, 1, 64, 128, "fp8", seed=1))
    small = torch.empty(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(pkg.SphattnError) as e:
        pkg.sphattn_fp8_fwd(q, k, v, small)
    assert e.value.code == -9
    q64, k64, v64 = (t.to(DEV) for t in si.make_qkv(1, 1, 64, 64, "fp8", seed=1))
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(pkg.SphattnError) as e:
        pkg.sphattn_fp8_fwd(q64, k64, v64, ws)
    assert e.value.code == -3


@pytest.mark.parametrize("B,H,N", [(1, 1, 77), (1, 2, 128), (2, 1, 300), (1, 1, 1000), (1, 2, 2049)])
def test_fp8_all_softmax_twin(pkg, oracle, B, H, N):
    """The all-E4M3 SoftMax twin against the oracle's SoftMax, on inputs of moderate size (N(0, 0.5)
    cast to E4M3).  Its weights are rounded to E4M3 like the spherical variant's scores, so the same
    statistical bounds apply: rms(err) <= 0.04 rms(O), max <= 0.25 rms(O).  Ragged N checks that
    keys past the end get no weight (a zero key row would get exp(-shift) > 0)."""
    print(f"case fp8-all softmax twin B={B} H={H} N={N}", flush=True)
    qf, kf, vf = si.gaussian_qkv(B, H, N, 128, seed=950 + N, factor=0.5)
    q, k, v = (t.to(torch.float8_e4m3fn) for t in (qf, kf, vf))
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(B, H, N, 128), dtype=torch.uint8, device=DEV)
    out = pkg.sphattn_fp8_softmax_fwd(q.to(DEV), k.to(DEV), v.to(DEV), ws)
    torch.cuda.synchronize()
    got = out.cpu().to(torch.float64).numpy()
    ref = oracle.softmax_attention(*_bits(q, k, v), kinds=("e4m3fn",) * 3)
    assert np.all(np.isfinite(got))
    rms = np.sqrt((ref ** 2).mean())
    err = got - ref
    err_rms, err_max = np.sqrt((err ** 2).mean()) / rms, np.abs(err).max() / rms
    print(f"softmax twin vs oracle: rms {err_rms:.3e} max {err_max:.3e}", flush=True)
    assert err_rms <= TOL_EXACT_RMS and err_max <= TOL_EXACT_MAX
