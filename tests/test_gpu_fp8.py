"""GPU parity for the all-E4M3 forward (sphattn_fp8_fwd): Q, K, V in E4M3, both contractions
on the fp8 matrix instructions, through the C ABI, against the CPU oracle.

Parity is against the paper-derived oracle (oracle.spherical_attention, exact fp64 on the stored
values).  The entry point rounds every score to E4M3 (3 mantissa bits), so its distance from the
exact result is not the 2e-2 / 6e-2 of the 16-bit-score paths; what it may be is derived, per
output element, from the exact scores alone (fp8_kernel_model.oracle_error_bounds, which states
the derivation and is checked for soundness on the CPU):
  * hard:  |err_ic| <= (sum_j eps_ij |v_jc| + |O_ic| |eps_i|) / (|s_i| - |eps_i|) + output rounding,
           eps_ij = 2^-4 |s_ij| + subnormal step + fp32 score error: every rounding error at its
           worst size and sign.  Must hold for every element, always.
  * 7 sigma: |err_ic| <= 7 sigma_ic + output rounding, sigma_ic the first-order standard deviation
           of the element's error for independent rounding errors of variance <= eps_ij^2 / 3.
           (7 sigma: < 1e-11 per element; the largest test has 1e7 elements.)
  * rms:   rms(err) <= rms(sigma) (+ output rounding): the sigma are upper bounds (worst place in a
           binade), so the observed rms must not exceed theirs.
A wrong column of V, a saturated or unscaled row, a coarser grid or a sum over the wrong scores
breaks at least one of them (tests/test_fp8_kernel_model.py plants such mistakes on the CPU).

Beside that, as a REGRESSION CHECK and not as parity: the output is compared with a model of
the kernel's own rounding (tests/fp8_kernel_model.py: same row exponents, same rounding, fp64
sums) to the bfloat16 path's 2e-2 of rms(O) plus, per element, one E4M3 step of one term (the
kernel's fp32 score can fall on the other side of a rounding boundary than the fp64 one); at
most 2 % of the rows may need that allowance.  Rows whose bound |q_i| max|k_j| / 440 is within
1e-5 of a power of two may take the neighbouring exponent in fp32 and are left out of this check.
"""
import numpy as np
import pytest
import torch

import fp8_kernel_model as km
import synthetic_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL_MODEL = 2e-2
K_SIGMA = 7.0


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


def _run(pkg, q, k, v, slack=0, mult=None):
    B, H, N, d = q.shape
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(B, k.shape[1], N, d) + slack, dtype=torch.uint8, device=DEV)
    if mult is None:
        out = pkg.sphattn_fp8_fwd(q.to(DEV), k.to(DEV), v.to(DEV), ws)
    else:
        out = pkg.sphattn_fp8_grn_fwd(q.to(DEV), k.to(DEV), v.to(DEV), mult.to(DEV), ws)
    torch.cuda.synchronize()
    return out.cpu().to(torch.float64).numpy()


def _bits(*tensors):
    return [si.storage_bits(t)[0] for t in tensors]


def _assert_within_oracle_bounds(got, exact, S, Vw, cap, d, what):
    """The three oracle-derived criteria of the module docstring."""
    hard, sigma, own = km.oracle_error_bounds(S, Vw, exact, cap, d)
    err = np.abs(got - exact)
    rms = np.sqrt((exact ** 2).mean())
    worst_hard = np.max(np.where(hard > 0, err / np.where(hard > 0, hard, 1.0), np.where(err > 0, np.inf, 0.0)))
    stat = K_SIGMA * sigma + own
    worst_stat = np.max(np.where(stat > 0, err / np.where(stat > 0, stat, 1.0), np.where(err > 0, np.inf, 0.0)))
    err_rms = np.sqrt((err ** 2).mean())
    bound_rms = np.sqrt((sigma ** 2).mean() + (own ** 2).mean())
    print(f"{what}: vs exact rms {err_rms / rms:.3e} (bound {bound_rms / rms:.3e}) max {err.max() / rms:.3e}; "
          f"worst err/hard {worst_hard:.3f}, err/(7 sigma) {worst_stat:.3f}", flush=True)
    assert worst_hard <= 1.0
    assert worst_stat <= 1.0
    assert err_rms <= bound_rms


def _check(oracle, got, q, k, v, mult=None):
    bits = _bits(q, k, v)
    kinds = ("e4m3fn",) * 3
    d = q.shape[-1]
    assert np.all(np.isfinite(got))
    Qw, Kw, Vw = (oracle.widen(b, "e4m3fn") for b in bits)
    if mult is None:
        # exact output and scores from the oracle: s_ij = w_ij sqrt(z_i)
        exact, W, Z = oracle.spherical_attention_full(*bits, kinds=kinds)
        S = W * np.sqrt(Z)[..., None]
        kn = np.sqrt((Kw * Kw).sum(-1))
    else:
        exact = oracle.grn_attention(*bits, mult, kinds=kinds)
        _, z = oracle.spherical_accumulate(*bits, mult, kinds=kinds)
        S = np.matmul(Qw, np.swapaxes(Kw, -1, -2)) * mult[:, None, None, :]
        assert np.allclose((S * S).sum(-1), z, rtol=1e-12)     # the bound is built on the oracle's scores
        kn = np.sqrt((Kw * Kw).sum(-1)) * np.abs(mult)[:, None, :]
    cap = np.sqrt((Qw * Qw).sum(-1)) * kn.max(-1)[..., None]
    _assert_within_oracle_bounds(got, exact, S, Vw, cap, d, "parity")

    # regression check against the model of the kernel's rounding (not parity)
    rms = np.sqrt((exact ** 2).mean())
    model = km.spherical_attention_e4m3_scores(Qw, Kw, Vw, mult)
    e, m = km.e4m3_row_exponents(Qw, Kw, mult)
    safe = (np.abs(m - 0.5) > 1e-5) & (np.abs(m - 1.0) > 1e-5)
    assert safe.mean() > 0.99
    # one E4M3 step of the largest score of the row, times the largest |v| of the column
    P = km.round_to_e4m3(S * np.ldexp(1.0, -e)[..., None])
    _, ex = np.frexp(np.abs(P).max(-1))
    step = np.ldexp(1.0, np.maximum(ex - 1, -6) - 3)
    z = (P * P).sum(-1)
    flip = (step / np.sqrt(np.where(z > 0, z, 1.0)))[..., None] * np.abs(Vw).max(-2)[..., None, :]
    diff = np.abs(got - model)
    assert np.all(diff[safe] <= (TOL_MODEL * rms + flip)[safe])
    rows_over = (diff > TOL_MODEL * rms).any(-1)[safe]
    assert rows_over.mean() <= 0.02 or rows_over.sum() <= 1
    print(f"regression vs kernel model {diff[safe].max() / rms:.3e}", flush=True)


SHAPES = [(1, 1, 1), (1, 2, 33), (2, 2, 77), (1, 1, 128), (1, 3, 129), (2, 1, 255), (1, 2, 256), (1, 1, 257),
          (1, 2, 300), (1, 1, 1000), (2, 2, 513), (1, 1, 2048), (1, 1, 2176)]


@pytest.mark.parametrize("B,H,N", SHAPES)
def test_fp8_all_small_full_compare(pkg, oracle, B, H, N):
    print(f"case fp8-all B={B} H={H} N={N}", flush=True)
    q, k, v = si.make_qkv(B, H, N, 128, "fp8", seed=900 + N)
    _check(oracle, _run(pkg, q, k, v), q, k, v)


@pytest.mark.parametrize("B,H,N", [(1, 1, 1), (1, 2, 33), (2, 2, 77), (1, 1, 128), (1, 3, 129), (1, 2, 256), (1, 1, 257),
                                   (1, 2, 300), (1, 1, 1000), (2, 2, 513), (1, 1, 2176)])
def test_fp8_all_d64_small_full_compare(pkg, oracle, B, H, N):
    """Head dimension 64: the first contraction runs with half of its k-slots zero, the output
    has four column blocks."""
    print(f"case fp8-all d=64 B={B} H={H} N={N}", flush=True)
    q, k, v = si.make_qkv(B, H, N, 64, "fp8", seed=1900 + N)
    _check(oracle, _run(pkg, q, k, v), q, k, v)


def _counts(B, N, seed):
    """Gene counts of a cell: mostly small integers, some zeros (genes that are absent)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    return torch.poisson(torch.full((B, N), 1.5), generator=g).to(torch.float32)


@pytest.mark.parametrize("B,H,H_kv,N,d", [(1, 1, 1, 1, 128), (1, 2, 2, 33, 128), (2, 2, 1, 77, 64), (1, 3, 3, 129, 128),
                                          (1, 2, 2, 256, 64), (1, 4, 2, 300, 128), (1, 1, 1, 1000, 64),
                                          (2, 2, 2, 513, 128), (1, 2, 1, 2176, 128)])
def test_fp8_all_multiplicities(pkg, oracle, B, H, H_kv, N, d):
    """s_ij = mult_j (q_i . k_j) (paper, Section 3.1), with shared K/V heads, both head dimensions,
    ragged N: against the oracle's gene-regulatory-network variant on K, V repeated per group."""
    print(f"case fp8-all multiplicities B={B} H={H} H_kv={H_kv} N={N} d={d}", flush=True)
    q, _, _ = si.make_qkv(B, H, N, d, "fp8", seed=2970 + N)
    _, k, v = si.make_qkv(B, H_kv, N, d, "fp8", seed=2980 + N)
    mult = _counts(B, N, 31 + N)
    if N == 1:
        mult[:] = 3.0
    got = _run(pkg, q, k, v, mult=mult)
    rep = H // H_kv
    k_full = k.view(torch.uint8).repeat_interleave(rep, dim=1).view(torch.float8_e4m3fn)
    v_full = v.view(torch.uint8).repeat_interleave(rep, dim=1).view(torch.float8_e4m3fn)
    _check(oracle, got, q, k_full, v_full, mult=mult.numpy().astype(np.float64))


def test_fp8_all_multiplicities_that_differ_by_orders_of_magnitude(pkg, oracle):
    """One gene counted 500 times among genes counted once: it sets the row bound for every row."""
    print("case fp8-all large multiplicity", flush=True)
    q, k, v = si.make_qkv(1, 2, 400, 128, "fp8", seed=61)
    mult = torch.ones((1, 400), dtype=torch.float32)
    mult[0, 123] = 500.0
    mult[0, 7] = 0.0
    got = _run(pkg, q, k, v, mult=mult)
    _check(oracle, got, q, k, v, mult=mult.numpy().astype(np.float64))


def test_fp8_all_without_multiplicities_equals_plain_call(pkg):
    q, k, v = (t.to(DEV) for t in si.make_qkv(1, 2, 700, 64, "fp8", seed=62))
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(1, 2, 700, 64), dtype=torch.uint8, device=DEV)
    a = pkg.sphattn_fp8_fwd(q, k, v, ws).clone()
    b = pkg.sphattn_fp8_grn_fwd(q, k, v, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    ones = torch.ones((1, 700), dtype=torch.float32, device=DEV)
    c = pkg.sphattn_fp8_grn_fwd(q, k, v, ones, ws)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), c.view(torch.int16))


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
    rng = np.random.default_rng(5)
    rows = sorted(set(rows) | set(rng.integers(0, N, size=56).tolist()))
    qb, kb, vb = _bits(q, k, v)
    for bh in (0, 17, B * H - 1):
        b, h = divmod(bh, H)
        Q, K, V = (oracle.widen(x[b, h], "e4m3fn") for x in (qb, kb, vb))
        exact = oracle.spherical_attention_rows(qb, kb, vb, bh, rows, kinds=("e4m3fn",) * 3)
        # exact scores of the sampled rows for the bound (fp64 products of E4M3 values: exact sums
        # up to fp64 rounding); the reference output itself comes from oracle/
        S = Q[rows] @ K.T
        cap = np.sqrt((Q[rows] ** 2).sum(-1)) * np.sqrt((K * K).sum(-1)).max()
        g = got[b, h][rows]
        _assert_within_oracle_bounds(g, exact, S, V, cap, d, f"bh={bh}")
        e, m = km.e4m3_row_exponents(Q[None, None], K[None, None])
        P = km.round_to_e4m3(S * np.ldexp(1.0, -e[0, 0, rows])[:, None])
        model = (P @ V) / np.sqrt((P * P).sum(-1))[:, None]
        rms = np.sqrt((exact ** 2).mean())
        err_model = np.abs(g - model).max() / rms
        print(f"bh={bh}: regression vs kernel model {err_model:.3e}", flush=True)
        # N = 16384: one step of one term is far below the tolerance
        assert err_model <= TOL_MODEL


def test_fp8_all_argument_errors_on_device(pkg):
    q, k, v = (t.to(DEV) for t in si.make_qkv(1, 1, 64, 128, "fp8", seed=1))
    small = torch.empty(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(pkg.SphattnError) as e:
        pkg.sphattn_fp8_fwd(q, k, v, small)
    assert e.value.code == -9
    q96 = torch.zeros((1, 1, 64, 96), dtype=torch.float8_e4m3fn, device=DEV)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=DEV)
    with pytest.raises(pkg.SphattnError) as e:
        pkg.sphattn_fp8_fwd(q96, q96, q96, ws)
    assert e.value.code == -3


# the SoftMax twin is a timing aid, not a row of the method: statistical bounds only
TWIN_RMS, TWIN_MAX = 0.04, 0.25


@pytest.mark.parametrize("d", [128, 64])
@pytest.mark.parametrize("B,H,N", [(1, 1, 77), (1, 2, 128), (2, 1, 300), (1, 1, 1000), (1, 2, 2049)])
def test_fp8_all_softmax_twin(pkg, oracle, B, H, N, d):
    """The all-E4M3 SoftMax twin against the oracle's SoftMax, on inputs of moderate size (N(0, 0.5)
    cast to E4M3).  Its weights are rounded to E4M3 like the spherical variant's scores, so the same
    statistical bounds apply: rms(err) <= 0.04 rms(O), max <= 0.25 rms(O).  Ragged N checks that
    keys past the end get no weight (a zero key row would get exp(-shift) > 0)."""
    print(f"case fp8-all softmax twin B={B} H={H} N={N} d={d}", flush=True)
    qf, kf, vf = si.gaussian_qkv(B, H, N, d, seed=950 + N, factor=0.5)
    q, k, v = (t.to(torch.float8_e4m3fn) for t in (qf, kf, vf))
    ws = torch.empty(pkg.sphattn_fp8_workspace_bytes(B, H, N, d), dtype=torch.uint8, device=DEV)
    out = pkg.sphattn_fp8_softmax_fwd(q.to(DEV), k.to(DEV), v.to(DEV), ws)
    torch.cuda.synchronize()
    got = out.cpu().to(torch.float64).numpy()
    ref = oracle.softmax_attention(*_bits(q, k, v), kinds=("e4m3fn",) * 3)
    assert np.all(np.isfinite(got))
    rms = np.sqrt((ref ** 2).mean())
    err = got - ref
    err_rms, err_max = np.sqrt((err ** 2).mean()) / rms, np.abs(err).max() / rms
    print(f"softmax twin vs oracle: rms {err_rms:.3e} max {err_max:.3e}", flush=True)
    assert err_rms <= TWIN_RMS and err_max <= TWIN_MAX


def test_fp8_all_backward_key_stream_with_ragged_tail(pkg, oracle):
    """More workgroups than run at once (330 at one per compute unit): every other batch of an XCD
    streams the keys from the last tile to the first, the ragged tile first.  Sampled rows of every
    head against the oracle-derived bounds."""
    B, H, N, d = 2, 5, 8237, 128
    print(f"case fp8-all key-stream direction B={B} H={H} N={N}", flush=True)
    q, k, v = si.make_qkv(B, H, N, d, "fp8", seed=4242)
    got = _run(pkg, q, k, v)
    assert np.all(np.isfinite(got))
    qb, kb, vb = _bits(q, k, v)
    rng = np.random.default_rng(6)
    for bh in range(B * H):
        b, h = divmod(bh, H)
        # one row of every 256-row query tile (each is one workgroup), first and last included
        rows = sorted({0, N - 1} | {int(t * 256 + rng.integers(min(256, N - t * 256))) for t in range((N + 255) // 256)})
        Q, K, V = (oracle.widen(x[b, h], "e4m3fn") for x in (qb, kb, vb))
        exact = oracle.spherical_attention_rows(qb, kb, vb, bh, rows, kinds=("e4m3fn",) * 3)
        S = Q[rows] @ K.T
        cap = np.sqrt((Q[rows] ** 2).sum(-1)) * np.sqrt((K * K).sum(-1)).max()
        _assert_within_oracle_bounds(got[b, h][rows], exact, S, V, cap, d, f"bh={bh}")
