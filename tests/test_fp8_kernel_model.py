"""CPU tests of tests/fp8_kernel_model.py: the model of the all-E4M3 kernel's rounding, and the
error bounds that test_gpu_fp8.py places around the paper-derived oracle.

The model is pinned by the library's own E4M3 cast, hand-computed cases and exact invariance
under power-of-two row scaling.  The bounds (oracle_error_bounds) are derived from the exact
scores alone; here they are checked for soundness with the model standing in for the kernel:
a rounding of the exact scores to E4M3 must fall inside them, and planted mistakes (a wrong
value column, a dropped key, truncation instead of rounding) must fall outside."""
import numpy as np
import pytest
import torch

import fp8_kernel_model as km
import synthetic_inputs as si


def _e4m3_values():
    """All finite E4M3 values, ascending, decoded by the library cast (not by the oracle)."""
    codes = torch.arange(256, dtype=torch.uint8)
    vals = codes.view(torch.float8_e4m3fn).to(torch.float64)
    return np.unique(vals[torch.isfinite(vals)].numpy())


def test_e4m3_rounding_fixed_points_midpoints_and_library_cast(oracle):
    vals = _e4m3_values()
    assert len(vals) == 253 and vals.max() == 448.0          # 2 * 126 non-zero magnitudes + zero
    # every representable value is a fixed point
    assert np.array_equal(km.round_to_e4m3(vals), vals)
    # a midpoint goes to the neighbour whose code is even (ties to even); just off it, to the nearer
    lo, hi = vals[:-1], vals[1:]
    mid = 0.5 * (lo + hi)
    codes = {float(v): int(c) for c, v in zip(range(256), torch.arange(256, dtype=torch.uint8)
                                              .view(torch.float8_e4m3fn).to(torch.float64).tolist()) if v == v}
    want = np.array([a if codes[float(a)] % 2 == 0 else b for a, b in zip(lo, hi)])
    nonzero = (lo != 0) | (hi != 0)
    assert np.array_equal(np.abs(km.round_to_e4m3(mid))[nonzero], np.abs(want)[nonzero])
    eps = 1e-9 * (hi - lo)
    assert np.array_equal(km.round_to_e4m3(mid - eps), lo)
    assert np.array_equal(km.round_to_e4m3(mid + eps), hi)
    # random values against the library's own cast
    g = torch.Generator().manual_seed(11)
    x = (torch.randn(100000, generator=g, dtype=torch.float64)
         * torch.logspace(-4, 2.4, 100000, dtype=torch.float64)).clamp(-448, 448)
    lib = x.to(torch.float32).to(torch.float8_e4m3fn).to(torch.float64).numpy()
    assert np.array_equal(km.round_to_e4m3(x.numpy()), lib)
    with pytest.raises(ValueError):
        km.round_to_e4m3(np.array([449.0]))


def test_e4m3_row_exponents_bound_the_scores(oracle):
    rng = np.random.default_rng(5)
    Q = rng.standard_normal((2, 2, 40, 16)) * np.exp(rng.standard_normal((2, 2, 40, 1)) * 3)
    K = rng.standard_normal((2, 2, 40, 16)) * np.exp(rng.standard_normal((2, 2, 40, 1)))
    Q[0, 0, 3] = 0.0
    e, m = km.e4m3_row_exponents(Q, K)
    S = Q @ np.swapaxes(K, -1, -2)
    scaled = np.abs(S) * np.ldexp(1.0, -e)[..., None]
    assert scaled.max() <= 440.0
    # the exponent is the smallest that does it for the Cauchy-Schwarz bound
    bound = np.sqrt((Q * Q).sum(-1)) * np.sqrt((K * K).sum(-1)).max(-1)[..., None]
    nz = bound > 0
    assert np.all(bound[nz] * np.ldexp(1.0, -e[nz]) > 220.0)
    assert e[0, 0, 3] == 0


def test_e4m3_model_close_to_exact_and_invariant_to_row_scaling(oracle):
    q, k, v = si.make_qkv(1, 2, 300, 64, "fp8", seed=21)
    bits = [si.storage_bits(t)[0] for t in (q, k, v)]
    kinds = ("e4m3fn",) * 3
    exact = oracle.spherical_attention(*bits, kinds=kinds)
    model = km.spherical_attention_e4m3_scores(*(oracle.widen(b, "e4m3fn") for b in bits))
    rms = np.sqrt((exact ** 2).mean())
    err = model - exact
    # rounding to 3 mantissa bits: relative error uniform in +-2^-4 at the bottom of a binade,
    # +-2^-5 at the top, about 0.026 rms; independent over the terms of the sum
    assert 0.015 <= np.sqrt((err ** 2).mean()) / rms <= 0.04
    assert np.abs(err).max() / rms <= 0.25
    # scaling a query row by a power of two shifts e_i and changes nothing else
    qs = oracle.widen(bits[0], "e4m3fn")
    ks, vs = oracle.widen(bits[1], "e4m3fn"), oracle.widen(bits[2], "e4m3fn")
    scale = np.ldexp(1.0, np.arange(300) % 7 - 3)[None, None, :, None]
    a = km.spherical_attention_e4m3_scores(qs, ks, vs)
    b = km.spherical_attention_e4m3_scores(qs * scale, ks, vs)
    assert np.array_equal(a, b)
    assert np.array_equal(a, model)
    # scaling all keys by a power of two: the same
    c = km.spherical_attention_e4m3_scores(qs, ks * 0.25, vs)
    assert np.array_equal(a, c)


def test_e4m3_model_brute_force_tiny(oracle):
    """Two keys, hand-checkable: q = (1, 0), k1 = (3, 0), k2 = (1, 1); v = 1, -1."""
    Q = np.array([[[[1.0, 0.0]]]])
    K = np.array([[[[3.0, 0.0], [1.0, 1.0]]]])
    V = np.array([[[[1.0], [-1.0]]]])
    # bound = 1 * 3 -> 3 / 440 = 0.8727.. * 2^-7 -> e = -7; scores 3, 1 -> 384, 128: both representable
    e, _ = km.e4m3_row_exponents(Q, K)
    assert e[0, 0, 0] == -7
    out = km.spherical_attention_e4m3_scores(Q, K, V)
    assert np.isclose(out[0, 0, 0, 0], (3.0 - 1.0) / np.sqrt(10.0), rtol=1e-15)
    # a score that is not representable: s = (1, 2.2) / bound 2.2 -> e = -7: 128, 281.6 -> 288
    K2 = np.array([[[[2.2, 0.0], [1.0, 0.0]]]])
    out2 = km.spherical_attention_e4m3_scores(Q, K2, V)
    assert np.isclose(out2[0, 0, 0, 0], (288.0 - 128.0) / np.sqrt(288.0 ** 2 + 128.0 ** 2), rtol=1e-15)


# ---------------------------------------------------------------------------
# Soundness of the oracle-derived bounds, the model standing in for the kernel
# ---------------------------------------------------------------------------
def _exact_parts(oracle, q, k, v):
    """Exact scores, values, output and score caps from the oracle's own outputs: s_ij = w_ij sqrt(z_i)."""
    bits = [si.storage_bits(t)[0] for t in (q, k, v)]
    kinds = ("e4m3fn",) * 3
    O, W, Z = oracle.spherical_attention_full(*bits, kinds=kinds)
    S = W * np.sqrt(Z)[..., None]
    Qw, Kw, Vw = (oracle.widen(b, "e4m3fn") for b in bits)
    cap = np.sqrt((Qw * Qw).sum(-1)) * np.sqrt((Kw * Kw).sum(-1)).max(-1)[..., None]
    return S, Vw, O, cap, (Qw, Kw, Vw)


@pytest.mark.parametrize("B,H,N,d,factor", [(1, 2, 33, 128, 1.0), (1, 1, 300, 128, 1.0), (2, 1, 1000, 64, 1.0),
                                            (1, 1, 400, 128, 2.0 ** -6), (1, 1, 2048, 128, 30.0)])
def test_bounds_hold_for_a_rounding_of_the_exact_scores(oracle, B, H, N, d, factor):
    q, k, v = si.make_qkv(B, H, N, d, "fp8", seed=40 + N, factor=factor)
    S, Vw, O, cap, (Qw, Kw, _) = _exact_parts(oracle, q, k, v)
    hard, sigma, own = km.oracle_error_bounds(S, Vw, O, cap, d)
    model = km.spherical_attention_e4m3_scores(Qw, Kw, Vw)
    err = np.abs(model - O)
    assert np.all(err <= hard)
    assert np.all(err <= 7.0 * sigma + own)
    # the bounds are not slack beyond use: typical sigma is a few percent of rms(O), and the
    # observed rms error is below the bound's rms but within a factor of two of it
    rms = np.sqrt((O ** 2).mean())
    assert np.sqrt((sigma ** 2).mean()) <= 0.06 * rms
    assert 0.4 * np.sqrt((sigma ** 2).mean()) <= np.sqrt((err ** 2).mean()) <= np.sqrt((sigma ** 2).mean())


def test_bounds_reject_planted_mistakes(oracle):
    q, k, v = si.make_qkv(1, 2, 300, 128, "fp8", seed=77)
    S, Vw, O, cap, (Qw, Kw, _) = _exact_parts(oracle, q, k, v)
    hard, sigma, own = km.oracle_error_bounds(S, Vw, O, cap, 128)
    stat = 7.0 * sigma + own

    def outside(out):
        return bool(np.any(np.abs(out - O) > stat))
    good = km.spherical_attention_e4m3_scores(Qw, Kw, Vw)
    assert not outside(good)
    # two value columns exchanged
    Vx = Vw.copy()
    Vx[..., [3, 4]] = Vx[..., [4, 3]]
    assert outside(km.spherical_attention_e4m3_scores(Qw, Kw, Vx))
    # the last 16 keys dropped (a ragged tail handled wrongly)
    assert outside(km.spherical_attention_e4m3_scores(Qw[:, :, :, :], Kw[:, :, :284], Vw[:, :, :284]))
    # scores rounded to two mantissa bits (the other 8-bit format's grid): twice the step
    e, _ = km.e4m3_row_exponents(Qw, Kw)
    T = S * np.ldexp(1.0, -e)[..., None]
    _, ex = np.frexp(np.abs(T))
    step = np.ldexp(1.0, np.maximum(ex - 1, -6) - 2)
    P = np.rint(T / step) * step
    coarse = (P @ Vw) / np.sqrt((P * P).sum(-1))[..., None]
    err = coarse - O
    assert np.sqrt((err ** 2).mean()) > np.sqrt((sigma ** 2).mean())     # fails the rms criterion
    # no row factor at all (scores far outside the E4M3 range would saturate or vanish): here
    # modelled as every score divided by 2^12 too much, so that most become subnormal
    Pt = km.round_to_e4m3(T * 2.0 ** -12)
    with np.errstate(invalid="ignore", divide="ignore"):
        tiny = np.nan_to_num((Pt @ Vw) / np.sqrt((Pt * Pt).sum(-1))[..., None])
    assert outside(tiny)


def test_bounds_with_multiplicities(oracle):
    """s_ij = m_j (q_i . k_j): the cap is |q_i| max_j m_j |k_j| and everything else is unchanged."""
    q, k, v = si.make_qkv(1, 2, 260, 128, "fp8", seed=78)
    Qw, Kw, Vw = (oracle.widen(si.storage_bits(t)[0], "e4m3fn") for t in (q, k, v))
    mult = np.random.default_rng(3).poisson(1.5, size=(1, 260)).astype(np.float64)
    bits = [si.storage_bits(t)[0] for t in (q, k, v)]
    O = oracle.grn_attention(*bits, mult, kinds=("e4m3fn",) * 3)
    o_raw, z = oracle.spherical_accumulate(*bits, mult, kinds=("e4m3fn",) * 3)
    S = np.matmul(Qw, np.swapaxes(Kw, -1, -2)) * mult[:, None, None, :]
    assert np.allclose((S * S).sum(-1), z, rtol=1e-12)                    # the scores used for the bound are the oracle's
    cap = np.sqrt((Qw * Qw).sum(-1)) * (np.sqrt((Kw * Kw).sum(-1)) * mult[:, None, :]).max(-1)[..., None]
    hard, sigma, own = km.oracle_error_bounds(S, Vw, O, cap, 128)
    model = km.spherical_attention_e4m3_scores(Qw, Kw, Vw, mult)
    err = np.abs(model - O)
    assert np.all(err <= hard) and np.all(err <= 7.0 * sigma + own)
