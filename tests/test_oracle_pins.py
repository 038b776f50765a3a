"""Pins for the CPU oracle: things the paper's definition and plain mathematics fix.

The oracle is the fp64 statement of spherical attention (paper, Appendix A.1,
Definition 2 with a1 = id, a2 = square, b = sqrt; Section 3).  None of these
tests calls the oracle to produce its own expected value: every expectation is
an exact-rational brute force, a hand-worked example, a closed form, a library
routine, or an invariant.  Each also lists the mistakes it would catch.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# ---------------------------------------------------------------- worked example
def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = line.split()
            vals[parts[0]] = [float(x) for x in parts[1:]]
    return vals


def test_hand_worked_example(oracle):
    """Catches: transposed K or V, missing sqrt, sum |s| instead of s^2, weights not signed."""
    g = _read_golden("hand_worked_2x2.txt")
    Q = np.array(g["Q"]).reshape(1, 1, 2, 2)
    K = np.array(g["K"]).reshape(1, 1, 2, 2)
    V = np.array(g["V"]).reshape(1, 1, 2, 2)
    O, W, Z = oracle.spherical_attention_full(Q, K, V)
    np.testing.assert_allclose(O[0, 0, 0] * math.sqrt(10.0), g["O_times_sqrt10_row0"], rtol=1e-15)
    np.testing.assert_allclose(O[0, 0, 1], g["O_row1"], rtol=1e-15)
    np.testing.assert_array_equal(Z[0, 0], g["z"])


# ---------------------------------------------------------------- exact brute force
def _brute_force_exact(Q, K, V):
    """Literal triple loop in exact rationals: returns (o_raw, z) per row."""
    N, d = len(Q), len(Q[0])
    dv = len(V[0])
    o_raw = [[Fraction(0)] * dv for _ in range(N)]
    z = [Fraction(0)] * N
    for i in range(N):
        for j in range(len(K)):
            s = sum(Q[i][k] * K[j][k] for k in range(d))
            z[i] += s * s
            for c in range(dv):
                o_raw[i][c] += s * V[j][c]
    return o_raw, z


@pytest.mark.parametrize("N,d,seed", [(1, 1, 0), (2, 3, 1), (5, 2, 2), (8, 4, 3), (7, 3, 4)])
def test_brute_force_rationals(oracle, N, d, seed):
    """Dyadic-rational inputs are exact in fp64, so the oracle must match the exact
    (o_raw, z) to the last few ulps.  Catches any dropped term, wrong index or sign."""
    rng = np.random.default_rng(seed)
    Qi = rng.integers(-9, 10, size=(N, d))
    Ki = rng.integers(-9, 10, size=(N, d))
    Vi = rng.integers(-9, 10, size=(N, d))
    Qf = [[Fraction(int(x), 4) for x in r] for r in Qi]
    Kf = [[Fraction(int(x), 2) for x in r] for r in Ki]
    Vf = [[Fraction(int(x), 8) for x in r] for r in Vi]
    o_raw, z = _brute_force_exact(Qf, Kf, Vf)
    O, W, Z = oracle.spherical_attention_full((Qi / 4.0).reshape(1, 1, N, d),
                                              (Ki / 2.0).reshape(1, 1, N, d),
                                              (Vi / 8.0).reshape(1, 1, N, d))
    for i in range(N):
        assert Z[0, 0, i] == float(z[i])            # exact: small dyadic rationals
        for c in range(d):
            if z[i] == 0:
                assert O[0, 0, i, c] == 0.0
            else:
                want = float(o_raw[i][c]) / math.sqrt(float(z[i]))
                assert O[0, 0, i, c] == pytest.approx(want, rel=4e-16, abs=1e-300)


# ---------------------------------------------------------------- invariants
def test_unit_norm_weight_rows(oracle):
    """Weights of each query row lie on the unit sphere (L2 normalization)."""
    Q, K, V = (_rand((2, 3, 37, 8), s) for s in (10, 11, 12))
    _, W, Z = oracle.spherical_attention_full(Q, K, V)
    np.testing.assert_allclose((W ** 2).sum(-1), 1.0, rtol=1e-13)
    # and the weights keep the sign of the raw scores (signed attention)
    S = np.einsum("bhik,bhjk->bhij", Q, K)
    assert np.array_equal(np.sign(W), np.sign(S))
    np.testing.assert_allclose(Z, (S ** 2).sum(-1), rtol=1e-13)


def test_output_is_weights_times_v(oracle):
    Q, K, V = (_rand((1, 2, 19, 5), s) for s in (13, 14, 15))
    O, W, _ = oracle.spherical_attention_full(Q, K, V)
    np.testing.assert_allclose(O, np.einsum("bhij,bhjc->bhic", W, V), rtol=1e-12, atol=1e-14)


def test_cauchy_schwarz_bound(oracle):
    Q, K, V = (_rand((1, 2, 50, 6), s) for s in (16, 17, 18))
    O = oracle.spherical_attention(Q, K, V)
    bound = np.sqrt((V ** 2).sum(axis=2, keepdims=True))
    assert np.all(np.abs(O) <= bound * (1 + 1e-12))


def test_scale_and_sign_invariance(oracle):
    """Positive per-query-row factors on Q and a positive scalar on K cancel; a sign flip
    of Q flips the output (the weights are signed).  Catches a stray 1/sqrt(d) or epsilon
    that does not cancel, and abs() in the weights."""
    Q, K, V = (_rand((2, 2, 23, 7), s) for s in (19, 20, 21))
    O = oracle.spherical_attention(Q, K, V)
    alpha = np.random.default_rng(22).uniform(0.01, 100.0, size=(2, 2, 23, 1))
    np.testing.assert_allclose(oracle.spherical_attention(alpha * Q, 37.5 * K, V), O,
                               rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.spherical_attention(1e-6 * Q, 1e-6 * K, V), O,
                               rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.spherical_attention(-Q, K, V), -O, rtol=1e-15)


def test_linearity_in_v(oracle):
    Q, K, V = (_rand((1, 3, 17, 4), s) for s in (23, 24, 25))
    V2 = _rand((1, 3, 17, 4), 26)
    lhs = oracle.spherical_attention(Q, K, 2.5 * V + V2)
    rhs = 2.5 * oracle.spherical_attention(Q, K, V) + oracle.spherical_attention(Q, K, V2)
    np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-13)


def test_single_key_closed_form(oracle):
    """N = 1: the only weight is s/|s| = sign(q.k), so O = sign(q.k) v."""
    q, k, v = (_rand((4, 2, 1, 6), s) for s in (27, 28, 29))
    O = oracle.spherical_attention(q, k, v)
    sgn = np.sign((q * k).sum(-1, keepdims=True))
    np.testing.assert_allclose(O, sgn * v, rtol=1e-15)


def test_orthonormal_keys_closed_form(oracle):
    """K = identity (N = d): scores are q itself, so O_i = q_i V / ||q_i||_2."""
    d = 9
    Q = _rand((1, 2, d, d), 30)
    V = _rand((1, 2, d, d), 31)
    K = np.broadcast_to(np.eye(d), (1, 2, d, d)).copy()
    O = oracle.spherical_attention(Q, K, V)
    want = np.matmul(Q, V) / np.linalg.norm(Q, axis=-1, keepdims=True)
    np.testing.assert_allclose(O, want, rtol=1e-13, atol=1e-15)


def test_gram_matrix_closed_form(oracle):
    """Because a1 is the identity, sum_j s_ij v_j = q_i (K^T V) and z_i = q_i (K^T K) q_i^T:
    the whole result follows from two d x d matrices and textbook matmuls.  N != d and
    unequal heads catch transposes and head mix-ups."""
    Q, K, V = (_rand((2, 3, 131, 16), s) for s in (32, 33, 34))
    O = oracle.spherical_attention(Q, K, V)
    KtV = np.matmul(K.transpose(0, 1, 3, 2), V)
    G = np.matmul(K.transpose(0, 1, 3, 2), K)
    z = np.einsum("bhik,bhkl,bhil->bhi", Q, G, Q)
    want = np.matmul(Q, KtV) / np.sqrt(z)[..., None]
    np.testing.assert_allclose(O, want, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("chunk", [1, 2, 3, 7, 16, 29, 30, 64])
def test_streaming_identity(oracle, chunk):
    """Lemma 1: carrying (o, z) over key chunks of any size reproduces the direct result."""
    Q, K, V = (_rand((1, 2, 29, 5), s) for s in (35, 36, 37))
    direct = oracle.spherical_attention(Q, K, V)
    np.testing.assert_allclose(oracle.spherical_attention_streamed(Q, K, V, chunk), direct,
                               rtol=1e-12, atol=1e-14)


def test_bag_invariances(oracle):
    """Keys form a bag: permuting (K,V) rows together changes nothing; appending zero key
    rows (with arbitrary value rows) changes nothing."""
    Q, K, V = (_rand((1, 2, 21, 6), s) for s in (38, 39, 40))
    O = oracle.spherical_attention(Q, K, V)
    perm = np.random.default_rng(41).permutation(21)
    # only K and V are permuted; Q (and hence the output rows) stay in place, so build by hand
    S = np.einsum("bhik,bhjk->bhij", Q, K[:, :, perm])
    Wp = S / np.sqrt((S ** 2).sum(-1, keepdims=True))
    np.testing.assert_allclose(np.matmul(Wp, V[:, :, perm]), O, rtol=1e-12, atol=1e-14)
    # zero padding through the oracle itself, on a rectangular brute-force check
    pad = 11
    Kp = np.concatenate([K, np.zeros((1, 2, pad, 6))], axis=2)
    Vp = np.concatenate([V, _rand((1, 2, pad, 6), 42)], axis=2)
    Qp = np.concatenate([Q, _rand((1, 2, pad, 6), 43)], axis=2)
    Op = oracle.spherical_attention(Qp, Kp, Vp)
    np.testing.assert_allclose(Op[:, :, :21], O, rtol=1e-13, atol=1e-15)


def test_zero_score_row_gives_zero(oracle):
    """No epsilon is defined; a row whose scores are all zero has a zero numerator and is 0."""
    Q, K, V = (_rand((1, 1, 6, 4), s) for s in (44, 45, 46))
    Q[0, 0, 2] = 0.0
    O = oracle.spherical_attention(Q, K, V)
    assert np.all(O[0, 0, 2] == 0.0)
    assert np.all(np.isfinite(O))


def test_rows_entry_matches_heads(oracle):
    """The sampled-row entry point reads the right head and rows (checked against the
    Gram closed form, not against the full entry point)."""
    Q, K, V = (_rand((2, 2, 40, 8), s) for s in (47, 48, 49))
    rows = [0, 39, 7, 7, 21]
    for bh in range(4):
        b, h = divmod(bh, 2)
        got = oracle.spherical_attention_rows(Q, K, V, bh, rows)
        q = Q[b, h, rows]
        KtV = K[b, h].T @ V[b, h]
        G = K[b, h].T @ K[b, h]
        want = (q @ KtV) / np.sqrt(np.einsum("ik,kl,il->i", q, G, q))[:, None]
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-13)


# ---------------------------------------------------------------- stored formats
def test_bf16_widening_all_codes(oracle):
    import torch
    bits = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.widen(bits, "bf16")
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    m = ~np.isnan(want)
    np.testing.assert_array_equal(got[m], want[m])


def test_e4m3fn_widening_all_codes(oracle):
    """All 256 codes against the published format: checked against torch's decoder and
    against the format's landmarks (max 448, min subnormal 2^-9, NaN only at S.1111.111)."""
    import torch
    bits = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(bits).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = oracle.widen(bits, "e4m3fn")
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    m = ~np.isnan(want)
    np.testing.assert_array_equal(got[m], want[m])
    assert got[0x7E] == 448.0 and got[0xFE] == -448.0
    assert got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6 and got[0x38] == 1.0
    assert np.isnan(got[0x7F]) and np.isnan(got[0xFF]) and np.isnan(got).sum() == 2


def test_stored_formats_feed_the_same_values(oracle):
    """bf16 / e4m3fn inputs give exactly what the widened fp64 values give."""
    import torch
    import synthetic_inputs as si
    q, k, v = si.make_qkv(1, 2, 33, 16, "fp8qk_bf16v", seed=5)
    (qb, qk), (kb, kk), (vb, vk) = (si.storage_bits(t) for t in (q, k, v))
    O1 = oracle.spherical_attention(qb, kb, vb, kinds=(qk, kk, vk))
    O2 = oracle.spherical_attention(q.to(torch.float64).numpy(), k.to(torch.float64).numpy(),
                                    v.to(torch.float64).numpy())
    np.testing.assert_array_equal(O1, O2)


# ---------------------------------------------------------------- softmax twin
def test_softmax_twin_against_library(oracle):
    """The comparison twin is textbook attention: check it against scipy's softmax."""
    from scipy.special import softmax
    Q, K, V = (_rand((2, 2, 45, 8), s) for s in (50, 51, 52))
    O = oracle.softmax_attention(Q, K, V)
    P = softmax(np.einsum("bhik,bhjk->bhij", Q, K) / math.sqrt(8), axis=-1)
    np.testing.assert_allclose(O, np.matmul(P, V), rtol=1e-12, atol=1e-14)
    ones = np.ones_like(V)
    np.testing.assert_allclose(oracle.softmax_attention(Q, K, ones), ones, rtol=1e-13)
    rows = [3, 44]
    np.testing.assert_allclose(oracle.softmax_attention_rows(Q, K, V, 3, rows), O[1, 1, rows],
                               rtol=1e-13)


# ---------------------------------------------------------------- GRN variant (Section 3.1)
def _grn_numpy(Q, K, V, mult, H_kv):
    """The same definition written with numpy primitives: keys scaled by multiplicity, K/V heads
    repeated over their query-head groups."""
    B, H, N, d = Q.shape
    rep = H // H_kv
    Kx = np.repeat(K, rep, axis=1)
    Vx = np.repeat(V, rep, axis=1)
    if mult is not None:
        Kx = Kx * mult[:, None, :, None]
    S = np.einsum("bhik,bhjk->bhij", Q, Kx)
    W = S / np.sqrt((S ** 2).sum(-1, keepdims=True))
    return np.matmul(W, Vx)


@pytest.mark.parametrize("H,H_kv", [(4, 4), (4, 2), (6, 1), (3, 3)])
def test_grn_variant_against_numpy_definition(oracle, H, H_kv):
    """Catches a wrong group index (h % H_kv instead of h // group), multiplicities applied per
    query instead of per key, or to the wrong batch row."""
    B, N, d = 2, 23, 5
    Q = _rand((B, H, N, d), 60)
    K = _rand((B, H_kv, N, d), 61)
    V = _rand((B, H_kv, N, d), 62)
    mult = np.random.default_rng(63).integers(0, 6, size=(B, N)).astype(np.float64)
    mult[:, 0] = 3.0
    np.testing.assert_allclose(oracle.grn_attention(Q, K, V, mult), _grn_numpy(Q, K, V, mult, H_kv),
                               rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.grn_attention(Q, K, V, None), _grn_numpy(Q, K, V, None, H_kv),
                               rtol=1e-12, atol=1e-14)
    rows = [0, 22, 9]
    for bh in range(B * H):
        b, h = divmod(bh, H)
        np.testing.assert_allclose(oracle.grn_attention_rows(Q, K, V, mult, bh, rows),
                                   _grn_numpy(Q, K, V, mult, H_kv)[b, h, rows], rtol=1e-12, atol=1e-14)


def test_grn_multiplicity_brute_force_rationals(oracle):
    """Exact rationals: s_ij = m_j (q_i . k_j); a gene with multiplicity 0 drops out, integer
    multiplicity m equals m copies of the key only through the score scale (not the bag size)."""
    rng = np.random.default_rng(64)
    N, d = 6, 3
    Qi, Ki, Vi = (rng.integers(-5, 6, size=(N, d)) for _ in range(3))
    m = [2, 0, 1, 3, 1, 5]
    Qf = [[Fraction(int(x), 2) for x in r] for r in Qi]
    Kf = [[Fraction(int(x)) * m[j] for x in r] for j, r in enumerate(Ki)]
    Vf = [[Fraction(int(x), 4) for x in r] for r in Vi]
    o_raw, z = _brute_force_exact(Qf, Kf, Vf)
    O = oracle.grn_attention((Qi / 2.0).reshape(1, 1, N, d), Ki.astype(np.float64).reshape(1, 1, N, d),
                             (Vi / 4.0).reshape(1, 1, N, d), np.array([m], dtype=np.float64))
    for i in range(N):
        for c in range(d):
            want = 0.0 if z[i] == 0 else float(o_raw[i][c]) / math.sqrt(float(z[i]))
            assert O[0, 0, i, c] == pytest.approx(want, rel=4e-16, abs=1e-300)


def test_grn_uniform_multiplicity_cancels(oracle):
    """A constant multiplicity is a positive scale on K and cancels in the normalisation."""
    Q, K, V = (_rand((1, 2, 17, 4), s) for s in (65, 66, 67))
    np.testing.assert_allclose(oracle.grn_attention(Q, K, V, np.full((1, 17), 7.0)),
                               oracle.spherical_attention(Q, K, V), rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- other normalizers (Theorem 1)
@pytest.mark.parametrize("name", ["l1", "sqrelu"])
def test_other_normalizers_against_numpy_definition(oracle, name):
    """N(x)_i = a1(x_i) / b(sum a2(x_j)) written with numpy; scale invariance; rows entry."""
    Q, K, V = (_rand((2, 2, 37, 6), s) for s in (70, 71, 72))
    S = np.einsum("bhik,bhjk->bhij", Q, K)
    if name == "l1":
        W = S / np.abs(S).sum(-1, keepdims=True)
        assert np.allclose(np.abs(W).sum(-1), 1.0)
    else:
        R = np.maximum(S, 0.0) ** 2
        W = R / R.sum(-1, keepdims=True)
        assert np.allclose(W.sum(-1), 1.0) and W.min() >= 0.0
    want = np.matmul(W, V)
    got = oracle.normalized_attention(Q, K, V, name)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oracle.normalized_attention(3.0 * Q, 0.25 * K, V, name), got, rtol=1e-12, atol=1e-14)
    rows = [0, 36, 5]
    np.testing.assert_allclose(oracle.normalized_attention_rows(Q, K, V, name, 3, rows), want[1, 1, rows],
                               rtol=1e-12, atol=1e-14)


def test_normalizer_names_agree_with_the_dedicated_entries(oracle):
    Q, K, V = (_rand((1, 2, 21, 4), s) for s in (73, 74, 75))
    np.testing.assert_array_equal(oracle.normalized_attention(Q, K, V, "l2"), oracle.spherical_attention(Q, K, V))
    np.testing.assert_array_equal(oracle.normalized_attention(Q, K, V, "softmax"), oracle.softmax_attention(Q, K, V))


def test_sqrelu_row_without_positive_scores_is_zero(oracle):
    Q = -np.abs(_rand((1, 1, 5, 3), 76))
    K = np.abs(_rand((1, 1, 5, 3), 77))
    V = _rand((1, 1, 5, 3), 78)
    assert np.all(oracle.normalized_attention(Q, K, V, "sqrelu") == 0.0)


def test_f16_widening_all_codes(oracle):
    """All 65536 binary16 codes against numpy's float16, plus landmarks of the format."""
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = oracle.widen(bits, "f16")
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want))
    m = ~np.isnan(want)
    np.testing.assert_array_equal(got[m], want[m])
    assert got[0x3C00] == 1.0 and got[0x7BFF] == 65504.0 and got[0x0001] == 2.0 ** -24
    assert got[0x7C00] == np.inf and got[0xFC00] == -np.inf


# ---------------------------------------------------------------- the bare accumulator of Lemma 1
def test_accumulator_brute_force_rationals_rectangular(oracle):
    """(o_raw, z) without the tail, N_q != N_k, two query heads sharing one K/V head, with
    multiplicities: exact rationals.  Catches a wrong N in an index, a missing multiplicity,
    a tail applied by mistake, z from |x| or from the unscaled score."""
    rng = np.random.default_rng(90)
    Nq, Nk, d = 3, 5, 2
    Qi = rng.integers(-5, 6, size=(2, Nq, d))
    Ki, Vi = rng.integers(-5, 6, size=(Nk, d)), rng.integers(-5, 6, size=(Nk, d))
    m = [1, 3, 0, 2, 1]
    o_raw, z = oracle.spherical_accumulate((Qi / 2.0).reshape(1, 2, Nq, d), Ki.astype(np.float64).reshape(1, 1, Nk, d),
                                           (Vi / 4.0).reshape(1, 1, Nk, d), np.array([m], dtype=np.float64))
    Kf = [[Fraction(int(x)) * m[j] for x in r] for j, r in enumerate(Ki)]
    Vf = [[Fraction(int(x), 4) for x in r] for r in Vi]
    for h in range(2):
        Qf = [[Fraction(int(x), 2) for x in r] for r in Qi[h]]
        want_o, want_z = _brute_force_exact(Qf, Kf, Vf)
        for i in range(Nq):
            assert z[0, h, i] == float(want_z[i])
            for c in range(d):
                assert o_raw[0, h, i, c] == float(want_o[i][c])


def test_accumulator_single_key_closed_form(oracle):
    """One key: o = (m q.k) v and z = (m q.k)^2, for any number of query rows."""
    Q = _rand((2, 3, 7, 4), 91)
    K, V = _rand((2, 3, 1, 4), 92), _rand((2, 3, 1, 4), 93)
    m = np.array([[2.5], [0.5]])
    o_raw, z = oracle.spherical_accumulate(Q, K, V, m)
    s = np.einsum("bhik,bhk->bhi", Q, K[:, :, 0]) * m[:, None, :]
    np.testing.assert_allclose(z, s * s, rtol=1e-14)
    np.testing.assert_allclose(o_raw, s[..., None] * V[:, :, 0][:, :, None, :], rtol=1e-14)


@pytest.mark.parametrize("cuts", [(0, 37), (0, 1, 37), (0, 16, 32, 37), (0, 5, 6, 30, 37)])
def test_accumulators_add_over_key_partitions_and_tail_gives_attention(oracle, cuts):
    """Lemma 1: the accumulators of the slices of any partition of the key axis add up, and the
    tail of the sum is the attention output (pinned above by other means)."""
    Q, K, V = _rand((2, 4, 37, 8), 94), _rand((2, 2, 37, 8), 95), _rand((2, 2, 37, 8), 96)
    m = np.random.default_rng(97).uniform(0.5, 4.0, size=(2, 37))
    parts = [oracle.spherical_accumulate(Q, K[:, :, a:b], V[:, :, a:b], m[:, a:b])
             for a, b in zip(cuts[:-1], cuts[1:])]
    O = oracle.spherical_tail(np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts]))
    np.testing.assert_allclose(O, _grn_numpy(Q, K, V, m, 2), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(O, oracle.grn_attention(Q, K, V, m), rtol=1e-11, atol=1e-13)


def test_tail_of_zero_accumulator_is_zero(oracle):
    o = np.zeros((2, 1, 1, 3, 4))
    z = np.zeros((2, 1, 1, 3))
    o[0, 0, 0, 1], z[0, 0, 0, 1] = [3.0, 0.0, -4.0, 1.0], 4.0
    out = oracle.spherical_tail(o, z)
    np.testing.assert_array_equal(out[0, 0, 0], 0.0)
    np.testing.assert_array_equal(out[0, 0, 2], 0.0)
    np.testing.assert_array_equal(out[0, 0, 1], [1.5, 0.0, -2.0, 0.5])


# ---------------------------------------------------------------- backward (derived, not in the paper)
def _loss(oracle, Q, K, V, dO):
    return float((oracle.spherical_attention(Q, K, V) * dO).sum())


def test_backward_against_central_differences(oracle):
    """Every gradient entry of a small problem against (L(x+h) - L(x-h)) / 2h of the forward
    oracle, L = sum(O * dO).  Catches a wrong sign or factor in the term through z, a missing
    r, swapped q/k in dK, and index slips."""
    Q, K, V, dO = (_rand((1, 2, 5, 3), s) for s in (110, 111, 112, 113))
    dQ, dK, dV = oracle.spherical_attention_bwd(Q, K, V, dO)
    h = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for idx in np.ndindex(X.shape):
            old = X[idx]
            X[idx] = old + h
            up = _loss(oracle, Q, K, V, dO)
            X[idx] = old - h
            dn = _loss(oracle, Q, K, V, dO)
            X[idx] = old
            assert G[idx] == pytest.approx((up - dn) / (2 * h), rel=2e-6, abs=2e-8), (name, idx)


def test_backward_against_library_autograd(oracle):
    """torch.autograd through a plain fp64 statement of Definition 2 (matmul, square, sum, sqrt)."""
    import torch
    Qn, Kn, Vn, Gn = (_rand((2, 3, 19, 8), s) for s in (114, 115, 116, 117))
    Q, K, V = (torch.tensor(x, requires_grad=True) for x in (Qn, Kn, Vn))
    S = Q @ K.transpose(-1, -2)
    O = (S @ V) / S.pow(2).sum(-1, keepdim=True).sqrt()
    (O * torch.tensor(Gn)).sum().backward()
    dQ, dK, dV = oracle.spherical_attention_bwd(Qn, Kn, Vn, Gn)
    np.testing.assert_allclose(dQ, Q.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, K.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, V.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_backward_structure(oracle):
    """dV = W^T dO with the forward oracle's weights (O is linear in V); Euler's identity for
    the scale invariances of the forward: q_i . dQ_i = 0 for every row and
    sum_j k_j . dK_j = 0 for every head."""
    Q, K, V, dO = (_rand((1, 2, 23, 6), s) for s in (118, 119, 120, 121))
    dQ, dK, dV = oracle.spherical_attention_bwd(Q, K, V, dO)
    _, W, _ = oracle.spherical_attention_full(Q, K, V)
    np.testing.assert_allclose(dV, np.einsum("bhij,bhik->bhjk", W, dO), rtol=1e-11, atol=1e-13)
    scale = np.abs(dQ).max() * np.abs(Q).max()
    assert np.abs((Q * dQ).sum(-1)).max() <= 1e-12 * scale * Q.shape[-1]
    assert np.abs((K * dK).sum((-1, -2))).max() <= 1e-12 * np.abs(dK).max() * np.abs(K).max() * K.shape[-1] * K.shape[-2]


def test_backward_takes_stored_formats(oracle):
    import torch
    import synthetic_inputs as si
    q, k, v = si.make_qkv(1, 2, 17, 8, "bf16", seed=122)
    g = torch.randn(q.shape, generator=torch.Generator().manual_seed(123)).to(torch.bfloat16)
    bits = [si.storage_bits(t)[0] for t in (q, k, v, g)]
    a = oracle.spherical_attention_bwd(*bits, kinds=("bf16",) * 4)
    b = oracle.spherical_attention_bwd(*(t.double().numpy() for t in (q, k, v, g)))
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_grn_backward_against_central_differences_and_autograd(oracle):
    """Multiplicities and shared K/V heads in the backward: central differences of the forward
    oracle on a tiny problem, library autograd on a larger one.  Catches a multiplicity applied
    once instead of twice on the way to dQ/dK, and K/V gradients not summed over a group."""
    import torch
    Q, dO = _rand((1, 4, 5, 3), 130), _rand((1, 4, 5, 3), 131)
    K, V = _rand((1, 2, 5, 3), 132), _rand((1, 2, 5, 3), 133)
    m = np.array([[2.0, 0.0, 1.0, 3.0, 0.5]])
    dQ, dK, dV = oracle.grn_attention_bwd(Q, K, V, dO, m)
    loss = lambda: float((oracle.grn_attention(Q, K, V, m) * dO).sum())
    h = 1e-6
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for idx in np.ndindex(X.shape):
            old = X[idx]
            X[idx] = old + h
            up = loss()
            X[idx] = old - h
            dn = loss()
            X[idx] = old
            assert G[idx] == pytest.approx((up - dn) / (2 * h), rel=2e-6, abs=2e-8), (name, idx)
    Qn, Gn = _rand((2, 6, 17, 8), 134), _rand((2, 6, 17, 8), 135)
    Kn, Vn = _rand((2, 3, 17, 8), 136), _rand((2, 3, 17, 8), 137)
    mn = np.random.default_rng(138).uniform(0.5, 3.0, size=(2, 17))
    Qt, Kt, Vt = (torch.tensor(x, requires_grad=True) for x in (Qn, Kn, Vn))
    Ke, Ve = Kt.repeat_interleave(2, dim=1), Vt.repeat_interleave(2, dim=1)
    S = (Qt @ Ke.transpose(-1, -2)) * torch.tensor(mn)[:, None, None, :]
    O = (S @ Ve) / S.pow(2).sum(-1, keepdim=True).sqrt()
    (O * torch.tensor(Gn)).sum().backward()
    dQ, dK, dV = oracle.grn_attention_bwd(Qn, Kn, Vn, Gn, mn)
    np.testing.assert_allclose(dQ, Qt.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dK, Kt.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(dV, Vt.grad.numpy(), rtol=1e-10, atol=1e-12)
