"""A MODEL OF THE KERNEL in csrc/sphattn_fp8.hpp (the all-E4M3 forward) -- not an oracle.

The paper defines spherical attention (Appendix A.1, Definition 2 with a1 = id, a2 = square,
b = sqrt); it says nothing about rounding the scores to E4M3.  How the kernel does that (each
row divided by a power of two chosen from the Cauchy-Schwarz bound, round to nearest even,
both sums over the rounded values) is this build's design, so a restatement of it cannot
serve as the reference that proves parity.  It lives here, with the tests, for two uses:
  * a regression check of the kernel's rounding (tests/test_gpu_fp8.py, "vs model"), and
  * a CPU stand-in for the kernel when the error bounds that ARE derived from the paper's
    oracle (oracle_error_bounds below) are checked for soundness without a GPU.
Parity of sphattn_fp8_fwd rests on oracle_error_bounds around oracle.spherical_attention.
"""
from __future__ import annotations

import numpy as np

E4M3_SCORE_LIMIT = 440.0       # the kernel scales each row so that no score can exceed this


def round_to_e4m3(x: np.ndarray) -> np.ndarray:
    """Nearest OCP E4M3 value (ties to even) of every element of the fp64 array x, |x| <= 448:
    three mantissa bits, least normal exponent -6, subnormals in steps of 2^-9."""
    x = np.asarray(x, dtype=np.float64)
    ax = np.abs(x)
    if ax.size and ax.max() > 448.0:
        raise ValueError("outside the E4M3 range")
    _, ex = np.frexp(ax)                       # ax = m 2^ex with m in [0.5, 1): leading bit is 2^(ex-1)
    lead = np.maximum(ex - 1, -6)              # subnormals share the exponent of the least normal
    step = np.ldexp(1.0, lead - 3)
    return np.copysign(np.rint(ax / step) * step, x)


def e4m3_row_exponents(Q, K, mult=None):
    """The power of two by which the kernel divides the scores of row i before it rounds them:
    e_i with |q_i| max_j (m_j |k_j|) / 440 = m 2^e_i, m in [0.5, 1) (e_i = 0 for a zero bound).
    Q [B,H,N,d], K [B,H,N,d] fp64, mult [B,N] or None; returns (e [B,H,N] int, m [B,H,N])."""
    qn = np.sqrt((Q * Q).sum(-1))
    kn = np.sqrt((K * K).sum(-1))
    if mult is not None:
        kn = kn * np.abs(np.asarray(mult, dtype=np.float64))[:, None, :]
    bound = qn * kn.max(-1)[..., None]
    m, e = np.frexp(bound / E4M3_SCORE_LIMIT)
    e = np.where(bound > 0.0, e, 0)
    return e, m


def spherical_attention_e4m3_scores(Q, K, V, mult=None) -> np.ndarray:
    """What the kernel computes, in fp64: the scores of row i (times the multiplicities, if
    any) are divided by 2^e_i and rounded to E4M3, and O_i = (sum_j p_ij v_j) / sqrt(sum_j
    p_ij^2) is formed from the ROUNDED scores p_ij.  Q, K, V fp64 [B,H,N,d] (same head count)."""
    e, _ = e4m3_row_exponents(Q, K, mult)
    S = np.matmul(Q, np.swapaxes(K, -1, -2))
    if mult is not None:
        S = S * np.asarray(mult, dtype=np.float64)[:, None, None, :]
    P = round_to_e4m3(S * np.ldexp(1.0, -e)[..., None])
    o = np.matmul(P, V)
    z = (P * P).sum(-1)
    out = np.zeros_like(o)
    nz = z > 0.0
    out[nz] = o[nz] / np.sqrt(z[nz])[:, None]
    return out


def oracle_error_bounds(S, V, O_ref, score_cap, d, out_half_ulp=2.0 ** -9):
    """Error bounds for an implementation that rounds every score to E4M3 before the second
    contraction, derived from the EXACT quantities of the paper's definition only.

    S [..., R, N] are the exact scores s_ij of R query rows (fp64, from the oracle), V [..., N, c]
    the values, O_ref [..., R, c] the oracle's output, score_cap [..., R] an upper bound c_i of the
    |s_ij| of row i (Cauchy-Schwarz: |q_i| max_j |k_j|) and d the head dimension.  The entry
    point's contract (its header) is that row i is divided by a power of two 2^e_i with
    c_i / 2^e_i in (220, 440], then rounded to nearest; nothing else about the implementation
    enters.  In the units of s:

      * a normal E4M3 value has 3 mantissa bits: |p - s| <= 2^-4 |s|;
      * below the least normal 2^-6 the grid step is 2^-9 (scaled units): |p - s| <= 2^-10 2^e_i
        <= 2^-10 c_i / 220;
      * the score that is rounded is an fp32 dot product of d products, off by at most
        eta = d 2^-24 c_i, which can also move it across a rounding boundary.
      So |p_ij - s_ij| <= eps_ij = 2^-4 |s_ij| + 2^-10 c_i / 220 + (1 + 2^-4) eta_i.

    With a = sum_j s_ij v_j, n = |s_i|_2 (O = a / n) and the same from p:
        O' - O = (a' - a) / n' + O (n - n') / n',   |a' - a| <= sum_j eps_ij |v_jc|,
        |n' - n| <= |eps_i|_2,   n' >= n - |eps_i|_2
    gives the WORST-CASE bound  hard = (sum_j eps_ij |v_jc| + |O_c| |eps_i|_2) / (n - |eps_i|_2),
    attained only if every rounding error had the worst size and sign.  To first order the
    output error is sum_j g_ijc (p_ij - s_ij) with g_ijc = (v_jc - O_c s_ij / n) / n; rounding
    errors are spread over +-eps_ij with variance at most eps_ij^2 / 3 and vary independently
    from score to score, so the error of one output has standard deviation at most
        sigma_ic = sqrt(sum_j g_ijc^2 eps_ij^2 / 3).
    Both get the output's own rounding added: |O| * out_half_ulp (bfloat16: 2^-9), plus fp32
    accumulation of N terms (2^-24 sqrt(N) relative, negligible but stated).

    Returns (hard, sigma, own), each shaped like O_ref; `own` is the output-rounding part, which
    is already inside `hard` and has to be added to k * sigma by the caller.  Rows with n = 0 get
    bound 0 (O must be 0); rows whose scores all lie below the E4M3 grid (n <= |eps|) get inf."""
    S = np.asarray(S, dtype=np.float64)
    absV = np.abs(V)
    cap = np.asarray(score_cap, dtype=np.float64)[..., None]
    eta = d * 2.0 ** -24 * cap
    eps = 2.0 ** -4 * np.abs(S) + 2.0 ** -10 * cap / 220.0 + (1.0 + 2.0 ** -4) * eta
    n = np.sqrt((S * S).sum(-1))[..., None]
    en = np.sqrt((eps * eps).sum(-1))[..., None]
    live = (n > en)
    den = np.where(live, n - en, 1.0)
    hard = (np.matmul(eps, absV) + np.abs(O_ref) * en) / den
    nn = np.where(n > 0, n, 1.0)
    # sigma^2 = sum_j (v_jc - O_c s_j / n)^2 eps_j^2 / (3 n^2), expanded so that no [R, N, c] array is formed
    e2 = eps * eps
    t0 = np.matmul(e2, V * V)
    t1 = np.matmul(e2 * S, V)
    t2 = (e2 * S * S).sum(-1)[..., None]
    var = (t0 - 2.0 * (O_ref / nn) * t1 + (O_ref / nn) ** 2 * t2) / (3.0 * nn * nn)
    sigma = np.sqrt(np.maximum(var, 0.0))
    N = S.shape[-1]
    own = np.abs(O_ref) * (out_half_ulp + 2.0 ** -24 * np.sqrt(N))
    hard = np.where(live, hard + own, np.inf)
    hard = np.where(n > 0, hard, 0.0)
    sigma = np.where(n > 0, sigma, 0.0)
    return hard, sigma, own
