/*
 * CPU oracle for spherical attention (forward).  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain, fp64 statement of what the GPU library must
 * compute.  It is used by the tests, by the smoke check and by the benchmark's
 * CPU-baseline leg.  It shares no code with the HIP path and the product never
 * calls it.
 *
 * What is computed (paper, Appendix A.1, definition of a normalized
 * contraction, with the spherical choice of Section 3: a1(x) = x,
 * a2(x) = x^2, b = sqrt, i.e. the score row is divided by its L2 norm):
 *
 *     s_ij = sum_k Q[b,h,i,k] * K[b,h,j,k]                 (Theorem 1: the Q/K
 *                                                           contraction feeding
 *                                                           the normalizer)
 *     z_i  = sum_j s_ij^2                                   (sum_j a2(x_j))
 *     O[b,h,i,:] = ( sum_j s_ij * V[b,h,j,:] ) / sqrt(z_i)  (NC(x, y))
 *
 * A row with z_i = 0 has an all-zero numerator as well; it is defined as 0
 * (the paper gives no epsilon, so none is used).
 *
 * No score scale (1/sqrt(d) or other) is applied: any positive factor on the
 * scores cancels between numerator and sqrt(z).
 *
 * Inputs are taken exactly as stored (fp64, fp32, bf16 or fp16 bit patterns, OCP
 * e4m3fn bytes) and widened exactly to fp64 before any arithmetic.  Layout is
 * dense row-major [B,H,N,d] with d contiguous.
 *
 * Gene-regulatory-network variant (paper, Section 3.1 and Appendix A.2): the key of
 * gene j is multiplied by that gene's multiplicity m_j before the scores are formed,
 * s_ij = sum_k Q[b,h,i,k] * (m[b,j] * K[b,g,j,k]), and K/V heads may be shared by
 * groups of query heads (grouped-query attention): g = h / (H / H_kv).
 *
 * The comparison twin (standard SoftMax attention, a1 = a2 = exp, b = id, with
 * the conventional 1/sqrt(d) score scale) is also given, from its textbook
 * definition.
 *
 * Parity pins (tests/test_oracle_*.py): exact-rational brute force on tiny
 * inputs, unit-norm weight rows, Cauchy-Schwarz bound, scale/sign invariance,
 * linearity in V, N = 1 and orthonormal-key closed forms, the Gram-matrix
 * closed form, and chunk-size / permutation / zero-padding invariance of the
 * streamed accumulator of Lemma 1.  The bare accumulator (no tail) is pinned by
 * exact rationals, by the one-key closed form on a rectangular shape, and by
 * additivity over key partitions followed by the tail against the direct form.  The
 * backward (derived here, not in the paper) is pinned by central finite differences of
 * the forward oracle, by automatic differentiation of a library statement of the
 * definition, by dV = W^T dO with W from the forward oracle, and by Euler's identity for
 * the scale invariances (q_i . dQ_i = 0 for every row, sum_j k_j . dK_j = 0 per head).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F64 = 0, ORACLE_F32 = 1, ORACLE_BF16 = 2, ORACLE_E4M3FN = 3, ORACLE_F16 = 4 };

/* ---- exact widening of stored formats to fp64 --------------------------- */

/* bfloat16: the upper 16 bits of an IEEE binary32. */
static double widen_bf16(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3 ("fn": finite, no infinities): 1 sign, 4 exponent
 * (bias 7), 3 mantissa bits; exponent field 0 is subnormal (2^-6 * m/8);
 * S.1111.111 is NaN; every other code is a finite number, max 448. */
static double widen_e4m3fn(uint8_t bits)
{
    int sign = bits >> 7;
    int e = (bits >> 3) & 0xF;
    int m = bits & 0x7;
    double v;
    if (e == 0xF && m == 0x7)
        v = NAN;
    else if (e == 0)
        v = ldexp((double)m, -9);              /* m/8 * 2^-6 */
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

/* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 mantissa bits; exponent field 0 is
 * subnormal (m * 2^-24), 31 is infinity (m == 0) or NaN. */
static double widen_f16(uint16_t bits)
{
    int sign = bits >> 15;
    int e = (bits >> 10) & 0x1F;
    int m = bits & 0x3FF;
    double v;
    if (e == 0x1F)
        v = m ? NAN : INFINITY;
    else if (e == 0)
        v = ldexp((double)m, -24);
    else
        v = ldexp(1.0 + (double)m / 1024.0, e - 15);
    return sign ? -v : v;
}

static double load_elem(const void *p, int kind, size_t idx)
{
    switch (kind) {
    case ORACLE_F64: return ((const double *)p)[idx];
    case ORACLE_F32: return (double)((const float *)p)[idx];
    case ORACLE_BF16: return widen_bf16(((const uint16_t *)p)[idx]);
    case ORACLE_E4M3FN: return widen_e4m3fn(((const uint8_t *)p)[idx]);
    case ORACLE_F16: return widen_f16(((const uint16_t *)p)[idx]);
    default: return NAN;
    }
}

/* Widen `count` stored elements starting at element offset `off`. */
void oracle_widen(const void *src, int kind, size_t off, size_t count, double *dst)
{
    for (size_t t = 0; t < count; ++t)
        dst[t] = load_elem(src, kind, off + t);
}

/* ---- one query row, given one head's K and V already widened ------------ */

/* Spherical row: two passes, exactly as the definition reads.
 * s (length N) is caller-provided scratch and holds the raw scores on return.
 * w, if not NULL, receives the normalized weights s_j / sqrt(z). */
static void spherical_row(const double *q, const double *Kh, const double *Vh, const double *m,
                          int N, int d, double *s, double *o, double *w, double *z_out)
{
    double z = 0.0;
    for (int j = 0; j < N; ++j) {
        double acc = 0.0;
        for (int k = 0; k < d; ++k)
            acc += q[k] * (m ? m[j] * Kh[(size_t)j * d + k] : Kh[(size_t)j * d + k]);
        s[j] = acc;
        z += acc * acc;
    }
    for (int k = 0; k < d; ++k)
        o[k] = 0.0;
    for (int j = 0; j < N; ++j)
        for (int k = 0; k < d; ++k)
            o[k] += s[j] * Vh[(size_t)j * d + k];
    double nrm = sqrt(z);
    for (int k = 0; k < d; ++k)
        o[k] = (z > 0.0) ? o[k] / nrm : 0.0;
    if (w)
        for (int j = 0; j < N; ++j)
            w[j] = (z > 0.0) ? s[j] / nrm : 0.0;
    if (z_out)
        *z_out = z;
}

/* SoftMax row (comparison twin): p_j = exp(c*s_j - max) / sum, c = 1/sqrt(d). */
static void softmax_row(const double *q, const double *Kh, const double *Vh,
                        int N, int d, double *s, double *o)
{
    double c = 1.0 / sqrt((double)d);
    double mx = -INFINITY;
    for (int j = 0; j < N; ++j) {
        double acc = 0.0;
        for (int k = 0; k < d; ++k)
            acc += q[k] * Kh[(size_t)j * d + k];
        s[j] = acc * c;
        if (s[j] > mx)
            mx = s[j];
    }
    double den = 0.0;
    for (int j = 0; j < N; ++j) {
        s[j] = exp(s[j] - mx);
        den += s[j];
    }
    for (int k = 0; k < d; ++k)
        o[k] = 0.0;
    for (int j = 0; j < N; ++j)
        for (int k = 0; k < d; ++k)
            o[k] += s[j] * Vh[(size_t)j * d + k];
    for (int k = 0; k < d; ++k)
        o[k] /= den;
}

/* Other normalizers of Definition 2, N(x)_i = a1(x_i) / b(sum_j a2(x_j)), as examples of
 * Theorem 1 (any such normalizer gives a streamable attention):
 *   mode 2  "L1":            a1(x) = x,            a2(x) = |x|,          b = id
 *   mode 3  "squared ReLU":  a1(x) = max(x,0)^2,   a2(x) = max(x,0)^2,   b = id
 * No score scale (both are homogeneous, so any positive scale cancels); a row whose
 * aggregate is 0 gives 0. */
static double norm_a1(int mode, double x)
{
    if (mode == 2) return x;
    double r = x > 0.0 ? x : 0.0;
    return r * r;
}

static double norm_a2(int mode, double x)
{
    if (mode == 2) return fabs(x);
    double r = x > 0.0 ? x : 0.0;
    return r * r;
}

static void normalized_row(int mode, const double *q, const double *Kh, const double *Vh,
                           int N, int d, double *s, double *o)
{
    double z = 0.0;
    for (int j = 0; j < N; ++j) {
        double x = 0.0;
        for (int k = 0; k < d; ++k)
            x += q[k] * Kh[(size_t)j * d + k];
        s[j] = norm_a1(mode, x);
        z += norm_a2(mode, x);
    }
    for (int k = 0; k < d; ++k)
        o[k] = 0.0;
    for (int j = 0; j < N; ++j)
        for (int k = 0; k < d; ++k)
            o[k] += s[j] * Vh[(size_t)j * d + k];
    for (int k = 0; k < d; ++k)
        o[k] = (z > 0.0) ? o[k] / z : 0.0;          /* b = id */
}

/* ---- whole-tensor entry points ------------------------------------------ */

/* mode 0 = spherical, 1 = softmax twin, 2 = L1, 3 = squared ReLU.
 * Q, K, V: [B,H,N,d] in the stored format named by q_kind/k_kind/v_kind.
 * O: [B,H,N,d] fp64.  W (may be NULL; spherical only): [B,H,N,N] weights.
 * Z (may be NULL; spherical only): [B,H,N] squared row norms.
 * Returns 0, or -1 on bad arguments / allocation failure. */
int oracle_attention_fwd_grn(int mode, const void *Q, int q_kind, const void *K, int k_kind,
                             const void *V, int v_kind, const double *mult,
                             double *O, double *W, double *Z,
                             int B, int H, int H_kv, int N, int d)
{
    if (!Q || !K || !V || !O || B <= 0 || H <= 0 || H_kv <= 0 || H % H_kv || N <= 0 || d <= 0)
        return -1;
    if (mode < 0 || mode > 3 || (mode != 0 && mult))
        return -1;
    size_t head = (size_t)N * d;
    double *Kh = malloc(head * sizeof *Kh);
    double *Vh = malloc(head * sizeof *Vh);
    int status = (Kh && Vh) ? 0 : -1;
    for (int bh = 0; bh < B * H && status == 0; ++bh) {
        const int b = bh / H, h = bh % H;
        const size_t kvh = (size_t)b * H_kv + h / (H / H_kv);   /* K/V head of this query head */
        const double *m = mult ? mult + (size_t)b * N : NULL;    /* multiplicities of this cell */
        oracle_widen(K, k_kind, kvh * head, head, Kh);
        oracle_widen(V, v_kind, kvh * head, head, Vh);
#pragma omp parallel
        {
            double *q = malloc((size_t)d * sizeof *q);
            double *s = malloc((size_t)N * sizeof *s);
            if (!q || !s) {
#pragma omp atomic write
                status = -1;
            } else {
#pragma omp for schedule(static)
                for (int i = 0; i < N; ++i) {
                    size_t row = (size_t)bh * N + i;
                    oracle_widen(Q, q_kind, row * d, (size_t)d, q);
                    if (mode == 0)
                        spherical_row(q, Kh, Vh, m, N, d, s, O + row * d,
                                      W ? W + row * N : NULL, Z ? Z + row : NULL);
                    else if (mode == 1)
                        softmax_row(q, Kh, Vh, N, d, s, O + row * d);
                    else
                        normalized_row(mode, q, Kh, Vh, N, d, s, O + row * d);
                }
            }
            free(q);
            free(s);
        }
    }
    free(Kh);
    free(Vh);
    return status;
}

/* The plain case: no multiplicities, one K/V head per query head. */
int oracle_attention_fwd(int mode, const void *Q, int q_kind, const void *K, int k_kind,
                         const void *V, int v_kind, double *O, double *W, double *Z,
                         int B, int H, int N, int d)
{
    return oracle_attention_fwd_grn(mode, Q, q_kind, K, k_kind, V, v_kind, NULL, O, W, Z, B, H, H, N, d);
}

/* Selected query rows of one head only (for full-size workloads, where the
 * whole tensor would take minutes): rows[r] in [0,N) of head index bh in
 * [0,B*H).  O_rows: [n_rows, d] fp64. */
int oracle_attention_rows_grn(int mode, const void *Q, int q_kind, const void *K, int k_kind,
                              const void *V, int v_kind, const double *mult, double *O_rows,
                              int B, int H, int H_kv, int N, int d, int bh, const int *rows, int n_rows)
{
    if (!Q || !K || !V || !O_rows || !rows || B <= 0 || H <= 0 || H_kv <= 0 || H % H_kv ||
        N <= 0 || d <= 0 || bh < 0 || bh >= B * H || n_rows < 0 || mode < 0 || mode > 3 ||
        (mode != 0 && mult))
        return -1;
    for (int r = 0; r < n_rows; ++r)
        if (rows[r] < 0 || rows[r] >= N)
            return -1;
    size_t head = (size_t)N * d;
    double *Kh = malloc(head * sizeof *Kh);
    double *Vh = malloc(head * sizeof *Vh);
    int status = (Kh && Vh) ? 0 : -1;
    if (status == 0) {
        const size_t kvh = (size_t)(bh / H) * H_kv + (bh % H) / (H / H_kv);
        const double *m = mult ? mult + (size_t)(bh / H) * N : NULL;
        oracle_widen(K, k_kind, kvh * head, head, Kh);
        oracle_widen(V, v_kind, kvh * head, head, Vh);
#pragma omp parallel
        {
            double *q = malloc((size_t)d * sizeof *q);
            double *s = malloc((size_t)N * sizeof *s);
            if (!q || !s) {
#pragma omp atomic write
                status = -1;
            } else {
#pragma omp for schedule(static)
                for (int r = 0; r < n_rows; ++r) {
                    size_t row = (size_t)bh * N + rows[r];
                    oracle_widen(Q, q_kind, row * d, (size_t)d, q);
                    if (mode == 0)
                        spherical_row(q, Kh, Vh, m, N, d, s, O_rows + (size_t)r * d, NULL, NULL);
                    else if (mode == 1)
                        softmax_row(q, Kh, Vh, N, d, s, O_rows + (size_t)r * d);
                    else
                        normalized_row(mode, q, Kh, Vh, N, d, s, O_rows + (size_t)r * d);
                }
            }
            free(q);
            free(s);
        }
    }
    free(Kh);
    free(Vh);
    return status;
}

int oracle_attention_rows(int mode, const void *Q, int q_kind, const void *K, int k_kind,
                          const void *V, int v_kind, double *O_rows,
                          int B, int H, int N, int d, int bh, const int *rows, int n_rows)
{
    return oracle_attention_rows_grn(mode, Q, q_kind, K, k_kind, V, v_kind, NULL, O_rows,
                                     B, H, H, N, d, bh, rows, n_rows);
}

/* Lemma 1 as a loop: the key axis is cut into chunks of `chunk` rows (the last
 * may be shorter); only (o, z) is carried between chunks, starting from (0,0),
 * updated by B((o,z),(x,y)) = (o + sum a1(x_i) y_i, z + sum a2(x_i)); the tail
 * t(o,z) = o / b(z) is applied once at the end.  fp64 inputs only.
 * Exists so the streaming identity can be tested against the direct form. */
int oracle_spherical_streamed(const double *Q, const double *K, const double *V, double *O,
                              int B, int H, int N, int d, int chunk)
{
    if (!Q || !K || !V || !O || B <= 0 || H <= 0 || N <= 0 || d <= 0 || chunk <= 0)
        return -1;
    size_t head = (size_t)N * d;
    double *o = malloc((size_t)d * sizeof *o);
    if (!o)
        return -1;
    for (int bh = 0; bh < B * H; ++bh) {
        const double *Kh = K + (size_t)bh * head, *Vh = V + (size_t)bh * head;
        for (int i = 0; i < N; ++i) {
            const double *q = Q + (size_t)bh * head + (size_t)i * d;
            double z = 0.0;
            for (int k = 0; k < d; ++k)
                o[k] = 0.0;
            for (int j0 = 0; j0 < N; j0 += chunk) {
                int j1 = j0 + chunk < N ? j0 + chunk : N;
                double dz = 0.0;
                for (int j = j0; j < j1; ++j) {
                    double x = 0.0;
                    for (int k = 0; k < d; ++k)
                        x += q[k] * Kh[(size_t)j * d + k];
                    dz += x * x;
                    for (int k = 0; k < d; ++k)
                        o[k] += x * Vh[(size_t)j * d + k];
                }
                z += dz;
            }
            double *out = O + (size_t)bh * head + (size_t)i * d;
            for (int k = 0; k < d; ++k)
                out[k] = (z > 0.0) ? o[k] / sqrt(z) : 0.0;
        }
    }
    free(o);
    return 0;
}

/* The accumulator of Lemma 1 over one set of keys, without the tail: for the N_q query rows
 * of every head against the N_k keys and values given,
 *     o_raw[b,h,i,:] = sum_j a1(s_ij) V[b,g,j,:] = sum_j s_ij V[b,g,j,:]
 *     z[b,h,i]       = sum_j a2(s_ij)            = sum_j s_ij^2
 * with s_ij = sum_k Q[b,h,i,k] * (m[b,j] * K[b,g,j,k]), g = h / (H / H_kv), m = 1 if mult is
 * NULL.  Q: [B,H,N_q,d]; K, V: [B,H_kv,N_k,d]; mult: [B,N_k]; O_raw: [B,H,N_q,d]; Z: [B,H,N_q].
 * The accumulators of disjoint key sets add up to the accumulator of their union, and
 * t(o, z) = o / sqrt(z) of the total is the attention output. */
int oracle_spherical_accumulate(const void *Q, int q_kind, const void *K, int k_kind,
                                const void *V, int v_kind, const double *mult,
                                double *O_raw, double *Z,
                                int B, int H, int H_kv, int N_q, int N_k, int d)
{
    if (!Q || !K || !V || !O_raw || !Z || B <= 0 || H <= 0 || H_kv <= 0 || H % H_kv ||
        N_q <= 0 || N_k <= 0 || d <= 0)
        return -1;
    size_t kv_head = (size_t)N_k * d;
    double *Kh = malloc(kv_head * sizeof *Kh);
    double *Vh = malloc(kv_head * sizeof *Vh);
    int status = (Kh && Vh) ? 0 : -1;
    for (int bh = 0; bh < B * H && status == 0; ++bh) {
        const int b = bh / H, h = bh % H;
        const size_t kvh = (size_t)b * H_kv + h / (H / H_kv);
        const double *m = mult ? mult + (size_t)b * N_k : NULL;
        oracle_widen(K, k_kind, kvh * kv_head, kv_head, Kh);
        oracle_widen(V, v_kind, kvh * kv_head, kv_head, Vh);
#pragma omp parallel
        {
            double *q = malloc((size_t)d * sizeof *q);
            if (!q) {
#pragma omp atomic write
                status = -1;
            } else {
#pragma omp for schedule(static)
                for (int i = 0; i < N_q; ++i) {
                    size_t row = (size_t)bh * N_q + i;
                    double *o = O_raw + row * d;
                    double z = 0.0;
                    oracle_widen(Q, q_kind, row * d, (size_t)d, q);
                    for (int k = 0; k < d; ++k)
                        o[k] = 0.0;
                    for (int j = 0; j < N_k; ++j) {
                        double x = 0.0;
                        for (int k = 0; k < d; ++k)
                            x += q[k] * (m ? m[j] * Kh[(size_t)j * d + k] : Kh[(size_t)j * d + k]);
                        z += x * x;
                        for (int k = 0; k < d; ++k)
                            o[k] += x * Vh[(size_t)j * d + k];
                    }
                    Z[row] = z;
                }
            }
            free(q);
        }
    }
    free(Kh);
    free(Vh);
    return status;
}

/* Backward of spherical attention.  The paper states no backward pass; this is the chain
 * rule applied to the definition above.  With r_i = z_i^(-1/2), O_i = r_i sum_j s_ij v_j and a
 * given upstream gradient dO:
 *     dV_j  = sum_i r_i s_ij dO_i
 *     ds_ij = r_i (dO_i . v_j) - (dO_i . O_i) r_i^2 s_ij     (through o, and through r via z)
 *     dQ_i  = sum_j ds_ij m_j k_j      dK_j = m_j sum_i ds_ij q_i
 * for the gene-regulatory-network variant s_ij = m_j (q_i . k_j) (m = 1 without multiplicities;
 * the multiplicities are data and get no gradient); with shared K/V heads the sums over i run
 * over the query rows of every head of the group.  A row with z_i = 0 has O_i = 0 by
 * definition and contributes no gradient.
 * Q, dO: [B,H,N,d], K, V: [B,H_kv,N,d] in their stored formats; mult: [B,N] or NULL;
 * dQ: [B,H,N,d], dK, dV: [B,H_kv,N,d] fp64.
 * Per query head, as the formulas read: rows i in parallel for dQ (and the row quantities),
 * then keys j in parallel, adding into dK and dV of the head's K/V head. */
int oracle_spherical_bwd_grn(const void *Q, int q_kind, const void *K, int k_kind,
                             const void *V, int v_kind, const void *dO, int g_kind,
                             const double *mult, double *dQ, double *dK, double *dV,
                             int B, int H, int H_kv, int N, int d)
{
    if (!Q || !K || !V || !dO || !dQ || !dK || !dV || B <= 0 || H <= 0 || H_kv <= 0 || H % H_kv ||
        N <= 0 || d <= 0)
        return -1;
    size_t head = (size_t)N * d;
    double *Qh = malloc(head * sizeof *Qh), *Kh = malloc(head * sizeof *Kh);
    double *Vh = malloc(head * sizeof *Vh), *Gh = malloc(head * sizeof *Gh);
    double *r = malloc((size_t)N * sizeof *r), *delta = malloc((size_t)N * sizeof *delta);
    int status = (Qh && Kh && Vh && Gh && r && delta) ? 0 : -1;
    if (status == 0)
        memset(dK, 0, (size_t)B * H_kv * head * sizeof *dK), memset(dV, 0, (size_t)B * H_kv * head * sizeof *dV);
    for (int bh = 0; bh < B * H && status == 0; ++bh) {
        const int b = bh / H, h = bh % H;
        const size_t kvh = (size_t)b * H_kv + h / (H / H_kv);
        const double *m = mult ? mult + (size_t)b * N : NULL;
        oracle_widen(Q, q_kind, bh * head, head, Qh);
        oracle_widen(K, k_kind, kvh * head, head, Kh);
        oracle_widen(V, v_kind, kvh * head, head, Vh);
        oracle_widen(dO, g_kind, bh * head, head, Gh);
        /* rows: r_i, delta_i = dO_i . O_i, dQ_i */
#pragma omp parallel for schedule(static)
        for (int i = 0; i < N; ++i) {
            const double *q = Qh + (size_t)i * d, *g = Gh + (size_t)i * d;
            double *dq = dQ + bh * head + (size_t)i * d;
            double z = 0.0, go = 0.0;                /* go = dO_i . o_raw_i */
            for (int j = 0; j < N; ++j) {
                double s = 0.0, gv = 0.0;
                for (int k = 0; k < d; ++k) {
                    s += q[k] * Kh[(size_t)j * d + k];
                    gv += g[k] * Vh[(size_t)j * d + k];
                }
                if (m)
                    s *= m[j];
                z += s * s;
                go += s * gv;
            }
            r[i] = z > 0.0 ? 1.0 / sqrt(z) : 0.0;
            delta[i] = r[i] * go;                    /* dO_i . O_i */
            for (int k = 0; k < d; ++k)
                dq[k] = 0.0;
            for (int j = 0; j < N; ++j) {
                double s = 0.0, gv = 0.0;
                for (int k = 0; k < d; ++k) {
                    s += q[k] * Kh[(size_t)j * d + k];
                    gv += g[k] * Vh[(size_t)j * d + k];
                }
                if (m)
                    s *= m[j];
                double ds = r[i] * gv - delta[i] * r[i] * r[i] * s;
                if (m)
                    ds *= m[j];                      /* d s_ij / d (q_i . k_j) */
                for (int k = 0; k < d; ++k)
                    dq[k] += ds * Kh[(size_t)j * d + k];
            }
        }
        /* keys: this head's share of dK_j, dV_j */
#pragma omp parallel for schedule(static)
        for (int j = 0; j < N; ++j) {
            const double *kj = Kh + (size_t)j * d, *vj = Vh + (size_t)j * d;
            double *dk = dK + kvh * head + (size_t)j * d, *dv = dV + kvh * head + (size_t)j * d;
            for (int i = 0; i < N; ++i) {
                const double *q = Qh + (size_t)i * d, *g = Gh + (size_t)i * d;
                double s = 0.0, gv = 0.0;
                for (int k = 0; k < d; ++k) {
                    s += q[k] * kj[k];
                    gv += g[k] * vj[k];
                }
                if (m)
                    s *= m[j];
                double w = r[i] * s;
                double ds = r[i] * gv - delta[i] * r[i] * r[i] * s;
                if (m)
                    ds *= m[j];
                for (int k = 0; k < d; ++k) {
                    dv[k] += w * g[k];
                    dk[k] += ds * q[k];
                }
            }
        }
    }
    free(Qh); free(Kh); free(Vh); free(Gh); free(r); free(delta);
    return status;
}

/* The plain case: no multiplicities, one K/V head per query head. */
int oracle_spherical_bwd(const void *Q, int q_kind, const void *K, int k_kind,
                         const void *V, int v_kind, const void *dO, int g_kind,
                         double *dQ, double *dK, double *dV, int B, int H, int N, int d)
{
    return oracle_spherical_bwd_grn(Q, q_kind, K, k_kind, V, v_kind, dO, g_kind, NULL, dQ, dK, dV, B, H, H, N, d);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
