/*
 * Sanitizer driver for oracle/sphattn_oracle.c (host code only; no GPU involved).
 *
 * Built by tests/test_sanitizers.py together with the oracle's source under
 * -fsanitize=address,undefined.  It fills EXACTLY sized heap buffers (so that any read or write
 * past an input or output lands in a red zone) with seeded values, calls every entry point of
 * the oracle on one problem shape, and writes inputs and outputs to a file; the Python test
 * feeds the same inputs to the ordinary build of the oracle and compares the outputs.
 *
 *   oracle_driver B H H_kv N_q N_k d kind seed out_file
 * kind: 0 f64, 1 f32, 2 bf16, 3 e4m3fn, 4 f16 (all of Q, K, V, dO).  With N_q != N_k only the
 * rectangular entry point (the accumulator) runs.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_attention_fwd_grn(int, const void *, int, const void *, int, const void *, int, const double *,
                             double *, double *, double *, int, int, int, int, int);
int oracle_attention_fwd(int, const void *, int, const void *, int, const void *, int, double *, double *,
                         double *, int, int, int, int);
int oracle_attention_rows_grn(int, const void *, int, const void *, int, const void *, int, const double *,
                              double *, int, int, int, int, int, int, const int *, int);
int oracle_attention_rows(int, const void *, int, const void *, int, const void *, int, double *,
                          int, int, int, int, int, const int *, int);
int oracle_spherical_streamed(const double *, const double *, const double *, double *, int, int, int, int, int);
int oracle_spherical_accumulate(const void *, int, const void *, int, const void *, int, const double *,
                                double *, double *, int, int, int, int, int, int);
int oracle_spherical_bwd_grn(const void *, int, const void *, int, const void *, int, const void *, int,
                             const double *, double *, double *, double *, int, int, int, int, int);
void oracle_widen(const void *, int, size_t, size_t, double *);

static uint64_t state;
static uint32_t next_u32(void)
{
    state = state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (uint32_t)(state >> 32);
}
static double next_unit(void) { return (double)next_u32() / 4294967296.0 * 2.0 - 1.0; }

static const size_t kind_bytes[5] = {8, 4, 2, 1, 2};

/* n finite values of the given kind, magnitude below 2 */
static void *fill(int kind, size_t n)
{
    void *p = malloc(n * kind_bytes[kind]);
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) {
        const double x = next_unit() * 1.5;
        if (kind == 0) ((double *)p)[i] = x;
        else if (kind == 1) ((float *)p)[i] = (float)x;
        else if (kind == 2) { float f = (float)x; uint32_t u; memcpy(&u, &f, 4); ((uint16_t *)p)[i] = (uint16_t)(u >> 16); }
        else if (kind == 3) {                      /* sign, exponent 0..8 of 15, 3 mantissa bits: finite */
            const uint32_t r = next_u32();
            ((uint8_t *)p)[i] = (uint8_t)(((r & 1) << 7) | (((r >> 1) % 9) << 3) | ((r >> 8) & 7));
        } else {                                   /* f16: sign, exponent 10..16 of 31, 10 mantissa bits */
            const uint32_t r = next_u32();
            ((uint16_t *)p)[i] = (uint16_t)(((r & 1) << 15) | ((10 + (r >> 1) % 7) << 10) | ((r >> 8) & 1023));
        }
    }
    return p;
}

static double *out_buf(size_t n)
{
    double *p = malloc(n * sizeof *p);
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) p[i] = -777.0;
    return p;
}

static void put(FILE *f, const void *p, size_t bytes)
{
    const uint64_t n = bytes;
    fwrite(&n, 8, 1, f);
    fwrite(p, 1, bytes, f);
}

#define CHECK(call) do { if ((call) != 0) { fprintf(stderr, "failed: %s\n", #call); return 4; } } while (0)

int main(int argc, char **argv)
{
    if (argc != 10) return 2;
    const int B = atoi(argv[1]), H = atoi(argv[2]), H_kv = atoi(argv[3]), Nq = atoi(argv[4]), Nk = atoi(argv[5]);
    const int d = atoi(argv[6]), kind = atoi(argv[7]);
    state = (uint64_t)atoll(argv[8]);
    FILE *f = fopen(argv[9], "wb");
    if (!f || kind < 0 || kind > 4) return 2;
    const size_t nq = (size_t)B * H * Nq * d, nkv = (size_t)B * H_kv * Nk * d, rows_q = (size_t)B * H * Nq;
    void *Q = fill(kind, nq), *K = fill(kind, nkv), *V = fill(kind, nkv), *G = fill(kind, nq);
    double *mult = malloc((size_t)B * Nk * sizeof *mult);
    for (size_t i = 0; i < (size_t)B * Nk; ++i) mult[i] = (double)(next_u32() % 4);   /* multiplicities 0..3 */
    put(f, Q, nq * kind_bytes[kind]);
    put(f, K, nkv * kind_bytes[kind]);
    put(f, V, nkv * kind_bytes[kind]);
    put(f, G, nq * kind_bytes[kind]);
    put(f, mult, (size_t)B * Nk * 8);

    double *o_raw = out_buf(nq), *z = out_buf(rows_q);
    CHECK(oracle_spherical_accumulate(Q, kind, K, kind, V, kind, mult, o_raw, z, B, H, H_kv, Nq, Nk, d));
    put(f, o_raw, nq * 8);
    put(f, z, rows_q * 8);
    if (Nq == Nk) {
        const int N = Nq;
        double *O = out_buf(nq), *W = out_buf(rows_q * N), *Z = out_buf(rows_q);
        CHECK(oracle_attention_fwd_grn(0, Q, kind, K, kind, V, kind, mult, O, W, Z, B, H, H_kv, N, d));
        put(f, O, nq * 8);
        put(f, W, rows_q * N * 8);
        put(f, Z, rows_q * 8);
        int rows[3] = {0, N - 1, N / 2};
        double *Or = out_buf((size_t)3 * d);
        CHECK(oracle_attention_rows_grn(0, Q, kind, K, kind, V, kind, mult, Or, B, H, H_kv, N, d, B * H - 1, rows, 3));
        put(f, Or, (size_t)3 * d * 8);
        double *dQ = out_buf(nq), *dK = out_buf(nkv), *dV = out_buf(nkv);
        CHECK(oracle_spherical_bwd_grn(Q, kind, K, kind, V, kind, G, kind, mult, dQ, dK, dV, B, H, H_kv, N, d));
        put(f, dQ, nq * 8);
        put(f, dK, nkv * 8);
        put(f, dV, nkv * 8);
        if (H_kv == H) {                           /* the other normalizers and the streamed loop: plain heads */
            for (int mode = 1; mode <= 3; ++mode) {
                CHECK(oracle_attention_fwd(mode, Q, kind, K, kind, V, kind, O, NULL, NULL, B, H, N, d));
                put(f, O, nq * 8);
                CHECK(oracle_attention_rows(mode, Q, kind, K, kind, V, kind, Or, B, H, N, d, 0, rows, 3));
                put(f, Or, (size_t)3 * d * 8);
            }
            double *Qd = out_buf(nq), *Kd = out_buf(nkv), *Vd = out_buf(nkv);
            oracle_widen(Q, kind, 0, nq, Qd);
            oracle_widen(K, kind, 0, nkv, Kd);
            oracle_widen(V, kind, 0, nkv, Vd);
            const int chunks[3] = {1, 7, N + 3};
            for (int c = 0; c < 3; ++c) {
                CHECK(oracle_spherical_streamed(Qd, Kd, Vd, O, B, H, N, d, chunks[c]));
                put(f, O, nq * 8);
            }
            free(Qd); free(Kd); free(Vd);
        }
        free(O); free(W); free(Z); free(Or); free(dQ); free(dK); free(dV);
    }
    /* bad arguments come back as -1 without touching anything */
    if (oracle_spherical_accumulate(NULL, kind, K, kind, V, kind, mult, o_raw, z, B, H, H_kv, Nq, Nk, d) != -1) return 5;
    if (oracle_attention_fwd(7, Q, kind, K, kind, V, kind, o_raw, NULL, NULL, B, H, Nq, d) != -1) return 5;
    free(Q); free(K); free(V); free(G); free(mult); free(o_raw); free(z);
    fclose(f);
    puts("ok");
    return 0;
}
