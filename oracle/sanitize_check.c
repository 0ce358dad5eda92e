/*
 * Sanitizer run of the CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * Built together with moe_oracle.c under -fsanitize=address,undefined (oracle/build.py,
 * build_sanitize_check) and run by tests/test_oracle_pins.py: it drives every oracle
 * function over a small seeded layer, including the edge cases (an empty expert, k == E,
 * T == 0, bf16 and fp32 weights), so that an out-of-bounds access, a misaligned or
 * overflowing index or an uninitialised read in the oracle aborts the run.  It prints one
 * checksum per function; the test compares them with the same calls through the ordinary
 * build of the oracle.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_route(const float*, long, int, int, int32_t*, double*);
int oracle_permute(const int32_t*, long, int, int, const double*, long, int32_t*, int32_t*,
                   int32_t*, int32_t*, double*);
int oracle_expert_ffn(const double*, const int32_t*, int, long, long, const void*, const void*,
                      const void*, int, double*);
int oracle_combine(const double*, const int32_t*, const double*, long, int, long, double*);
int oracle_rmsnorm(const double*, long, long, double, double*);
int oracle_router_logits(const double*, const float*, long, long, int, float*);

/* the generator the test repeats: x_{n+1} = 1664525 x_n + 1013904223 (mod 2^32) */
static uint32_t lcg_state;
static double lcg_unit(void) {
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (double)(lcg_state >> 8) / 16777216.0 - 0.5;
}

static int run(int T, int d, int f, int E, int k, int bf16, uint32_t seed) {
    lcg_state = seed;
    const long N = (long)T * k;
    float* logits = malloc(sizeof(float) * (size_t)(T * E + 1));
    double* x = malloc(sizeof(double) * (size_t)(T * d + 1));
    const size_t wn = (size_t)E * d * f;
    void *w1, *w3, *w2;
    if (bf16) {
        uint16_t *a = malloc(2 * wn), *b = malloc(2 * wn), *c = malloc(2 * wn);
        for (size_t i = 0; i < wn; i++) {
            /* bf16 patterns of small values: sign, exponent around 2^-3, 7 mantissa bits */
            a[i] = (uint16_t)(0x3d00u + ((uint32_t)(lcg_unit() * 256 + 128) & 0xffu) + (lcg_unit() < 0 ? 0x8000u : 0));
            b[i] = (uint16_t)(0x3d00u + ((uint32_t)(lcg_unit() * 256 + 128) & 0xffu) + (lcg_unit() < 0 ? 0x8000u : 0));
            c[i] = (uint16_t)(0x3d00u + ((uint32_t)(lcg_unit() * 256 + 128) & 0xffu) + (lcg_unit() < 0 ? 0x8000u : 0));
        }
        w1 = a; w3 = b; w2 = c;
    } else {
        float *a = malloc(4 * wn), *b = malloc(4 * wn), *c = malloc(4 * wn);
        for (size_t i = 0; i < wn; i++) { a[i] = (float)lcg_unit(); b[i] = (float)lcg_unit(); c[i] = (float)lcg_unit(); }
        w1 = a; w3 = b; w2 = c;
    }
    for (int i = 0; i < T * E; i++) logits[i] = (float)(4.0 * lcg_unit());
    for (int t = 0; t < T; t++) if (E > 2) logits[t * E + 1] = -30.0f;   /* expert 1 stays empty */
    for (int i = 0; i < T * d; i++) x[i] = 2.0 * lcg_unit();
    int32_t* idx = malloc(sizeof(int32_t) * (size_t)(N + 1));
    double* w = malloc(sizeof(double) * (size_t)(N + 1));
    int32_t* counts = malloc(sizeof(int32_t) * (size_t)E);
    int32_t* offsets = malloc(sizeof(int32_t) * (size_t)(E + 1));
    int32_t* perm = malloc(sizeof(int32_t) * (size_t)(N + 1));
    int32_t* inv = malloc(sizeof(int32_t) * (size_t)(N + 1));
    double* xg = malloc(sizeof(double) * (size_t)(N * d + 1));
    double* yg = malloc(sizeof(double) * (size_t)(N * d + 1));
    double* y = malloc(sizeof(double) * (size_t)(T * d + 1));
    double* h = malloc(sizeof(double) * (size_t)(T * d + 1));
    float* wg = malloc(sizeof(float) * (size_t)(d * E));
    float* lg2 = malloc(sizeof(float) * (size_t)(T * E + 1));
    for (int i = 0; i < d * E; i++) wg[i] = (float)lcg_unit();
    int rc = 0;
    rc |= oracle_route(logits, T, E, k, idx, w);
    rc |= oracle_permute(idx, T, E, k, x, d, counts, offsets, perm, inv, xg);
    rc |= oracle_expert_ffn(xg, offsets, E, d, f, w1, w3, w2, bf16, yg);
    rc |= oracle_combine(yg, inv, w, T, k, d, y);
    rc |= oracle_rmsnorm(x, T, d, 1e-5, h);
    rc |= oracle_router_logits(h, wg, T, d, E, lg2);
    double s_w = 0, s_y = 0, s_h = 0, s_l = 0;
    long s_i = 0;
    for (long i = 0; i < N; i++) { s_w += w[i] * (double)(i + 1); s_i += (long)idx[i] * (i + 1) + 3L * perm[i] * (i + 1) + 7L * inv[i]; }
    for (int e = 0; e <= E; e++) s_i += 11L * offsets[e] * (e + 1);
    for (long i = 0; i < (long)T * d; i++) { s_y += y[i] * (double)((i % 7) + 1); s_h += h[i] * (double)((i % 5) + 1); }
    for (int i = 0; i < T * E; i++) s_l += (double)lg2[i] * (double)((i % 3) + 1);
    printf("case T=%d d=%d f=%d E=%d k=%d bf16=%d rc=%d idx=%ld w=%.17g y=%.17g h=%.17g logits=%.17g\n", T, d, f,
           E, k, bf16, rc, s_i, s_w, s_y, s_h, s_l);
    free(logits); free(x); free(w1); free(w3); free(w2); free(idx); free(w); free(counts);
    free(offsets); free(perm); free(inv); free(xg); free(yg); free(y); free(h); free(wg); free(lg2);
    return rc;
}

int main(void) {
    int rc = 0;
    rc |= run(9, 16, 24, 4, 2, 1, 11u);
    rc |= run(5, 8, 12, 3, 3, 0, 12u);   /* k == E */
    rc |= run(0, 8, 8, 4, 2, 1, 13u);    /* no tokens */
    rc |= run(33, 32, 16, 8, 1, 0, 14u);
    return rc;
}
