/*
 * CPU oracle for the MoE expert layer -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain fp64 loops that write out the definition of what the layer computes:
 * the gating function picks the experts of every token (paper Sec. 2.1,
 * Sec. 3.3 "Execution"), the tokens of each expert are batched (the inp_size
 * array of Algorithm 1), every expert with at least one token runs its FFN
 * (Algorithm 1 skips experts whose input size is zero; Sec. 3.2 gives the
 * three 4096 x 14336 matrices, Sec. 2.2 names SiLU as the activation) and the
 * expert outputs return to the token stream.  The paper does not print the
 * layer's equations; the readings used here (top-k on raw logits, softmax over
 * the selected k, ties to the lower index, silu(x.w1)*(x.w3) then .w2, gate-
 * weighted sum) are the Mixtral layer the paper evaluates (Sec. 4.1).
 *
 * Nothing here is shared with the HIP path and nothing in the product imports
 * it: only tests, the smoke check and the bench's CPU-baseline leg call it.
 * There is no blocking, fusion or reordering: every output element is one
 * ascending-index sum.  OpenMP only splits independent output columns over
 * threads.
 *
 * Pins (tests/test_oracle_pins.py): dense brute force with a sort-based top-k
 * on tiny inputs, closed forms (sigmoid for k=2, full softmax for k=E, scalar
 * case 1/(1+e^-1)), invariants (weights sum to 1, counts sum to T*k, perm is
 * a bijection and stable), identical-experts => dense FFN, numpy matmul.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG (-1)
#define ORACLE_NONFINITE (-2)

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static inline double widen_bf16(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Gating (Sec. 2.1; Sec. 3.3): per token the k largest logits, a larger logit
 * first and the lower expert index first among equal logits; weights are the
 * softmax over the selected k (= full softmax renormalised over them). */
int oracle_route(const float* logits, long T, int E, int k, int32_t* idx, double* w) {
    if (T < 0 || E < 1 || k < 1 || k > E) return ORACLE_BAD_ARG;
    for (long t = 0; t < T; t++) {
        const float* l = logits + t * E;
        int32_t* sel = idx + t * k;
        int n = 0;
        for (int e = 0; e < E; e++) {
            if (!isfinite(l[e])) return ORACLE_NONFINITE;
            double v = (double)l[e];
            /* position of e in the list kept in (logit desc, index asc) order */
            int pos = n;
            while (pos > 0 && (double)l[sel[pos - 1]] < v) pos--;
            if (pos >= k) continue;
            int last = (n < k) ? n : k - 1;
            for (int j = last; j > pos; j--) sel[j] = sel[j - 1];
            sel[pos] = e;
            if (n < k) n++;
        }
        double m = (double)l[sel[0]];
        double s = 0.0;
        for (int j = 0; j < k; j++) {
            w[t * k + j] = exp((double)l[sel[j]] - m);
            s += w[t * k + j];
        }
        for (int j = 0; j < k; j++) w[t * k + j] /= s;
    }
    return ORACLE_OK;
}

/* Per-expert input sizes and batching (Algorithm 1's inp_size; Sec. 3.3):
 * counts, exclusive-scan offsets, and the stable ordering of the flat slots
 * p = t*k + j by expert.  perm[pos] = p, inv_perm[p] = pos, xg[pos] = x[t]. */
int oracle_permute(const int32_t* idx, long T, int E, int k, const double* x, long d,
                   int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                   double* xg) {
    if (T < 0 || E < 1 || k < 1 || d < 0) return ORACLE_BAD_ARG;
    long N = T * k;
    for (int e = 0; e < E; e++) counts[e] = 0;
    for (long p = 0; p < N; p++) {
        if (idx[p] < 0 || idx[p] >= E) return ORACLE_BAD_ARG;
        counts[idx[p]]++;
    }
    offsets[0] = 0;
    for (int e = 0; e < E; e++) offsets[e + 1] = offsets[e] + counts[e];
    int32_t* seen = (int32_t*)calloc((size_t)E, sizeof(int32_t));
    if (!seen) return ORACLE_BAD_ARG;
    for (long p = 0; p < N; p++) {
        int e = idx[p];
        long pos = offsets[e] + seen[e]++;
        perm[pos] = (int32_t)p;
        inv_perm[p] = (int32_t)pos;
        if (xg && x) {
            long t = p / k;
            for (long r = 0; r < d; r++) xg[pos * d + r] = x[t * d + r];
        }
    }
    free(seen);
    return ORACLE_OK;
}

/* out[c] = sum_{r=0..K-1} v[r] * W[r,c] for c in [0,C), W row-major [K,C].
 * Each out[c] is one ascending-r sum; threads own disjoint column ranges. */
static void vec_times_matrix(const double* v, const void* W, int w_is_bf16, long K, long C,
                             double* out) {
#pragma omp parallel
    {
#ifdef _OPENMP
        int nt = omp_get_num_threads(), id = omp_get_thread_num();
#else
        int nt = 1, id = 0;
#endif
        long c0 = C * id / nt, c1 = C * (id + 1) / nt;
        for (long c = c0; c < c1; c++) out[c] = 0.0;
        for (long r = 0; r < K; r++) {
            double vr = v[r];
            if (w_is_bf16) {
                const uint16_t* row = (const uint16_t*)W + r * C;
                for (long c = c0; c < c1; c++) out[c] += vr * widen_bf16(row[c]);
            } else {
                const float* row = (const float*)W + r * C;
                for (long c = c0; c < c1; c++) out[c] += vr * (double)row[c];
            }
        }
    }
}

/* Expert FFN on the batched rows (Sec. 3.2 shapes; SiLU per Sec. 2.2):
 * for every expert e with rows [offsets[e], offsets[e+1]) (none => skipped, as
 * Algorithm 1 does): a = x.w1_e, b = x.w3_e, h = a/(1+exp(-a)) * b, y = h.w2_e.
 * w1, w3: [E,d,f]; w2: [E,f,d]; fp32 or bf16 bit patterns, widened exactly. */
int oracle_expert_ffn(const double* xg, const int32_t* offsets, int E, long d, long f,
                      const void* w1, const void* w3, const void* w2, int w_is_bf16,
                      double* yg) {
    if (E < 1 || d < 1 || f < 1) return ORACLE_BAD_ARG;
    size_t esz = w_is_bf16 ? 2 : 4;
    double* a = (double*)malloc(sizeof(double) * (size_t)f);
    double* b = (double*)malloc(sizeof(double) * (size_t)f);
    if (!a || !b) { free(a); free(b); return ORACLE_BAD_ARG; }
    for (int e = 0; e < E; e++) {
        if (offsets[e + 1] < offsets[e]) { free(a); free(b); return ORACLE_BAD_ARG; }
        if (offsets[e + 1] == offsets[e]) continue;
        const char* w1e = (const char*)w1 + (size_t)e * d * f * esz;
        const char* w3e = (const char*)w3 + (size_t)e * d * f * esz;
        const char* w2e = (const char*)w2 + (size_t)e * f * d * esz;
        for (long i = offsets[e]; i < offsets[e + 1]; i++) {
            vec_times_matrix(xg + i * d, w1e, w_is_bf16, d, f, a);
            vec_times_matrix(xg + i * d, w3e, w_is_bf16, d, f, b);
            for (long c = 0; c < f; c++) a[c] = a[c] / (1.0 + exp(-a[c])) * b[c];
            vec_times_matrix(a, w2e, w_is_bf16, f, d, yg + i * d);
        }
    }
    free(a);
    free(b);
    return ORACLE_OK;
}

/* Expert outputs return to token order, weighted by the gate (Sec. 3.2 step 4
 * of case (c) is the only mention; the weighting is Mixtral's):
 * y[t] = sum_{j<k, ascending} w[t,j] * yg[inv_perm[t*k+j]]. */
int oracle_combine(const double* yg, const int32_t* inv_perm, const double* w, long T, int k,
                   long d, double* y) {
    if (T < 0 || k < 1 || d < 0) return ORACLE_BAD_ARG;
    for (long t = 0; t < T; t++) {
        for (long q = 0; q < d; q++) {
            double s = 0.0;
            for (int j = 0; j < k; j++)
                s += w[t * k + j] * yg[(long)inv_perm[t * k + j] * d + q];
            y[t * d + q] = s;
        }
    }
    return ORACLE_OK;
}

/* Support steps of the layer-stack workload (not part of the paper's text:
 * the stack workload places an RMSNorm with no gain before each router).
 * h[t] = x[t] / sqrt(mean(x[t]^2) + eps). */
int oracle_rmsnorm(const double* x, long T, long d, double eps, double* h) {
    if (T < 0 || d < 1) return ORACLE_BAD_ARG;
    for (long t = 0; t < T; t++) {
        double ss = 0.0;
        for (long r = 0; r < d; r++) ss += x[t * d + r] * x[t * d + r];
        double inv = 1.0 / sqrt(ss / (double)d + eps);
        for (long r = 0; r < d; r++) h[t * d + r] = x[t * d + r] * inv;
    }
    return ORACLE_OK;
}

/* logits[t,e] = fp32( sum_r h[t,r] * Wg[r,e] ), Wg fp32 [d,E]. */
int oracle_router_logits(const double* h, const float* Wg, long T, long d, int E, float* logits) {
    if (T < 0 || d < 1 || E < 1) return ORACLE_BAD_ARG;
    for (long t = 0; t < T; t++)
        for (int e = 0; e < E; e++) {
            double s = 0.0;
            for (long r = 0; r < d; r++) s += h[t * d + r] * (double)Wg[r * E + e];
            logits[t * E + e] = (float)s;
        }
    return ORACLE_OK;
}
