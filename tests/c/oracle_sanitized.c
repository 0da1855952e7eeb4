/* Drives the C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host only): every
 * mask over a few rounds on small ragged sizes, fp32 and bf16 gradients, with and without the
 * update rule, threaded and scalar.  Integer-valued data keep fp32 exact, so conservation
 * (every gradient delivered exactly once, Section 6.1 of the paper) is checked exactly.
 * Built and run by tests/test_oracle_pins.py. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void eager_oracle_round_ex(int P, int64_t n, const void *const *G, int grad_is_bf16,
                           float *const *R, uint64_t valid, uint64_t mask, float *w, float *v,
                           float lr, float mu, float wd, int nesterov, float *recv, int nthreads);

static uint16_t to_bf16(float f)            /* the test values are exactly representable */
{
    uint32_t b;
    memcpy(&b, &f, sizeof b);
    return (uint16_t)(b >> 16);
}

static int run(int P, int64_t n, int bf16, int nthreads)
{
    const int T = 3;
    uint64_t seq, nseq = 1;
    int t, p;
    int64_t i;
    for (t = 0; t < T; ++t) nseq *= (1u << P);
    for (seq = 0; seq < nseq; ++seq) {
        void **G = malloc(sizeof(void *) * P);
        float **R = malloc(sizeof(float *) * P);
        float *recv = malloc(sizeof(float) * (n ? n : 1));
        float *w = malloc(sizeof(float) * (n ? n : 1)), *v = malloc(sizeof(float) * (n ? n : 1));
        double delivered = 0.0, produced = 0.0, pending = 0.0;
        uint64_t valid = 0, s = seq;
        for (p = 0; p < P; ++p) {
            G[p] = malloc((bf16 ? 2 : 4) * (n ? n : 1));
            R[p] = malloc(sizeof(float) * (n ? n : 1));   /* left uninitialised: reading an empty */
        }                                                 /* send buffer would break the check   */
        for (i = 0; i < n; ++i) { w[i] = 0.0f; v[i] = 0.0f; }
        for (t = 0; t <= T; ++t) {
            const uint64_t mask = t < T ? s % (1u << P) : (1u << P) - 1;   /* last round: flush */
            s /= (1u << P);
            for (p = 0; p < P; ++p)
                for (i = 0; i < n; ++i) {
                    const float g = t < T ? (float)((t * 7 + p * 3 + i) % 5 - 2) : 0.0f;
                    if (bf16) ((uint16_t *)G[p])[i] = to_bf16(g);
                    else ((float *)G[p])[i] = g;
                    produced += g;
                }
            eager_oracle_round_ex(P, n, (const void *const *)G, bf16, R, valid, mask,
                                  (t & 1) ? w : NULL, (t & 1) ? v : NULL, 0.5f, 0.5f, 0.0f, t == 3,
                                  recv, nthreads);
            valid = ~mask & ((1u << P) - 1);
            for (i = 0; i < n; ++i) delivered += (double)recv[i] * P;
        }
        for (p = 0; p < P; ++p)
            if ((valid >> p) & 1u)
                for (i = 0; i < n; ++i) pending += R[p][i];
        if (valid != 0 || delivered + pending != produced) {
            fprintf(stderr, "conservation failed: P=%d n=%lld seq=%llu\n", P, (long long)n,
                    (unsigned long long)seq);
            return 1;
        }
        for (p = 0; p < P; ++p) { free(G[p]); free(R[p]); }
        free(G); free(R); free(recv); free(w); free(v);
    }
    return 0;
}

int main(void)
{
    static const int64_t sizes[] = {0, 1, 5, 17};
    int P, k, bf16;
    for (P = 1; P <= 4; P *= 2)           /* powers of two keep the 1/P scaling exact */
        for (k = 0; k < 4; ++k)
            for (bf16 = 0; bf16 < 2; ++bf16)
                if (run(P, sizes[k], bf16, 1 + (k & 1) * 2)) return 1;
    puts("ok");
    return 0;
}
