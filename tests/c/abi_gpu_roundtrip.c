/* The library used from plain C, without Python or torch: device memory from hipMalloc, rounds
 * of each mode through the C ABI, a stash, the unfused path, results copied back and compared
 * bit for bit with the C oracle (fixed-order mode, integer-valued data not required: both sides
 * define every rounding).  Needs a GPU; built with gcc and run by tests/test_gpu_parity.py. */
#include "eager.h"

#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void eager_oracle_round_async(int P, int64_t n, const void *const *G, int grad_is_bf16,
                              float *const *R, uint64_t valid, uint64_t mask, uint64_t absent,
                              float *w, float *v, float lr, float mu, float wd, int nesterov,
                              float *recv, int nthreads);
void eager_oracle_stash(int64_t n, const void *G, int grad_is_bf16, float *R, int has_stale);
void eager_oracle_sgd_ex(int64_t n, const float *u, float *w, float *v, float lr, float mu,
                         float wd, int nesterov, int nthreads);

#define P 3
#define NB 3
#define CHECK(cond)                                                     \
    do {                                                                \
        if (!(cond)) {                                                  \
            printf("line %d: %s\n", __LINE__, #cond);                   \
            return 1;                                                   \
        }                                                               \
    } while (0)
#define HIP(call) CHECK((call) == hipSuccess)

static const int64_t off[NB] = {0, 8, 1032}, num[NB] = {5, 1021, 4099};
enum { ARENA = 1032 + 4099 + 1 };

static float value(unsigned step, unsigned p, unsigned i)      /* a few thousand distinct floats */
{
    unsigned h = (step * 2654435761u) ^ (p * 40503u + 17u) ^ (i * 2246822519u);
    h ^= h >> 15; h *= 2654435761u; h ^= h >> 13;
    return ((float)(h & 0xffffu) - 32768.0f) * (1.0f / 4194304.0f);
}

int main(void)
{
    eager_ctx *ctx = NULL;
    float *hG[P], *hR[P], *dG[P], *dR[P], *hw, *hv, *hrecv, *dw, *dv, *drecv, *back;
    const void *dGc[P];
    uint64_t valid[NB] = {0, 0, 0}, got;
    const float lr = 0.1f, mu = 0.9f;
    const size_t bytes = ARENA * sizeof(float);
    int p, b, t;
    int64_t i;

    CHECK(eager_create(&ctx, P, NB, off, num, EAGER_F32, EAGER_ORDER_FIXED) == EAGER_OK);
    CHECK(eager_set_update_rule(ctx, 0.001f, 1) == EAGER_OK);
    hw = calloc(ARENA, sizeof(float)); hv = calloc(ARENA, sizeof(float));
    hrecv = calloc(ARENA, sizeof(float)); back = malloc(bytes);
    HIP(hipMalloc((void **)&dw, bytes)); HIP(hipMalloc((void **)&dv, bytes));
    HIP(hipMalloc((void **)&drecv, bytes));
    for (i = 0; i < ARENA; ++i) hw[i] = value(99, 7, (unsigned)i) * 16.0f;
    HIP(hipMemcpy(dw, hw, bytes, hipMemcpyHostToDevice));
    HIP(hipMemset(dv, 0, bytes));
    for (p = 0; p < P; ++p) {
        hG[p] = calloc(ARENA, sizeof(float)); hR[p] = calloc(ARENA, sizeof(float));
        HIP(hipMalloc((void **)&dG[p], bytes)); HIP(hipMalloc((void **)&dR[p], bytes));
        HIP(hipMemset(dR[p], 0xff, bytes));           /* empty send buffers hold NaN patterns */
        dGc[p] = dG[p];
    }

    for (t = 0; t < 6; ++t) {
        const double arrival[P] = {1.0 + (t * 7 % 5), 2.0 + (t * 3 % 4), 1.5 + (t % 3)};
        eager_plan plan;
        const eager_opt opt = {dw, dv, lr, mu};
        const int unfused = t == 4;
        for (p = 0; p < P; ++p) {
            for (i = 0; i < ARENA; ++i) hG[p][i] = value((unsigned)t, (unsigned)p, (unsigned)i);
            HIP(hipMemcpy(dG[p], hG[p], bytes, hipMemcpyHostToDevice));
        }
        if (t % 3 == 0) {
            CHECK(eager_plan_participation(EAGER_SOLO, P, arrival, 5u, (uint64_t)t, 0.0, 0u, &plan) == EAGER_OK);
            CHECK(eager_partial_allreduce_solo(ctx, &plan, 0, NB, dGc, dR, drecv, unfused ? NULL : &opt, NULL) == EAGER_OK);
        } else if (t % 3 == 1) {
            CHECK(eager_plan_participation(EAGER_MAJORITY, P, arrival, 5u, (uint64_t)t, 0.0, 0u, &plan) == EAGER_OK);
            CHECK(eager_partial_allreduce_majority(ctx, &plan, 0, NB, dGc, dR, drecv, unfused ? NULL : &opt, NULL) == EAGER_OK);
        } else {
            CHECK(eager_plan_quorum(P, arrival, 2, (uint64_t)t, 0.0, &plan) == EAGER_OK);
            CHECK(eager_partial_allreduce_quorum(ctx, &plan, 0, NB, dGc, dR, drecv, unfused ? NULL : &opt, NULL) == EAGER_OK);
        }
        if (unfused) CHECK(eager_sgd_step(ctx, 0, NB, drecv, &opt, NULL) == EAGER_OK);
        for (b = 0; b < NB; ++b) {                    /* the same round in the oracle */
            const void *g[P];
            float *r[P];
            for (p = 0; p < P; ++p) { g[p] = hG[p] + off[b]; r[p] = hR[p] + off[b]; }
            eager_oracle_round_async(P, num[b], g, 0, r, valid[b], plan.mask, 0u,
                                     unfused ? NULL : hw + off[b], unfused ? NULL : hv + off[b],
                                     lr, mu, 0.001f, 1, hrecv + off[b], 1);
            if (unfused)
                eager_oracle_sgd_ex(num[b], hrecv + off[b], hw + off[b], hv + off[b], lr, mu, 0.001f, 1, 1);
            valid[b] = ~plan.mask & ((1u << P) - 1u);
        }
        if (t == 2) {                                 /* a gradient that finished between rounds */
            for (i = 0; i < ARENA; ++i) hG[1][i] = value(77u, 1u, (unsigned)i);
            HIP(hipMemcpy(dG[1], hG[1], bytes, hipMemcpyHostToDevice));
            CHECK(eager_stash(ctx, 1, 0, NB, dG[1], dR[1], NULL) == EAGER_OK);
            for (b = 0; b < NB; ++b) {
                eager_oracle_stash(num[b], hG[1] + off[b], 0, hR[1] + off[b], (int)((valid[b] >> 1) & 1u));
                valid[b] |= 2u;
            }
        }
        HIP(hipDeviceSynchronize());
        for (b = 0; b < NB; ++b) {
            const size_t nb = (size_t)num[b] * sizeof(float);
            CHECK(eager_get_valid(ctx, b, &got) == EAGER_OK && got == valid[b]);
            HIP(hipMemcpy(back, dw + off[b], nb, hipMemcpyDeviceToHost));
            CHECK(memcmp(back, hw + off[b], nb) == 0);
            HIP(hipMemcpy(back, dv + off[b], nb, hipMemcpyDeviceToHost));
            CHECK(memcmp(back, hv + off[b], nb) == 0);
            HIP(hipMemcpy(back, drecv + off[b], nb, hipMemcpyDeviceToHost));
            CHECK(memcmp(back, hrecv + off[b], nb) == 0);
            for (p = 0; p < P; ++p)
                if ((valid[b] >> p) & 1u) {
                    HIP(hipMemcpy(back, dR[p] + off[b], nb, hipMemcpyDeviceToHost));
                    CHECK(memcmp(back, hR[p] + off[b], nb) == 0);
                }
        }
    }
    CHECK(eager_destroy(ctx) == EAGER_OK);
    for (p = 0; p < P; ++p) { HIP(hipFree(dG[p])); HIP(hipFree(dR[p])); free(hG[p]); free(hR[p]); }
    HIP(hipFree(dw)); HIP(hipFree(dv)); HIP(hipFree(drecv));
    free(hw); free(hv); free(hrecv); free(back);
    printf("ok\n");
    return 0;
}
