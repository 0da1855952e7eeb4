/*
 * CPU oracle for the eager-SGD hot path: one partial-allreduce round with stale-gradient
 * carry, averaged over P and applied as a momentum-SGD update.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU library is
 * checked against.  It shares no code with the GPU library and must never be called
 * from the product path; only the tests, the smoke check and the benchmark's
 * cpu_baseline leg may use it.
 *
 * What it follows (paper: "Taming Unbalanced Training Workloads in Deep Learning with
 * Partial Collective Operations"):
 *   - Section 5, the two-process walk-through of Fig. 7: a process that is late at round
 *     t contributes only what its send buffer holds (nothing, or the gradient it finished
 *     late in the previous round); the gradient it finishes late becomes the new content
 *     of the send buffer; a process that is on time contributes send buffer + fresh
 *     gradient and its send buffer becomes empty (G_null).
 *   - Algorithm 2, line 6: the result is the sum of the contributions times 1/P (P, not
 *     the number of contributors); lines 7-8: the update rule U is applied to it.
 *   - Section 6.1: the per-process bit s_t^i (did this process's update enter the result
 *     of round t) is the participation mask; a rejected update is added in the next round,
 *     exactly once.
 *
 * Readings where the paper is silent (they are conventions of this repository):
 *   - U is heavy-ball momentum SGD, v <- mu*v + u, w <- w - lr*v, each as one fused
 *     multiply-add (single rounding).  The paper leaves U generic (Algorithm 2, line 7);
 *     two common variants are available and off by default: weight decay (g = u + wd*w
 *     enters the rule in place of u) and Nesterov momentum (the step is g + mu*v' instead
 *     of v'), each again one fused multiply-add.
 *   - fp32 throughout, round-to-nearest-even; the P contributions are added in
 *     ascending rank order starting from +0.0f; 1/P is computed once in fp32 and
 *     multiplied.  This fixed order is what makes a bit-exact comparison possible.
 *     "parity unpinned" for the ORDER itself: the paper fixes no order, so nothing
 *     outside this repository can confirm it; every value-level property is pinned by
 *     the tests (brute-force ledger, worked example, allreduce special case,
 *     conservation, Lemma-2 identity, closed-form momentum).
 *
 * Compile with -ffp-contract=off so that no multiply-add is fused except where fmaf is
 * written out.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static inline float widen_bf16(uint16_t h)
{
    uint32_t b = (uint32_t)h << 16;   /* bf16 is the top half of an fp32: exact */
    float f;
    memcpy(&f, &b, sizeof f);
    return f;
}

/* The update rule U on one element (Algorithm 2, lines 7-8), with the optional variants. */
static inline void update_rule(float u, float *w, float *v, float lr, float mu, float wd,
                               int nesterov)
{
    float g = u, vn, step;
    if (wd != 0.0f)
        g = fmaf(wd, *w, u);
    vn = fmaf(mu, *v, g);
    step = vn;
    if (nesterov)
        step = fmaf(mu, vn, g);
    *v = vn;
    *w = fmaf(-lr, step, *w);
}

/*
 * One round over one bucket of n elements.
 *
 *   P            number of processes (1..64)
 *   G[p]         fresh gradient of process p, n elements, fp32 or bf16 (grad_is_bf16)
 *   R[p]         send buffer of process p (fp32, n elements); read only where bit p of
 *                `valid` is set, written for every process whose bit in `mask` is clear
 *   valid        bit p set: R[p] holds a gradient that has not been delivered yet
 *   mask         bit p set: process p is active in this round (s_t^p = true)
 *   w, v         parameters and momentum (fp32, n elements), updated in place; both may
 *                be NULL to skip the update rule
 *   absent       bit p set (only where mask's bit is clear): process p has not finished a
 *                gradient in this round's window either (it lags by more than one round,
 *                last paragraph of Section 5): it contributes what its send buffer holds
 *                and stores nothing; G[p] is not read
 *   wd, nesterov variants of the update rule (0, 0 = heavy-ball momentum SGD)
 *   recv         receive buffer, gets the averaged result u; may be NULL
 *   nthreads     1 = the scalar reference; >1 = same loop body, elements partitioned
 *                statically over threads (per-element arithmetic and order unchanged)
 *
 * After the call the caller sets valid' = ~mask (on-time processes emptied their send
 * buffer, late ones stored the gradient they finished late).
 */
void eager_oracle_round_async(int P, int64_t n,
                              const void *const *G, int grad_is_bf16,
                              float *const *R, uint64_t valid, uint64_t mask, uint64_t absent,
                              float *w, float *v, float lr, float mu, float wd, int nesterov,
                              float *recv, int nthreads)
{
    const float inv_P = 1.0f / (float)P;
    int64_t i;
    (void)nthreads;
#pragma omp parallel for schedule(static) num_threads(nthreads) if (nthreads > 1)
    for (i = 0; i < n; ++i) {
        float s = 0.0f;
        int p;
        for (p = 0; p < P; ++p) {
            const int on_time = (int)((mask >> p) & 1u);
            const int has_stale = (int)((valid >> p) & 1u);
            const int is_absent = (int)((absent >> p) & 1u);
            float g = 0.0f;
            if (!is_absent)
                g = grad_is_bf16 ? widen_bf16(((const uint16_t *)G[p])[i])
                                 : ((const float *)G[p])[i];
            if (on_time) {
                /* contributes stale + fresh; its send buffer becomes G_null */
                float c = g;
                if (has_stale)
                    c = R[p][i] + g;
                s = s + c;
            } else {
                /* contributes only what was pending; the late gradient is stored (a process
                 * that is still computing has none to store) */
                if (has_stale)
                    s = s + R[p][i];
                if (!is_absent)
                    R[p][i] = g;
            }
        }
        {
            const float u = s * inv_P;
            if (w)
                update_rule(u, &w[i], &v[i], lr, mu, wd, nesterov);
            if (recv)
                recv[i] = u;
        }
    }
}

void eager_oracle_round_ex(int P, int64_t n,
                           const void *const *G, int grad_is_bf16,
                           float *const *R, uint64_t valid, uint64_t mask,
                           float *w, float *v, float lr, float mu, float wd, int nesterov,
                           float *recv, int nthreads)
{
    eager_oracle_round_async(P, n, G, grad_is_bf16, R, valid, mask, 0u, w, v, lr, mu, wd,
                             nesterov, recv, nthreads);
}

/* A process that finishes a gradient after the round it was computed for has been executed
 * puts it into its send buffer (Section 5): the buffer holds it alone if it was empty,
 * else the sum of what it held and the new gradient (a process that lags by several
 * rounds may finish two gradients between two executions). */
void eager_oracle_stash(int64_t n, const void *G, int grad_is_bf16, float *R, int has_stale)
{
    int64_t i;
    for (i = 0; i < n; ++i) {
        const float g = grad_is_bf16 ? widen_bf16(((const uint16_t *)G)[i]) : ((const float *)G)[i];
        R[i] = has_stale ? R[i] + g : g;
    }
}

void eager_oracle_round(int P, int64_t n,
                        const void *const *G, int grad_is_bf16,
                        float *const *R, uint64_t valid, uint64_t mask,
                        float *w, float *v, float lr, float mu,
                        float *recv, int nthreads)
{
    eager_oracle_round_ex(P, n, G, grad_is_bf16, R, valid, mask, w, v, lr, mu, 0.0f, 0, recv,
                          nthreads);
}

/* The update rule alone, applied to an already averaged result u (the unfused path:
 * receive buffer first, optimizer afterwards). */
void eager_oracle_sgd_ex(int64_t n, const float *u, float *w, float *v, float lr, float mu,
                         float wd, int nesterov, int nthreads)
{
    int64_t i;
    (void)nthreads;
#pragma omp parallel for schedule(static) num_threads(nthreads) if (nthreads > 1)
    for (i = 0; i < n; ++i)
        update_rule(u[i], &w[i], &v[i], lr, mu, wd, nesterov);
}

/*
 * The update rule with a rate per layer (bucket), one more instance of the generic U of
 * Algorithm 2, line 7: layer-wise adaptive rate scaling as published by You, Gitman and
 * Ginsburg (2017), the large-batch recipe behind the work the paper points to in
 * Section 7.3 for batch sizes that need tuned rates.  For a bucket with averaged update u
 * and parameters w (both before the step), over the finite elements only:
 *
 *     rate = trust * ||w|| / (||u|| + wd * ||w|| + eps)     if ||w|| > 0 and ||u|| > 0
 *          = 1                                              otherwise (e.g. biases at zero)
 *
 * norms from fp64 sums of squares in index order, the rate computed in fp64 and rounded to
 * fp32 once.  Then per element
 *
 *     g = rate * (u + wd * w);  v' = mu * v + g;  step = nesterov ? g + mu * v' : v';
 *     w' = w - lr * step
 *
 * (the scaled gradient enters the momentum, as in the publication).  Returns the rate.
 */
float eager_oracle_sgd_lars(int64_t n, const float *u, float *w, float *v, float lr, float mu,
                            float wd, int nesterov, float trust, float eps)
{
    double ssu = 0.0, ssw = 0.0, nu, nw;
    float rate = 1.0f;
    int64_t i;
    for (i = 0; i < n; ++i) {
        if (isfinite(u[i]))
            ssu += (double)u[i] * (double)u[i];
        if (isfinite(w[i]))
            ssw += (double)w[i] * (double)w[i];
    }
    nu = sqrt(ssu);
    nw = sqrt(ssw);
    if (nu > 0.0 && nw > 0.0)
        rate = (float)((double)trust * nw / (nu + (double)wd * nw + (double)eps));
    for (i = 0; i < n; ++i) {
        float g = u[i];
        if (wd != 0.0f)
            g = fmaf(wd, w[i], u[i]);
        /* the decay is already in g: the plain rule on the scaled gradient */
        update_rule(rate * g, &w[i], &v[i], lr, mu, 0.0f, nesterov);
    }
    return rate;
}

void eager_oracle_sgd(int64_t n, const float *u, float *w, float *v, float lr, float mu,
                      int nthreads)
{
    eager_oracle_sgd_ex(n, u, w, v, lr, mu, 0.0f, 0, nthreads);
}
