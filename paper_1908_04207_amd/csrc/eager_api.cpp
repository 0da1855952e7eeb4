// Host side of the C ABI: context state (bucket table, send-buffer validity per bucket),
// argument checking, the participation plan, and the split of a bucket range into runs
// that one kernel launch each can cover.  All arithmetic of a round runs in the kernels.
#include "../../include/eager_tuning.h"
#include "eager_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

struct eager_ctx {
    int P = 0;
    int n_buckets = 0;
    bool bf16 = false;
    bool fast = false;
    std::vector<int64_t> offset, numel;
    std::vector<uint64_t> valid;       // per bucket: bit p = R_p holds an undelivered gradient
    std::vector<uint64_t> last_step;   // per bucket: round it was last stepped with
    std::vector<uint8_t> stepped;      // per bucket: last_step is meaningful
    eager::Launch launch;
    float weight_decay = 0.0f;         // update rule variants (eager_set_update_rule)
    int nesterov = 0;
    std::vector<long long> table;      // start, end of every bucket (the device copy lives in the
                                       // statistics workspace)
    eager::BucketStats *stats = nullptr;   // device, caller-owned; NULL: no by-products
    char *workspace = nullptr;             // device, caller-owned: bucket table, then records
    std::string err;
};

namespace {

int fail(eager_ctx *ctx, int status, const char *fmt, ...)
{
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        ctx->err = buf;
    }
    return status;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int popcount64(uint64_t x) { return __builtin_popcountll(x); }

uint64_t low_bits(int P) { return P >= 64 ? ~0ull : ((1ull << P) - 1ull); }

// SplitMix64 output function on seed + (step+1)*gamma: the shared-seed draw of the
// designated initiator (paper Section 4.2).
uint64_t initiator_hash(uint64_t seed, uint64_t step)
{
    uint64_t z = seed + (step + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// wavefronts a round kernel may be launched with over the whole arena, whatever the block size
int64_t max_records(const eager_ctx *ctx)
{
    const int64_t span = ctx->offset.back() + ctx->numel.back() - ctx->offset.front();
    return span / 256 + 8;
}

// Fills the parts of the statistics arguments that do not depend on the run: where the bucket
// table, the records, the lane records and the partials live in the caller's workspace.
void stats_layout(const eager_ctx *ctx, char *workspace, eager::BucketStats *stats,
                  eager::StatsArgs &st)
{
    st.table = reinterpret_cast<const long long *>(workspace);
    st.stats = stats;
    st.records = reinterpret_cast<eager::StatsRecord *>(
        workspace + static_cast<size_t>(ctx->n_buckets) * 16);
    st.lane_records = st.records + max_records(ctx);
    st.partials = st.lane_records + (static_cast<int64_t>(ctx->n_buckets) + 1) * 64;
    st.n_buckets = ctx->n_buckets;
}

// Workgroups that add up the records of one bucket before the finishing kernel: from the
// largest bucket of the run (one record per 256 elements)
int stats_slices(const eager_ctx *ctx, int b0, int b1)
{
    int64_t most = 0;
    for (int b = b0; b < b1; ++b) most = std::max(most, ctx->numel[b] / 256);
    const int64_t s = (most + eager::kStatsRecordsPerSlice - 1) / eager::kStatsRecordsPerSlice;
    return static_cast<int>(std::min<int64_t>(std::max<int64_t>(s, 1), eager::kStatsMaxSlices));
}

// Whether the send-buffer rewrite of the late processes runs as its own copy kernel after
// the reduction instead of inside it.
bool use_split(const eager::Launch &l, int P, uint64_t mask, uint64_t valid, int64_t n)
{
    if (l.split == 1) return false;
    if (l.split == 2) return true;
    // Measured on MI355X: a copy that streams one source and one destination at a time
    // reaches 6.7 TB/s, whereas the same bytes written as several interleaved streams next
    // to the reduction's reads cost 5-10 % of the round (P = 8, 7 late: 6.1 fused, 6.7 split).
    // The fused pass wins while few processes are late and all of its streams fit one chunk
    // of 16 loads, and on short runs, where the second launch costs more than it saves
    // (25 M elements, P = 8: 7.03 fused against 6.82 TB/s split).  The same holds with bf16
    // gradients (P = 16, 15 late: 6.43 split against 5.91 TB/s fused on 67 M elements, 6.31
    // against 6.19 on 1.56e9; P = 16, 2 late, 16 M elements: 6.68 split against 6.71 fused).
    const uint64_t late = ~mask & low_bits(P);
    const int n_late = popcount64(late);
    if (n_late == 0) return false;
    const int fused_streams = P + popcount64(valid);   // every G_p, every non-empty R_p
    return fused_streams > 16 || n_late >= 8 || (n_late >= 3 && n >= (int64_t{1} << 25));
}

int check_range(eager_ctx *ctx, int b0, int b1)
{
    if (b0 < 0 || b1 > ctx->n_buckets || b0 >= b1)
        return fail(ctx, EAGER_EINVAL, "bucket range [%d, %d) is empty or outside 0..%d", b0, b1,
                    ctx->n_buckets);
    return EAGER_OK;
}

int check_opt(eager_ctx *ctx, const eager_opt *opt)
{
    if (!opt->params || !opt->momentum)
        return fail(ctx, EAGER_EINVAL, "opt->params and opt->momentum must not be NULL");
    if (!aligned16(opt->params) || !aligned16(opt->momentum))
        return fail(ctx, EAGER_EINVAL, "opt->params / opt->momentum must be 16-byte aligned");
    return EAGER_OK;
}

// What becomes of the gradient a late process finishes:
//   kCopy      it is copied into the send buffer (in the round's pass, or by the copy kernel)
//   kExchange  its buffer becomes the send buffer: the caller of partial_allreduce exchanges
//              the two pointers in the user's tables on success, and the round neither reads
//              nor writes the late gradients
//   kFlush     there is none: the round in which nobody hands over a gradient (every process
//              absent, nobody active); `plan` is then a stand-in without an initiator and
//              belongs to no round index
enum RoundKind { kCopy, kExchange, kFlush };

// want_mode < 0: any mode.  absent: processes outside the mask that store no gradient.
int partial_allreduce(eager_ctx *ctx, int want_mode, const eager_plan *plan, uint64_t absent,
                      int b0, int b1, const void *const *grads, float *const *resid,
                      float *recv, const eager_opt *opt, void *stream, RoundKind kind = kCopy)
{
    const bool exchange = kind == kExchange, flush = kind == kFlush;
    if (!ctx) return EAGER_EINVAL;
    if (!plan || (!grads && !flush) || !resid)
        return fail(ctx, EAGER_EINVAL, "plan, grads and resid must not be NULL");
    if (int st = check_range(ctx, b0, b1)) return st;
    if (!opt && !recv)
        return fail(ctx, EAGER_EINVAL, "nothing to produce: recv and opt are both NULL");
    if (opt) {
        if (int st = check_opt(ctx, opt)) return st;
    }
    if (recv && !aligned16(recv)) return fail(ctx, EAGER_EINVAL, "recv must be 16-byte aligned");
    const int P = ctx->P;
    if (want_mode >= 0 && plan->mode != want_mode)
        return fail(ctx, EAGER_ESTATE, "plan->mode %d does not match this entry point (%d)",
                    plan->mode, want_mode);
    if (plan->mode < EAGER_SOLO || plan->mode > EAGER_QUORUM)
        return fail(ctx, EAGER_ESTATE, "plan->mode %d is not a mode", plan->mode);
    if (absent & plan->mask) return fail(ctx, EAGER_ESTATE, "an absent process cannot be active");
    if (absent & ~low_bits(P)) return fail(ctx, EAGER_ESTATE, "absent mask has bits beyond P");
    if (plan->P != P) return fail(ctx, EAGER_ESTATE, "plan->P %d != context P %d", plan->P, P);
    if (plan->mask & ~low_bits(P)) return fail(ctx, EAGER_ESTATE, "plan->mask has bits beyond P");
    if (plan->nap != popcount64(plan->mask) || (plan->nap < 1 && !flush))
        return fail(ctx, EAGER_ESTATE, "plan->nap %d is not popcount(mask) >= 1", plan->nap);
    if (!flush &&
        (plan->initiator < 0 || plan->initiator >= P || !((plan->mask >> plan->initiator) & 1ull)))
        return fail(ctx, EAGER_ESTATE, "initiator %d is not in the mask", plan->initiator);
    if (plan->flags & ~EAGER_FLAG_STRICT_QUORUM)
        return fail(ctx, EAGER_ESTATE, "plan->flags %#x holds unknown bits", plan->flags);
    if (want_mode == EAGER_MAJORITY && (plan->flags & EAGER_FLAG_STRICT_QUORUM) &&
        plan->nap < (P + 1) / 2)
        return fail(ctx, EAGER_ESTATE, "a strict majority round needs %d of %d processes, the plan has %d",
                    (P + 1) / 2, P, plan->nap);
    for (int p = 0; p < P; ++p) {
        const bool needs_g = !((absent >> p) & 1ull);       // an absent process has no gradient
        if ((needs_g && !grads[p]) || !resid[p])
            return fail(ctx, EAGER_EINVAL, "grads[%d] or resid[%d] is NULL", p, p);
        if ((needs_g && !aligned16(grads[p])) || !aligned16(resid[p]))
            return fail(ctx, EAGER_EINVAL, "grads[%d] / resid[%d] must be 16-byte aligned", p, p);
    }
    for (int b = b0; b < b1 && !flush; ++b)
        if (ctx->stepped[b] && ctx->last_step[b] == plan->step)
            return fail(ctx, EAGER_ESTATE, "bucket %d was already stepped with round %llu", b,
                        static_cast<unsigned long long>(plan->step));

    eager::RoundArgs a;
    std::memset(&a, 0, sizeof a);
    for (int p = 0; p < P; ++p) {
        a.g[p] = grads ? grads[p] : nullptr;
        a.r[p] = resid[p];
    }
    a.active = plan->mask;
    a.w = opt ? opt->params : nullptr;
    a.v = opt ? opt->momentum : nullptr;
    a.recv = recv;
    a.P = P;
    a.elem_bytes = ctx->bf16 ? 2 : 4;
    a.inv_P = 1.0f / static_cast<float>(P);
    a.neg_lr = opt ? -opt->lr : 0.0f;
    a.mu = opt ? opt->mu : 0.0f;
    a.wd = ctx->weight_decay;
    a.nesterov = ctx->nesterov;
    const bool round_stats = ctx->stats && ctx->launch.round_stats;
    if (round_stats) {
        if (ctx->launch.chunk != 0 && ctx->launch.chunk != 16)
            return fail(ctx, EAGER_ESTATE, "bucket statistics need the default chunk size (16)");
        stats_layout(ctx, ctx->workspace, ctx->stats, a.stats);
    }

    // Everything that could make a launcher refuse is checked for every run before the first
    // kernel is enqueued (the launch keys are validated when they are set): a run longer than
    // one grid covers.  After this point only the HIP runtime can fail.
    for (int b = b0; b < b1;) {
        int e = b + 1;
        while (e < b1 && ctx->valid[e] == ctx->valid[b]) ++e;
        const int64_t n = ctx->offset[e - 1] + ctx->numel[e - 1] - ctx->offset[b];
        if (n > (int64_t{1} << 33))
            return fail(ctx, EAGER_EINVAL, "buckets %d..%d span %lld elements in one send-buffer state; "
                                           "one call covers at most 2^33 per such stretch: use smaller ranges",
                        b, e - 1, static_cast<long long>(n));
        b = e;
    }

    // Consecutive buckets whose send buffers are in the same state form one run = one
    // launch over a contiguous element range (after a whole-model round every bucket is
    // in the same state, so a round is normally a single launch however small the
    // buckets are).
    int b = b0;
    while (b < b1) {
        int e = b + 1;
        while (e < b1 && ctx->valid[e] == ctx->valid[b]) ++e;
        a.valid = ctx->valid[b];
        a.e0 = ctx->offset[b];
        a.n = ctx->offset[e - 1] + ctx->numel[e - 1] - ctx->offset[b];
        const uint64_t late = ~plan->mask & ~absent & low_bits(P);   // finish a gradient late
        const bool split = exchange ||
                           use_split(ctx->launch, P, plan->mask | absent, a.valid, a.n);
        a.gload = split ? plan->mask : (plan->mask | late);
        a.store = split ? 0 : late;
        if (round_stats) {
            a.stats.e0 = a.e0;
            a.stats.b_lo = b;
            a.stats.b_hi = e;
            a.stats.n_records = eager::slot_records(a.n, ctx->bf16, ctx->launch.block);
            a.stats.tail_count = eager::slot_tail(a.n, ctx->bf16);
            a.stats.slices = stats_slices(ctx, b, e);
        }
        hipError_t he = eager::launch_round(a, ctx->bf16, ctx->fast, ctx->launch,
                                            static_cast<hipStream_t>(stream));
        if (he != hipSuccess)
            return fail(ctx, EAGER_EDEVICE, "round kernel launch failed: %s", hipGetErrorString(he));
        if (round_stats) {
            he = eager::launch_stats_finish(a.stats, static_cast<hipStream_t>(stream));
            if (he != hipSuccess)
                return fail(ctx, EAGER_EDEVICE, "statistics kernel launch failed: %s",
                            hipGetErrorString(he));
        }
        if (split && !exchange) {
            // same stream: the reduction has read every pending R_p before it is overwritten
            eager::CarryArgs c;
            std::memset(&c, 0, sizeof c);
            for (int p = 0; p < P; ++p)
                if ((late >> p) & 1ull) {
                    c.src[c.count] = grads[p];
                    c.dst[c.count] = resid[p];
                    ++c.count;
                }
            c.e0 = a.e0;
            c.n = a.n;
            he = eager::launch_carry(c, ctx->bf16, ctx->launch, static_cast<hipStream_t>(stream));
            if (he != hipSuccess)
                return fail(ctx, EAGER_EDEVICE, "carry kernel launch failed: %s",
                            hipGetErrorString(he));
        }
        for (int k = b; k < e; ++k) {
            ctx->valid[k] = late;
            ctx->last_step[k] = plan->step;
            ctx->stepped[k] = flush ? 0 : 1;
        }
        b = e;
    }
    ctx->err.clear();
    return EAGER_OK;
}

}  // namespace

extern "C" {

int eager_create(eager_ctx **out, int P, int n_buckets, const int64_t *bucket_offset,
                 const int64_t *bucket_numel, int grad_dtype, int order)
{
    if (!out) return EAGER_EINVAL;
    *out = nullptr;
    if (!bucket_offset || !bucket_numel) return EAGER_EINVAL;
    if (P < 1 || P > EAGER_MAX_P || n_buckets < 1) return EAGER_EINVAL;
    if (grad_dtype != EAGER_F32 && grad_dtype != EAGER_BF16) return EAGER_EINVAL;
    if (order != EAGER_ORDER_FIXED && order != EAGER_ORDER_FAST) return EAGER_EINVAL;
    const int64_t align = grad_dtype == EAGER_BF16 ? 8 : 4;
    int64_t end = 0;
    for (int b = 0; b < n_buckets; ++b) {
        if (bucket_numel[b] < 0 || bucket_offset[b] < end || bucket_offset[b] % align != 0)
            return EAGER_ESHAPE;
        if (bucket_numel[b] > INT64_MAX / 8 - bucket_offset[b]) return EAGER_ESHAPE;
        end = bucket_offset[b] + bucket_numel[b];
    }
    eager_ctx *c = new (std::nothrow) eager_ctx;
    if (!c) return EAGER_ENOMEM;
    try {
        c->P = P;
        c->n_buckets = n_buckets;
        c->bf16 = grad_dtype == EAGER_BF16;
        c->fast = order == EAGER_ORDER_FAST;
        c->offset.assign(bucket_offset, bucket_offset + n_buckets);
        c->numel.assign(bucket_numel, bucket_numel + n_buckets);
        c->valid.assign(n_buckets, 0);
        c->last_step.assign(n_buckets, 0);
        c->stepped.assign(n_buckets, 0);
        c->table.resize(static_cast<size_t>(n_buckets) * 2);
        for (int b = 0; b < n_buckets; ++b) {
            c->table[2 * b] = bucket_offset[b];
            c->table[2 * b + 1] = bucket_offset[b] + bucket_numel[b];
        }
    } catch (const std::bad_alloc &) {
        delete c;
        return EAGER_ENOMEM;
    }
    *out = c;
    return EAGER_OK;
}

int eager_destroy(eager_ctx *ctx)
{
    delete ctx;
    return EAGER_OK;
}

const char *eager_last_error(const eager_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

#ifndef EAGER_SOURCE_HASH
#define EAGER_SOURCE_HASH "unknown"
#endif
const char *eager_source_hash(void) { return EAGER_SOURCE_HASH; }

const char *eager_status_string(int status)
{
    switch (status) {
    case EAGER_OK: return "EAGER_OK";
    case EAGER_EINVAL: return "EAGER_EINVAL";
    case EAGER_ESHAPE: return "EAGER_ESHAPE";
    case EAGER_ESTATE: return "EAGER_ESTATE";
    case EAGER_EDEVICE: return "EAGER_EDEVICE";
    case EAGER_ENOMEM: return "EAGER_ENOMEM";
    case EAGER_ELIMIT: return "EAGER_ELIMIT";
    default: return "EAGER_<unknown>";
    }
}

int eager_plan_participation(int mode, int P, const double *arrival_ms, uint64_t seed,
                             uint64_t step, double window_ms, uint32_t flags, eager_plan *out)
{
    if (!arrival_ms || !out) return EAGER_EINVAL;
    if (P < 1 || P > EAGER_MAX_P) return EAGER_EINVAL;
    if (mode != EAGER_SOLO && mode != EAGER_MAJORITY) return EAGER_EINVAL;
    if (!(window_ms >= 0.0)) return EAGER_EINVAL;
    if (flags & ~EAGER_FLAG_STRICT_QUORUM) return EAGER_EINVAL;
    for (int p = 0; p < P; ++p)
        if (std::isnan(arrival_ms[p])) return EAGER_EINVAL;

    int init = 0;
    if (mode == EAGER_SOLO) {
        for (int p = 1; p < P; ++p)
            if (arrival_ms[p] < arrival_ms[init]) init = p;   // strict: lowest rank wins a tie
    } else {
        init = static_cast<int>(initiator_hash(seed, step) % static_cast<uint64_t>(P));
    }
    double threshold = arrival_ms[init] + window_ms;
    if (mode == EAGER_MAJORITY && (flags & EAGER_FLAG_STRICT_QUORUM)) {
        // the time by which ceil(P/2) processes have arrived
        const int need = (P + 1) / 2;
        double sorted[EAGER_MAX_P];
        for (int p = 0; p < P; ++p) sorted[p] = arrival_ms[p];
        for (int i = 1; i < P; ++i) {
            const double x = sorted[i];
            int j = i - 1;
            while (j >= 0 && sorted[j] > x) { sorted[j + 1] = sorted[j]; --j; }
            sorted[j + 1] = x;
        }
        if (sorted[need - 1] > threshold) threshold = sorted[need - 1];
    }
    uint64_t mask = 0;
    for (int p = 0; p < P; ++p)
        if (arrival_ms[p] <= threshold) mask |= 1ull << p;
    out->mode = mode;
    out->P = P;
    out->step = step;
    out->mask = mask;
    out->initiator = init;
    out->nap = popcount64(mask);
    out->flags = mode == EAGER_MAJORITY ? (flags & EAGER_FLAG_STRICT_QUORUM) : 0u;
    out->reserved = 0u;
    return EAGER_OK;
}

int eager_plan_quorum(int P, const double *arrival_ms, int quorum, uint64_t step,
                      double window_ms, eager_plan *out)
{
    if (!arrival_ms || !out) return EAGER_EINVAL;
    if (P < 1 || P > EAGER_MAX_P || quorum < 1 || quorum > P) return EAGER_EINVAL;
    if (!(window_ms >= 0.0)) return EAGER_EINVAL;
    for (int p = 0; p < P; ++p)
        if (std::isnan(arrival_ms[p])) return EAGER_EINVAL;
    // ranks in order of arrival, equal times by rank (stable insertion sort, P <= 64)
    int order[EAGER_MAX_P];
    for (int i = 0; i < P; ++i) {
        int j = i - 1;
        while (j >= 0 && arrival_ms[order[j]] > arrival_ms[i]) { order[j + 1] = order[j]; --j; }
        order[j + 1] = i;
    }
    const int init = order[quorum - 1];
    const double threshold = arrival_ms[init] + window_ms;
    uint64_t mask = 0;
    for (int p = 0; p < P; ++p)
        if (arrival_ms[p] <= threshold) mask |= 1ull << p;
    out->mode = EAGER_QUORUM;
    out->P = P;
    out->step = step;
    out->mask = mask;
    out->initiator = init;
    out->nap = popcount64(mask);
    out->flags = 0u;
    out->reserved = 0u;
    return EAGER_OK;
}

int eager_designated_initiator(uint64_t seed, uint64_t round, int P, int *rank)
{
    if (!rank || P < 1 || P > EAGER_MAX_P) return EAGER_EINVAL;
    *rank = static_cast<int>(initiator_hash(seed, round) % static_cast<uint64_t>(P));
    return EAGER_OK;
}

int eager_plan_open_round(int mode, int P, uint64_t waiting, int newest, int quorum,
                          uint64_t seed, uint64_t round, int *triggered, eager_plan *out)
{
    if (!triggered || !out || P < 1 || P > EAGER_MAX_P) return EAGER_EINVAL;
    if (mode < EAGER_SOLO || mode > EAGER_QUORUM) return EAGER_EINVAL;
    if (waiting == 0 || (waiting & ~low_bits(P))) return EAGER_EINVAL;
    if (newest < 0 || newest >= P || !((waiting >> newest) & 1ull)) return EAGER_EINVAL;
    if (mode == EAGER_QUORUM && (quorum < 1 || quorum > P)) return EAGER_EINVAL;
    int init = 0;
    bool go = false;
    if (mode == EAGER_SOLO) {
        go = true;
        init = __builtin_ctzll(waiting);
    } else if (mode == EAGER_MAJORITY) {
        init = static_cast<int>(initiator_hash(seed, round) % static_cast<uint64_t>(P));
        go = (waiting >> init) & 1ull;
    } else {
        go = popcount64(waiting) >= quorum;
        init = newest;
    }
    *triggered = go ? 1 : 0;
    if (go) {
        out->mode = mode;
        out->P = P;
        out->step = round;
        out->mask = waiting;
        out->initiator = init;
        out->nap = popcount64(waiting);
        out->flags = 0u;
        out->reserved = 0u;
    }
    return EAGER_OK;
}

int eager_partial_allreduce_solo(eager_ctx *ctx, const eager_plan *plan, int b0, int b1,
                                 const void *const *grads, float *const *resid, float *recv,
                                 const eager_opt *opt, void *stream)
{
    return partial_allreduce(ctx, EAGER_SOLO, plan, 0, b0, b1, grads, resid, recv, opt, stream);
}

int eager_partial_allreduce_majority(eager_ctx *ctx, const eager_plan *plan, int b0, int b1,
                                     const void *const *grads, float *const *resid, float *recv,
                                     const eager_opt *opt, void *stream)
{
    return partial_allreduce(ctx, EAGER_MAJORITY, plan, 0, b0, b1, grads, resid, recv, opt, stream);
}

int eager_partial_allreduce_quorum(eager_ctx *ctx, const eager_plan *plan, int b0, int b1,
                                   const void *const *grads, float *const *resid, float *recv,
                                   const eager_opt *opt, void *stream)
{
    return partial_allreduce(ctx, EAGER_QUORUM, plan, 0, b0, b1, grads, resid, recv, opt, stream);
}

int eager_partial_allreduce_lagging(eager_ctx *ctx, const eager_plan *plan, uint64_t absent,
                                    int b0, int b1, const void *const *grads,
                                    float *const *resid, float *recv, const eager_opt *opt,
                                    void *stream)
{
    return partial_allreduce(ctx, -1, plan, absent, b0, b1, grads, resid, recv, opt, stream);
}

int eager_partial_allreduce_exchange(eager_ctx *ctx, const eager_plan *plan, const void **grads,
                                     float **resid, float *recv, const eager_opt *opt, void *stream)
{
    if (!ctx) return EAGER_EINVAL;
    if (ctx->bf16)
        return fail(ctx, EAGER_ESTATE, "a gradient buffer can only become a send buffer when both "
                                       "hold fp32 (this context has bf16 gradients)");
    const int st = partial_allreduce(ctx, -1, plan, 0, 0, ctx->n_buckets, grads, resid, recv, opt,
                                     stream, kExchange);
    if (st != EAGER_OK) return st;
    const uint64_t late = ~plan->mask & low_bits(ctx->P);
    for (int p = 0; p < ctx->P; ++p)
        if ((late >> p) & 1ull) {
            float *pending = const_cast<float *>(static_cast<const float *>(grads[p]));
            grads[p] = resid[p];
            resid[p] = pending;
        }
    return EAGER_OK;
}

int eager_flush(eager_ctx *ctx, int b0, int b1, float *const *resid, float *recv,
                const eager_opt *opt, void *stream)
{
    if (!ctx) return EAGER_EINVAL;
    eager_plan nobody;
    std::memset(&nobody, 0, sizeof nobody);
    nobody.mode = EAGER_SOLO;
    nobody.P = ctx->P;
    return partial_allreduce(ctx, -1, &nobody, low_bits(ctx->P), b0, b1, nullptr, resid, recv, opt,
                             stream, kFlush);
}

int eager_stash(eager_ctx *ctx, int process, int b0, int b1, const void *grad, float *resid,
                void *stream)
{
    if (!ctx) return EAGER_EINVAL;
    if (process < 0 || process >= ctx->P) return fail(ctx, EAGER_EINVAL, "process %d out of range", process);
    if (!grad || !resid) return fail(ctx, EAGER_EINVAL, "grad and resid must not be NULL");
    if (!aligned16(grad) || !aligned16(resid))
        return fail(ctx, EAGER_EINVAL, "grad and resid must be 16-byte aligned");
    if (int st = check_range(ctx, b0, b1)) return st;
    const uint64_t bit = 1ull << process;
    int b = b0;
    while (b < b1) {                     // runs of buckets whose send buffer is in the same state
        int e = b + 1;
        while (e < b1 && ((ctx->valid[e] ^ ctx->valid[b]) & bit) == 0) ++e;
        eager::StashArgs a;
        a.g = grad;
        a.r = resid;
        a.e0 = ctx->offset[b];
        a.n = ctx->offset[e - 1] + ctx->numel[e - 1] - ctx->offset[b];
        a.accumulate = (ctx->valid[b] & bit) ? 1 : 0;
        hipError_t he = eager::launch_stash(a, ctx->bf16, static_cast<hipStream_t>(stream));
        if (he != hipSuccess)
            return fail(ctx, EAGER_EDEVICE, "stash kernel launch failed: %s", hipGetErrorString(he));
        for (int k = b; k < e; ++k) ctx->valid[k] |= bit;
        b = e;
    }
    ctx->err.clear();
    return EAGER_OK;
}

int eager_sgd_step(eager_ctx *ctx, int b0, int b1, const float *update, const eager_opt *opt,
                   void *stream)
{
    if (!ctx) return EAGER_EINVAL;
    if (!update || !opt) return fail(ctx, EAGER_EINVAL, "update and opt must not be NULL");
    if (!aligned16(update)) return fail(ctx, EAGER_EINVAL, "update must be 16-byte aligned");
    if (int st = check_range(ctx, b0, b1)) return st;
    if (int st = check_opt(ctx, opt)) return st;
    eager::SgdArgs a;
    a.u = update;
    a.w = opt->params;
    a.v = opt->momentum;
    a.e0 = ctx->offset[b0];
    a.n = ctx->offset[b1 - 1] + ctx->numel[b1 - 1] - ctx->offset[b0];
    a.neg_lr = -opt->lr;
    a.mu = opt->mu;
    a.wd = ctx->weight_decay;
    a.nesterov = ctx->nesterov;
    hipError_t he = eager::launch_sgd(a, ctx->fast, ctx->launch, static_cast<hipStream_t>(stream));
    if (he != hipSuccess)
        return fail(ctx, EAGER_EDEVICE, "sgd kernel launch failed: %s", hipGetErrorString(he));
    ctx->err.clear();
    return EAGER_OK;
}

namespace {
// The layer-wise update with its statistics workspace at `workspace` and its per-bucket output
// at `stats` (both device memory laid out as eager_stats_attach describes).
int sgd_step_lars(eager_ctx *ctx, int b0, int b1, const float *update, const eager_opt *opt,
                  float trust, float eps, char *workspace, eager::BucketStats *stats,
                  bool fill_table, void *stream)
{
    eager::SgdArgs a;
    a.u = update;
    a.w = opt->params;
    a.v = opt->momentum;
    a.e0 = ctx->offset[b0];
    a.n = ctx->offset[b1 - 1] + ctx->numel[b1 - 1] - ctx->offset[b0];
    a.neg_lr = -opt->lr;
    a.mu = opt->mu;
    a.wd = ctx->weight_decay;
    a.nesterov = ctx->nesterov;
    eager::StatsArgs st;
    std::memset(&st, 0, sizeof st);
    stats_layout(ctx, workspace, stats, st);
    st.slices = stats_slices(ctx, b0, b1);
    st.e0 = a.e0;
    st.b_lo = b0;
    st.b_hi = b1;
    st.n_records = eager::norms_records(a.n);
    st.tail_count = static_cast<int>(a.n % 4);
    st.want_rate = 1;
    st.trust = trust;
    st.wd = ctx->weight_decay;
    st.eps = eps;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t he = hipSuccess;
    if (fill_table)
        he = eager::launch_table_fill(reinterpret_cast<long long *>(workspace), ctx->table.data(),
                                      ctx->n_buckets, s);
    if (he == hipSuccess) he = eager::launch_norms(a, st, s);
    if (he == hipSuccess) he = eager::launch_stats_finish(st, s);
    if (he == hipSuccess) he = eager::launch_sgd_lars(a, st, ctx->fast, s);
    if (he != hipSuccess)
        return fail(ctx, EAGER_EDEVICE, "layer-wise update launch failed: %s", hipGetErrorString(he));
    ctx->err.clear();
    return EAGER_OK;
}

int check_lars(eager_ctx *ctx, int b0, int b1, const float *update, const eager_opt *opt,
               float trust, float eps)
{
    if (!update || !opt) return fail(ctx, EAGER_EINVAL, "update and opt must not be NULL");
    if (!aligned16(update)) return fail(ctx, EAGER_EINVAL, "update must be 16-byte aligned");
    if (!(trust > 0.0f) || std::isinf(trust) || !(eps >= 0.0f) || std::isinf(eps))
        return fail(ctx, EAGER_EINVAL, "trust must be finite and > 0, eps finite and >= 0");
    if (int st = check_range(ctx, b0, b1)) return st;
    return check_opt(ctx, opt);
}
}  // namespace

int eager_sgd_step_lars(eager_ctx *ctx, int b0, int b1, const float *update, const eager_opt *opt,
                        float trust, float eps, void *stream)
{
    if (!ctx) return EAGER_EINVAL;
    if (int st = check_lars(ctx, b0, b1, update, opt, trust, eps)) return st;
    if (!ctx->stats)
        return fail(ctx, EAGER_ESTATE, "the layer-wise rate needs eager_stats_attach (norms and rates "
                                       "are written to the attached array)");
    return sgd_step_lars(ctx, b0, b1, update, opt, trust, eps, ctx->workspace, ctx->stats, false,
                         stream);
}

int eager_sgd_step_lars_static(eager_ctx *ctx, int b0, int b1, const float *update,
                               const eager_opt *opt, float trust, float eps,
                               eager_bucket_stats *stats, void *stream)
{
    static_assert(EAGER_STATIC_MAX_BUCKETS == eager::kStaticMaxBuckets &&
                      EAGER_STATIC_MAX_ELEMENTS == eager::kStaticMaxElements &&
                      EAGER_STATIC_SCRATCH_BYTES == eager::kStaticScratchBytes,
                  "the header states the capacity of the fixed scratch");
    if (!ctx) return EAGER_EINVAL;
    if (int st = check_lars(ctx, b0, b1, update, opt, trust, eps)) return st;
    if (!stats || !aligned16(stats))
        return fail(ctx, EAGER_EINVAL, "stats must be a 16-byte aligned device array of n_buckets entries");
    const int64_t span = ctx->offset.back() + ctx->numel.back() - ctx->offset.front();
    if (ctx->n_buckets > eager::kStaticMaxBuckets || span > eager::kStaticMaxElements)
        return fail(ctx, EAGER_ELIMIT,
                    "the library's fixed scratch holds the statistics of at most %d buckets spanning "
                    "%lld elements; this context has %d buckets spanning %lld (use eager_stats_attach "
                    "and eager_sgd_step_lars with a workspace of your own)",
                    eager::kStaticMaxBuckets, static_cast<long long>(eager::kStaticMaxElements),
                    ctx->n_buckets, static_cast<long long>(span));
    int64_t need = 0;
    eager_stats_workspace_bytes(ctx, &need);
    if (need > eager::kStaticScratchBytes)     // cannot happen within the two limits above
        return fail(ctx, EAGER_ELIMIT, "statistics workspace of %lld bytes exceeds the fixed scratch",
                    static_cast<long long>(need));
    char *scratch = nullptr;
    if (hipError_t he = eager::static_scratch(&scratch); he != hipSuccess)
        return fail(ctx, EAGER_EDEVICE, "address of the fixed scratch: %s", hipGetErrorString(he));
    return sgd_step_lars(ctx, b0, b1, update, opt, trust, eps, scratch,
                         reinterpret_cast<eager::BucketStats *>(stats), true, stream);
}

namespace {
int fill_views(eager_ctx *ctx, eager::ViewsArgs &a, int b0, int b1, int n_views,
               float *const *params, float *const *momentum)
{
    if (n_views < 1 || n_views > EAGER_MAX_P)
        return fail(ctx, EAGER_EINVAL, "n_views must be 1..%d", EAGER_MAX_P);
    if (!params) return fail(ctx, EAGER_EINVAL, "params must not be NULL");
    if (int st = check_range(ctx, b0, b1)) return st;
    std::memset(&a, 0, sizeof a);
    for (int p = 0; p < n_views; ++p) {
        if (!params[p] || !aligned16(params[p]) ||
            (momentum && (!momentum[p] || !aligned16(momentum[p]))))
            return fail(ctx, EAGER_EINVAL, "view %d is NULL or not 16-byte aligned", p);
        for (int q = 0; q < p; ++q)
            if (params[q] == params[p] || (momentum && momentum[q] == momentum[p]))
                return fail(ctx, EAGER_EINVAL, "views %d and %d are the same buffer", q, p);
        a.w[p] = params[p];
        a.v[p] = momentum ? momentum[p] : nullptr;
    }
    a.n_views = n_views;
    a.e0 = ctx->offset[b0];
    a.n = ctx->offset[b1 - 1] + ctx->numel[b1 - 1] - ctx->offset[b0];
    return EAGER_OK;
}
}  // namespace

int eager_sgd_step_views(eager_ctx *ctx, int b0, int b1, const float *update, int n_views,
                         float *const *params, float *const *momentum, float lr, float mu,
                         void *stream)
{
    if (!ctx) return EAGER_EINVAL;
    if (!update || !aligned16(update) || !momentum)
        return fail(ctx, EAGER_EINVAL, "update and momentum must not be NULL, update 16-byte aligned");
    eager::ViewsArgs a;
    if (int st = fill_views(ctx, a, b0, b1, n_views, params, momentum)) return st;
    a.u = update;
    a.neg_lr = -lr;
    a.mu = mu;
    a.wd = ctx->weight_decay;
    a.nesterov = ctx->nesterov;
    hipError_t he = eager::launch_views_sgd(a, ctx->fast, ctx->launch, static_cast<hipStream_t>(stream));
    if (he != hipSuccess)
        return fail(ctx, EAGER_EDEVICE, "views kernel launch failed: %s", hipGetErrorString(he));
    ctx->err.clear();
    return EAGER_OK;
}

int eager_average_views(eager_ctx *ctx, int b0, int b1, int n_views, float *const *views,
                        void *stream)
{
    if (!ctx) return EAGER_EINVAL;
    eager::ViewsArgs a;
    if (int st = fill_views(ctx, a, b0, b1, n_views, views, nullptr)) return st;
    a.inv_views = 1.0f / static_cast<float>(n_views);
    hipError_t he = eager::launch_views_average(a, ctx->launch, static_cast<hipStream_t>(stream));
    if (he != hipSuccess)
        return fail(ctx, EAGER_EDEVICE, "views kernel launch failed: %s", hipGetErrorString(he));
    ctx->err.clear();
    return EAGER_OK;
}

int eager_get_valid(const eager_ctx *ctx, int bucket, uint64_t *valid_mask)
{
    if (!ctx || !valid_mask || bucket < 0 || bucket >= ctx->n_buckets) return EAGER_EINVAL;
    *valid_mask = ctx->valid[bucket];
    return EAGER_OK;
}

int eager_set_valid(eager_ctx *ctx, int bucket, uint64_t valid_mask)
{
    if (!ctx) return EAGER_EINVAL;
    if (bucket < 0 || bucket >= ctx->n_buckets) return fail(ctx, EAGER_EINVAL, "bucket %d out of range", bucket);
    if (valid_mask & ~low_bits(ctx->P)) return fail(ctx, EAGER_EINVAL, "validity mask has bits beyond P");
    ctx->valid[bucket] = valid_mask;
    ctx->stepped[bucket] = 0;
    return EAGER_OK;
}

int eager_stats_workspace_bytes(const eager_ctx *ctx, int64_t *bytes)
{
    if (!ctx || !bytes) return EAGER_EINVAL;
    // bucket table, one record per wavefront, (n_buckets + 1) blocks of 64 lane records, one
    // block of partials per bucket
    *bytes = static_cast<int64_t>(ctx->n_buckets) * 16 +
             (max_records(ctx) + (static_cast<int64_t>(ctx->n_buckets) + 1) * 64 +
              static_cast<int64_t>(ctx->n_buckets) * eager::kStatsMaxSlices) *
                 static_cast<int64_t>(sizeof(eager::StatsRecord));
    return EAGER_OK;
}

int eager_stats_attach(eager_ctx *ctx, eager_bucket_stats *stats, void *workspace,
                       int64_t workspace_bytes, void *stream)
{
    static_assert(sizeof(eager_bucket_stats) == sizeof(eager::BucketStats), "layout");
    static_assert(sizeof(eager::StatsRecord) == 32, "layout");
    if (!ctx) return EAGER_EINVAL;
    if (!stats) {                       // detach
        ctx->stats = nullptr;
        ctx->workspace = nullptr;
        return EAGER_OK;
    }
    int64_t need = 0;
    eager_stats_workspace_bytes(ctx, &need);
    if (!workspace || workspace_bytes < need)
        return fail(ctx, EAGER_EINVAL, "statistics workspace must hold %lld bytes",
                    static_cast<long long>(need));
    if (!aligned16(stats) || !aligned16(workspace))
        return fail(ctx, EAGER_EINVAL, "stats and workspace must be 16-byte aligned");
    // written by a small kernel from the kernel arguments: no host-to-device copy, so the call
    // can be captured in a graph like every other
    hipError_t he = eager::launch_table_fill(static_cast<long long *>(workspace), ctx->table.data(),
                                             ctx->n_buckets, static_cast<hipStream_t>(stream));
    if (he != hipSuccess)
        return fail(ctx, EAGER_EDEVICE, "writing the bucket table failed: %s", hipGetErrorString(he));
    ctx->stats = reinterpret_cast<eager::BucketStats *>(stats);
    ctx->workspace = static_cast<char *>(workspace);
    return EAGER_OK;
}

int eager_set_update_rule(eager_ctx *ctx, float weight_decay, int nesterov)
{
    if (!ctx) return EAGER_EINVAL;
    if (!(weight_decay >= 0.0f) || std::isinf(weight_decay))
        return fail(ctx, EAGER_EINVAL, "weight_decay must be finite and >= 0");
    if (nesterov != 0 && nesterov != 1) return fail(ctx, EAGER_EINVAL, "nesterov must be 0 or 1");
    ctx->weight_decay = weight_decay;
    ctx->nesterov = nesterov;
    return EAGER_OK;
}

int eager_set_launch(eager_ctx *ctx, const char *key, int value)
{
    if (!ctx) return EAGER_EINVAL;
    if (!key) return fail(ctx, EAGER_EINVAL, "key is NULL");
    if (!std::strcmp(key, "block")) {
        if (value != 64 && value != 128 && value != 256)
            return fail(ctx, EAGER_EINVAL, "block must be 64, 128 or 256");
        ctx->launch.block = value;
    } else if (!std::strcmp(key, "split")) {
        if (value < 0 || value > 2) return fail(ctx, EAGER_EINVAL, "split must be 0, 1 or 2");
        ctx->launch.split = value;
    } else if (!std::strcmp(key, "chunk")) {
        if (value != 0 && value != 8 && value != 16)
            return fail(ctx, EAGER_EINVAL, "chunk must be 0, 8 or 16");
        ctx->launch.chunk = value;
    } else if (!std::strcmp(key, "blocks_per_cu")) {
        if (value < -1 || value > 32) return fail(ctx, EAGER_EINVAL, "blocks_per_cu must be -1..32");
        ctx->launch.blocks_per_cu = value;
    } else if (!std::strcmp(key, "nt_state")) {
        if (value < -1 || value > 1) return fail(ctx, EAGER_EINVAL, "nt_state must be -1, 0 or 1");
        ctx->launch.nt_state = value;
    } else if (!std::strcmp(key, "xcd_map")) {
        if (value != 0 && value != 1) return fail(ctx, EAGER_EINVAL, "xcd_map must be 0 or 1");
        ctx->launch.xcd_map = value;
    } else if (!std::strcmp(key, "carry_block")) {
        if (value != 64 && value != 128 && value != 256)
            return fail(ctx, EAGER_EINVAL, "carry_block must be 64, 128 or 256");
        ctx->launch.carry_block = value;
    } else if (!std::strcmp(key, "carry_vec")) {
        if (value != 1 && value != 2 && value != 4)
            return fail(ctx, EAGER_EINVAL, "carry_vec must be 1, 2 or 4");
        ctx->launch.carry_vec = value;
    } else if (!std::strcmp(key, "carry_blocks_per_cu")) {
        if (value < -1 || value == 0 || value > 32)
            return fail(ctx, EAGER_EINVAL, "carry_blocks_per_cu must be -1 or 1..32");
        ctx->launch.carry_blocks_per_cu = value;
    } else if (!std::strcmp(key, "round_stats")) {
        if (value != 0 && value != 1) return fail(ctx, EAGER_EINVAL, "round_stats must be 0 or 1");
        ctx->launch.round_stats = value;
    } else {
        return fail(ctx, EAGER_EINVAL, "unknown launch key '%s'", key);
    }
    return EAGER_OK;
}

int eager_calib_copy(void *dst, const void *src, int64_t nbytes, void *stream)
{
    if (!dst || !src || nbytes < 0 || nbytes % 16 || !aligned16(dst) || !aligned16(src))
        return EAGER_EINVAL;
    return eager::launch_copy(dst, src, nbytes, static_cast<hipStream_t>(stream)) == hipSuccess
               ? EAGER_OK : EAGER_EDEVICE;
}

int eager_calib_read(const void *src, int64_t nbytes, float *sink, void *stream)
{
    if (!src || !sink || nbytes < 0 || nbytes % 16 || !aligned16(src)) return EAGER_EINVAL;
    return eager::launch_read(src, nbytes, sink, static_cast<hipStream_t>(stream)) == hipSuccess
               ? EAGER_OK : EAGER_EDEVICE;
}

int eager_calib_mix(const void *const *read, int n_read, uint64_t read_half_mask,
                    void *const *write, int n_write, int64_t n_vec, int waves_per_cu, float *sink,
                    void *stream)
{
    if (!read || n_read < 1 || n_read > eager::kMixMaxRead || n_write < 0 ||
        n_write > eager::kMixMaxWrite || (n_write > 0 && !write) || (n_write == 0 && !sink) ||
        n_vec < 0 || waves_per_cu < 0 || waves_per_cu > 32)
        return EAGER_EINVAL;
    if (read_half_mask && (n_vec & 1)) return EAGER_EINVAL;
    if (n_read < 64 && (read_half_mask >> n_read)) return EAGER_EINVAL;
    eager::MixArgs a;
    std::memset(&a, 0, sizeof a);
    for (int j = 0; j < n_read; ++j) {
        if (!read[j] || !aligned16(read[j])) return EAGER_EINVAL;
        a.src[j] = read[j];
    }
    for (int j = 0; j < n_write; ++j) {
        if (!write[j] || !aligned16(write[j])) return EAGER_EINVAL;
        a.dst[j] = write[j];
    }
    a.half = read_half_mask;
    a.sink = sink;
    a.n_read = n_read;
    a.n_write = n_write;
    a.nvec = n_vec;
    return eager::launch_mix(a, waves_per_cu, static_cast<hipStream_t>(stream)) == hipSuccess
               ? EAGER_OK : EAGER_EDEVICE;
}

}  // extern "C"
