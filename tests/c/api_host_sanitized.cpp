// The host side of the library (eager_api.cpp: context state, validation, how a bucket range
// is cut into runs = launches, which form a round takes) compiled WITHOUT the kernels and run
// under AddressSanitizer and UndefinedBehaviorSanitizer on the CPU.  The launchers and the one
// HIP runtime call the host side uses are replaced by recorders, so every launch the host
// side would make is checked for its element range, masks and order, and nothing needs a
// GPU.  Built and run by tests/test_host_library.py.
#include "../../include/eager_tuning.h"
#include "../../paper_1908_04207_amd/csrc/eager_internal.h"

#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

struct Launched {
    std::string kind;
    long long e0 = 0, n = 0;
    unsigned long long active = 0, valid = 0, gload = 0, store = 0;
    int count = 0;          // carry: pairs; views: views; finish: slices; stash: accumulate
    int b_lo = 0, b_hi = 0;
    bool has_w = false, has_recv = false, has_stats = false;
};
static std::vector<Launched> g_log;
static int g_fail_round = -1;       // the round launch with this index in g_log reports a failure

extern "C" const char *hipGetErrorString(hipError_t) { return "stub"; }

namespace eager {
hipError_t launch_round(const RoundArgs &a, bool, bool, const Launch &, hipStream_t)
{
    Launched l;
    l.kind = "round";
    l.e0 = a.e0; l.n = a.n; l.active = a.active; l.valid = a.valid; l.gload = a.gload; l.store = a.store;
    l.has_w = a.w != nullptr; l.has_recv = a.recv != nullptr; l.has_stats = a.stats.stats != nullptr;
    if (static_cast<int>(g_log.size()) == g_fail_round) return hipErrorLaunchFailure;
    g_log.push_back(l);
    return hipSuccess;
}
hipError_t launch_carry(const CarryArgs &a, bool, const Launch &, hipStream_t)
{
    Launched l;
    l.kind = "carry";
    l.e0 = a.e0; l.n = a.n; l.count = a.count;
    g_log.push_back(l);
    return hipSuccess;
}
hipError_t launch_stats_finish(const StatsArgs &a, hipStream_t)
{
    Launched l;
    l.kind = "finish";
    l.e0 = a.e0; l.b_lo = a.b_lo; l.b_hi = a.b_hi; l.count = a.slices;
    g_log.push_back(l);
    return hipSuccess;
}
long long slot_records(long long n, bool, int) { return n / 256 + 1; }
int slot_tail(long long n, bool bf16) { return static_cast<int>(n % (bf16 ? 8 : 4)); }
hipError_t launch_stash(const StashArgs &a, bool, hipStream_t)
{
    Launched l;
    l.kind = "stash";
    l.e0 = a.e0; l.n = a.n; l.count = a.accumulate;
    g_log.push_back(l);
    return hipSuccess;
}
static hipError_t views(const char *kind, const ViewsArgs &a)
{
    Launched l;
    l.kind = kind;
    l.e0 = a.e0; l.n = a.n; l.count = a.n_views;
    g_log.push_back(l);
    return hipSuccess;
}
hipError_t launch_views_sgd(const ViewsArgs &a, bool, const Launch &, hipStream_t) { return views("views_sgd", a); }
hipError_t launch_views_average(const ViewsArgs &a, const Launch &, hipStream_t) { return views("views_avg", a); }
static hipError_t sgd(const char *kind, const SgdArgs &a)
{
    Launched l;
    l.kind = kind;
    l.e0 = a.e0; l.n = a.n;
    g_log.push_back(l);
    return hipSuccess;
}
hipError_t launch_sgd(const SgdArgs &a, bool, const Launch &, hipStream_t) { return sgd("sgd", a); }
hipError_t launch_norms(const SgdArgs &a, const StatsArgs &, hipStream_t) { return sgd("norms", a); }
hipError_t launch_sgd_lars(const SgdArgs &a, const StatsArgs &, bool, hipStream_t) { return sgd("lars", a); }
long long norms_records(long long n) { return n / 256 + 4; }
static char g_scratch[64];
hipError_t static_scratch(char **ptr) { *ptr = g_scratch; return hipSuccess; }
hipError_t launch_table_fill(long long *table, const long long *start_end, int n_buckets, hipStream_t)
{
    Launched l;
    l.kind = "table";
    l.count = n_buckets;
    // the host copy of the table is read here, under the sanitizers
    for (int i = 0; i < 2 * n_buckets; ++i) l.n += start_end[i];
    l.has_w = reinterpret_cast<char *>(table) == g_scratch;
    g_log.push_back(l);
    return hipSuccess;
}
hipError_t launch_copy(void *, const void *, long long, hipStream_t) { return hipSuccess; }
hipError_t launch_read(const void *, long long, float *, hipStream_t) { return hipSuccess; }
hipError_t launch_mix(const MixArgs &a, int, hipStream_t)
{
    Launched l;
    l.kind = "mix";
    l.n = a.nvec; l.count = a.n_read; l.b_hi = a.n_write; l.active = a.half;
    g_log.push_back(l);
    return hipSuccess;
}
}  // namespace eager

#define CHECK(cond)                                                              \
    do {                                                                         \
        if (!(cond)) {                                                           \
            std::printf("line %d: %s\n", __LINE__, #cond);                       \
            return 1;                                                            \
        }                                                                        \
    } while (0)

static eager_plan plan_of(int mode, int P, uint64_t step, uint64_t mask, int initiator)
{
    eager_plan p;
    p.mode = mode; p.P = P; p.step = step; p.mask = mask; p.initiator = initiator;
    p.nap = __builtin_popcountll(mask);
    p.flags = 0;
    p.reserved = 0;
    return p;
}

int main()
{
    const int P = 4, NB = 4;
    const int64_t off[NB] = {0, 8, 16, 1024}, num[NB] = {5, 8, 1000, 40};
    const long long whole = 1024 + 40;
    eager_ctx *ctx = nullptr;
    CHECK(eager_create(&ctx, P, NB, off, num, EAGER_F32, EAGER_ORDER_FIXED) == EAGER_OK);
    // fake, aligned device addresses: the recorders never touch them
    const void *G[P];
    float *R[P];
    for (int p = 0; p < P; ++p) {
        G[p] = reinterpret_cast<const void *>(0x100000ull * (p + 1));
        R[p] = reinterpret_cast<float *>(0x1000000ull * (p + 1));
    }
    float *w = reinterpret_cast<float *>(0x20000000ull), *v = reinterpret_cast<float *>(0x30000000ull);
    float *recv = reinterpret_cast<float *>(0x40000000ull);
    const eager_opt opt = {w, v, 0.1f, 0.9f};
    uint64_t valid = 99;

    // a fused round over the whole model: ONE launch, late processes stored in the same pass
    eager_plan p0 = plan_of(EAGER_SOLO, P, 0, 0b0011, 0);
    CHECK(eager_partial_allreduce_solo(ctx, &p0, 0, NB, G, R, nullptr, &opt, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 1 && g_log[0].kind == "round" && g_log[0].e0 == 0 && g_log[0].n == whole);
    CHECK(g_log[0].active == 0b0011 && g_log[0].valid == 0 && g_log[0].store == 0b1100 &&
          g_log[0].gload == 0b1111 && g_log[0].has_w && !g_log[0].has_recv && !g_log[0].has_stats);
    for (int b = 0; b < NB; ++b) CHECK(eager_get_valid(ctx, b, &valid) == EAGER_OK && valid == 0b1100);
    // the same round again is refused and launches nothing
    CHECK(eager_partial_allreduce_solo(ctx, &p0, 0, NB, G, R, nullptr, &opt, nullptr) == EAGER_ESTATE);
    CHECK(g_log.size() == 1 && std::string(eager_last_error(ctx)).find("already") != std::string::npos);

    // a majority plan made under the strict reading needs its quorum at the entry point too
    {
        eager_plan strict = plan_of(EAGER_MAJORITY, P, 77, 0b0001, 0);
        strict.flags = EAGER_FLAG_STRICT_QUORUM;
        CHECK(eager_partial_allreduce_majority(ctx, &strict, 0, NB, G, R, nullptr, &opt, nullptr) == EAGER_ESTATE);
        CHECK(std::string(eager_last_error(ctx)).find("strict majority") != std::string::npos);
        strict.flags = 2u;
        CHECK(eager_partial_allreduce_majority(ctx, &strict, 0, NB, G, R, nullptr, &opt, nullptr) == EAGER_ESTATE);
        CHECK(g_log.size() == 1);
        const double t4[4] = {4.0, 1.0, 3.0, 2.0};
        eager_plan made;
        CHECK(eager_plan_participation(EAGER_MAJORITY, P, t4, 5u, 0u, 0.0, EAGER_FLAG_STRICT_QUORUM, &made) == EAGER_OK);
        CHECK(made.flags == EAGER_FLAG_STRICT_QUORUM && made.nap >= 2 && made.reserved == 0);
        CHECK(eager_plan_participation(EAGER_SOLO, P, t4, 5u, 0u, 0.0, EAGER_FLAG_STRICT_QUORUM, &made) == EAGER_OK);
        CHECK(made.flags == 0);
        CHECK(eager_plan_participation(EAGER_MAJORITY, P, t4, 5u, 0u, 0.0, 4u, &made) == EAGER_EINVAL);
    }

    // buckets in different send-buffer states: one launch per run of equal state
    g_log.clear();
    CHECK(eager_set_valid(ctx, 1, 0b0100) == EAGER_OK);
    eager_plan p1 = plan_of(EAGER_MAJORITY, P, 1, 0b1111, 2);
    CHECK(eager_partial_allreduce_majority(ctx, &p1, 0, NB, G, R, recv, &opt, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 3);
    CHECK(g_log[0].e0 == 0 && g_log[0].n == 5 && g_log[0].valid == 0b1100);
    CHECK(g_log[1].e0 == 8 && g_log[1].n == 8 && g_log[1].valid == 0b0100);
    CHECK(g_log[2].e0 == 16 && g_log[2].n == whole - 16 && g_log[2].valid == 0b1100 && g_log[2].store == 0 &&
          g_log[2].has_recv);
    for (int b = 0; b < NB; ++b) CHECK(eager_get_valid(ctx, b, &valid) == EAGER_OK && valid == 0);

    // a launch that the runtime refuses in the middle of a call: EDEVICE; the runs enqueued before
    // it stay stepped (documented: the range is in an undefined state), and setting the validity
    // again makes the buckets usable
    {
        g_log.clear();
        CHECK(eager_set_valid(ctx, 1, 0b0100) == EAGER_OK);
        g_fail_round = 1;
        eager_plan pf = plan_of(EAGER_SOLO, P, 40, 0b0001, 0);
        CHECK(eager_partial_allreduce_solo(ctx, &pf, 0, NB, G, R, nullptr, &opt, nullptr) == EAGER_EDEVICE);
        g_fail_round = -1;
        CHECK(g_log.size() == 1 && g_log[0].e0 == 0 && g_log[0].n == 5);
        CHECK(std::string(eager_last_error(ctx)).find("launch failed") != std::string::npos);
        CHECK(eager_partial_allreduce_solo(ctx, &pf, 0, NB, G, R, nullptr, &opt, nullptr) == EAGER_ESTATE);
        for (int b = 0; b < NB; ++b) CHECK(eager_set_valid(ctx, b, 0) == EAGER_OK);
        CHECK(eager_partial_allreduce_solo(ctx, &pf, 0, NB, G, R, nullptr, &opt, nullptr) == EAGER_OK);
        for (int b = 0; b < NB; ++b) CHECK(eager_set_valid(ctx, b, 0) == EAGER_OK);
    }

    // the split form: the reduction reads only the on-time gradients, a copy kernel follows
    g_log.clear();
    CHECK(eager_set_launch(ctx, "split", 2) == EAGER_OK);
    eager_plan p2 = plan_of(EAGER_QUORUM, P, 2, 0b0110, 1);
    CHECK(eager_partial_allreduce_quorum(ctx, &p2, 1, 3, G, R, nullptr, &opt, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 2 && g_log[0].kind == "round" && g_log[0].gload == 0b0110 && g_log[0].store == 0 &&
          g_log[0].e0 == 8 && g_log[0].n == 1008);
    CHECK(g_log[1].kind == "carry" && g_log[1].count == 2 && g_log[1].e0 == 8 && g_log[1].n == 1008);
    CHECK(eager_get_valid(ctx, 0, &valid) == EAGER_OK && valid == 0);
    CHECK(eager_get_valid(ctx, 2, &valid) == EAGER_OK && valid == 0b1001);
    CHECK(eager_set_launch(ctx, "split", 0) == EAGER_OK);

    // processes that finish nothing in the round's window store nothing and stay pending
    g_log.clear();
    const void *G_absent[P] = {G[0], G[1], G[2], nullptr};
    eager_plan p3 = plan_of(EAGER_SOLO, P, 3, 0b0010, 1);
    CHECK(eager_partial_allreduce_lagging(ctx, &p3, 0b1000, 1, 3, G_absent, R, nullptr, &opt, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 1 && g_log[0].store == 0b0101 && g_log[0].gload == 0b0111 && g_log[0].valid == 0b1001);
    CHECK(eager_get_valid(ctx, 1, &valid) == EAGER_OK && valid == 0b0101);
    CHECK(eager_partial_allreduce_lagging(ctx, &p3, 0b0010, 0, 1, G, R, nullptr, &opt, nullptr) == EAGER_ESTATE);

    // the gradient buffer of a late process becomes its send buffer: the reduction alone (it reads
    // only the on-time gradients), no copy kernel, the two table entries exchanged
    {
        g_log.clear();
        const void *Gx[P] = {G[0], G[1], G[2], G[3]};
        float *Rx[P] = {R[0], R[1], R[2], R[3]};
        uint64_t before[NB];
        for (int b = 0; b < NB; ++b) CHECK(eager_get_valid(ctx, b, &before[b]) == EAGER_OK);
        eager_plan px = plan_of(EAGER_MAJORITY, P, 30, 0b0101, 2);
        CHECK(eager_partial_allreduce_exchange(ctx, &px, Gx, Rx, nullptr, &opt, nullptr) == EAGER_OK);
        for (const Launched &l : g_log) CHECK(l.kind == "round" && l.gload == 0b0101 && l.store == 0);
        CHECK(!g_log.empty() && g_log.front().e0 == 0 && g_log.back().e0 + g_log.back().n == whole);
        CHECK(Gx[0] == G[0] && Rx[0] == R[0] && Gx[2] == G[2] && Rx[2] == R[2]);
        CHECK(Gx[1] == R[1] && Rx[1] == G[1] && Gx[3] == R[3] && Rx[3] == G[3]);
        for (int b = 0; b < NB; ++b) CHECK(eager_get_valid(ctx, b, &valid) == EAGER_OK && valid == 0b1010);
        // refused calls leave the tables alone
        CHECK(eager_partial_allreduce_exchange(ctx, &px, Gx, Rx, nullptr, &opt, nullptr) == EAGER_ESTATE);
        CHECK(Gx[1] == R[1] && Rx[1] == G[1]);
        // back to the state the following checks expect
        for (int b = 0; b < NB; ++b) CHECK(eager_set_valid(ctx, b, before[b]) == EAGER_OK);
    }

    // the flush: nobody active, everybody absent, no gradient table; validity cleared, and the
    // same round index may be used again afterwards
    {
        g_log.clear();
        uint64_t before[NB];
        for (int b = 0; b < NB; ++b) CHECK(eager_get_valid(ctx, b, &before[b]) == EAGER_OK);
        CHECK(eager_flush(ctx, 1, 3, R, recv, &opt, nullptr) == EAGER_OK);
        for (const Launched &l : g_log) CHECK(l.kind == "round" && l.active == 0 && l.gload == 0 && l.store == 0);
        CHECK(!g_log.empty() && g_log.front().e0 == 8 && g_log.back().e0 + g_log.back().n == 1016);
        CHECK(eager_get_valid(ctx, 1, &valid) == EAGER_OK && valid == 0);
        CHECK(eager_get_valid(ctx, 0, &valid) == EAGER_OK && valid == before[0]);
        CHECK(eager_flush(ctx, 1, 3, R, nullptr, nullptr, nullptr) == EAGER_EINVAL);
        CHECK(eager_flush(ctx, 1, 3, nullptr, recv, &opt, nullptr) == EAGER_EINVAL);
        for (int b = 0; b < NB; ++b) CHECK(eager_set_valid(ctx, b, before[b]) == EAGER_OK);
    }

    // a stash runs per stretch of buckets in which the process's buffer is in the same state
    g_log.clear();
    CHECK(eager_stash(ctx, 0, 0, NB, G[0], R[0], nullptr) == EAGER_OK);     // bit 0: 0, 1, 1, 0
    CHECK(g_log.size() == 3 && g_log[0].count == 0 && g_log[0].e0 == 0 && g_log[0].n == 5);
    CHECK(g_log[1].count == 1 && g_log[1].e0 == 8 && g_log[1].n == 1008);
    CHECK(g_log[2].count == 0 && g_log[2].e0 == 1024 && g_log[2].n == 40);
    for (int b = 0; b < NB; ++b) CHECK(eager_get_valid(ctx, b, &valid) == EAGER_OK && (valid & 1));
    CHECK(eager_stash(ctx, P, 0, NB, G[0], R[0], nullptr) == EAGER_EINVAL);

    // update rule on a receive buffer, on views, the average
    g_log.clear();
    float *views_w[3] = {w, w + 4096, w + 8192}, *views_v[3] = {v, v + 4096, v + 8192};
    CHECK(eager_sgd_step(ctx, 2, 4, recv, &opt, nullptr) == EAGER_OK);
    CHECK(eager_sgd_step_views(ctx, 0, NB, recv, 3, views_w, views_v, 0.1f, 0.9f, nullptr) == EAGER_OK);
    CHECK(eager_average_views(ctx, 0, 2, 3, views_w, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 3 && g_log[0].kind == "sgd" && g_log[0].e0 == 16 && g_log[0].n == whole - 16);
    CHECK(g_log[1].kind == "views_sgd" && g_log[1].count == 3 && g_log[1].n == whole);
    CHECK(g_log[2].kind == "views_avg" && g_log[2].n == 16);
    float *twice[2] = {w, w};
    CHECK(eager_average_views(ctx, 0, 2, 2, twice, nullptr) == EAGER_EINVAL);
    CHECK(eager_sgd_step_views(ctx, 0, NB, recv, 65, views_w, views_v, 0.1f, 0.9f, nullptr) == EAGER_EINVAL);

    // statistics: the workspace must be large enough; attached, a round is followed by the
    // finishing step and the layer-wise rule is norms, finish, update
    g_log.clear();
    int64_t need = 0;
    CHECK(eager_stats_workspace_bytes(ctx, &need) == EAGER_OK && need > 0);
    eager_bucket_stats *stats = reinterpret_cast<eager_bucket_stats *>(0x50000000ull);
    void *ws = reinterpret_cast<void *>(0x60000000ull);
    CHECK(eager_sgd_step_lars(ctx, 0, NB, recv, &opt, 0.02f, 0.0f, nullptr) == EAGER_ESTATE);
    CHECK(eager_stats_attach(ctx, stats, ws, need - 1, nullptr) == EAGER_EINVAL);
    CHECK(eager_stats_attach(ctx, stats, ws, need, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 1 && g_log[0].kind == "table" && g_log[0].count == NB && !g_log[0].has_w);
    g_log.clear();
    for (int b = 0; b < NB; ++b) CHECK(eager_set_valid(ctx, b, 0) == EAGER_OK);
    eager_plan p4 = plan_of(EAGER_SOLO, P, 4, 0b1111, 0);
    CHECK(eager_partial_allreduce_solo(ctx, &p4, 0, NB, G, R, recv, nullptr, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 2 && g_log[0].kind == "round" && g_log[0].has_stats && g_log[1].kind == "finish" &&
          g_log[1].b_lo == 0 && g_log[1].b_hi == NB && g_log[1].count == 1);
    g_log.clear();
    CHECK(eager_sgd_step_lars(ctx, 1, 3, recv, &opt, 0.02f, 1e-9f, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 3 && g_log[0].kind == "norms" && g_log[1].kind == "finish" && g_log[2].kind == "lars");
    CHECK(g_log[0].e0 == 8 && g_log[0].n == 1008 && g_log[1].b_lo == 1 && g_log[1].b_hi == 3 && g_log[2].n == 1008);
    CHECK(eager_sgd_step_lars(ctx, 1, 3, recv, &opt, -1.0f, 0.0f, nullptr) == EAGER_EINVAL);
    // the same rule with the library's fixed scratch as workspace: the bucket table is written by
    // a kernel first, nothing needs to be attached, and the attached workspace is left alone
    g_log.clear();
    CHECK(eager_sgd_step_lars_static(ctx, 1, 3, recv, &opt, 0.02f, 1e-9f, stats, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 4 && g_log[0].kind == "table" && g_log[0].count == NB && g_log[0].has_w &&
          g_log[0].n == 0 + 5 + 8 + 16 + 16 + 1016 + 1024 + 1064);
    CHECK(g_log[1].kind == "norms" && g_log[2].kind == "finish" && g_log[3].kind == "lars" && g_log[3].n == 1008);
    CHECK(eager_sgd_step_lars_static(ctx, 1, 3, recv, &opt, 0.02f, 1e-9f, nullptr, nullptr) == EAGER_EINVAL);
    CHECK(eager_sgd_step_lars_static(ctx, 3, 1, recv, &opt, 0.02f, 1e-9f, stats, nullptr) == EAGER_EINVAL);
    CHECK(g_log.size() == 4);
    // by-products switched off for rounds: the round alone
    g_log.clear();
    CHECK(eager_set_launch(ctx, "round_stats", 0) == EAGER_OK);
    eager_plan p5 = plan_of(EAGER_SOLO, P, 5, 0b1111, 0);
    CHECK(eager_partial_allreduce_solo(ctx, &p5, 0, NB, G, R, recv, nullptr, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 1 && !g_log[0].has_stats);
    CHECK(eager_stats_attach(ctx, nullptr, nullptr, 0, nullptr) == EAGER_OK);
    CHECK(eager_destroy(ctx) == EAGER_OK);

    // a model with one bucket of 2^31 elements: many records, so the finishing step is sliced;
    // nothing is allocated per element on the host
    const int64_t big_off[1] = {0}, big_num[1] = {int64_t{1} << 31};
    CHECK(eager_create(&ctx, 2, 1, big_off, big_num, EAGER_BF16, EAGER_ORDER_FAST) == EAGER_OK);
    CHECK(eager_stats_workspace_bytes(ctx, &need) == EAGER_OK && need > (int64_t{1} << 31) / 256 * 32);
    CHECK(eager_stats_attach(ctx, stats, ws, need, nullptr) == EAGER_OK);
    g_log.clear();
    eager_plan p6 = plan_of(EAGER_MAJORITY, 2, 0, 0b01, 0);
    CHECK(eager_partial_allreduce_majority(ctx, &p6, 0, 1, G, R, nullptr, &opt, nullptr) == EAGER_OK);
    CHECK(g_log.size() == 2 && g_log[1].kind == "finish" && g_log[1].count == eager::kStatsMaxSlices);
    // beyond the capacity of the fixed scratch: refused, nothing launched
    g_log.clear();
    CHECK(eager_sgd_step_lars_static(ctx, 0, 1, recv, &opt, 0.02f, 0.0f, stats, nullptr) == EAGER_ELIMIT);
    CHECK(g_log.empty() && std::string(eager_last_error(ctx)).find("fixed scratch") != std::string::npos);
    CHECK(eager_destroy(ctx) == EAGER_OK);
    {
        std::vector<int64_t> many_off(EAGER_STATIC_MAX_BUCKETS + 1), many_num(EAGER_STATIC_MAX_BUCKETS + 1, 4);
        for (size_t b = 0; b < many_off.size(); ++b) many_off[b] = 4 * static_cast<int64_t>(b);
        CHECK(eager_create(&ctx, 2, EAGER_STATIC_MAX_BUCKETS + 1, many_off.data(), many_num.data(), EAGER_F32,
                           EAGER_ORDER_FIXED) == EAGER_OK);
        CHECK(eager_sgd_step_lars_static(ctx, 0, 1, recv, &opt, 0.02f, 0.0f, stats, nullptr) == EAGER_ELIMIT);
        CHECK(eager_destroy(ctx) == EAGER_OK);
        CHECK(eager_create(&ctx, 2, EAGER_STATIC_MAX_BUCKETS, many_off.data(), many_num.data(), EAGER_F32,
                           EAGER_ORDER_FIXED) == EAGER_OK);
        CHECK(eager_sgd_step_lars_static(ctx, 0, EAGER_STATIC_MAX_BUCKETS, recv, &opt, 0.02f, 0.0f, stats, nullptr) ==
              EAGER_OK);
        CHECK(g_log.size() == 4 && g_log[0].count == EAGER_STATIC_MAX_BUCKETS);
        CHECK(eager_destroy(ctx) == EAGER_OK);
    }

    // the calibration kernel checks its stream tables before it launches
    {
        g_log.clear();
        const void *rd[3] = {G[0], G[1], G[2]};
        void *wr[2] = {R[0], R[1]};
        CHECK(eager_calib_mix(rd, 3, 0b100, wr, 2, 1024, 4, nullptr, nullptr) == EAGER_OK);
        CHECK(g_log.size() == 1 && g_log[0].kind == "mix" && g_log[0].count == 3 && g_log[0].b_hi == 2 &&
              g_log[0].active == 0b100 && g_log[0].n == 1024);
        CHECK(eager_calib_mix(rd, 3, 0b1000, wr, 2, 1024, 4, nullptr, nullptr) == EAGER_EINVAL);   // mask beyond n_read
        CHECK(eager_calib_mix(rd, 3, 0b001, wr, 2, 1023, 4, nullptr, nullptr) == EAGER_EINVAL);    // odd with half-width
        CHECK(eager_calib_mix(rd, 3, 0, wr, 0, 1024, 4, nullptr, nullptr) == EAGER_EINVAL);        // no sink
        CHECK(eager_calib_mix(rd, 81, 0, wr, 2, 1024, 4, nullptr, nullptr) == EAGER_EINVAL);
        CHECK(eager_calib_mix(rd, 3, 0, wr, 2, 1024, 33, nullptr, nullptr) == EAGER_EINVAL);
        rd[1] = nullptr;
        CHECK(eager_calib_mix(rd, 3, 0, wr, 2, 1024, 4, nullptr, nullptr) == EAGER_EINVAL);
        CHECK(g_log.size() == 1);
    }

    // creation errors leave nothing behind
    const int64_t bad_off[2] = {0, 2}, bad_num[2] = {2, 4};
    ctx = nullptr;
    CHECK(eager_create(&ctx, 2, 2, bad_off, bad_num, EAGER_F32, EAGER_ORDER_FIXED) == EAGER_ESHAPE && ctx == nullptr);
    CHECK(eager_create(&ctx, 0, 2, off, num, EAGER_F32, EAGER_ORDER_FIXED) == EAGER_EINVAL);
    std::printf("ok\n");
    return 0;
}
