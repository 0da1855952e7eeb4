// gfx950 kernels around the round: the second stage of the per-bucket statistics, the update
// rule alone on a receive buffer (plain, or with a layer-wise rate per bucket: norms pass, rate,
// update pass), and what processes that lag by more than one round need - a late gradient
// stashed into a send buffer, the update of several weight views from one read of the result, the
// model average (paper Section 5, last paragraph).  All of them are HBM streams: a lane owns 4 consecutive elements, 64-thread
// workgroups, nontemporal accesses, occupancy chosen for the bytes in flight.
#include "eager_device.h"

namespace eager {
namespace {

// Adds the plain records (one per wavefront whose elements all lie in one bucket) with index in
// [lo, hi) that belong to bucket b: 8 independent loads per thread in flight, wavefront sums by
// DPP, the 4 wavefronts of the workgroup through LDS.  The totals arrive in thread 0.
__device__ __forceinline__ void add_records(const StatsRecord *records, long long lo, long long hi,
                                            int b, double &su, double &sw, double &nf)
{
    constexpr int K = 8;
    for (long long wb = lo + threadIdx.x; wb < hi; wb += static_cast<long long>(blockDim.x) * K) {
        StatsRecord r[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const long long w = wb + static_cast<long long>(k) * blockDim.x;
            if (w < hi) r[k] = records[w];
            else r[k].bucket = -2;
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            if (r[k].bucket == b) {
                su += r[k].ssu;
                sw += r[k].ssw;
                nf += r[k].nf;
            }
        }
    }
}

// (the count travels as a double: integers below 2^53 add exactly, and a 32-bit sum could
// overflow on a bucket of billions of elements)
__device__ __forceinline__ void workgroup_sum(double &su, double &sw, double &nf)
{
    __shared__ double part_u[4], part_w[4], part_n[4];
    su = wave_sum(su);
    sw = wave_sum(sw);
    nf = wave_sum(nf);
    const unsigned wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63u) == 0u) {
        part_u[wave] = su;
        part_w[wave] = sw;
        part_n[wave] = nf;
    }
    __syncthreads();
    su = (part_u[0] + part_u[1]) + (part_u[2] + part_u[3]);
    sw = (part_w[0] + part_w[1]) + (part_w[2] + part_w[3]);
    nf = (part_n[0] + part_n[1]) + (part_n[2] + part_n[3]);
}

// records of bucket b: [w0, w1)
__device__ __forceinline__ void bucket_records(const StatsArgs &a, int b, long long &w0, long long &w1)
{
    const long long start = a.table[2 * b], end = a.table[2 * b + 1];
    w0 = (start - a.e0) / 256;
    w1 = (end - a.e0 + 255) / 256;
    if (w1 > a.n_records) w1 = a.n_records;
}

// First stage for buckets with many records (a flat model is ONE bucket: millions of records):
// workgroup (bucket, slice) adds one slice of the bucket's plain records and leaves a partial.
__global__ __launch_bounds__(256) void stats_slice_kernel(const StatsArgs a)
{
    const int b = a.b_lo + static_cast<int>(blockIdx.x);
    const int s = static_cast<int>(blockIdx.y);
    long long w0, w1;
    bucket_records(a, b, w0, w1);
    const long long len = (w1 - w0 + a.slices - 1) / a.slices;
    const long long lo = w0 + s * len, hi = lo + len < w1 ? lo + len : w1;
    double su = 0.0, sw = 0.0, nf = 0.0;
    add_records(a.records, lo, hi, b, su, sw, nf);
    workgroup_sum(su, sw, nf);
    if (threadIdx.x == 0) {
        // a slice holds at most 2^33 / 256 / slices records of 256 elements: the count fits
        const StatsRecord out = {su, sw, b, static_cast<unsigned>(nf), 0};
        a.partials[static_cast<long long>(b) * kStatsMaxSlices + s] = out;
    }
}

// One workgroup per bucket of the run: adds the records of the wavefronts whose 256 elements
// touch the bucket (they are consecutive) - a uniform wavefront's sums (or the partials of the
// first stage), a mixed wavefront's lane records of this bucket - and the records of the ragged
// tail; one thread writes the bucket's totals.
__global__ __launch_bounds__(256) void stats_finish_kernel(const StatsArgs a)
{
    const int b = a.b_lo + static_cast<int>(blockIdx.x);
    long long w0, w1;
    bucket_records(a, b, w0, w1);
    double su = 0.0, sw = 0.0, nf = 0.0;
    if (a.slices > 1) {
        if (static_cast<int>(threadIdx.x) < a.slices) {
            const StatsRecord r = a.partials[static_cast<long long>(b) * kStatsMaxSlices + threadIdx.x];
            su = r.ssu;
            sw = r.ssw;
            nf = r.nf;
        }
    } else {
        add_records(a.records, w0, w1, b, su, sw, nf);
    }
    // Only the first and the last wavefront of the bucket can be mixed: wavefront 0 of this
    // workgroup takes the lane records of the first, wavefront 1 those of the last, one lane
    // each; wavefront 2 takes the ragged tail.
    const unsigned which = threadIdx.x >> 6, lane = threadIdx.x & 63u;
    if (which < 2 && w1 > w0 && (which == 0 || w1 - 1 != w0)) {
        const StatsRecord r = a.records[which == 0 ? w0 : w1 - 1];
        if (r.bucket == -1) {
            const StatsRecord lr = a.lane_records[static_cast<long long>(r.nf) * 64 + lane];
            if (lr.bucket == b) {
                su += lr.ssu;
                sw += lr.ssw;
                nf += lr.nf;
            }
        }
    }
    if (which == 2 && static_cast<int>(lane) < a.tail_count) {
        const StatsRecord tr = a.lane_records[static_cast<long long>(a.n_buckets) * 64 + lane];
        if (tr.bucket == b) {
            su += tr.ssu;
            sw += tr.ssw;
            nf += tr.nf;
        }
    }
    workgroup_sum(su, sw, nf);
    if (threadIdx.x == 0) {
        BucketStats out;
        out.sumsq_update = su;
        out.sumsq_params = sw;
        out.nonfinite = static_cast<unsigned long long>(nf);
        out.rate = 0.0f;
        if (a.want_rate) {
            // fp64 square roots and division, one rounding to fp32 at the end
            const double nu = __builtin_sqrt(out.sumsq_update), nw = __builtin_sqrt(out.sumsq_params);
            out.rate = (nu > 0.0 && nw > 0.0)
                           ? static_cast<float>(static_cast<double>(a.trust) * nw /
                                                (nu + static_cast<double>(a.wd) * nw +
                                                 static_cast<double>(a.eps)))
                           : 1.0f;
        }
        out.reserved = 0u;
        a.stats[b] = out;
    }
}

// A late gradient outside a round (a process that lags by more than one round, last
// paragraph of Section 5): R <- G, or R <- R + G if the send buffer still holds an
// undelivered gradient.  A plain stream, a lane owns 4 elements.
// STRIDE: the grid does not cover the range and every lane loops.  Where it does cover it the
// body stands alone: a wavefront then ends right after its store instead of reaching a loop
// end first, and such short-lived wavefronts are measurably faster that way.
template <bool BF16, bool STRIDE>
__global__ __launch_bounds__(64) void stash_kernel(const StashArgs a)
{
    const long long nvec = a.n / 4;
    const char *src = static_cast<const char *>(a.g);
    auto body = [&](long long vi) {
        const long long e = a.e0 + vi * 4;
        f32x4 x;
        if (BF16) {
            const u32x2 g = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(src + e * 2));
            x.x = __uint_as_float(g.x << 16);
            x.y = __uint_as_float(g.x & 0xffff0000u);
            x.z = __uint_as_float(g.y << 16);
            x.w = __uint_as_float(g.y & 0xffff0000u);
        } else {
            x = ld_f4<true>(reinterpret_cast<const float *>(src + e * 4));
        }
        if (a.accumulate) x = ld_f4<true>(a.r + e) + x;
        st_f4<true>(a.r + e, x);
    };
    const long long first = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if constexpr (STRIDE) {
        const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
        for (long long vi = first; vi < nvec; vi += stride) body(vi);
    } else {
        if (first < nvec) body(first);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        const float g = load_grad_scalar<BF16>(src, i);
        a.r[i] = a.accumulate ? a.r[i] + g : g;
    }
}

// ---------------------------------------------------------------------------------------
// Weight views (one per process).  Both kernels: a lane owns 4 elements, the pointer table is
// read from the kernel-argument segment, views are taken in chunks whose loads are all issued
// before the first use, the last chunk has its exact size.
typedef const ViewsArgs __attribute__((address_space(4))) KViewsArgs;

// the update rule on C views from one value of u: 2C loads, then the arithmetic, then 2C stores
template <bool FAST, int C>
__device__ __forceinline__ void views_sgd_chunk(KViewsArgs &a, int p0, long long e, f32x4 u)
{
    f32x4 wo[C], vo[C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        vo[j] = ld_f4<true>(a.v[p0 + j] + e);
        wo[j] = ld_f4<true>(a.w[p0 + j] + e);
    }
    const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
    f32x4 vn[C], wn[C];
#pragma unroll
    for (int j = 0; j < C; ++j) update_rule<FAST>(rule, u, vo[j], wo[j], vn[j], wn[j]);
#pragma unroll
    for (int j = 0; j < C; ++j) {
        st_f4<true>(a.v[p0 + j] + e, vn[j]);
        st_f4<true>(a.w[p0 + j] + e, wn[j]);
    }
}
template <bool FAST, int R>
__device__ __forceinline__ void views_sgd_rest(KViewsArgs &a, int p0, int rem, long long e, f32x4 u)
{
    if constexpr (R >= 1) {
        if (rem == R) views_sgd_chunk<FAST, R>(a, p0, e, u);
        else views_sgd_rest<FAST, R - 1>(a, p0, rem, e, u);
    }
}

template <bool FAST>
__global__ __launch_bounds__(64) void views_sgd_kernel(const ViewsArgs)
{
    KViewsArgs &a = kernarg<ViewsArgs>();
    constexpr int CH = 8;
    const long long nvec = a.n / 4;
    const long long vi = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (vi < nvec) {
        const long long e = a.e0 + vi * 4;
        const f32x4 u = ld_f4<true>(a.u + e);
        const int V = a.n_views;
#pragma unroll
        for (int c = 0; c < kMaxP / CH; ++c)
            if ((c + 1) * CH <= V) views_sgd_chunk<FAST, CH>(a, c * CH, e, u);
        views_sgd_rest<FAST, CH - 1>(a, V / CH * CH, V % CH, e, u);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
        const float u = a.u[i];
        for (int p = 0; p < a.n_views; ++p) {
            float v = a.v[p][i], w = a.w[p][i];
            update_rule_scalar(rule, u, v, w);
            a.v[p][i] = v;
            a.w[p][i] = w;
        }
    }
}

// model synchronisation: every view <- (sum of the views in ascending order from +0.0f) * 1/V,
// the arithmetic of a round in which everybody is on time with an empty send buffer
template <int C>
__device__ __forceinline__ f32x4 views_sum_chunk(KViewsArgs &a, int p0, long long e, f32x4 s)
{
    f32x4 x[C];
#pragma unroll
    for (int j = 0; j < C; ++j) x[j] = ld_f4<true>(a.w[p0 + j] + e);
#pragma unroll
    for (int j = 0; j < C; ++j) s = s + x[j];
    return s;
}
template <int R>
__device__ __forceinline__ f32x4 views_sum_rest(KViewsArgs &a, int p0, int rem, long long e, f32x4 s)
{
    if constexpr (R >= 1) {
        if (rem == R) return views_sum_chunk<R>(a, p0, e, s);
        return views_sum_rest<R - 1>(a, p0, rem, e, s);
    }
    return s;
}

__global__ __launch_bounds__(64) void views_average_kernel(const ViewsArgs)
{
    KViewsArgs &a = kernarg<ViewsArgs>();
    constexpr int CH = 16;
    const long long nvec = a.n / 4;
    const long long vi = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int V = a.n_views;
    if (vi < nvec) {
        const long long e = a.e0 + vi * 4;
        f32x4 s = (f32x4)(0.0f);
#pragma unroll
        for (int c = 0; c < kMaxP / CH; ++c)
            if ((c + 1) * CH <= V) s = views_sum_chunk<CH>(a, c * CH, e, s);
        s = views_sum_rest<CH - 1>(a, V / CH * CH, V % CH, e, s);
        const f32x4 mean = s * a.inv_views;
        for (int p = 0; p < V; ++p) st_f4<true>(a.w[p] + e, mean);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        float s = 0.0f;
        for (int p = 0; p < V; ++p) s = s + a.w[p][i];
        const float mean = s * a.inv_views;
        for (int p = 0; p < V; ++p) a.w[p][i] = mean;
    }
}

// NT: w and v are too large to stay in the last-level cache until they are touched again
// STRIDE: as in stash_kernel
template <bool FAST, bool NT, bool STRIDE>
__global__ __launch_bounds__(256) void sgd_kernel(const SgdArgs a)
{
    const long long nvec = a.n / 4;
    auto body = [&](long long vi) {
        const long long i = a.e0 + vi * 4;
        const f32x4 u = ld_f4<true>(a.u + i);
        const f32x4 vo = ld_f4<NT>(a.v + i);
        const f32x4 wo = ld_f4<NT>(a.w + i);
        f32x4 vn, wn;
        const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
        update_rule<FAST>(rule, u, vo, wo, vn, wn);
        st_f4<NT>(a.v + i, vn);
        st_f4<NT>(a.w + i, wn);
    };
    const long long first = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if constexpr (STRIDE) {
        const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
        for (long long vi = first; vi < nvec; vi += stride) body(vi);
    } else {
        if (first < nvec) body(first);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
        float v = a.v[i], w = a.w[i];
        update_rule_scalar(rule, a.u[i], v, w);
        a.v[i] = v;
        a.w[i] = w;
    }
}

// ---- update rule with a rate per bucket (layer-wise adaptive rate scaling) ------------------
// Two passes, because the norms of a bucket must be complete before its first element moves:
// norms_kernel leaves the same per-wavefront records as a round with statistics (finished by
// stats_finish_kernel, which also forms the rate), lars_kernel applies
//     g = rate_b * (u + wd*w);  v' = mu*v + g;  step = nesterov ? g + mu*v' : v';  w' = w - lr*step
// One lane-vector per lane in both, so that record k belongs to elements [256k, 256k + 256).

// the wavefront's first lane-vector as a uniform value
__device__ __forceinline__ long long wave_first(long long vi)
{
    const long long v0 = vi - (threadIdx.x & 63u);
    return (static_cast<long long>(__builtin_amdgcn_readfirstlane(static_cast<int>(v0 >> 32))) << 32) |
           static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(v0)));
}

// bucket of the lane's 4 elements (they never straddle a bucket start: starts are multiples
// of 4) and how many of them lie inside it; the search starts at the wavefront's bucket
__device__ __forceinline__ int lane_bucket(const long long *tbl, int nb, int wave_bucket, long long e,
                                           int &n_valid)
{
    int b = wave_bucket;
    while (b + 1 < nb && tbl[2 * (b + 1)] <= e) ++b;
    const long long left = tbl[2 * b + 1] - e;
    n_valid = left >= 4 ? 4 : left > 0 ? static_cast<int>(left) : 0;
    return b;
}

// A wavefront takes K consecutive tiles of 256 elements: all 2K loads are issued before the
// first is used, and every tile leaves its own record.
constexpr int kNormsTiles = 4;

template <bool NT>
__global__ __launch_bounds__(64) void norms_kernel(const SgdArgs a, const StatsArgs st)
{
    constexpr int K = kNormsTiles;
    const long long nvec = a.n / 4;
    const long long tile0 = static_cast<long long>(blockIdx.x) * K;
    int bucket = find_bucket(st.table, st.n_buckets, a.e0 + tile0 * 256);
    f32x4 u[K], w[K];
    if (nvec > 0) {
#pragma unroll
        for (int k = 0; k < K; ++k) {
            // beyond the end: the last lane-vector again, discarded below
            long long vi = (tile0 + k) * 64 + threadIdx.x;
            if (vi >= nvec) vi = nvec - 1;
            u[k] = ld_f4<NT>(a.u + a.e0 + vi * 4);
            w[k] = ld_f4<NT>(a.w + a.e0 + vi * 4);
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const long long vi = (tile0 + k) * 64 + threadIdx.x;
        LaneStats ls = {0.0, 0.0, 0u, -1};
        if (vi < nvec) {
            int n_valid;
            bucket = lane_bucket(st.table, st.n_buckets, bucket, a.e0 + vi * 4, n_valid);
            ls.bucket = bucket;
            if (n_valid > 0) stats_add(ls, u[k].x, w[k].x, true);
            if (n_valid > 1) stats_add(ls, u[k].y, w[k].y, true);
            if (n_valid > 2) stats_add(ls, u[k].z, w[k].z, true);
            if (n_valid > 3) stats_add(ls, u[k].w, w[k].w, true);
        }
        stats_commit(st.records, st.lane_records, ls, tile0 + k);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        LaneStats t = {0.0, 0.0, 0u, find_bucket(st.table, st.n_buckets, i)};
        if (i < st.table[2 * t.bucket + 1]) stats_add(t, a.u[i], a.w[i], true);
        else t.bucket = -2;
        const StatsRecord mine = {t.ssu, t.ssw, t.bucket, t.nf, 0};
        st.lane_records[static_cast<long long>(st.n_buckets) * 64 + threadIdx.x] = mine;
    }
}

template <bool FAST>
__device__ __forceinline__ f32x4 scaled_gradient(float rate, float wd, f32x4 u, f32x4 w)
{
    if (FAST) {
#pragma clang fp contract(fast)
        f32x4 g = u;
        if (wd != 0.0f) g = wd * w + u;
        return rate * g;
    }
    f32x4 g = u;
    if (wd != 0.0f) g = fma4(wd, w, u);
    return rate * g;
}

template <bool FAST, bool NT>
__global__ __launch_bounds__(64) void lars_kernel(const SgdArgs a, const StatsArgs st)
{
    const long long nvec = a.n / 4;
    const long long vi = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    const int wave_bucket = find_bucket(st.table, st.n_buckets, a.e0 + 4 * wave_first(vi));
    // the decay is part of the scaled gradient, so the plain rule follows with wd = 0
    const UpdateRule rule = {a.neg_lr, a.mu, 0.0f, a.nesterov};
    if (vi < nvec) {
        const long long e = a.e0 + vi * 4;
        const f32x4 u = ld_f4<true>(a.u + e);
        const f32x4 vo = ld_f4<NT>(a.v + e);
        const f32x4 wo = ld_f4<NT>(a.w + e);
        int n_valid;
        const int b = lane_bucket(st.table, st.n_buckets, wave_bucket, e, n_valid);
        const float rate = st.stats[b].rate;
        f32x4 vn, wn;
        update_rule<FAST>(rule, scaled_gradient<FAST>(rate, a.wd, u, wo), vo, wo, vn, wn);
        st_f4<NT>(a.v + e, vn);
        st_f4<NT>(a.w + e, wn);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        const float rate = st.stats[find_bucket(st.table, st.n_buckets, i)].rate;
        float v = a.v[i], w = a.w[i];
        float g = a.u[i];
        if (a.wd != 0.0f) g = fma1(a.wd, w, g);
        update_rule_scalar(rule, rate * g, v, w);
        a.v[i] = v;
        a.w[i] = w;
    }
}

// Resident wavefronts per CU of the weight-view kernels when the caller leaves it open: what
// counts is the KiB of loads in flight per CU, about 38 for the update (1 + 2 per view loads
// per lane, views in chunks of 8) and 32 for the average (one load per view, chunks of 16).
// Measured optima, update: 12, 8, 4, 3, 2 wavefronts for 1, 2, 4, 8, 16 views (6.8, 6.6, 6.5,
// 6.4, 6.2 TB/s; uncapped 6.7, 6.2, 5.8, 5.7, 5.5); average: uncapped, 16, 8, 4, 4 (6.8, 6.8,
// 6.7, 6.5, 6.3 TB/s; uncapped 6.8, 6.5, 6.0, 5.8, 5.7).
int views_sgd_waves(int n_views)
{
    const int loads = 1 + 2 * (n_views < 8 ? n_views : 8);
    const int w = (38 + loads / 2) / loads;
    return w < 2 ? 2 : w;
}
int views_average_waves(int n_views)
{
    const int loads = n_views < 16 ? n_views : 16;
    const int w = 32 / loads;
    return w > 16 ? -1 : w < 4 ? 4 : w;
}

}  // namespace

hipError_t launch_stats_finish(const StatsArgs &a, hipStream_t stream)
{
    const int n = a.b_hi - a.b_lo;
    if (n <= 0) return hipSuccess;
    if (a.slices > kStatsMaxSlices || a.slices < 1) return hipErrorInvalidValue;
    if (a.slices > 1) {
        hipLaunchKernelGGL(stats_slice_kernel, dim3(n, a.slices), dim3(256), 0, stream, a);
        if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(stats_finish_kernel, dim3(n), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_stash(const StashArgs &a, bool bf16, hipStream_t stream)
{
    if (a.n <= 0) return hipSuccess;
    long long g = (a.n / 4 + 63) / 64;
    if (g < 1) g = 1;
    const bool stride = g > kMaxGridThreads / 64;
    if (stride) g = kMaxGridThreads / 64;
    const dim3 grid(static_cast<unsigned>(g)), block(64);
    if (bf16) {
        if (stride) hipLaunchKernelGGL((stash_kernel<true, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((stash_kernel<true, false>), grid, block, 0, stream, a);
    } else {
        if (stride) hipLaunchKernelGGL((stash_kernel<false, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((stash_kernel<false, false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

namespace {
template <typename K>
hipError_t launch_views(K kernel, const ViewsArgs &a, const Launch &cfg, int auto_waves,
                        hipStream_t stream)
{
    if (a.n <= 0 || a.n_views <= 0) return hipSuccess;
    long long g = (a.n / 4 + 63) / 64;
    if (g < 1) g = 1;
    if (g * 64 > kMaxGridThreads) return hipErrorInvalidValue;    // these kernels do not stride
    Launch l = cfg;
    l.block = 64;
    // half of the traffic is stores: few wavefronts per CU, as for the rounds
    const int bpc = cfg.blocks_per_cu == 0 ? auto_waves : cfg.blocks_per_cu;
    return launch_capped(kernel, a, bpc, l, static_cast<unsigned>(g), stream);
}
}  // namespace

hipError_t launch_views_sgd(const ViewsArgs &a, bool fast, const Launch &cfg, hipStream_t stream)
{
    const int waves = views_sgd_waves(a.n_views);
    return fast ? launch_views(views_sgd_kernel<true>, a, cfg, waves, stream)
                : launch_views(views_sgd_kernel<false>, a, cfg, waves, stream);
}

hipError_t launch_views_average(const ViewsArgs &a, const Launch &cfg, hipStream_t stream)
{
    return launch_views(views_average_kernel, a, cfg, views_average_waves(a.n_views), stream);
}

hipError_t launch_sgd(const SgdArgs &a, bool fast, const Launch &cfg, hipStream_t stream)
{
    if (a.n <= 0) return hipSuccess;
    // 64-thread workgroups, one lane-vector per lane unless the grid is capped (measured on
    // 355 M elements: 1.12 ms against 1.22 ms with 256-thread workgroups and cached state)
    const long long nvec = a.n / 4;
    const dim3 grid(grid_for(nvec, 64, 0)), block(64);
    const bool stride = static_cast<long long>(grid.x) * 64 < nvec;
    const bool nt = a.n * 8 > kStateCacheBytes;
    switch ((fast ? 4 : 0) | (nt ? 2 : 0) | (stride ? 1 : 0)) {
    case 0: hipLaunchKernelGGL((sgd_kernel<false, false, false>), grid, block, 0, stream, a); break;
    case 1: hipLaunchKernelGGL((sgd_kernel<false, false, true>), grid, block, 0, stream, a); break;
    case 2: hipLaunchKernelGGL((sgd_kernel<false, true, false>), grid, block, 0, stream, a); break;
    case 3: hipLaunchKernelGGL((sgd_kernel<false, true, true>), grid, block, 0, stream, a); break;
    case 4: hipLaunchKernelGGL((sgd_kernel<true, false, false>), grid, block, 0, stream, a); break;
    case 5: hipLaunchKernelGGL((sgd_kernel<true, false, true>), grid, block, 0, stream, a); break;
    case 6: hipLaunchKernelGGL((sgd_kernel<true, true, false>), grid, block, 0, stream, a); break;
    default: hipLaunchKernelGGL((sgd_kernel<true, true, true>), grid, block, 0, stream, a); break;
    }
    return hipGetLastError();
}

// tiles of 256 elements that the norms kernel leaves a record for
long long norms_records(long long n)
{
    long long g = (n / 4 + 64 * kNormsTiles - 1) / (64 * kNormsTiles);
    return (g < 1 ? 1 : g) * kNormsTiles;
}

hipError_t launch_norms(const SgdArgs &a, const StatsArgs &st, hipStream_t stream)
{
    if (a.n <= 0) return hipSuccess;
    const long long g = norms_records(a.n) / kNormsTiles;
    if (g * 64 > kMaxGridThreads) return hipErrorInvalidValue;    // the kernel does not stride
    // u and w are read again by the update right after: leave them in the last-level cache
    // when both fit
    if (a.n * 8 <= kStateCacheBytes)
        hipLaunchKernelGGL(norms_kernel<false>, dim3(static_cast<unsigned>(g)), dim3(64), 0, stream, a, st);
    else
        hipLaunchKernelGGL(norms_kernel<true>, dim3(static_cast<unsigned>(g)), dim3(64), 0, stream, a, st);
    return hipGetLastError();
}

hipError_t launch_sgd_lars(const SgdArgs &a, const StatsArgs &st, bool fast, hipStream_t stream)
{
    if (a.n <= 0) return hipSuccess;
    long long g = (a.n / 4 + 63) / 64;                            // one lane-vector per lane
    if (g < 1) g = 1;
    if (g * 64 > kMaxGridThreads) return hipErrorInvalidValue;
    const bool nt = a.n * 8 > kStateCacheBytes;
    const dim3 grid(static_cast<unsigned>(g)), block(64);
    if (fast) {
        if (nt) hipLaunchKernelGGL((lars_kernel<true, true>), grid, block, 0, stream, a, st);
        else hipLaunchKernelGGL((lars_kernel<true, false>), grid, block, 0, stream, a, st);
    } else {
        if (nt) hipLaunchKernelGGL((lars_kernel<false, true>), grid, block, 0, stream, a, st);
        else hipLaunchKernelGGL((lars_kernel<false, false>), grid, block, 0, stream, a, st);
    }
    return hipGetLastError();
}

}  // namespace eager
