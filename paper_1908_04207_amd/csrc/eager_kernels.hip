// gfx950 kernels of the eager-SGD round: partial-allreduce arithmetic with stale-gradient
// carry (paper Section 5, walk-through of Fig. 7), the 1/P average (Algorithm 2 line 6)
// and the momentum-SGD update rule (lines 7-8) in ONE pass over HBM.
//
// The path is a pure stream: per element <= 2P adds, one multiply and two FMAs against
// >= 4P bytes, so HBM bandwidth is the only roofline that matters and there is no
// contraction for the matrix cores.  Design for CDNA4:
//   * slot_kernel (the default): the host compacts the round into a list of streams that
//     must be read, in summation order; a lane owns 4 consecutive elements of every stream,
//     so a 64-lane wavefront reads or writes one contiguous KiB per fp32 stream and
//     instruction; the loads of a chunk of 16 streams are all issued before the first add,
//     which keeps 16-18 x 16 B per lane in flight - that, together with a deliberately
//     capped occupancy, is what suits HBM with mixed reads and writes;
//   * which streams exist and what is done with each is decided on the host and applied in
//     the kernel with scalar bit masks: no branch around a load, empty send buffers cost
//     no bytes, the send buffer of an on-time process is "cleared" by a flag on the host,
//     not by writing zeros;
//   * the accumulator stays in fp32 registers; in fixed-order mode contributions are added
//     in ascending rank order from +0.0f with contraction off, so the result is defined
//     bit for bit; fast mode keeps two partial sums and lets the compiler fuse;
//   * carry_kernel: the send-buffer rewrite of late processes as a plain pair-by-pair
//     copy, when a round is split;
//   * round_kernel: the earlier form (fixed chunks of ranks, stand-in loads for absent
//     streams), kept for comparison;
//   * optional per-bucket norms as by-products: DPP sums inside wavefronts, LDS across
//     them (stats_*); norms_kernel + lars_kernel use them for an update rule with a rate
//     per bucket;
//   * around the round, for processes that lag by more than one round: stash_kernel (a late
//     gradient into a send buffer), views_sgd_kernel / views_average_kernel (a weight view
//     per process: update of several views from one read of the result, model average);
//   * sgd_kernel: the update rule alone on a receive buffer (the unfused path).
#include "eager_internal.h"

#include <mutex>
#include <set>

namespace eager {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// Kernel arguments are read straight from the kernel-argument segment (constant address
// space, scalar loads).  Going through the by-value parameter instead makes the compiler
// keep a private copy of the whole struct in scratch memory as soon as it is indexed
// dynamically in more places than its copy-elision looks at.
typedef const RoundArgs __attribute__((address_space(4))) KRoundArgs;
typedef const SlotArgs __attribute__((address_space(4))) KSlotArgs;
template <typename T>
__device__ __forceinline__ const T __attribute__((address_space(4))) &kernarg()
{
    return *(const T __attribute__((address_space(4))) *)__builtin_amdgcn_kernarg_segment_ptr();
}

template <bool NT>
__device__ __forceinline__ f32x4 ld_f4(const float *p)
{
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
    return *reinterpret_cast<const f32x4 *>(p);
}
template <bool NT>
__device__ __forceinline__ void st_f4(float *p, f32x4 x)
{
    if (NT) __builtin_nontemporal_store(x, reinterpret_cast<f32x4 *>(p));
    else *reinterpret_cast<f32x4 *>(p) = x;
}
template <bool NT>
__device__ __forceinline__ u32x4 ld_u4(const void *p)
{
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return *reinterpret_cast<const u32x4 *>(p);
}

// bf16 is the upper half of an fp32: widening is a shift or a mask, exact.
__device__ __forceinline__ f32x4 widen_lo(u32x4 x, int half)   // elements 0..3 or 4..7
{
    const unsigned a = half ? x.z : x.x, b = half ? x.w : x.y;
    f32x4 r;
    r.x = __uint_as_float(a << 16);
    r.y = __uint_as_float(a & 0xffff0000u);
    r.z = __uint_as_float(b << 16);
    r.w = __uint_as_float(b & 0xffff0000u);
    return r;
}

// The update rule U of Algorithm 2, lines 7-8, for one element or one vector of 4:
//   g = u + wd*w  (only if wd != 0);  v' = mu*v + g;  step = nesterov ? g + mu*v' : v';
//   w' = w - lr*step
// every line one fused multiply-add (single rounding) in fixed-order mode.  wd and nesterov
// are uniform over the grid; with wd = 0 and nesterov = 0 this is plain heavy-ball momentum.
struct UpdateRule {
    float neg_lr, mu, wd;
    int nesterov;
};

__device__ __forceinline__ float fma1(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ f32x4 fma4(float a, f32x4 b, f32x4 c)
{
    f32x4 r;
    r.x = __builtin_fmaf(a, b.x, c.x);
    r.y = __builtin_fmaf(a, b.y, c.y);
    r.z = __builtin_fmaf(a, b.z, c.z);
    r.w = __builtin_fmaf(a, b.w, c.w);
    return r;
}

template <bool FAST>
__device__ __forceinline__ void update_rule(const UpdateRule &r, f32x4 u, f32x4 vo, f32x4 wo,
                                            f32x4 &vn, f32x4 &wn)
{
    if (FAST) {
#pragma clang fp contract(fast)
        f32x4 g = u;
        if (r.wd != 0.0f) g = r.wd * wo + u;
        vn = r.mu * vo + g;
        f32x4 step = vn;
        if (r.nesterov) step = r.mu * vn + g;
        wn = r.neg_lr * step + wo;
    } else {
        f32x4 g = u;
        if (r.wd != 0.0f) g = fma4(r.wd, wo, u);
        vn = fma4(r.mu, vo, g);
        f32x4 step = vn;
        if (r.nesterov) step = fma4(r.mu, vn, g);
        wn = fma4(r.neg_lr, step, wo);
    }
}

__device__ __forceinline__ void update_rule_scalar(const UpdateRule &r, float u, float &v, float &w)
{
    float g = u;
    if (r.wd != 0.0f) g = fma1(r.wd, w, u);
    const float vn = fma1(r.mu, v, g);
    float step = vn;
    if (r.nesterov) step = fma1(r.mu, vn, g);
    v = vn;
    w = fma1(r.neg_lr, step, w);
}

// One thread-vector: W = 4 (fp32 gradients) or 8 (bf16 gradients) consecutive elements,
// i.e. NV = W/4 fp32 quads of state; U vectors are processed together.  Ranks are taken
// CH at a time.
//
// The load phase of a chunk is straight-line code with no branch in it: a stream that
// must not be read (an empty send buffer, or a rank index beyond P in the last chunk)
// has its address replaced by one fixed 16-byte location (`dummy`, the first vector of
// the run in G_0), which every lane of every wavefront hits in cache; the value is
// discarded by a select, never by arithmetic.  With branches around the loads the
// compiler can no longer count outstanding loads and falls back to waiting for each
// one, which leaves a single load in flight per wavefront.
template <bool BF16, bool FAST, bool NT, int U, int CH>
__device__ __forceinline__ void round_vectors(KRoundArgs &a, const long long (&e)[U])
{
    constexpr int NV = BF16 ? 2 : 1;
    constexpr int GB = BF16 ? 2 : 4;
    f32x4 s[U][NV];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < NV; ++k) s[u][k] = (f32x4)(0.0f);

    // parameters and momentum are requested first so that their latency hides behind
    // the gradient streams
    f32x4 vo_[U][NV], wo_[U][NV];
    if (a.w) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                vo_[u][k] = ld_f4<false>(a.v + e[u] + 4 * k);
                wo_[u][k] = ld_f4<false>(a.w + e[u] + 4 * k);
            }
    }

    const char *const dummy = static_cast<const char *>(a.dummy);
    for (int p0 = 0; p0 < a.P; p0 += CH) {
        u32x4 g[U][CH];
        f32x4 r[U][CH][NV];
        // 1. every gradient of the chunk (each is needed: summed if on time, stored if late)
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int p = p0 + j;
            const bool real = (a.gload >> p) & 1ull;
            const char *gp = static_cast<const char *>(a.g[p]);
#pragma unroll
            for (int u = 0; u < U; ++u)
                g[u][j] = ld_u4<NT>(real ? gp + e[u] * GB : dummy);
        }
        // 2. the send buffers that hold something
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int p = p0 + j;
            const bool has_stale = (a.valid >> p) & 1ull;
            const char *rp = reinterpret_cast<const char *>(a.r[p]);
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int k = 0; k < NV; ++k)
                    r[u][j][k] = ld_f4<NT>(reinterpret_cast<const float *>(
                        has_stale ? rp + (e[u] + 4 * k) * 4 : dummy));
        }
        // 3. contributions, in registers
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                if (!FAST) {
                    // ascending rank order; an absent contribution adds nothing
#pragma unroll
                    for (int j = 0; j < CH; ++j) {
                        const int p = p0 + j;
                        const bool on_time = (a.active >> p) & 1ull;
                        const bool has_stale = (a.valid >> p) & 1ull;
                        const f32x4 gf = BF16 ? widen_lo(g[u][j], k)
                                              : __builtin_bit_cast(f32x4, g[u][j]);
                        if (on_time) {
                            f32x4 c = gf;
                            if (has_stale) c = r[u][j][k] + gf;
                            s[u][k] = s[u][k] + c;
                        } else if (has_stale) {
                            s[u][k] = s[u][k] + r[u][j][k];
                        }
                    }
                } else {
                    // contributions of the chunk form a tree; absent terms are +0
                    f32x4 c[CH];
#pragma unroll
                    for (int j = 0; j < CH; ++j) {
                        const int p = p0 + j;
                        const bool on_time = (a.active >> p) & 1ull;
                        const bool has_stale = (a.valid >> p) & 1ull;
                        const f32x4 gf = BF16 ? widen_lo(g[u][j], k)
                                              : __builtin_bit_cast(f32x4, g[u][j]);
                        const f32x4 z = (f32x4)(0.0f);
                        c[j] = (on_time ? gf : z) + (has_stale ? r[u][j][k] : z);
                    }
#pragma unroll
                    for (int w = CH / 2; w >= 1; w >>= 1)
#pragma unroll
                        for (int j = 0; j < w; ++j) c[j] = c[j] + c[j + w];
                    s[u][k] = s[u][k] + c[0];
                }
            }
        // 4. late gradients become the new content of the send buffer
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int p = p0 + j;
            if ((a.store >> p) & 1ull) {
                float *rp = a.r[p];
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int k = 0; k < NV; ++k)
                        st_f4<NT>(rp + e[u] + 4 * k, BF16 ? widen_lo(g[u][j], k)
                                                           : __builtin_bit_cast(f32x4, g[u][j]));
            }
        }
    }

    // 5. average over P (not over the contributors) and the update rule
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const f32x4 avg = s[u][k] * a.inv_P;
            const long long i = e[u] + 4 * k;
            if (a.recv) st_f4<false>(a.recv + i, avg);
            if (a.w) {
                f32x4 vn, wn;
                const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
                update_rule<FAST>(rule, avg, vo_[u][k], wo_[u][k], vn, wn);
                st_f4<false>(a.v + i, vn);
                st_f4<false>(a.w + i, wn);
            }
        }
}

// Ragged tail (fewer elements than a vector): plain scalar code, fixed order in both
// modes - at most 7 elements per launch.
template <bool BF16>
__device__ __forceinline__ float load_grad_scalar(const void *g, long long i)
{
    if (BF16) {
        const unsigned short h = static_cast<const unsigned short *>(g)[i];
        return __uint_as_float(static_cast<unsigned>(h) << 16);
    }
    return static_cast<const float *>(g)[i];
}

template <bool BF16>
__device__ __forceinline__ void round_scalar(KRoundArgs &a, long long i)
{
    float s = 0.0f;
    for (int p = 0; p < a.P; ++p) {
        const bool on_time = (a.active >> p) & 1ull;
        const bool has_stale = (a.valid >> p) & 1ull;
        if (on_time) {
            const float g = load_grad_scalar<BF16>(a.g[p], i);
            float c = g;
            if (has_stale) c = a.r[p][i] + g;
            s = s + c;
        } else {
            if (has_stale) s = s + a.r[p][i];
            if ((a.store >> p) & 1ull) a.r[p][i] = load_grad_scalar<BF16>(a.g[p], i);
        }
    }
    const float avg = s * a.inv_P;
    if (a.recv) a.recv[i] = avg;
    if (a.w) {
        const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
        float v = a.v[i], w = a.w[i];
        update_rule_scalar(rule, avg, v, w);
        a.v[i] = v;
        a.w[i] = w;
    }
}

template <bool BF16, bool FAST, bool NT, int U, int CH, int LB>
__global__ __launch_bounds__(LB) void round_kernel(const RoundArgs)
{
    KRoundArgs &a = kernarg<RoundArgs>();
    constexpr int W = BF16 ? 8 : 4;
    const long long nvec = a.n / W;
    const long long tile = static_cast<long long>(blockDim.x) * U;
    for (long long base = static_cast<long long>(blockIdx.x) * tile; base < nvec;
         base += static_cast<long long>(gridDim.x) * tile) {
        if (base + tile <= nvec) {
            long long e[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                e[u] = a.e0 + (base + static_cast<long long>(u) * blockDim.x + threadIdx.x) * W;
            round_vectors<BF16, FAST, NT, U, CH>(a, e);
        } else {
            for (int u = 0; u < U; ++u) {
                const long long vi = base + static_cast<long long>(u) * blockDim.x + threadIdx.x;
                if (vi < nvec) {
                    const long long e1[1] = {a.e0 + vi * W};
                    round_vectors<BF16, FAST, NT, 1, CH>(a, e1);
                }
            }
        }
    }
    const long long rem = a.n - nvec * W;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem)
        round_scalar<BF16>(a, a.e0 + nvec * W + threadIdx.x);
}

// ---------------------------------------------------------------------------------------
// Per-bucket by-products (optional): sum of squares of the averaged update and of the
// parameters, count of non-finite elements.  They are reductions ACROSS elements, the one
// place on this path where cross-lane work belongs: a lane sums its 4 elements, the 64 lanes
// of a wavefront are combined with DPP moves inside rows of 16 lanes and lane reads across
// the 4 rows, and one lane writes one record per wavefront.  A wavefront whose elements lie in
// several buckets leaves one record per lane instead.  No atomics anywhere and fixed trees:
// the result is reproducible bit for bit.  A finishing kernel adds the records of a bucket,
// combining the wavefronts of its workgroup through LDS.
struct LaneStats {
    double ssu, ssw;   // squares of the update / of the old parameters
    unsigned nf;       // non-finite elements of the update
    int bucket;        // -1: the lane holds no element
};

// DPP controls: quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.  Applied
// in this order every lane ends with the sum over its row of 16; all lanes must be active.
constexpr int kDppXor1 = 0xB1, kDppXor2 = 0x4E, kDppHalfMirror = 0x141, kDppMirror = 0x140;

template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x)
{
    const unsigned long long b = __builtin_bit_cast(unsigned long long, x);
    const int lo = __builtin_amdgcn_update_dpp(0, static_cast<int>(b), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, static_cast<int>(b >> 32), CTRL, 0xf, 0xf, true);
    return __builtin_bit_cast(double, (static_cast<unsigned long long>(static_cast<unsigned>(hi)) << 32) |
                                          static_cast<unsigned>(lo));
}
template <int CTRL>
__device__ __forceinline__ unsigned dpp_u32(unsigned x)
{
    return static_cast<unsigned>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ double readlane_f64(double x, int lane)
{
    const unsigned long long b = __builtin_bit_cast(unsigned long long, x);
    const unsigned lo = __builtin_amdgcn_readlane(static_cast<int>(b), lane);
    const unsigned hi = __builtin_amdgcn_readlane(static_cast<int>(b >> 32), lane);
    return __builtin_bit_cast(double, (static_cast<unsigned long long>(hi) << 32) | lo);
}
// sum over the 64 lanes of the wavefront, the same value in every lane (uniform)
__device__ __forceinline__ double wave_sum(double x)
{
    x = x + dpp_f64<kDppXor1>(x);
    x = x + dpp_f64<kDppXor2>(x);
    x = x + dpp_f64<kDppHalfMirror>(x);
    x = x + dpp_f64<kDppMirror>(x);
    return (readlane_f64(x, 0) + readlane_f64(x, 16)) + (readlane_f64(x, 32) + readlane_f64(x, 48));
}
__device__ __forceinline__ unsigned wave_sum(unsigned x)
{
    x = x + dpp_u32<kDppXor1>(x);
    x = x + dpp_u32<kDppXor2>(x);
    x = x + dpp_u32<kDppHalfMirror>(x);
    x = x + dpp_u32<kDppMirror>(x);
    return static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(x), 0)) +
           static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(x), 16)) +
           static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(x), 32)) +
           static_cast<unsigned>(__builtin_amdgcn_readlane(static_cast<int>(x), 48));
}

// the bucket that holds element e: the last one that starts at or before e
__device__ __forceinline__ int find_bucket(const long long *tbl, int nb, long long e)
{
    int lo = 0, hi = nb;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tbl[2 * mid] <= e) lo = mid;
        else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ void stats_add(LaneStats &ls, float u, float w_old, bool has_w)
{
    // the square of an fp32 value is exact in fp64, so the fused form rounds exactly like a
    // product followed by a sum
    const double ud = static_cast<double>(u), wd = static_cast<double>(w_old);
    if (__builtin_isfinite(u)) ls.ssu = __builtin_fma(ud, ud, ls.ssu);
    else ls.nf += 1u;
    if (has_w && __builtin_isfinite(w_old)) ls.ssw = __builtin_fma(wd, wd, ls.ssw);
}

// Called by every lane of a wavefront (all active).  The lanes that hold elements are a
// prefix of the wavefront and buckets ascend with the lane, so a mixed wavefront is the only
// one whose first lane lies in bucket b0 while a later lane does not: block b0 of the lane
// records is its own.
__device__ __forceinline__ void stats_commit(StatsRecord *records, StatsRecord *lane_records,
                                             const LaneStats &ls, long long wave_index)
{
    const int b0 = __builtin_amdgcn_readfirstlane(ls.bucket);
    const bool mixed = __builtin_amdgcn_ballot_w64(ls.bucket != b0) != 0ull;
    StatsRecord rec = {0.0, 0.0, b0 >= 0 ? b0 : -2, 0u, 0};
    if (mixed) {
        const StatsRecord mine = {ls.ssu, ls.ssw, ls.bucket, ls.nf, 0};
        lane_records[static_cast<long long>(b0) * 64 + (threadIdx.x & 63u)] = mine;
        rec.bucket = -1;
        rec.nf = static_cast<unsigned>(b0);
    } else if (b0 >= 0) {
        rec.ssu = wave_sum(ls.ssu);
        rec.ssw = wave_sum(ls.ssw);
        if (__builtin_amdgcn_ballot_w64(ls.nf != 0u) != 0ull) rec.nf = wave_sum(ls.nf);
    }
    if ((threadIdx.x & 63u) == 0u) records[wave_index] = rec;
}

// ---------------------------------------------------------------------------------------
// Compacted form: a list of streams ("slots"), each with one action, in summation order.  A
// chunk of C slots is C loads issued back to back, then the adds, then the stores; the list
// is consumed in chunks of CH and one remainder chunk of its exact size, so that not a
// single stand-in load is issued.
//
// A lane owns 4 consecutive elements of every stream, so that each load or store instruction
// of a wavefront covers one contiguous kilobyte of an fp32 stream.  With bf16 gradients
// (BF16) the lane's 4 gradient elements are 8 bytes, one half of an aligned 16-byte piece:
// lanes 2k and 2k+1 load the same piece and each keeps its half.  That way every load of a
// chunk is the same 16-byte instruction whatever the type of its stream - the type, like the
// action, is a scalar select and never a branch around a load.
struct LaneVec {
    long long e;        // first of the lane's 4 elements (arena index)
    long long off_bf;   // byte offset of the 16-byte piece of a bf16 stream that holds them
    bool odd;           // the lane's elements are the upper half of that piece
};

template <bool BF16>
__device__ __forceinline__ f32x4 slot_value(u32x4 raw, bool is_bf, bool odd)
{
    const f32x4 plain = __builtin_bit_cast(f32x4, raw);
    if (!BF16) return plain;
    const unsigned a = odd ? raw.z : raw.x, b = odd ? raw.w : raw.y;
    f32x4 wide;
    wide.x = __uint_as_float(a << 16);
    wide.y = __uint_as_float(a & 0xffff0000u);
    wide.z = __uint_as_float(b << 16);
    wide.w = __uint_as_float(b & 0xffff0000u);
    return is_bf ? wide : plain;
}

__device__ __forceinline__ f32x4 masked(f32x4 x, unsigned m)
{
    return __builtin_bit_cast(f32x4, __builtin_bit_cast(u32x4, x) & m);
}

template <bool BF16, bool FAST, bool NT, int U, int C>
__device__ __forceinline__ void slot_chunk(KSlotArgs &a, int k0, const LaneVec (&lv)[U],
                                           f32x4 (&s)[U][2], f32x4 (&hold)[U])
{
    // a chunk starts at a multiple of its size (8, 16 or 32): its bits never straddle a
    // mask word
    const unsigned long long b0 = a.kind0[k0 >> 6] >> (k0 & 63);
    const unsigned long long b1 = a.kind1[k0 >> 6] >> (k0 & 63);
    const unsigned long long bf = BF16 ? a.bf[k0 >> 6] >> (k0 & 63) : 0ull;
    u32x4 raw[U][C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        const char *sp = static_cast<const char *>(a.src[k0 + j]);
        const bool is_bf = BF16 && ((bf >> j) & 1ull);
#pragma unroll
        for (int u = 0; u < U; ++u)
            raw[u][j] = ld_u4<NT>(sp + (is_bf ? lv[u].off_bf : lv[u].e * 4));
    }
    // Every loaded value is used unconditionally and the action of a slot is applied with
    // bit masks built from scalar conditions, never with a branch: if a path existed on
    // which a load is not consumed, the compiler would have to drain all memory operations
    // before its registers could be reused.
    //   fixed order:  c = x + (prev & pair) ;  s = s + (c & adds)
    // where prev is the value of the slot before (a HOLD is always directly followed by its
    // PAIR; `hold` carries the last value of the previous chunk), pair = all ones for a PAIR
    // slot, adds = all ones for ADD and PAIR.  A masked-out term is +0.0f, and adding +0.0f
    // changes nothing here: s starts at +0.0f and a sum of two floats is -0.0f only if both
    // are, so s is never -0.0f; and c = x + 0.0f differs from x only for x = -0.0f, which
    // adds the same as +0.0f to an s that is not -0.0f.
    f32x4 x[U][C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        const unsigned lo = static_cast<unsigned>(b0 >> j) & 1u;
        const unsigned hi = static_cast<unsigned>(b1 >> j) & 1u;
        const unsigned m_pair = 0u - (hi & ~lo & 1u);          // PAIR
        const unsigned m_adds = 0u - (~lo & 1u);               // ADD or PAIR
        const unsigned m_sum = ~(0u - (lo & hi));              // everything but STORE
#pragma unroll
        for (int u = 0; u < U; ++u) {
            x[u][j] = slot_value<BF16>(raw[u][j], (bf >> j) & 1ull, lv[u].odd);
            if (FAST) {
                // any order: two interleaved partial sums
                s[u][j & 1] = s[u][j & 1] + masked(x[u][j], m_sum);
            } else {
                const f32x4 prev = j == 0 ? hold[u] : x[u][j - 1];
                const f32x4 c = x[u][j] + masked(prev, m_pair);
                s[u][0] = s[u][0] + masked(c, m_adds);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) hold[u] = x[u][C - 1];
    // Stores stay behind the adds: moved ahead of them (the compiler likes to sink the add
    // chain below the store branches), the in-order memory counter would make every add
    // wait for the acknowledgement of a store instead of for its load.  The empty
    // statement pins the sums here and orders the stores after it.
#pragma unroll
    for (int u = 0; u < U; ++u)
        asm volatile("" : "+v"(s[u][0]), "+v"(s[u][1]), "+v"(hold[u]) : : "memory");
#pragma unroll
    for (int j = 0; j < C; ++j) {
        if (((b0 >> j) & 1ull) && ((b1 >> j) & 1ull)) {          // STORE
            float *dp = a.dst[k0 + j];
#pragma unroll
            for (int u = 0; u < U; ++u) st_f4<NT>(dp + lv[u].e, x[u][j]);
        }
    }
}

template <bool BF16, bool FAST, bool NT, int U, int R>
__device__ __forceinline__ void slot_remainder(KSlotArgs &a, int k0, int rem,
                                               const LaneVec (&lv)[U], f32x4 (&s)[U][2],
                                               f32x4 (&hold)[U])
{
    if constexpr (R >= 1) {
        if (rem == R) slot_chunk<BF16, FAST, NT, U, R>(a, k0, lv, s, hold);
        else slot_remainder<BF16, FAST, NT, U, R - 1>(a, k0, rem, lv, s, hold);
    }
}

// NTS: parameters, momentum and the receive buffer are streamed with the nontemporal hint
// too (right when they are too large to stay in the last-level cache until the next round).
template <bool BF16, bool FAST, bool NT, bool NTS, int U, int CH, bool STATS>
__device__ __forceinline__ void slot_vectors(KSlotArgs &a, const LaneVec (&lv)[U], int n_valid,
                                             LaneStats &ls)
{
    f32x4 s[U][2], hold[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        s[u][0] = (f32x4)(0.0f);
        s[u][1] = (f32x4)(0.0f);
        hold[u] = (f32x4)(0.0f);
    }
    f32x4 vo[U], wo[U];
    if (a.w) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            vo[u] = ld_f4<NTS>(a.v + lv[u].e);
            wo[u] = ld_f4<NTS>(a.w + lv[u].e);
        }
    }
    // The chunk sequence is unrolled to its maximum length with forward exits only: in a
    // real loop the compiler drains every outstanding store at the loop head before the
    // next chunk's loads may issue, which puts a store round trip between chunks.
    const int n = a.n_slots;
#pragma unroll
    for (int c = 0; c < kMaxSlots / CH; ++c)
        if ((c + 1) * CH <= n) slot_chunk<BF16, FAST, NT, U, CH>(a, c * CH, lv, s, hold);
    // the remainder is ONE chunk of its exact size: every chunk costs a memory round
    // trip per wavefront, so a cascade of smaller and smaller chunks would be slow
    slot_remainder<BF16, FAST, NT, U, CH - 1>(a, n / CH * CH, n % CH, lv, s, hold);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const long long e = lv[u].e;
        f32x4 sum = s[u][0];
        if (FAST) sum = sum + s[u][1];
        const f32x4 avg = sum * a.inv_P;
        if (a.recv) st_f4<NTS>(a.recv + e, avg);
        if (STATS) {
            // n_valid: how many of the lane's 4 elements lie inside their bucket (the rest
            // is padding between buckets)
            const bool has_w = a.w != nullptr;
            const f32x4 w_old = has_w ? wo[u] : (f32x4)(0.0f);
            if (n_valid > 0) stats_add(ls, avg.x, w_old.x, has_w);
            if (n_valid > 1) stats_add(ls, avg.y, w_old.y, has_w);
            if (n_valid > 2) stats_add(ls, avg.z, w_old.z, has_w);
            if (n_valid > 3) stats_add(ls, avg.w, w_old.w, has_w);
        }
        if (a.w) {
            f32x4 vn, wn;
            const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
            update_rule<FAST>(rule, avg, vo[u], wo[u], vn, wn);
            st_f4<NTS>(a.v + e, vn);
            st_f4<NTS>(a.w + e, wn);
        }
    }
}

// ragged tail: at most 3 (7 with bf16 gradients) elements per launch, fixed order in both
// modes
template <bool BF16, bool STATS>
__device__ __forceinline__ void slot_scalar(KSlotArgs &a, long long i)
{
    float s = 0.0f, hold = 0.0f;
    for (int k = 0; k < a.n_slots; ++k) {
        const int kind = static_cast<int>((a.kind0[k >> 6] >> (k & 63)) & 1ull) |
                         static_cast<int>(((a.kind1[k >> 6] >> (k & 63)) & 1ull) << 1);
        float x;
        if (BF16 && ((a.bf[k >> 6] >> (k & 63)) & 1ull))
            x = load_grad_scalar<true>(a.src[k], i);
        else
            x = load_grad_scalar<false>(a.src[k], i);
        if (kind == kAdd) s = s + x;
        else if (kind == kHold) hold = x;
        else if (kind == kPair) { const float c = hold + x; s = s + c; }
        else a.dst[k][i] = x;
    }
    const float avg = s * a.inv_P;
    if (a.recv) a.recv[i] = avg;
    if (STATS) {
        // a handful of single elements per launch: one record each, in the block after the
        // last bucket's
        const long long *tbl = a.stats.table;
        LaneStats ls = {0.0, 0.0, 0u, find_bucket(tbl, a.stats.n_buckets, i)};
        if (i < tbl[2 * ls.bucket + 1]) stats_add(ls, avg, a.w ? a.w[i] : 0.0f, a.w != nullptr);
        else ls.bucket = -2;                                   // padding
        const StatsRecord mine = {ls.ssu, ls.ssw, ls.bucket, ls.nf, 0};
        a.stats.lane_records[static_cast<long long>(a.stats.n_buckets) * 64 + threadIdx.x] = mine;
    }
    if (a.w) {
        const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
        float v = a.v[i], w = a.w[i];
        update_rule_scalar(rule, avg, v, w);
        a.v[i] = v;
        a.w[i] = w;
    }
}

// Lane-vectors (groups of 4 elements) of a run that the vector path covers.  With bf16
// gradients two lanes share one 16-byte piece, so the vector path ends at a multiple of 8
// elements and never reads beyond the run.
template <bool BF16>
__host__ __device__ __forceinline__ long long slot_nvec(long long n)
{
    return BF16 ? (n / 8) * 2 : n / 4;
}

// One lane-vector per lane and no loop over tiles: inside a loop every scalar condition of
// every slot is loop invariant, the compiler hoists hundreds of them out of it and then
// spills scalar registers.  The grid always covers the run.
template <bool BF16, bool FAST, bool NT, bool NTS, int CH, bool STATS>
__global__ __launch_bounds__(256) void slot_kernel(const SlotArgs)
{
    KSlotArgs &a = kernarg<SlotArgs>();
    const long long nvec = slot_nvec<BF16>(a.n);
    // Workgroups are dealt to the 8 XCDs round robin.  xcd_map = 1 gives every XCD one
    // contiguous eighth of the run instead of every eighth tile (a launch option, for A/B).
    unsigned bid = blockIdx.x;
    if (a.xcd_map) {
        const unsigned per = gridDim.x / 8u;
        if (bid < per * 8u) bid = (bid % 8u) * per + bid / 8u;
    }
    const long long vi = static_cast<long long>(bid) * blockDim.x + threadIdx.x;
    LaneStats ls = {0.0, 0.0, 0u, -1};
    int n_valid = 0;
    int wave_bucket = 0;
    if (STATS) {
        // bucket of the wavefront's first element: a uniform search (scalar loads), started
        // before the streams are requested
        const long long v0 = vi - (threadIdx.x & 63u);
        const long long e_wave =
            a.e0 + 4 * ((static_cast<long long>(__builtin_amdgcn_readfirstlane(
                             static_cast<int>(v0 >> 32))) << 32) |
                        static_cast<unsigned>(__builtin_amdgcn_readfirstlane(static_cast<int>(v0))));
        wave_bucket = find_bucket(a.stats.table, a.stats.n_buckets, e_wave);
    }
    if (vi < nvec) {
        // bucket starts are multiples of 8 elements with bf16 gradients, so e0 * 2 is a
        // multiple of 16 bytes
        const LaneVec lv[1] = {{a.e0 + vi * 4, a.e0 * 2 + (vi >> 1) * 16, (vi & 1) != 0}};
        if (STATS) {
            // a lane's 4 elements never straddle a bucket start (starts are multiples of 4)
            const long long *tbl = a.stats.table;
            int b = wave_bucket;
            while (b + 1 < a.stats.n_buckets && tbl[2 * (b + 1)] <= lv[0].e) ++b;
            const long long left = tbl[2 * b + 1] - lv[0].e;
            n_valid = left >= 4 ? 4 : left > 0 ? static_cast<int>(left) : 0;
            ls.bucket = b;
        }
        slot_vectors<BF16, FAST, NT, NTS, 1, CH, STATS>(a, lv, n_valid, ls);
    }
    if (STATS) stats_commit(a.stats.records, a.stats.lane_records, ls, vi >> 6);
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem)
        slot_scalar<BF16, STATS>(a, a.e0 + nvec * 4 + threadIdx.x);
}

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

// R_p <- G_p for the late processes, as a plain copy: pair after pair (blockIdx is
// pair-major), so that at any time the device streams one source and one destination.
// A copy of few streams runs near the read-only rate on MI355X, whereas the same bytes
// written as 8-31 interleaved streams next to the reduction's reads cost 10-15 %.
// A lane owns 4 elements: every store instruction of a wavefront writes one contiguous
// kilobyte (a bf16 source is read 8 bytes per lane and widened).
template <bool BF16, int V>
__global__ __launch_bounds__(256) void carry_kernel(const CarryArgs a, unsigned blocks_per_pair)
{
    const unsigned pair = blockIdx.x / blocks_per_pair;
    const unsigned blk = blockIdx.x - pair * blocks_per_pair;
    const long long nvec = a.n / 4;
    const char *src = static_cast<const char *>(a.src[pair]);
    float *dst = a.dst[pair];
    // a workgroup copies V * blockDim consecutive lane-vectors per iteration: all loads
    // first, then the stores
    const long long tile = static_cast<long long>(blockDim.x) * V;
    for (long long base = static_cast<long long>(blk) * tile; base < nvec;
         base += static_cast<long long>(blocks_per_pair) * tile) {
        f32x4 x[V];
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const long long vi = base + static_cast<long long>(k) * blockDim.x + threadIdx.x;
            if (vi < nvec) {
                const long long e = a.e0 + vi * 4;
                if (BF16) {
                    const u32x2 g = __builtin_nontemporal_load(
                        reinterpret_cast<const u32x2 *>(src + e * 2));
                    x[k].x = __uint_as_float(g.x << 16);
                    x[k].y = __uint_as_float(g.x & 0xffff0000u);
                    x[k].z = __uint_as_float(g.y << 16);
                    x[k].w = __uint_as_float(g.y & 0xffff0000u);
                } else {
                    x[k] = ld_f4<true>(reinterpret_cast<const float *>(src + e * 4));
                }
            }
        }
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const long long vi = base + static_cast<long long>(k) * blockDim.x + threadIdx.x;
            if (vi < nvec) st_f4<true>(dst + a.e0 + vi * 4, x[k]);
        }
    }
    const long long rem = a.n - nvec * 4;
    if (blk == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        dst[i] = load_grad_scalar<BF16>(src, i);
    }
}

// A late gradient outside a round (a process that lags by more than one round, last
// paragraph of Section 5): R <- G, or R <- R + G if the send buffer still holds an
// undelivered gradient.  A plain stream, a lane owns 4 elements.
template <bool BF16>
__global__ __launch_bounds__(64) void stash_kernel(const StashArgs a)
{
    const long long nvec = a.n / 4;
    const char *src = static_cast<const char *>(a.g);
    const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
    for (long long vi = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x; vi < nvec;
         vi += stride) {
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
template <bool FAST, bool NT>
__global__ __launch_bounds__(256) void sgd_kernel(const SgdArgs a)
{
    const long long nvec = a.n / 4;
    const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
    for (long long vi = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x; vi < nvec;
         vi += stride) {
        const long long i = a.e0 + vi * 4;
        const f32x4 u = ld_f4<true>(a.u + i);
        const f32x4 vo = ld_f4<NT>(a.v + i);
        const f32x4 wo = ld_f4<NT>(a.w + i);
        f32x4 vn, wn;
        const UpdateRule rule = {a.neg_lr, a.mu, a.wd, a.nesterov};
        update_rule<FAST>(rule, u, vo, wo, vn, wn);
        st_f4<NT>(a.v + i, vn);
        st_f4<NT>(a.w + i, wn);
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

__global__ __launch_bounds__(64) void copy_kernel(f32x4 *dst, const f32x4 *src, long long nvec)
{
    const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
    for (long long i = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec;
         i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

__global__ __launch_bounds__(256) void read_kernel(const f32x4 *src, long long nvec, float *sink)
{
    const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
    f32x4 acc = (f32x4)(0.0f);
    for (long long i = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x; i < nvec;
         i += stride)
        acc = acc + __builtin_nontemporal_load(src + i);
    const float t = acc.x + acc.y + acc.z + acc.w;
    if (t == 123.456f) *sink = t;   // keeps the loads alive; practically never taken
}

// LDS is not used by the kernel; a dynamic allocation only caps how many workgroups a CU
// holds at once.  A stream that mixes reads with 30-35 % writes runs 5-10 % faster on
// MI355X with a few wavefronts per CU, each with 12-16 KiB of loads in flight, than at
// full occupancy (measured: about 64-110 KiB in flight per CU is the optimum; beyond it
// HBM throughput falls again).
constexpr int kLdsPerCu = 160 * 1024;

// A grid must hold fewer than 2^32 threads in total; a launch beyond that is not refused
// by the runtime, its thread count wraps.  Every launcher stays at or below 2^31.
constexpr long long kMaxGridThreads = 1ll << 31;

// Parameters and momentum above this size are streamed past the caches (see slot_vectors).
constexpr long long kStateCacheBytes = 256ll << 20;

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

// Resident workgroups per CU when the caller leaves the choice to the library: measured
// optima of the rank-chunk kernel with 64-thread workgroups for 1, 2 and 4 chunks of 8.
int auto_blocks_per_cu(int P, int block, bool bf16)
{
    const int chunks = (P + 7) / 8;
    const int waves = chunks <= 1 ? 10 : chunks == 2 ? (bf16 ? 8 : 5) : 6;
    const int b = (waves * 64 + block - 1) / block;
    return b < 1 ? 1 : b;
}

template <typename K, typename A, typename... Extra>
hipError_t launch_capped(K kernel, const A &a, int bpc, const Launch &cfg, unsigned grid,
                         hipStream_t st, Extra... extra)
{
    unsigned lds = 0;
    if (bpc > 0) {
        lds = static_cast<unsigned>(kLdsPerCu / bpc) & ~2047u;
        // Kernels of one signature share this function, so the flag is kept per kernel
        // address (a handful of entries; a context is not used from several threads, the
        // mutex covers several contexts).
        static std::mutex mu;
        static std::set<const void *> raised;
        const void *fn = reinterpret_cast<const void *>(kernel);
        std::lock_guard<std::mutex> lock(mu);
        if (!raised.count(fn)) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               kLdsPerCu);
            if (e != hipSuccess) return e;
            raised.insert(fn);
        }
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(cfg.block), lds, st, a, extra...);
    return hipGetLastError();
}

template <typename K>
hipError_t launch_capped(K kernel, const RoundArgs &a, const Launch &cfg, unsigned grid,
                         hipStream_t st)
{
    const bool bf16 = a.elem_bytes == 2;
    const int bpc = cfg.blocks_per_cu == 0 ? auto_blocks_per_cu(a.P, cfg.block, bf16)
                                           : cfg.blocks_per_cu;
    return launch_capped(kernel, a, bpc, cfg, grid, st);
}

// ---- slot kernel: build the stream list from the rank masks, pick the instantiation
void build_slots(const RoundArgs &a, SlotArgs &s)
{
    s.n_slots = 0;
    s.kind0[0] = s.kind0[1] = s.kind1[0] = s.kind1[1] = s.bf[0] = s.bf[1] = 0;
    const bool bf16 = a.elem_bytes == 2;
    auto push = [&s](const void *src, float *dst, int kind, bool is_bf) {
        const int k = s.n_slots++;
        s.src[k] = src;
        s.dst[k] = dst;
        if (kind & 1) s.kind0[k >> 6] |= 1ull << (k & 63);
        if (kind & 2) s.kind1[k >> 6] |= 1ull << (k & 63);
        if (is_bf) s.bf[k >> 6] |= 1ull << (k & 63);
    };
    for (int p = 0; p < a.P; ++p) {
        const bool on_time = (a.active >> p) & 1ull, has_stale = (a.valid >> p) & 1ull;
        const void *g = a.g[p];
        if (on_time) {
            if (has_stale) {
                push(a.r[p], nullptr, kHold, false);
                push(g, nullptr, kPair, bf16);
            } else {
                push(g, nullptr, kAdd, bf16);
            }
        } else {
            if (has_stale) push(a.r[p], nullptr, kAdd, false);
            if ((a.store >> p) & 1ull) push(g, a.r[p], kStore, bf16);
        }
    }
    s.w = a.w;
    s.v = a.v;
    s.recv = a.recv;
    s.e0 = a.e0;
    s.n = a.n;
    s.inv_P = a.inv_P;
    s.neg_lr = a.neg_lr;
    s.mu = a.mu;
    s.wd = a.wd;
    s.nesterov = a.nesterov;
    s.stats = a.stats;
    s.xcd_map = 0;
}

// Resident 64-lane wavefronts per CU for the slot kernel (measured optima): with stores of
// late gradients in the same pass few wavefronts are best once there are many streams; a
// pass that only reads (apart from w and v) likes more while one chunk holds all streams.
// What counts is the bytes in flight per CU: a bf16 stream carries half as many per load, so
// the count grows with the share of bf16 streams (all bf16: twice as many wavefronts).
int auto_waves_for_slots(const SlotArgs &s, bool has_stores)
{
    const int n = s.n_slots;
    const int base = has_stores ? (n <= 16 ? 8 : 5) : (n <= 20 ? 10 : 5);
    const int n_bf = __builtin_popcountll(s.bf[0]) + __builtin_popcountll(s.bf[1]);
    // (one chunk with stores: the stores are full-width fp32 whatever the gradient type, and
    // 8 stays the best count - P = 8, bf16, majority: 6.46 against 6.23 TB/s with 12)
    if (n_bf == 0 || n == 0 || (has_stores && n <= 16)) return base;
    // base / (1 - share/2), rounded
    const int waves = (2 * base * n + (2 * n - n_bf) / 2) / (2 * n - n_bf);
    return waves > 16 ? 16 : waves;
}

template <bool BF16, bool FAST>
hipError_t launch_slots(const RoundArgs &a, const Launch &cfg, hipStream_t st)
{
    SlotArgs s;
    build_slots(a, s);
    int bpc = cfg.blocks_per_cu;
    if (bpc == 0) {
        int waves = auto_waves_for_slots(s, a.store != 0);
        // With the by-products a wavefront ends in arithmetic (fp64 squares, DPP sums) during
        // which it has nothing in flight; a little more occupancy covers that (measured: 355 M
        // elements, P = 32, 6 instead of 5: 15.28 against 15.78 ms, 15.08 without by-products;
        // 25.6 M elements, P = 8, 12 instead of 8: 0.287 against 0.296 ms, 0.271 without).
        if (s.stats.stats) waves = waves <= 7 ? waves + 1 : waves == 8 ? 12 : waves;
        bpc = (waves * 64 + cfg.block - 1) / cfg.block;
        if (bpc < 1) bpc = 1;
        // A run whose streams all fit the last-level cache is not an HBM stream: it is bound
        // by latency, and full occupancy is fastest (1 M elements, P = 4: 8.9 against 10 us).
        const long long run_bytes = s.n * (4ll * s.n_slots + 16);
        if (run_bytes < kStateCacheBytes / 2) bpc = -1;
    }
    // one vector per lane, the grid covers the run ("unroll" and "max_blocks" do not apply);
    // always nontemporal (the A/B against plain loads and stores lives in the rank-chunk
    // kernel)
    const long long nvec = slot_nvec<BF16>(s.n);
    long long g = (nvec + cfg.block - 1) / cfg.block;
    if (g < 1) g = 1;
    // this kernel does not stride: a run beyond the thread limit of a grid (more than
    // 2^33 elements) is refused
    if (g * cfg.block > kMaxGridThreads) return hipErrorInvalidValue;
    const unsigned grid = static_cast<unsigned>(g);
    int ch = cfg.chunk;
    if (ch == 0) ch = 16;
    // w, v (and recv) of a run that cannot stay in the 256 MiB last-level cache until the
    // next round are streamed; smaller ones are left to the cache
    const long long state_bytes = s.n * 4 * ((s.w ? 2 : 0) + (s.recv ? 1 : 0));
    const bool nts = cfg.nt_state < 0 ? state_bytes > kStateCacheBytes : cfg.nt_state != 0;
    s.xcd_map = cfg.xcd_map;
    if (s.stats.stats) {
        // the by-products exist for the default chunk size only
        if (ch != 16) return hipErrorInvalidValue;
        s.stats.n_records = (static_cast<long long>(grid) * cfg.block + 63) / 64;
        return nts ? launch_capped(slot_kernel<BF16, FAST, true, true, 16, true>, s, bpc, cfg, grid, st)
                   : launch_capped(slot_kernel<BF16, FAST, true, false, 16, true>, s, bpc, cfg, grid, st);
    }
    switch (ch * 2 + (nts ? 1 : 0)) {
    case 16: return launch_capped(slot_kernel<BF16, FAST, true, false, 8, false>, s, bpc, cfg, grid, st);
    case 17: return launch_capped(slot_kernel<BF16, FAST, true, true, 8, false>, s, bpc, cfg, grid, st);
    case 32: return launch_capped(slot_kernel<BF16, FAST, true, false, 16, false>, s, bpc, cfg, grid, st);
    case 33: return launch_capped(slot_kernel<BF16, FAST, true, true, 16, false>, s, bpc, cfg, grid, st);
    case 64: return launch_capped(slot_kernel<BF16, FAST, true, false, 32, false>, s, bpc, cfg, grid, st);
    case 65: return launch_capped(slot_kernel<BF16, FAST, true, true, 32, false>, s, bpc, cfg, grid, st);
    default: return hipErrorInvalidValue;   // more streams per chunk exceed the scalar registers
    }
}

template <bool BF16, bool FAST, bool NT, int U>
hipError_t launch_round_ch(const RoundArgs &a, const Launch &cfg, unsigned grid, hipStream_t st)
{
    // ranks per chunk: all loads of a chunk are in flight together.  Few processes take
    // a short chunk so that the rank loop is not padded with dummy streams.
    int ch = cfg.chunk;
    if (ch == 0) ch = a.P <= 4 ? 4 : 8;
    switch (ch) {
    case 4: return launch_capped(round_kernel<BF16, FAST, NT, U, 4, 256>, a, cfg, grid, st);
    case 8: return launch_capped(round_kernel<BF16, FAST, NT, U, 8, 256>, a, cfg, grid, st);
    case 16:
        // combinations that would spill registers are not built
        if constexpr (BF16 && U > 1) return hipErrorInvalidValue;
        else return launch_capped(round_kernel<BF16, FAST, NT, U, 16, 256>, a, cfg, grid, st);
    case 32:
        if constexpr (BF16 || U > 1) return hipErrorInvalidValue;
        else return launch_capped(round_kernel<BF16, FAST, NT, 1, 32, 256>, a, cfg, grid, st);
    default: return hipErrorInvalidValue;
    }
}

template <bool BF16, bool FAST, bool NT>
hipError_t launch_round_u(const RoundArgs &a, const Launch &cfg, unsigned grid, hipStream_t st)
{
    switch (cfg.unroll) {
    case 1: return launch_round_ch<BF16, FAST, NT, 1>(a, cfg, grid, st);
    case 2: return launch_round_ch<BF16, FAST, NT, 2>(a, cfg, grid, st);
    default: return hipErrorInvalidValue;
    }
}

template <bool BF16, bool FAST>
hipError_t launch_round_nt(const RoundArgs &a, const Launch &cfg, unsigned grid, hipStream_t st)
{
    return cfg.nontemporal ? launch_round_u<BF16, FAST, true>(a, cfg, grid, st)
                           : launch_round_u<BF16, FAST, false>(a, cfg, grid, st);
}

unsigned grid_for(long long nvec, long long per_block, int max_blocks)
{
    long long g = (nvec + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (max_blocks > 0 && g > max_blocks) g = max_blocks;
    // the kernels stride, so a cap is safe; workgroups have at most 256 threads
    if (g > kMaxGridThreads / 256) g = kMaxGridThreads / 256;
    return static_cast<unsigned>(g);
}

}  // namespace

hipError_t launch_round(const RoundArgs &a, bool bf16, bool fast, const Launch &cfg,
                        hipStream_t stream)
{
    if (a.n <= 0) return hipSuccess;
    const long long nvec = a.n / (bf16 ? 8 : 4);
    const unsigned grid = grid_for(nvec, static_cast<long long>(cfg.block) * cfg.unroll,
                                   cfg.max_blocks);
    if (cfg.compact) {
        if (bf16)
            return fast ? launch_slots<true, true>(a, cfg, stream)
                        : launch_slots<true, false>(a, cfg, stream);
        return fast ? launch_slots<false, true>(a, cfg, stream)
                    : launch_slots<false, false>(a, cfg, stream);
    }
    if (bf16)
        return fast ? launch_round_nt<true, true>(a, cfg, grid, stream)
                    : launch_round_nt<true, false>(a, cfg, grid, stream);
    return fast ? launch_round_nt<false, true>(a, cfg, grid, stream)
                : launch_round_nt<false, false>(a, cfg, grid, stream);
}

template <bool BF16, int V>
hipError_t launch_carry_v(const CarryArgs &a, const Launch &cfg, hipStream_t stream)
{
    const long long nvec = a.n / 4;
    const long long tile = static_cast<long long>(cfg.carry_block) * V;
    long long bpp = (nvec + tile - 1) / tile;
    if (bpp < 1) bpp = 1;
    // a grid may hold fewer than 2^32 threads in all; beyond that the kernel strides
    const long long cap = kMaxGridThreads / cfg.carry_block / a.count;
    if (bpp > cap) bpp = cap;
    const unsigned grid = static_cast<unsigned>(bpp) * static_cast<unsigned>(a.count);
    Launch l = cfg;
    l.block = cfg.carry_block;
    return launch_capped(carry_kernel<BF16, V>, a, cfg.carry_blocks_per_cu, l, grid, stream,
                         static_cast<unsigned>(bpp));
}

template <bool BF16>
hipError_t launch_carry_t(const CarryArgs &a, const Launch &cfg, hipStream_t stream)
{
    switch (cfg.carry_vec) {
    case 1: return launch_carry_v<BF16, 1>(a, cfg, stream);
    case 2: return launch_carry_v<BF16, 2>(a, cfg, stream);
    case 4: return launch_carry_v<BF16, 4>(a, cfg, stream);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_carry(const CarryArgs &a, bool bf16, const Launch &cfg, hipStream_t stream)
{
    if (a.n <= 0 || a.count <= 0) return hipSuccess;
    return bf16 ? launch_carry_t<true>(a, cfg, stream) : launch_carry_t<false>(a, cfg, stream);
}

long long slot_records(long long n, bool bf16, int block)
{
    const long long nvec = bf16 ? slot_nvec<true>(n) : slot_nvec<false>(n);
    long long g = (nvec + block - 1) / block;
    if (g < 1) g = 1;
    return (g * block + 63) / 64;
}

int slot_tail(long long n, bool bf16)
{
    return static_cast<int>(n - (bf16 ? slot_nvec<true>(n) : slot_nvec<false>(n)) * 4);
}

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
    if (g > kMaxGridThreads / 64) g = kMaxGridThreads / 64;   // the kernel strides
    if (bf16) hipLaunchKernelGGL(stash_kernel<true>, dim3(static_cast<unsigned>(g)), dim3(64), 0, stream, a);
    else hipLaunchKernelGGL(stash_kernel<false>, dim3(static_cast<unsigned>(g)), dim3(64), 0, stream, a);
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
    const dim3 grid(grid_for(a.n / 4, 64, cfg.max_blocks)), block(64);
    const bool nt = a.n * 8 > kStateCacheBytes;
    if (fast) {
        if (nt) hipLaunchKernelGGL((sgd_kernel<true, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((sgd_kernel<true, false>), grid, block, 0, stream, a);
    } else {
        if (nt) hipLaunchKernelGGL((sgd_kernel<false, true>), grid, block, 0, stream, a);
        else hipLaunchKernelGGL((sgd_kernel<false, false>), grid, block, 0, stream, a);
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

hipError_t launch_copy(void *dst, const void *src, long long nbytes, hipStream_t stream)
{
    const long long nvec = nbytes / 16;
    if (nvec <= 0) return hipSuccess;
    // the fastest plain copy found on MI355X: 64-thread workgroups, one vector per lane
    long long g = (nvec + 63) / 64;
    if (g > kMaxGridThreads / 64) g = kMaxGridThreads / 64;   // the kernel strides
    hipLaunchKernelGGL(copy_kernel, dim3(static_cast<unsigned>(g)), dim3(64), 0, stream,
                       static_cast<f32x4 *>(dst), static_cast<const f32x4 *>(src), nvec);
    return hipGetLastError();
}

hipError_t launch_read(const void *src, long long nbytes, float *sink, hipStream_t stream)
{
    const long long nvec = nbytes / 16;
    if (nvec <= 0) return hipSuccess;
    hipLaunchKernelGGL(read_kernel, dim3(grid_for(nvec, 256, 256 * 32)), dim3(256), 0, stream,
                       static_cast<const f32x4 *>(src), nvec, sink);
    return hipGetLastError();
}

}  // namespace eager
