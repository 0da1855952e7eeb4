// Device-side helpers shared by the kernel files: vector types and nontemporal accesses, the
// update rule, the per-bucket statistics (DPP wavefront sums, records) and the launch helper that
// caps occupancy.  Everything here has internal linkage; not part of the public ABI.
#pragma once

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

// One gradient element of a ragged tail (fewer elements than a vector; scalar code, at most 7
// elements per launch).
template <bool BF16>
__device__ __forceinline__ float load_grad_scalar(const void *g, long long i)
{
    if (BF16) {
        const unsigned short h = static_cast<const unsigned short *>(g)[i];
        return __uint_as_float(static_cast<unsigned>(h) << 16);
    }
    return static_cast<const float *>(g)[i];
}

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

template <typename K, typename A, typename... Extra>
hipError_t launch_capped(K kernel, const A &a, int bpc, const Launch &cfg, dim3 grid,
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
    hipLaunchKernelGGL(kernel, grid, dim3(cfg.block), lds, st, a, extra...);
    return hipGetLastError();
}

inline unsigned grid_for(long long nvec, long long per_block, int max_blocks)
{
    long long g = (nvec + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (max_blocks > 0 && g > max_blocks) g = max_blocks;
    // the kernels stride, so a cap is safe; workgroups have at most 256 threads
    if (g > kMaxGridThreads / 256) g = kMaxGridThreads / 256;
    return static_cast<unsigned>(g);
}

}  // namespace
}  // namespace eager
