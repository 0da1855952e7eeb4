// gfx950 kernels of the eager-SGD round: partial-allreduce arithmetic with stale-gradient
// carry (paper Section 5, walk-through of Fig. 7), the 1/P average (Algorithm 2 line 6)
// and the momentum-SGD update rule (lines 7-8) in ONE pass over HBM.
//
// The path is a pure stream: per element <= 2P adds, one multiply and two FMAs against
// >= 4P bytes, so HBM bandwidth is the only roofline that matters and there is no
// contraction for the matrix cores.  Design for CDNA4:
//   * a thread owns one 16-byte vector of each gradient stream (4 fp32 or 8 bf16
//     elements), so a 64-lane wavefront reads 1 KiB contiguous per stream per load;
//   * the P gradient loads and the loads of the non-empty send buffers of a chunk of
//     ranks are all issued before the first add, which keeps (2*CH+2) x 16 B per lane in
//     flight - that, not occupancy, is what covers HBM latency;
//   * which streams are read or written is decided from two 64-bit masks that live in
//     scalar registers: every branch is uniform, empty send buffers cost no bytes, the
//     send buffer of an on-time process is "cleared" by a flag on the host, not by
//     writing zeros;
//   * the accumulator stays in fp32 registers; in fixed-order mode contributions are
//     added in ascending rank order from +0.0f with contraction off, so the result is
//     defined bit for bit; fast mode sums a chunk as a tree and lets the compiler fuse.
#include "eager_internal.h"

namespace eager {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

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
__device__ __forceinline__ void round_vectors(const RoundArgs &a, const long long (&e)[U])
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
                const f32x4 vo = vo_[u][k];
                const f32x4 wo = wo_[u][k];
                f32x4 vn, wn;
                if (FAST) {
#pragma clang fp contract(fast)
                    vn = a.mu * vo + avg;
                    wn = a.neg_lr * vn + wo;
                } else {
                    vn.x = __builtin_fmaf(a.mu, vo.x, avg.x);
                    vn.y = __builtin_fmaf(a.mu, vo.y, avg.y);
                    vn.z = __builtin_fmaf(a.mu, vo.z, avg.z);
                    vn.w = __builtin_fmaf(a.mu, vo.w, avg.w);
                    wn.x = __builtin_fmaf(a.neg_lr, vn.x, wo.x);
                    wn.y = __builtin_fmaf(a.neg_lr, vn.y, wo.y);
                    wn.z = __builtin_fmaf(a.neg_lr, vn.z, wo.z);
                    wn.w = __builtin_fmaf(a.neg_lr, vn.w, wo.w);
                }
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
__device__ __forceinline__ void round_scalar(const RoundArgs &a, long long i)
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
        const float vn = __builtin_fmaf(a.mu, a.v[i], avg);
        a.v[i] = vn;
        a.w[i] = __builtin_fmaf(a.neg_lr, vn, a.w[i]);
    }
}

template <bool BF16, bool FAST, bool NT, int U, int CH, int LB>
__global__ __launch_bounds__(LB) void round_kernel(const RoundArgs a)
{
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

// R_p <- G_p for the late processes, as a plain copy: pair after pair (blockIdx is
// pair-major), so that at any time the device streams one source and one destination.
// A copy of few streams runs near the read-only rate on MI355X, whereas the same bytes
// written as 8-31 interleaved streams next to the reduction's reads cost 10-15 %.
template <bool BF16>
__global__ __launch_bounds__(256) void carry_kernel(const CarryArgs a, unsigned blocks_per_pair)
{
    constexpr int W = BF16 ? 8 : 4;
    const unsigned pair = blockIdx.x / blocks_per_pair;
    const unsigned blk = blockIdx.x - pair * blocks_per_pair;
    const long long nvec = a.n / W;
    const char *src = static_cast<const char *>(a.src[pair]);
    float *dst = a.dst[pair];
    const long long stride = static_cast<long long>(blocks_per_pair) * blockDim.x;
    for (long long vi = static_cast<long long>(blk) * blockDim.x + threadIdx.x; vi < nvec;
         vi += stride) {
        const long long e = a.e0 + vi * W;
        const u32x4 g = ld_u4<true>(src + e * (BF16 ? 2 : 4));
        if (BF16) {
            st_f4<true>(dst + e, widen_lo(g, 0));
            st_f4<true>(dst + e + 4, widen_lo(g, 1));
        } else {
            st_f4<true>(dst + e, __builtin_bit_cast(f32x4, g));
        }
    }
    const long long rem = a.n - nvec * W;
    if (blk == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * W + threadIdx.x;
        dst[i] = load_grad_scalar<BF16>(src, i);
    }
}

template <bool FAST>
__global__ __launch_bounds__(256) void sgd_kernel(const SgdArgs a)
{
    const long long nvec = a.n / 4;
    const long long stride = static_cast<long long>(gridDim.x) * blockDim.x;
    for (long long vi = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x; vi < nvec;
         vi += stride) {
        const long long i = a.e0 + vi * 4;
        const f32x4 u = ld_f4<true>(a.u + i);
        const f32x4 vo = ld_f4<false>(a.v + i);
        const f32x4 wo = ld_f4<false>(a.w + i);
        f32x4 vn, wn;
        if (FAST) {
#pragma clang fp contract(fast)
            vn = a.mu * vo + u;
            wn = a.neg_lr * vn + wo;
        } else {
            vn.x = __builtin_fmaf(a.mu, vo.x, u.x);
            vn.y = __builtin_fmaf(a.mu, vo.y, u.y);
            vn.z = __builtin_fmaf(a.mu, vo.z, u.z);
            vn.w = __builtin_fmaf(a.mu, vo.w, u.w);
            wn.x = __builtin_fmaf(a.neg_lr, vn.x, wo.x);
            wn.y = __builtin_fmaf(a.neg_lr, vn.y, wo.y);
            wn.z = __builtin_fmaf(a.neg_lr, vn.z, wo.z);
            wn.w = __builtin_fmaf(a.neg_lr, vn.w, wo.w);
        }
        st_f4<false>(a.v + i, vn);
        st_f4<false>(a.w + i, wn);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        const float vn = __builtin_fmaf(a.mu, a.v[i], a.u[i]);
        a.v[i] = vn;
        a.w[i] = __builtin_fmaf(a.neg_lr, vn, a.w[i]);
    }
}

__global__ __launch_bounds__(256) void copy_kernel(f32x4 *dst, const f32x4 *src, long long nvec)
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

// Resident workgroups per CU when the caller leaves the choice to the library: measured
// optima with 64-thread workgroups for 1, 2 and 4 rank chunks of 8.
int auto_blocks_per_cu(int P, int block)
{
    const int chunks = (P + 7) / 8;
    const int waves = chunks <= 1 ? 10 : chunks == 2 ? 5 : 6;
    const int b = (waves * 64 + block - 1) / block;
    return b < 1 ? 1 : b;
}

template <typename K>
hipError_t launch_capped(K kernel, const RoundArgs &a, const Launch &cfg, unsigned grid,
                         hipStream_t st)
{
    unsigned lds = 0;
    const int bpc = cfg.blocks_per_cu == 0 ? auto_blocks_per_cu(a.P, cfg.block) : cfg.blocks_per_cu;
    if (bpc > 0) {
        lds = static_cast<unsigned>(kLdsPerCu / bpc) & ~2047u;
        static bool raised = false;   // one flag per kernel instantiation
        if (!raised) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                               hipFuncAttributeMaxDynamicSharedMemorySize,
                                               kLdsPerCu);
            if (e != hipSuccess) return e;
            raised = true;
        }
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(cfg.block), lds, st, a);
    return hipGetLastError();
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
    if (g > 0x7fffffffLL) g = 0x7fffffffLL;   // the kernels stride, so a cap is safe
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
    if (bf16)
        return fast ? launch_round_nt<true, true>(a, cfg, grid, stream)
                    : launch_round_nt<true, false>(a, cfg, grid, stream);
    return fast ? launch_round_nt<false, true>(a, cfg, grid, stream)
                : launch_round_nt<false, false>(a, cfg, grid, stream);
}

hipError_t launch_carry(const CarryArgs &a, bool bf16, hipStream_t stream)
{
    if (a.n <= 0 || a.count <= 0) return hipSuccess;
    const long long nvec = a.n / (bf16 ? 8 : 4);
    long long bpp = (nvec + 255) / 256;
    if (bpp < 1) bpp = 1;
    if (bpp > 0x7fffffffLL / a.count) bpp = 0x7fffffffLL / a.count;   // the kernel strides
    const unsigned grid = static_cast<unsigned>(bpp) * static_cast<unsigned>(a.count);
    if (bf16)
        hipLaunchKernelGGL(carry_kernel<true>, dim3(grid), dim3(256), 0, stream, a,
                           static_cast<unsigned>(bpp));
    else
        hipLaunchKernelGGL(carry_kernel<false>, dim3(grid), dim3(256), 0, stream, a,
                           static_cast<unsigned>(bpp));
    return hipGetLastError();
}

hipError_t launch_sgd(const SgdArgs &a, bool fast, const Launch &cfg, hipStream_t stream)
{
    if (a.n <= 0) return hipSuccess;
    const unsigned grid = grid_for(a.n / 4, 256, cfg.max_blocks);
    if (fast) hipLaunchKernelGGL(sgd_kernel<true>, dim3(grid), dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(sgd_kernel<false>, dim3(grid), dim3(256), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_copy(void *dst, const void *src, long long nbytes, hipStream_t stream)
{
    const long long nvec = nbytes / 16;
    if (nvec <= 0) return hipSuccess;
    hipLaunchKernelGGL(copy_kernel, dim3(grid_for(nvec, 256, 256 * 32)), dim3(256), 0, stream,
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
