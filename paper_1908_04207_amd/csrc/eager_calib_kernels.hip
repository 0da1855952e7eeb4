// Plain streaming kernels of known traffic: they calibrate what the device reaches (and what the
// profiler's byte counters read) against the round kernels.  copy and read are one stream in,
// one out / one stream in; mix reads n_read streams and writes n_write streams with the access
// shape of a round - a lane owns 16 bytes of every stream, one tile per wavefront, the loads of
// up to 16 streams issued before the first use, nontemporal, occupancy capped through an unused
// LDS allocation - but without a round's slot list, masks or update rule: what a plain kernel
// with a round's mix of streams reaches.
#include "eager_device.h"

namespace eager {
namespace {

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

typedef const MixArgs __attribute__((address_space(4))) KMixArgs;

// C streams from slot k0 on: all loads first, then the adds.  A half-width stream holds 8 bytes
// per lane-vector: lanes 2k and 2k+1 load the same 16-byte piece and each keeps its half (the
// access shape of a bf16 gradient stream in a round).
template <int C>
__device__ __forceinline__ f32x4 mix_chunk(KMixArgs &a, int k0, long long vi, f32x4 s)
{
    const unsigned long long half = a.half >> k0;
    u32x4 raw[C];
#pragma unroll
    for (int j = 0; j < C; ++j) {
        const char *sp = static_cast<const char *>(a.src[k0 + j]);
        const bool h = (half >> j) & 1ull;
        raw[j] = ld_u4<true>(sp + (h ? (vi >> 1) * 16 : vi * 16));
    }
#pragma unroll
    for (int j = 0; j < C; ++j) {
        const bool h = (half >> j) & 1ull;
        u32x4 x = raw[j];
        if (h) {
            const bool odd = (vi & 1) != 0;
            x.x = odd ? x.z : x.x;
            x.y = odd ? x.w : x.y;
            x.z = 0u;
            x.w = 0u;
        }
        s = s + __builtin_bit_cast(f32x4, x);
    }
    return s;
}
template <int R>
__device__ __forceinline__ f32x4 mix_rest(KMixArgs &a, int k0, int rem, long long vi, f32x4 s)
{
    if constexpr (R >= 1) {
        if (rem == R) return mix_chunk<R>(a, k0, vi, s);
        return mix_rest<R - 1>(a, k0, rem, vi, s);
    }
    return s;
}

__global__ __launch_bounds__(64) void mix_kernel(const MixArgs)
{
    KMixArgs &a = kernarg<MixArgs>();
    constexpr int CH = 16;
    const long long vi = static_cast<long long>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (vi >= a.nvec) return;
    f32x4 s = (f32x4)(0.0f);
    const int n = a.n_read;
#pragma unroll
    for (int c = 0; c < kMixMaxRead / CH; ++c)
        if ((c + 1) * CH <= n) s = mix_chunk<CH>(a, c * CH, vi, s);
    s = mix_rest<CH - 1>(a, n / CH * CH, n % CH, vi, s);
    asm volatile("" : "+v"(s) : : "memory");
    for (int w = 0; w < a.n_write; ++w)
        __builtin_nontemporal_store(s, static_cast<f32x4 *>(a.dst[w]) + vi);
    if (a.n_write == 0 && s.x == 123.456f) *static_cast<float *>(a.sink) = s.x;
}

}  // namespace

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

hipError_t launch_mix(const MixArgs &a, int waves_per_cu, hipStream_t stream)
{
    if (a.nvec <= 0) return hipSuccess;
    const long long g = (a.nvec + 63) / 64;
    if (g * 64 > kMaxGridThreads) return hipErrorInvalidValue;    // the kernel does not stride
    Launch l;
    l.block = 64;
    return launch_capped(mix_kernel, a, waves_per_cu > 0 ? waves_per_cu : -1, l,
                         static_cast<unsigned>(g), stream);
}

}  // namespace eager
