// The earlier form of the round kernel, kept for comparison (launch option "compact" = 0): the P
// processes are taken in fixed chunks of ranks; a stream that must not be read gets a stand-in
// address instead of being left out.  Same arithmetic, same bits as slot_kernel
// (eager_round_kernels.hip), which replaced it as the default: it cannot drop the streams a round
// does not need, and with bf16 gradients its lanes own 8 elements, so its fp32 streams are read and
// written at a 32-byte stride.
#include "eager_device.h"

namespace eager {
namespace {

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

// Ragged tail of the rank-chunk kernel: plain scalar code, fixed order in both modes.
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

// Resident workgroups per CU when the caller leaves the choice to the library: measured
// optima of the rank-chunk kernel with 64-thread workgroups for 1, 2 and 4 chunks of 8.
int auto_blocks_per_cu(int P, int block, bool bf16)
{
    const int chunks = (P + 7) / 8;
    const int waves = chunks <= 1 ? 10 : chunks == 2 ? (bf16 ? 8 : 5) : 6;
    const int b = (waves * 64 + block - 1) / block;
    return b < 1 ? 1 : b;
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

}  // namespace

hipError_t launch_round_chunks(const RoundArgs &a, bool bf16, bool fast, const Launch &cfg,
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

}  // namespace eager
