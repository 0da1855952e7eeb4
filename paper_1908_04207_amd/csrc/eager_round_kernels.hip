// gfx950 kernels of the eager-SGD round: partial-allreduce arithmetic with stale-gradient
// carry (paper Section 5, walk-through of Fig. 7), the 1/P average (Algorithm 2 line 6)
// and the momentum-SGD update rule (lines 7-8) in ONE pass over HBM.
//
// The path is a pure stream: per element <= 2P adds, one multiply and two FMAs against
// >= 4P bytes, so HBM bandwidth is the only roofline that matters and there is no
// contraction for the matrix cores.  Design for CDNA4:
//   * slot_kernel: the host compacts the round into a list of streams that
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
//   * optional per-bucket norms as by-products of the same pass: DPP sums inside wavefronts,
//     one record per wavefront (the helpers live in eager_device.h, the kernels that finish
//     them in eager_aux_kernels.hip).
#include "eager_device.h"

#include <algorithm>

namespace eager {
namespace {

// The round as a list of streams ("slots"), each with one action, in summation order.  A
// chunk of C slots is C loads issued back to back, then the adds, then the stores; the list
// is consumed in chunks of CH and one remainder chunk of its exact size, so that no load is
// issued for a stream the round does not need.
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
// spills scalar registers.  The grid always covers the run.  (Two consecutive tiles per
// wavefront, every stream requested 2 KiB at a time, were measured as well: 3-6 % faster in a
// plain kernel of 16-34 read and 2 write streams, but on the rounds themselves the same with
// 18 streams and 2-5 % slower with 13 or 28.)
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

// R_p <- G_p for the late processes, as a plain copy: pair after pair (blockIdx.y is the
// pair, and workgroups are dealt out x first), so that at any time the device streams one
// source and one destination.  A copy of few streams runs near the read-only rate on MI355X,
// whereas the same bytes written as 8-31 interleaved streams next to the reduction's reads
// cost 10-15 %.  A lane owns 4 elements: every store instruction of a wavefront writes one
// contiguous kilobyte (a bf16 source is read 8 bytes per lane and widened).  No loop and no
// division: a wavefront lives for one load and one store, so whatever stands before its load
// counts (bf16 source, 1.1e9 elements per pair: 6.73 TB/s in this form, 6.62 with the pair
// taken from blockIdx.x by a division, 6.46 with a striding loop around the body).
template <bool BF16, int V>
__global__ __launch_bounds__(256) void carry_kernel(const CarryArgs a)
{
    const unsigned pair = blockIdx.y;
    const long long nvec = a.n / 4;
    const char *src = static_cast<const char *>(a.src[pair]);
    float *dst = a.dst[pair];
    // a workgroup copies V * blockDim consecutive lane-vectors: all loads first, then the stores
    const long long base = static_cast<long long>(blockIdx.x) * blockDim.x * V + threadIdx.x;
    f32x4 x[V];
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const long long vi = base + static_cast<long long>(k) * blockDim.x;
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
        const long long vi = base + static_cast<long long>(k) * blockDim.x;
        if (vi < nvec) st_f4<true>(dst + a.e0 + vi * 4, x[k]);
    }
    const long long rem = a.n - nvec * 4;
    if (blockIdx.x == 0 && static_cast<long long>(threadIdx.x) < rem) {
        const long long i = a.e0 + nvec * 4 + threadIdx.x;
        dst[i] = load_grad_scalar<BF16>(src, i);
    }
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
    const int n_bf = __builtin_popcountll(s.bf[0]) + __builtin_popcountll(s.bf[1]);
    if (has_stores && n <= 16) {
        // One chunk with stores: about 84 KiB of loads in flight per CU, between 8 and 12
        // wavefronts.  A wavefront requests a KiB per fp32 stream (w and v included), half of
        // that per bf16 stream.  Measured, 2e8 elements: 3 fp32 streams 6.64 TB/s with 12
        // against 6.17 with 8; 4 bf16 + 1 fp32 streams 6.64 against 5.72; 8 bf16 + 1 fp32
        // (2.6e7 elements) 6.94 against 6.43; from 9 fp32 streams on 8 stays the best count.
        const int half_kib = 2 * (n - n_bf) + n_bf + 4;
        const int waves = (2 * 84 + half_kib / 2) / half_kib;
        return waves < 8 ? 8 : waves > 12 ? 12 : waves;
    }
    const int base = has_stores ? 5 : (n <= 20 ? 10 : 5);
    if (n_bf == 0 || n == 0) return base;
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
    // one vector per lane, the grid covers the run; always nontemporal
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
    default: return hipErrorInvalidValue;   // more streams per chunk exceed the scalar registers
    }
}

}  // namespace

hipError_t launch_round(const RoundArgs &a, bool bf16, bool fast, const Launch &cfg,
                        hipStream_t stream)
{
    if (a.n <= 0) return hipSuccess;
    if (bf16)
        return fast ? launch_slots<true, true>(a, cfg, stream)
                    : launch_slots<true, false>(a, cfg, stream);
    return fast ? launch_slots<false, true>(a, cfg, stream)
                : launch_slots<false, false>(a, cfg, stream);
}

template <bool BF16, int V>
hipError_t launch_carry_v(const CarryArgs &a, const Launch &cfg, hipStream_t stream)
{
    const long long nvec = a.n / 4;
    const long long tile = static_cast<long long>(cfg.carry_block) * V;
    long long bpp = (nvec + tile - 1) / tile;     // workgroups per pair: they cover it
    if (bpp < 1) bpp = 1;
    // A grid may hold fewer than 2^32 threads in all: the pairs go into as many launches as it
    // takes.  (One pair always fits: a call covers at most 2^33 elements per run.)
    const long long limit = kMaxGridThreads / cfg.carry_block;
    if (bpp > limit) return hipErrorInvalidValue;
    long long pairs_per_launch = std::min<long long>(limit / bpp, 65535);
    Launch l = cfg;
    l.block = cfg.carry_block;
    for (int first = 0; first < a.count; first += static_cast<int>(pairs_per_launch)) {
        CarryArgs part = a;
        part.count = static_cast<int>(std::min<long long>(pairs_per_launch, a.count - first));
        for (int k = 0; k < part.count; ++k) {
            part.src[k] = a.src[first + k];
            part.dst[k] = a.dst[first + k];
        }
        const hipError_t e = launch_capped(carry_kernel<BF16, V>, part, cfg.carry_blocks_per_cu, l,
                                           dim3(static_cast<unsigned>(bpp),
                                                static_cast<unsigned>(part.count)),
                                           stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
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

}  // namespace eager
