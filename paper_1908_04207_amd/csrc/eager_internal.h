// Internal interface between the host side of the library (argument checking, context
// state, run building) and the gfx950 kernels.  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace eager {

constexpr int kMaxP = 64;

// Optional by-products of a round, per bucket (same layout as eager_bucket_stats of the public
// header): squared norm of the averaged update and of the parameters before the update (finite
// elements only), number of non-finite elements of the update.
struct BucketStats {
    double sumsq_update;
    double sumsq_params;
    unsigned long long nonfinite;
    float rate;
    unsigned reserved;
};

// What one wavefront of the round kernel leaves for the finishing kernel: the sums over its
// 256 elements if they all lie in one bucket (bucket >= 0); bucket = -1 if they lie in several
// (then every lane has left a record of its own in block `nf` of the lane records); bucket =
// -2 if the wavefront holds no element.  Lane records and the records of the ragged tail
// (at most 7 single elements, in the block after the last bucket's) have the same layout.
struct StatsRecord {
    double ssu, ssw;
    int bucket;
    unsigned nf;
    long long pad;
};

struct StatsArgs {
    const long long *table;      // device: start, end of every bucket (2 per bucket)
    BucketStats *stats;          // device: one per bucket
    StatsRecord *records;        // device: one per wavefront of the round kernel
    StatsRecord *lane_records;   // device: (n_buckets + 1) blocks of 64
    int tail_count;              // elements of the run's ragged tail (0..7)
    long long e0;                // first element of the run
    long long n_records;         // wavefronts the round kernel was launched with
    int b_lo, b_hi;              // buckets of the run
    int n_buckets;
    // layer-wise rate, written next to the totals when want_rate is set:
    // trust * |w| / (|u| + wd * |w| + eps), or 1 where a norm is zero
    int want_rate;
    float trust, wd, eps;
    // A bucket with many records is added up by `slices` workgroups first, one partial each
    // (partials[bucket * kStatsMaxSlices + slice]); 1: the finishing kernel reads the records.
    StatsRecord *partials;
    int slices;
};
constexpr int kStatsMaxSlices = 64;
constexpr long long kStatsRecordsPerSlice = 4096;

// Capacity of the entry point that allocates nothing: its statistics workspace is a fixed
// device array inside the library (bucket table, one record per 256 elements, lane records,
// partials - the layout of the caller-provided workspace), so the context may hold at most this
// many buckets and span at most this many elements.
constexpr int kStaticMaxBuckets = 512;
constexpr long long kStaticMaxElements = 1ll << 27;
constexpr long long kStaticMaxRecords = kStaticMaxElements / 256 + 8;
constexpr long long kStaticScratchBytes =
    kStaticMaxBuckets * 16ll +
    (kStaticMaxRecords + (kStaticMaxBuckets + 1ll) * 64 + kStaticMaxBuckets * 1ll * kStatsMaxSlices) * 32;

// Bucket table entries handed to the device in one kernel-argument block.
constexpr int kTableChunk = 120;
struct TableArgs {
    long long *table;            // device: start, end of every bucket
    int first, count;            // buckets [first, first + count) are written
    long long start_end[2 * kTableChunk];
};

// Everything one launch of the round kernel needs, passed by value in the kernel
// argument segment: the P gradient and send-buffer bases stay in scalar registers and
// every per-rank decision is uniform across the grid.
struct RoundArgs {
    const void *g[kMaxP];        // G_p arena bases (fp32 or bf16)
    float *r[kMaxP];             // R_p arena bases (fp32)
    unsigned long long active;   // bit p: process p is on time in this round
    unsigned long long valid;    // bit p: R_p holds an undelivered gradient
    unsigned long long gload;    // bit p: this launch reads G_p (every process that has a gradient
                                 // when fused; only on-time processes when the carry runs as
                                 // its own kernel)
    unsigned long long store;    // bit p: this launch stores G_p into R_p (late processes when
                                 // fused; none otherwise)
    float *w;                    // parameters (NULL: no update rule)
    float *v;                    // momentum
    float *recv;                 // receive buffer (NULL: not wanted)
    long long e0;                // first element of the run (arena index)
    long long n;                 // elements in the run
    int P;
    int elem_bytes;              // bytes per gradient element: 4 (fp32) or 2 (bf16)
    float inv_P;                 // 1.0f / (float)P
    float neg_lr;                // -lr
    float mu;
    float wd;                    // weight decay (0: none)
    int nesterov;                // 1: Nesterov momentum
    StatsArgs stats;             // stats.stats == NULL: no by-products
};

// The same round as the kernel takes it: a list of streams.  Slot k is one stream and one
// action; slots are listed in the order in which they enter the sum (ascending rank, send
// buffer before gradient):
//   ADD    s = s + x                       (a pending R_p of a late process, or the G_p
//                                           of an on-time process with an empty buffer)
//   HOLD   c = x                           (R_p of an on-time process ...)
//   PAIR   s = s + (c + x)                 (... followed by its G_p)
//   STORE  dst <- x, nothing added         (G_p of a late process, fused mode only)
// Streams that need not be read do not appear at all, so no load is wasted.  A stream is
// fp32 (send buffers; fp32 gradients) or bf16 (bf16 gradients); a lane owns 4 consecutive
// elements of every stream either way.
constexpr int kMaxSlots = 2 * kMaxP;
enum SlotKind { kAdd = 0, kHold = 1, kPair = 2, kStore = 3 };
struct SlotArgs {
    const void *src[kMaxSlots];        // arena bases
    float *dst[kMaxSlots];             // meaningful for STORE slots only
    unsigned long long kind0[2];       // bit k: low bit of the kind of slot k
    unsigned long long kind1[2];       // bit k: high bit
    unsigned long long bf[2];          // bit k: the stream of slot k is bf16
    int n_slots;
    float *w, *v, *recv;
    long long e0, n;
    float inv_P, neg_lr, mu, wd;
    int nesterov;
    int xcd_map;                       // 1: every XCD takes a contiguous eighth of the run
    StatsArgs stats;
};

// The carry as a kernel of its own: R_p <- G_p for every late process, one (source,
// destination) pair after the other.
struct CarryArgs {
    const void *src[kMaxP];      // G_p arena bases of the late processes
    float *dst[kMaxP];           // their R_p arena bases
    int count;                   // number of pairs
    long long e0;                // first element of the run
    long long n;                 // elements in the run
};

// A gradient finished after its round: R <- G (empty send buffer) or R <- R + G.
struct StashArgs {
    const void *g;               // gradient arena base of the process
    float *r;                    // its send-buffer arena base
    long long e0, n;             // run
    int accumulate;              // 1: the send buffer holds an undelivered gradient
};

// Several weight views at once (a weight view per process, for processes that lag by more
// than one round): the update rule applied to every listed view from one read of u, or
// every view replaced by the average of all of them.
struct ViewsArgs {
    float *w[kMaxP];             // parameter views
    float *v[kMaxP];             // momentum views (update rule only)
    const float *u;              // averaged update (update rule only)
    int n_views;
    long long e0, n;
    float neg_lr, mu, wd, inv_views;
    int nesterov;
};

struct SgdArgs {
    const float *u;
    float *w;
    float *v;
    long long e0;
    long long n;
    float neg_lr;
    float mu;
    float wd;
    int nesterov;
};

struct Launch {
    int block = 64;        // threads per workgroup
    int chunk = 0;         // streams whose loads are in flight together; 0: 16
    int split = 0;         // 0: chosen from the round; 1: one fused kernel; 2: reduce+update
                           // kernel followed by a carry (copy) kernel
    int blocks_per_cu = 0; // 0: chosen from the round; -1: no cap; else max workgroups resident per CU
    int nt_state = -1;     // w, v, recv nontemporal: -1 chosen from their size, 0 no, 1 yes
    int xcd_map = 0;       // slot kernel: 1 = contiguous eighth of the run per XCD
    int carry_block = 64;  // carry kernel: threads per workgroup
    int carry_vec = 1;     // carry kernel: lane-vectors per thread and iteration (1, 2, 4)
    int round_stats = 1;           // 0: rounds skip the by-products although statistics are attached
    int carry_blocks_per_cu = -1;  // carry kernel: -1 no cap, else max workgroups per CU
};

hipError_t launch_round(const RoundArgs &a, bool bf16, bool fast, const Launch &cfg,
                        hipStream_t stream);
hipError_t launch_carry(const CarryArgs &a, bool bf16, const Launch &cfg, hipStream_t stream);
hipError_t launch_stats_finish(const StatsArgs &a, hipStream_t stream);
long long slot_records(long long n, bool bf16, int block);   // wavefronts of a slot launch
int slot_tail(long long n, bool bf16);                       // elements of its ragged tail
hipError_t launch_stash(const StashArgs &a, bool bf16, hipStream_t stream);
hipError_t launch_views_sgd(const ViewsArgs &a, bool fast, const Launch &cfg, hipStream_t stream);
hipError_t launch_views_average(const ViewsArgs &a, const Launch &cfg, hipStream_t stream);
hipError_t launch_sgd(const SgdArgs &a, bool fast, const Launch &cfg, hipStream_t stream);
// norms of update and parameters per bucket (records for launch_stats_finish), then the update
// rule with the rate of each element's bucket read from st.stats
hipError_t launch_norms(const SgdArgs &a, const StatsArgs &st, hipStream_t stream);
hipError_t launch_sgd_lars(const SgdArgs &a, const StatsArgs &st, bool fast, hipStream_t stream);
long long norms_records(long long n);
// This device's copy of the library's fixed scratch array (kStaticScratchBytes bytes, 256-byte
// aligned); the address is looked up once per device.  launch_table_fill writes the bucket
// table there with a kernel, so that the call needs no host-to-device copy.
hipError_t static_scratch(char **ptr);
hipError_t launch_table_fill(long long *table, const long long *start_end, int n_buckets,
                             hipStream_t stream);
hipError_t launch_copy(void *dst, const void *src, long long nbytes, hipStream_t stream);
hipError_t launch_read(const void *src, long long nbytes, float *sink, hipStream_t stream);

// A plain kernel with a round's mix of streams (calibration): n_read streams are summed per
// lane-vector and the sum is written to n_write streams.
constexpr int kMixMaxRead = 80, kMixMaxWrite = 80;
struct MixArgs {
    const void *src[kMixMaxRead];
    void *dst[kMixMaxWrite];
    unsigned long long half;     // bit j: read stream j holds 8 bytes per lane-vector, not 16
    void *sink;                  // 4 writable bytes (only touched when nothing is written)
    int n_read, n_write;
    long long nvec;              // lane-vectors per stream
};
hipError_t launch_mix(const MixArgs &a, int waves_per_cu, hipStream_t stream);

}  // namespace eager
