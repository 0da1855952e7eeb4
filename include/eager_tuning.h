/*
 * eager_tuning.h - measurement interface of the eager-SGD library: the launch shape of the round
 * kernels (for sweeps) and plain streaming kernels of known traffic (to calibrate bandwidth and
 * the profiler's byte counters).  Nothing here is needed to use the library; eager.h is the
 * product interface.  The paper states no kernel design for this path (its reduction runs on the
 * host inside a communication schedule, Section 4.1.1), so nothing in this file follows a passage
 * of it.
 */
#ifndef EAGER_TUNING_H
#define EAGER_TUNING_H

#include "eager.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Launch shape of the round kernels of a context.  Unknown keys and values outside the listed
 * ones: EINVAL.  Every combination of listed values has a kernel.
 *   "split"      0 = chosen per round (default): the send-buffer rewrite of the late
 *                processes runs as a copy kernel of its own after the reduction when somebody
 *                is late and the fused pass would read more than 16 streams, when 8 or more
 *                processes are late, or when 3 or more are late and the run has 2^25 elements
 *                or more.  1 = always one fused kernel; 2 = always reduction + update kernel
 *                followed by the copy kernel
 *   "chunk"      streams whose loads are in flight together per wavefront: 0 (default) = 16, 8, 16.
 *                Per-bucket statistics need 16
 *   "block"      threads per workgroup: 64 (default), 128 or 256
 *   "blocks_per_cu" 0 = chosen from the round (default); -1 = no cap; 1..32 = at most that many
 *                workgroups resident per CU
 *   "nt_state"   nontemporal hint on w, v and recv too: -1 (default) = when they exceed 256 MiB
 *                in the call (they cannot stay in the last-level cache until the next round),
 *                0 = never, 1 = always
 *   "xcd_map"    0 (default) = consecutive workgroups, which the hardware deals to the 8 XCDs
 *                round robin, take consecutive tiles; 1 = every XCD takes one contiguous eighth
 *                of the range (measured 2.5 % slower: kept for A/B)
 *   "carry_block", "carry_vec", "carry_blocks_per_cu"  shape of the copy kernel of a split
 *                round: threads per workgroup (64 default, 128, 256), groups of 4 elements per
 *                thread (1 default, 2, 4), resident workgroups per CU (-1 = no cap, default;
 *                1..32)
 *   "round_stats" 1 (default) = with statistics attached every round writes the by-products;
 *                0 = rounds leave them alone (for callers that attach the statistics only as
 *                the workspace of eager_sgd_step_lars, which forms its own norms)
 */
int eager_set_launch(eager_ctx *ctx, const char *key, int value);

/*
 * Plain streaming kernels.  All pointers are 16-byte aligned device memory owned by the caller;
 * kernels go to `stream` (NULL = default stream); nothing synchronises.  Errors: EINVAL (NULL,
 * alignment, sizes or counts outside the stated ranges), EDEVICE.
 *   copy  dst <- src, nbytes a multiple of 16
 *   read  sums src (nbytes, a multiple of 16) in registers; *sink is written practically never
 *   mix   what a plain kernel with a round's mix of streams reaches: lane-vector i (16 bytes) of
 *         each of the n_read (1..80) streams is loaded, the values are added up, and the sum is
 *         stored to lane-vector i of each of the n_write (0..80) streams; same access shape as a
 *         round (one tile of 256 elements per wavefront, up to 16 loads in flight per lane,
 *         nontemporal).  n_vec lane-vectors per stream.  Bit j of read_half_mask marks read stream (one of the first 64)
 *         j as half-width: it holds 8 bytes per lane-vector (n_vec * 8 bytes, n_vec even), read the
 *         way a round reads bf16 gradients.  waves_per_cu: 0 = no cap, 1..32 = at most that many
 *         64-lane workgroups resident per CU.  sink: 4 writable bytes, needed when n_write is 0.
 */
int eager_calib_copy(void *dst, const void *src, int64_t nbytes, void *stream);
int eager_calib_read(const void *src, int64_t nbytes, float *sink, void *stream);
int eager_calib_mix(const void *const *read, int n_read, uint64_t read_half_mask,
                    void *const *write, int n_write, int64_t n_vec, int waves_per_cu,
                    float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EAGER_TUNING_H */
