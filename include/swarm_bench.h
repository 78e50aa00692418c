/*
 * swarm_bench.h -- measurement aids exported by the same library as swarm.h.
 *
 * Nothing here is a step of the swarm interaction: these calls exist so that a benchmark can time
 * the library's kernels on the stream they run on and compare them with plain streaming copies on
 * the same GPU.  Conventions as in swarm.h.
 */
#ifndef SWARM_BENCH_H
#define SWARM_BENCH_H

#include "swarm.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Timing aid.  Off by default.  After the first swarm_timing_reset on a handle the library brackets
 * the gossip pass of every swarm_gossip_round / swarm_round_fused / swarm_interact, every whole
 * swarm_run_sequential call and the kernels of every swarm_local_steps with HIP events on the
 * handle's stream (up to 1024 calls of each kind between resets; later calls are not recorded).
 * swarm_kernel_times synchronises and returns the summed device milliseconds and the number of
 * recorded calls since the last swarm_timing_reset. */
swarm_status swarm_timing_reset(swarm_t h);
swarm_status swarm_kernel_times(swarm_t h, double *gossip_ms, uint32_t *gossip_calls,
                                double *local_ms, uint32_t *local_calls);

/* Measurement aid: plain streaming copy of nbytes (a multiple of 16, at most 2^36) between
 * device buffers on the given stream -- the copy rate the gossip pass is compared with. */
swarm_status swarm_stream_copy(void *dst_dev, const void *src_dev, uint64_t nbytes, void *hip_stream);

/* Measurement aid: the same streaming access with n_read concurrent read streams (consecutive
 * blocks of stream_bytes in src_dev) summed into n_write write streams (consecutive blocks in
 * dst_dev; write stream w holds the sum plus w).  Shapes (n_read, n_write): (2,1), (3,1), (2,2),
 * (4,2), (6,2); others return SWARM_EINVAL.  stream_bytes a multiple of 16. */
swarm_status swarm_stream_mix(void *dst_dev, const void *src_dev, uint64_t stream_bytes, uint32_t n_read,
                              uint32_t n_write, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SWARM_BENCH_H */
