/*
 * libsvdp_probe — measurement helpers for the benchmark of libsvdp on MI355X (gfx950).
 * NOT part of the decode path: these calls measure the fixed costs and the ceilings of the
 * machine that the decode step's time is set against (cost of a dependent kernel node,
 * latency of a dependent load, streaming-read ceiling, time stamps between graph nodes).
 * C ABI; pointers named "device" are device pointers owned by the caller.  Every call that
 * takes a stream is asynchronous on it, allocates nothing and can be captured in a HIP graph.
 * Return value: 0 on success, 1 for an invalid argument, 4 if the HIP runtime refused a launch.
 */
#ifndef SVDP_PROBE_H
#define SVDP_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A kernel that does nothing: `blocks` x `threads`.  A chain of them in a graph gives the cost of
 * a dependent kernel node. */
int32_t svdp_probe_null(int32_t blocks, int32_t threads, void *stream);

/* One thread stores the GPU's constant-rate counter (100 MHz: 10 ns units) to slot[0].  Placed
 * between the steps of a captured sequence it gives each step's own duration (plus one node). */
int32_t svdp_probe_stamp(uint64_t *slot, void *stream);

/* One thread adds 1 to cell[0] (a load that depends on the previous node's store, then a store):
 * a chain of these is the cheapest possible hand-over of a value from one kernel to the next. */
int32_t svdp_probe_handover(uint32_t *cell, void *stream);

/* Reads `bytes` (a multiple of 16) from src once, 16 bytes per lane and load, with `blocks` blocks
 * of 512 threads; the streaming-read ceiling of the device.  sink: device, 4 bytes (written only if
 * an impossible checksum occurs, so that the loads cannot be removed). */
int32_t svdp_probe_stream_read(const void *src, size_t bytes, int32_t blocks, uint32_t *sink, void *stream);

/* One thread follows ring[i] -> ring[ring[i]] ... for `hops` dependent 4-byte loads starting at
 * index 0 (ring: device, a permutation of 0..n-1 written by the caller; every entry must be < n,
 * entries are reduced modulo n on the device) and stores the elapsed counter ticks (10 ns units) to
 * ticks[0] and the last index to ticks[1]: latency of one dependent load at the ring's footprint. */
int32_t svdp_probe_chase(const uint32_t *ring, uint32_t n, int32_t hops, uint64_t *ticks, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SVDP_PROBE_H */
