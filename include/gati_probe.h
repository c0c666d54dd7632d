/*
 * gati_probe.h - measurement probes shipped with the learned-cache library.  They compute nothing of
 * the method: they exist so that a benchmark run can state, on the box it runs on, what a plain
 * streaming read reaches (the ceiling the pooling kernels are compared with, beside the published
 * HBM peak), so that hardware byte counters can be scaled by a dispatch of exactly known traffic, and
 * what a launch costs that consumes its predecessor's output and does nothing else (the floor under
 * the predictor / selector kernels, which are chains of such launches).
 * Same conventions as gati.h: device pointers, caller-owned buffers, enqueue on the caller's stream,
 * status return, nothing allocated.
 */
#ifndef GATI_PROBE_H
#define GATI_PROBE_H

#include <stddef.h>
#include <stdint.h>

#include "gati.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Read `bytes` bytes (a multiple of 16, 16-byte aligned) of device memory once, with the same
 * non-temporal 16-byte loads the pooling kernels use, and fold them into one float per lane that is
 * stored only under a condition that never holds.  blocks_per_cu (1..32) workgroups of 256 lanes per
 * compute unit stride over the buffer, 8 loads in flight per lane; blocks_per_cu = 0 launches one wave
 * per contiguous 8 KB chunk instead, with no loop.  Which shape reads fastest depends on the box, so a
 * caller after the ceiling tries a few.  sink: device, at least
 * 256 * 4 * blocks_per_cu * CUs bytes.  Algorithmic traffic: `bytes` read, nothing written. */
gati_status_t gati_probe_stream_read(const void *buf, size_t bytes, float *sink, int32_t blocks_per_cu, void *stream);

/* Copy `bytes` bytes (a multiple of 16, both pointers 16-byte aligned, no overlap) with 16-byte loads
 * and stores.  Algorithmic traffic: `bytes` read and `bytes` written - the known quantity against
 * which FETCH_SIZE / WRITE_SIZE counter readings are scaled. */
gati_status_t gati_probe_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Enqueue `links` (0..4096) launches of `workgroups` (1..65536) workgroups of 256 lanes, one after the
 * other on `stream`; every lane of a link follows `loads` (0..8) dependent 4-byte loads starting at a
 * cell that the previous link wrote, and one lane writes that cell for the next link.  cell: device,
 * two int32, zero before the first call and zero afterwards.  Time per link = the cost of a launch
 * that waits for its predecessor's result and has nothing to compute. */
gati_status_t gati_probe_launch_chain(int32_t *cell, int32_t links, int32_t workgroups, int32_t loads, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GATI_PROBE_H */
