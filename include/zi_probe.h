/*
 * zi_probe.h — measurement aids of the zi library.
 *
 * These calls compute nothing of the optimizer step.  They measure what the hardware under the step
 * can do — HBM streams, the host link, the storage — with the library's own streams, staging memory
 * and thread pools, so that a benchmark can put the step's rates beside ceilings obtained in the same
 * process.  They are exported by the same shared library but are not part of the product interface
 * declared in zi.h (Section 4.1 and Section 5.2.2 motivate the ceilings: the step is bound by the
 * bandwidth of whichever memory holds the state).
 */
#ifndef ZI_PROBE_H
#define ZI_PROBE_H

#include "zi.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * HBM stream probe: one launch that streams `bytes` (positive multiple of 16) of 16-byte aligned
 * device memory with no arithmetic, shaped the way that measured best for a plain stream on this
 * device (single-wavefront workgroups, 4 KiB contiguous per wavefront, non-temporal accesses, six
 * wavefronts per compute unit, XCD-aware tile order).
 * mode 0 = read d_a; mode 1 = copy d_a to d_b (non-overlapping); mode 2 = update d_a in place
 * (every fp32 value + 1).  Asynchronous on hip_stream.  Timing it gives the bandwidth a pure
 * read, a 1:1 copy and an in-place read-modify-write reach on this device, i.e. the practical
 * ceilings of the norm pass and of the fused step.
 */
zi_status zi_hbm_probe(void* d_a, void* d_b, size_t bytes, int32_t mode, void* hip_stream);

/*
 * Host-link probe: moves `bytes` between pinned host buffers and the engine's staging memory in
 * pieces of `piece_bytes` on the engine's two copy streams and reports the elapsed seconds.
 * mode 0 = host-to-device only, 1 = device-to-host only, 2 = both directions at once (then `bytes`
 * move in EACH direction, from host_src and into host_dst).
 * piece_bytes: 0 = the engine's chunk size; at most half of the engine's staging memory.
 * depth: pieces per direction the host keeps in flight (1..8); 0 = no limit (everything is queued
 * at once).  The independent peak of the link is the best figure over a sweep of piece sizes and
 * depths; the streamed step's own pacing (ZI_OPT_MAX_INFLIGHT, chunk size) is one point of it.
 * Buffers must be pinned and hold `bytes` each; host_dst may be NULL for mode 0 and host_src for
 * mode 1.  host_dst is overwritten with staging contents.  Blocking.
 */
zi_status zi_engine_link_probe(zi_engine* e, const void* host_src, void* host_dst, size_t bytes, int32_t mode,
                               size_t piece_bytes, int32_t depth, double* seconds_out);

/*
 * Storage probe: with the engine's thread pools and pinned ring, read `bytes` from fd_read
 * (from offset 0) and, at the same time, write `bytes` to fd_write (from offset 0); either
 * descriptor may be -1 to measure one direction alone.  bytes: positive multiple of 4096.
 * Reports the elapsed seconds: the file-tier bandwidth the streamed step is bounded by.  The number
 * of requests in flight is the engine's ZI_OPT_HOST_COPY_THREADS per direction: sweep it for the
 * storage's own peak.
 */
zi_status zi_engine_file_probe(zi_engine* e, int32_t fd_read, int32_t fd_write, size_t bytes,
                               double* seconds_out);

#ifdef __cplusplus
}
#endif
#endif /* ZI_PROBE_H */
