/*
 * razor_bench.h -- measurement hooks of the razor library.  Not part of the product ABI
 * (razor.h): nothing here is on the hot path, and a serving stack never calls it.  The
 * benchmark uses these entry points to time the dominant kernel alone and to measure what
 * the device's memory system gives kernels that do nothing but move bytes.
 */
#ifndef RAZOR_BENCH_H
#define RAZOR_BENCH_H

#include "razor.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * After this call, every razor_decode_attn issued by the CALLING THREAD records ev_start (a
 * hipEvent_t) on its stream right before the kernel that streams the cache and ev_stop right
 * after it, so a benchmark can time that kernel alone.  Pass NULL, NULL to switch the hook off
 * (the default; do so before destroying the events).  This is per-thread state inside the
 * library, the one exception to "keeps no state between calls".  The events stay owned by
 * the caller.  While the hook is on, a decode call whose hipEventRecord fails returns
 * RAZOR_EHIP; work enqueued before the failing record stays enqueued.  Always returns RAZOR_OK.
 */
RAZOR_API int razor_profile_events(void *ev_start, void *ev_stop);

/* How a probe kernel hands 4 KB pieces to its W wavefronts (`pattern`): 0 = wavefront w gets one
 * contiguous range; n >= 1 (at most 65536) = the buffer is cut into chunks of n pieces and wavefront
 * w gets chunks w, w + W, w + 2W, ..., so that at any moment the chip works inside one moving window
 * of W * n pieces; -G (G >= 1, at most RAZOR_MAX_WORKERS) = the wavefronts form groups of G, every group
 * owns one contiguous range, and wave j of a group takes pieces j, j + G, j + 2G, ... of that range
 * (W / G moving windows of G pieces; G is lowered to the next divisor of W). */
#define RAZOR_PROBE_CONTIGUOUS 0
#define RAZOR_PROBE_INTERLEAVED 1

/*
 * Read-stream probe.  Reads the first bytes / 4096 * 4096 bytes at buf (device, 16-byte aligned,
 * at least 4096 bytes) exactly once with 128-bit loads and does no other work, so the duration
 * of this launch is what the device gives a kernel that only reads.
 *   n_workers    wavefronts; 0 = four per compute unit (one per SIMD); at most RAZOR_MAX_WORKERS
 *   pattern      RAZOR_PROBE_CONTIGUOUS, RAZOR_PROBE_INTERLEAVED, or a chunk length in pieces (see above)
 *   depth        4 KB pieces a wavefront keeps in flight: 1, 2, 4 or 8
 *   nontemporal  non-zero: non-temporal loads (what the streaming kernels use)
 *   sink         device, at least 4 * RAZOR_MAX_WORKERS bytes, may be written (keeps the loads alive)
 * Enqueued on `stream`; time it with events.  RAZOR_EINVAL for anything outside these ranges.
 */
RAZOR_API int razor_probe_read_stream(const void *buf, size_t bytes, int n_workers, int pattern,
                            int depth, int nontemporal, void *sink, void *stream);

/*
 * Copy probe: dst[0 .. bytes / 4096 * 4096) = src[...] with 128-bit loads and stores, two 4 KB
 * pieces in flight per wavefront; the read + write counterpart of the probe above (what a kernel
 * that only moves rows, like the compaction step, can reach).  dst and src: device, 16-byte
 * aligned, not overlapping.  nontemporal: bit 0 = non-temporal loads, bit 1 = non-temporal stores.
 */
RAZOR_API int razor_probe_copy(void *dst, const void *src, size_t bytes, int n_workers, int pattern,
                     int nontemporal, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RAZOR_BENCH_H */
