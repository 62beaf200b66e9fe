/* kmq_probe.h -- measurement probes, built into their own library (libkmq_probe.so).
 *
 * Not part of the product: nothing in libkmq.so calls these and no result depends on
 * them.  They exist so that the benchmark can state, measured on the machine it runs on,
 * the two figures a memory-bound call is judged against (the paper's App. E
 * "Micro-benchmarks" quotes effective bandwidth against what the memory system delivers):
 * what one launch costs when it does nothing, and how fast the same bytes can be read
 * when nothing is done with them.
 *
 * All pointers are DEVICE pointers; calls enqueue on `hip_stream` (a hipStream_t passed as
 * void*), allocate nothing and do not synchronise.  Return value: 0, or a nonzero
 * hipError_t / -1 for a bad argument.
 */
#ifndef KMQ_PROBE_H
#define KMQ_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* A kernel that does nothing, `grid` workgroups of `block` threads (block in {64, 256, 512,
 * 1024}): the cost of a launch.  `sink` (4 bytes, may be NULL) is never written in practice. */
int kmq_probe_empty(int grid, int block, void* sink, void* hip_stream);

/* Number of read-probe variants and their names (static strings, NULL past the end).
 * One-shot variants ("oneshot_l<L>_<nt|t>"): every wave issues L 16-byte loads per lane at
 * once and ends; the grid covers the buffer.  Persistent variants ("persist_g<G>_l<L>_nt"):
 * G workgroups of 256 threads loop over the buffer with L loads per lane in flight.  "nt"
 * marks loads with the non-temporal hint. */
int kmq_probe_read_variants(void);
const char* kmq_probe_read_name(int variant);

/* Reads `bytes` (>= 16, rounded down to a multiple of 16) at `data` (16-byte aligned) once with
 * the given variant and discards them.  `sink` as above. */
int kmq_probe_read(const void* data, size_t bytes, int variant, void* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* KMQ_PROBE_H */
