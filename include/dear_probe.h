/*
 * dear_probe.h -- HBM stream-pattern probe for the MI355X (gfx950).
 *
 * Not part of the aggregation path: a measurement aid for its rooflines.  Each pattern is
 * the bare memory traffic of one of the path's kernels with the arithmetic and the
 * tensor indexing taken out, so its rate is the ceiling that kernel's access pattern
 * allows on this chip (the 8 TB/s peak is what the roofline is priced against; these
 * figures say how much of the gap is the pattern's and how much the kernel's).
 *
 * The probe allocates its own device buffers (hipMalloc), fills them, times `reps`
 * launches with HIP events on the default stream, frees the buffers and returns.
 */
#ifndef DEAR_PROBE_H
#define DEAR_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    /* k input streams read at the same offset by every workgroup, summed, one output
     * stream written: the reduce-scatter's pattern (k = P workers' gradients) */
    DEAR_PROBE_READ_K_WRITE_1 = 0,
    /* one input stream read once, the value written to k output streams by the same
     * workgroup: an all-gather that stores to all replicas at once */
    DEAR_PROBE_READ_1_WRITE_K = 1,
    /* one input stream, k output streams written one after another in chunks of
     * chunk_bytes (workgroups ordered chunk, stream, part): the all-gather as built */
    DEAR_PROBE_READ_1_WRITE_K_CHUNKED = 2,
    /* three input streams, two of them written back: the shard update's pattern */
    DEAR_PROBE_READ_3_WRITE_2 = 3
};

/* dear_probe_streams -- run one pattern.
 *   pattern           one of the DEAR_PROBE_* values
 *   k                 number of parallel streams (1..64; ignored by READ_3_WRITE_2)
 *   bytes_per_stream  length of every stream in bytes (multiple of 4096, >= 4096); choose
 *                     it well above the 256 MB last-level cache
 *   chunk_bytes       chunk of the CHUNKED pattern (multiple of 4096), ignored otherwise
 *   elem_bytes_in     2 or 4: bytes read per output element in READ_K_WRITE_1 (2 = bf16
 *                     inputs widened to a 4-byte output); 4 for the other patterns
 *   skew_bytes        stream j starts j * skew_bytes into its own allocation (multiple of 256,
 *                     at most 64 MiB; 0 = every stream starts at its allocation's base): shifts
 *                     which HBM channel and bank the k streams touch at the same moment
 *   reps              timed launches (>= 1), after two untimed ones
 *   gbytes_per_s      host, receives (bytes read + bytes written per launch) / time, in 1e9 B/s
 *   avg_ms            host, receives the average launch time in milliseconds (may be NULL)
 * Returns 0, -1 for a bad argument, -2 if an allocation failed, -3 for a HIP error. */
int dear_probe_streams(int32_t pattern, int32_t k, int64_t bytes_per_stream, int64_t chunk_bytes,
                       int32_t elem_bytes_in, int64_t skew_bytes, int32_t reps, double *gbytes_per_s,
                       double *avg_ms);

#ifdef __cplusplus
}
#endif
#endif /* DEAR_PROBE_H */
