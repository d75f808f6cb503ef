/*
 * cagra_probe.h -- C ABI of libcagra_probe.so: a measurement aid that ships beside libcagra_hip.so,
 * not inside it.  It reads device memory the way the search does and computes nothing of the method;
 * bench.py uses it for the bandwidth references it prints beside the search's roofline figure.
 * Conventions (pointers, streams, return codes) as in cagra_hip.h.
 */
#ifndef CAGRA_PROBE_H
#define CAGRA_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif


/*
 * Device-memory bandwidth references for the search, whose limiter is the memory bandwidth
 * (Sec. IV-C.1, Sec. V-D): reads `data` (rows of row_bytes bytes, stride_bytes apart, both multiples
 * of 16) and computes nothing of the method.
 *   pattern 0: one streaming read of the whole block (stride_bytes must equal row_bytes);
 *   pattern 1: n_read whole rows at pseudo-random positions (a counter hash of `seed`), fetched the
 *              way the distance step fetches them (Sec. IV-B.1): teams of team_size lanes (0 =
 *              automatic; 4, 8, 16, 32), 16-byte pieces, rows_in_flight rows per team at once
 *              (0 = 4; 2, 4, 8), waves_per_cu single-wavefront workgroups per compute unit (0 = 16).
 * sink: one device word that may or may not be written.  The caller times the call (events on the
 * stream); bytes moved are rows * row_bytes (pattern 0) or n_read * row_bytes (pattern 1).
 */
int cagra_probe_bandwidth(const void *data, int64_t rows, int64_t row_bytes, int64_t stride_bytes,
                          int32_t pattern, int64_t n_read, int32_t team_size, int32_t rows_in_flight,
                          int32_t waves_per_cu, uint64_t seed, uint32_t *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* CAGRA_PROBE_H */
