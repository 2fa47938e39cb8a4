/* Measurement aids of the library (no part of the method).
 *
 * Section 3.2 of the paper computes a binary product on a vector ALU as one AND (or XNOR) and one
 * popcount per 32 binary MACs of a lane.  The benchmark's metric is named after that form, so the
 * benchmark measures its ceiling on the chip at hand instead of trusting a data-sheet clock:
 * lane-popcounts per second, and the shader clock the chip sustains meanwhile.
 */
#ifndef DAB_PROBE_H
#define DAB_PROBE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One launch of `grid` workgroups of 256 lanes; every lane issues `iters` x 64 accumulating vector
 * popcounts (pair = 0), or that many AND + popcount pairs (pair != 0), back to back.
 *   out     device, uint32 [grid * 256]: the accumulated counts (written so that the work is kept)
 *   clocks  device, uint64 [grid * 2]:   per workgroup, shader-clock ticks and constant-rate-clock ticks
 *                                        between the first and the last popcount of its first lane
 *   lane_ops, ref_clock_khz  host: the number of lane-popcounts the launch issues (grid * 256 * iters * 64)
 *                                        and the rate of the constant-rate clock in kHz
 * Asynchronous on `stream`; the caller times the launch and owns all buffers.  Returns DAB_OK, DAB_ERR_NULL
 * for a missing pointer, DAB_ERR_SHAPE for iters <= 0, grid <= 0 or grid > 2^20, DAB_ERR_HIP for a failed launch. */
int dab_probe_popcount(int pair, int iters, int grid, uint32_t* out, uint64_t* clocks, int64_t* lane_ops,
                       int32_t* ref_clock_khz, void* stream);

#ifdef __cplusplus
}
#endif
#endif
