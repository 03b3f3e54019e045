/*
 * liblaplex diagnostics: hooks for benchmarks and tests.  None of them is part
 * of the method or needed to use the library (that is laplex.h); they time
 * kernels, expose the launch geometry and measure a device ceiling.
 */
#ifndef LAPLEX_DIAG_H
#define LAPLEX_DIAG_H

#include "laplex.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Kernel-family timing.  Between begin and end,
 * every launch of the named kernel family ("sort_hist", "radix_scatter", "merge",
 * "decay", "rowdot", "sum_slabs", "fill", and "scan_meta.T", "scan_reduce.T",
 * "scan_spine.T", "scan_down.T", "scan_down_sparse.T" with T = "fwd" for the
 * forward scans of x, "bwd" for the backward scans of gy, "rescan" for the
 * backward's repeat of the forward scans when they were not saved) is bracketed by a pair of HIP
 * events on the stream it is launched on.  laplex_profile_end waits for those
 * events and returns their summed elapsed time and the number of launches
 * (host pointers).  Creates and destroys HIP events; process-wide; not for
 * use under stream capture.
 */
int laplex_profile_begin(const char* family /* host string */);
int laplex_profile_end(double* total_ms, int64_t* launches);

/*
 * With the family "*" every family is timed.  After laplex_profile_end, family number `index`
 * (0, 1, ... in the order of first launch; LAPLEX_ERR_SIZE past the last) of that measurement: its
 * name (copied to the host buffer `name` of name_bytes bytes, truncated if need be), its summed
 * time and its launches.
 */
int laplex_profile_family(int64_t index, char* name /* host */, size_t name_bytes, double* total_ms, int64_t* launches);

/*
 * Diagnostics: rows of the merged sequence that one workgroup (for batches of
 * 253 columns and more with 128-bit lanes: one wavefront) of the downsweep
 * kernels owns, a "block", for a given batch, with 128-bit lanes (wide != 0:
 * batch and leading dimensions multiples of 4, 16-byte aligned pointers) or
 * scalar lanes.  Lets a benchmark count which blocks a launch visits.  `rows`
 * is a host pointer.
 */
int laplex_scan_tile_rows(int64_t batch, int wide, int64_t* rows);

/*
 * Diagnostics: the device's ceiling for a kernel that does nothing but move
 * whole rows at scattered positions, the access pattern of the heavy scan
 * kernels at wide batches (rows of the batch-minor matrices in sorted-anchor
 * order).  Row r of the launch is row row_ids[r] of both matrices:
 *   dst != NULL:  dst[row_ids[r]*cols + c] = src[row_ids[r]*cols + c]   (read + write)
 *   dst == NULL:  the rows are read and summed into nothing              (read only)
 * src, dst: (max id + 1) x cols floats, contiguous, 16-byte aligned; cols a
 * multiple of 4; row_ids: `rows` device words, each below the number of rows of
 * src and dst (the caller guarantees it; a permutation gives every row once).
 * Nontemporal 16-byte loads and stores, one wavefront per row, eight rows in
 * flight per wavefront.  A benchmark times it to put a measured ceiling beside
 * the nominal HBM peak; it is not part of the method.
 */
int laplex_diag_move_rows(const float* src, float* dst, const uint32_t* row_ids, int64_t rows, int64_t cols,
                          laplex_stream_t stream);

/*
 * Test hook: overwrite the status word of the plan in `ws` (count as for
 * laplex_get_plan_status; plans of more than 8192 positions only) with `value`
 * (0 = valid, 1 = invalid), so that the behaviour of the compute calls on an
 * invalid plan can be tested without making any kernel wait.
 */
int laplex_diag_set_plan_status(void* ws, size_t ws_bytes, int64_t count, uint32_t value, laplex_stream_t stream);

/*
 * Test hook (host, process-wide): batch-1 problems with at least this many merged positions k + n (and more
 * than 8192) move x, gy and the results between the caller's order and the sorted order through partition
 * passes instead of random accesses (default 2^22: below, the tables fit the device's caches and the random accesses are as fast).  Lets tests
 * run that route on small problems.  A plan must be reused under the setting it was built with.
 */
int laplex_diag_set_route_min(int64_t merged_positions);

#ifdef __cplusplus
}
#endif
#endif /* LAPLEX_DIAG_H */
