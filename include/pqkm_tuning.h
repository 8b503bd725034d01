/*
 * pqkm_tuning.h -- tuning and measurement hooks of libpqkm.so.
 *
 * Not part of the method and not needed to use it: the entry points of pqkm.h choose their kernels and launch
 * shapes themselves.  These hooks exist so that tests can force every compiled kernel and so that a benchmark can
 * time the scan kernel on the stream it runs on.
 *
 * The options are PROCESS-WIDE.  Every pqkm.h entry point reads them once, when it is called, and works from that
 * copy, so a change made while a call runs does not affect it; but two callers in one process cannot hold
 * different settings, and setting an option while another thread is between two calls that belong together
 * (say pqkm_assign then pqkm_update) changes the second.  None of the options changes pqkm_workspace_bytes.
 */
#ifndef PQKM_TUNING_H
#define PQKM_TUNING_H

#include "pqkm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * pqkm_set_option: integer knobs, by name (host string).  Unknown
 * name or out-of-range value -> PQKM_ERR_SHAPE.  Names:
 *   "assign_kernel"      0 = choose automatically (default), 1 = force the generic
 *                        scan that reads the tables through the cache hierarchy,
 *                        2 = force the LDS-tiled scan (M in {4, 8, 16, 32} only)
 *   "scan_variant"       0 = default scan of the LDS-tiled assignment (for M = 4: codes regrouped for
 *                        conflict-free LDS reads when K >= 128 and N exceeds one round of 2048-code
 *                        workgroups, else the subspace-skewed scan in a launch shape chosen by N),
 *                        1..99 = one specific compiled scan and launch shape (for tuning sweeps;
 *                        e.g. 34 = the skewed M = 4 scan without regrouping, 70 = the regrouped one)
 *   "hist_kernel"        0 = choose automatically (default; inside pqkm_fit / pqkm_fit_until with M = 4 this
 *                        includes counting from records the scan files by cluster group), 1 = force one global atomic
 *                        per code and subspace, 2 = force the LDS-privatised histogram over cluster
 *                        groups (falls back when K needs more than 255 groups), 3 = force the
 *                        histogram over code indices sorted by cluster
 *   "launch_codes_log2"  the scan is issued in launches of 2^value codes (default 26)
 *   "scan_rounds_per_launch"  the large scans (two-lane M = 4 scan, regrouped M = 8 scan, sliding-window
 *                        scan) issue the workgroups of such a launch in kernel launches of `value`
 *                        rounds (one workgroup per compute unit) each, so that the workgroups start
 *                        in step and share the tile images through the L2 (default 1); 0 = one
 *                        kernel launch for all of them
 *   "profile"            bit 0 (value 1) = bracket every scan-kernel launch with a pair of HIP
 *                        events on the caller's stream; bit 1 (value 2) = bracket every whole
 *                        assignment step (tile images, regrouping of the codes where it is
 *                        due, scan launches) the same way; 3 = both; 0 = off (default).
 *                        Events are created on first use and reused; this is the one place
 *                        the library creates HIP objects.
 *
 * pqkm_profile_read / pqkm_profile_read_steps: wait for the recorded stop events, return the
 * summed elapsed time of the bracketed scan kernels / assignment steps in milliseconds and
 * their number, and reset that record.  A pair of events brackets the scan kernels of one
 * stretch of codes (one launch, or one per round of workgroups, back to back on the stream);
 * `launches` counts the kernels, so total_ms / launches is the average duration of a scan
 * kernel, the short gaps between consecutive launches included.  They block the host.
 *   total_ms, launches / steps   host pointers, out
 */
pqkm_status pqkm_set_option(const char *name, int32_t value);
pqkm_status pqkm_profile_read(double *total_ms, int64_t *launches);
pqkm_status pqkm_profile_read_steps(double *total_ms, int64_t *steps);

#ifdef __cplusplus
}
#endif
#endif /* PQKM_TUNING_H */
