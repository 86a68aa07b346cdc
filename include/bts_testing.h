/*
 * bts_testing -- measurement and testing aids of libbts.  NOT part of the contract of
 * bts.h: nothing here is needed to run a step, and these calls may synchronise the host.
 * They exist so that the tests can assert which select path ran and exercise the
 * recovery paths, and so that the benchmark can time the dominant kernel on the stream it
 * is launched on.  Conventions (device pointers, return codes) as in bts.h.
 */
#ifndef BTS_TESTING_H
#define BTS_TESTING_H

#include "bts.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Timing of the dominant kernel (the dense pass over g and eps in topk_compress).  While
 * enabled, the library brackets that kernel with HIP events on the context's stream.
 * bts_profile_read synchronises those events and returns the summed kernel time in
 * milliseconds and the number of launches since the last read (both host pointers).
 */
int bts_profile_enable(bts_ctx* ctx, int on);
int bts_profile_read(bts_ctx* ctx, double* ms_total, uint64_t* launches);

/* Path taken by the last topk_compress / downlink_topk on this context, for tests and
 * reports: a host-synchronous read of per-row flags.  rows_fast = rows finished by the
 * single-pass path, rows_dense = all others (dense multi-pass path, the three-launch path of
 * middling rows, or the one-workgroup path of short rows); rows_fast + rows_dense == rows.
 * which: 0 = uplink, 1 = downlink. */
int bts_last_path(bts_ctx* ctx, int which, uint32_t* rows_fast, uint32_t* rows_dense);

/* Testing aid: which select path later calls on this context take.  0 (default): chosen
 * by shape (one workgroup per row up to d = 8192; the three-launch select for K <= 3072,
 * K <= d/64 on rows up to 2^22 coordinates and calls of at most 2.4e7 coordinates, which are
 * bound by their launches; otherwise the single-pass select from about 1.1e7 coordinates per
 * call, 8e6 for a single row; else the dense multi-pass select); 1: the dense multi-pass
 * path only (the path that also serves as the fallback); 2: the single-pass path wherever the
 * shape allows it (d >= 65536 and K <= d/64), whatever its size; 3: the three-launch path
 * wherever the shape allows it (1 <= K <= 8192, K <= d/64, 8192 < d <= 2^22, at most 2^25
 * coordinates per call).
 * Results are identical in every mode. */
int bts_set_path(bts_ctx* ctx, int mode);

/* Testing aid, no device needed: how a select of `rows` rows of d coordinates with K kept
 * coordinates is planned.  out (host pointer, 16 words): [0] the path that serves the shape
 * by default (0 one workgroup per row, 1 dense multi-pass, 2 single-pass, 3 three-launch);
 * single-pass select: [1] possible for the shape, [2] capacity of one candidate list,
 * [3] sample stride in slices, [4] sampled coordinates wanted at or above the lower bound,
 * [5] the rank the handed-on lower bound aims at, [6] directory tiles per row, [7] directory
 * entries per row, [8] waves per SIMD the dense pass is held to; three-launch select:
 * [9] possible for the shape, [10] capacity of one list, [11] tiles, [12] directory entries
 * per row, [13] blocks per row of the capture, [14] of the histogram pass; [15] candidate
 * lists per row.  BTS_EINVAL for rows == 0, d == 0, d >= 2^32, K > d or a null pointer. */
int bts_testing_plan(uint32_t rows, uint64_t d, uint32_t K, uint32_t* out);

/* Testing aid: makes the next calls on this context behave as after a call that failed
 * half way (a HIP launch error): the select scratch is taken to be dirty, so the next
 * select clears its histograms, directory and sample counts before it starts, and the
 * aggregation stops using its range tables and finds its ranges by binary search.
 * Results must be unchanged.  No fault is involved; only host flags are set. */
int bts_testing_mark_dirty(bts_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* BTS_TESTING_H */
