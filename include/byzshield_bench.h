/*
 * byzshield_bench.h -- measurement aids of libbyzshield.  Not part of the aggregation ABI
 * (byzshield.h): reference kernels of known HBM traffic for reading hardware counters, event
 * timing of the dominant kernel, and a counter of the worst-case search.  Same conventions as
 * byzshield.h (byz_status returns, device pointers owned by the caller, hipStream_t as void*).
 */
#ifndef BYZSHIELD_BENCH_H
#define BYZSHIELD_BENCH_H

#include "byzshield.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Timing aid for benchmarks.  byz_profile_enable(n) with n > 0 creates n HIP event pairs for
 * the calling thread; from then on each byz_aggregate call of that thread records one pair
 * around its dominant kernel -- the single-pass kernel (its main launch, not the probe or the
 * finalisation), or the vote kernel for shapes without one -- on the call's stream, until n
 * calls have been recorded.
 * byz_profile_enable(0) releases the events.  Errors: BYZ_EINVAL (n < 0 or n > 100000),
 * BYZ_ENOMEM, BYZ_EDEVICE.
 * byz_profile_collect waits for the recorded events, writes the kernel durations in
 * milliseconds to host ms_out[0..*n_out-1] (at most `capacity`), and restarts recording at
 * the first pair.
 */
int byz_profile_enable(int max_calls);
int byz_profile_collect(float *ms_out, int capacity, int *n_out);

/*
 * Reference kernel for hardware HBM counters: copies `bytes` (a multiple of 16) from device
 * src to device dst, non-overlapping, with the same 16-byte non-temporal loads and stores the
 * streaming kernels use, so that it reads exactly `bytes` and writes exactly `bytes`.
 * Asynchronous on `stream`.  Errors: BYZ_EINVAL, BYZ_EDEVICE.
 */
int byz_calibration_copy(const void *src, void *dst, size_t bytes, void *stream);

/*
 * Reference kernel for the single pass's ceiling: reads the first 4*floor(d/4) words of rows
 * 0..n_rows-1 of the device matrix rows_base (row pitch ld words) with the access pattern of
 * byz_aggregate's single pass -- every thread 16 bytes of each row, non-temporal -- and does
 * nothing with them but XOR; with store != 0 it writes the XOR to out[0..4*floor(d/4)-1]
 * (device, non-temporal 16-byte stores), with store == 0 it writes nothing (out must still be
 * a valid device pointer).  The two timings bound what a kernel of this shape can reach with
 * and without its output.  4 <= d <= 2^30, 1 <= n_rows <= BYZ_MAX_F_WIDE * BYZ_MAX_R.
 * Asynchronous on `stream`.  Errors: BYZ_EINVAL, BYZ_EDEVICE.
 */
int byz_calibration_read_rows(const void *rows_base, int64_t d, int64_t ld, int n_rows, void *out,
                              int store, void *stream);

/* Subsets evaluated by the calling thread's last byz_worst_case / byz_worst_case_opts call. */
uint64_t byz_worst_case_last_visited(void);

#ifdef __cplusplus
}
#endif
#endif /* BYZSHIELD_BENCH_H */
