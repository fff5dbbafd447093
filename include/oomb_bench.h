/*
 * oomb_bench.h -- benchmark aids of the paged sparse attention library (same shared object as
 * oomb.h).  None of this is part of the paper's method and none of it belongs in a training
 * step: oomb_profile_read and oomb_calibrate WAIT for the device, and the profiling switch is
 * process-wide.  The product entry points of oomb.h never synchronise.
 */
#ifndef OOMB_BENCH_H_
#define OOMB_BENCH_H_

#include "oomb.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Benchmark aid (not part of the paper's method): per-kernel device time.  While
 * enabled (on = 1), every kernel the library launches is bracketed by two HIP events
 * recorded on the caller's stream (events are host objects created on demand; no
 * device memory is allocated).  on = 2 brackets only the four large kernels (page
 * scoring, forward, dQ, dK/dV), which disturbs back-to-back launches less; on = 0
 * switches the timing off.  oomb_profile_read waits for the recorded events of
 * entry idx (0 <= idx < oomb_profile_count()) and returns the kernel's name, its
 * accumulated device time in milliseconds and its launch count; it returns
 * OOMB_ERR_INVALID_ARG for a bad index or NULL outputs.  oomb_profile_reset drops
 * all entries.  Not thread-safe against concurrent launches on other threads.
 */
void oomb_profile_enable(int32_t on);
void oomb_profile_reset(void);
int32_t oomb_profile_count(void);
int32_t oomb_profile_read(int32_t idx, char* name, int32_t name_cap, double* total_ms, int64_t* launches);

/*
 * Benchmark aid (not part of the paper's method): a measured ceiling of the device,
 * to set kernel rates against something other than the data-sheet peaks.
 *   which = 0: every SIMD issues independent 32x32x16 bf16 matrix instructions back
 *              to back on constant operands; *result = TFLOP/s.  buf is only a sink
 *              (>= 4096 bytes).
 *   which = 2: the same instruction stream on operands with random signs and mantissas
 *              that change from one instruction to the next (the clock of the part
 *              follows the switching activity of the matrix units, so this is the
 *              ceiling of a kernel that multiplies real data); *result = TFLOP/s.
 *   which = 1: a streaming kernel copies the first half of buf (device memory,
 *              16-byte aligned, `bytes` long) to its second half; *result = GB/s
 *              counting bytes read + bytes written.
 * Runs on hip_stream and WAITS for the measurement (one warm-up launch, one timed
 * launch).  Returns OOMB_ERR_INVALID_ARG for NULL / misaligned / too small buffers
 * or an unknown `which`, OOMB_ERR_LAUNCH if HIP reports an error.
 */
oomb_status oomb_calibrate(int32_t which, void* buf, size_t bytes, double* result, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* OOMB_BENCH_H_ */
