/*
 * dbw_measure.h - measurement helpers of the dbw library (not part of a training round):
 * per-kernel timing of a context's launches and the device's achievable ceilings.
 * Same conventions as dbw.h.
 */
#ifndef DBW_MEASURE_H
#define DBW_MEASURE_H

#include "dbw.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Names, total durations (milliseconds, measured with HIP events on the launch stream) and
 * launch counts of the kernels of all calls on the context since timing was switched on with
 * dbw_set_timing(ctx, 1) (switching it on or off discards what was collected); used to report
 * achieved bandwidth / FLOP rate per kernel.  Two event records per kernel slow launch-bound
 * rounds down noticeably: time throughput with timing off.  dbw_get_timing synchronises the
 * device, writes up to `cap` entries and returns the entry count. */
typedef struct {
    const char *name;
    double ms_total;
    int64_t launches;
} dbw_kernel_time;
int dbw_set_timing(dbw_ctx *ctx, int32_t on);
int dbw_get_timing(dbw_ctx *ctx, dbw_kernel_time *out, int32_t cap);

/* Achievable ceilings of the device the roofline figures are read against, measured with
 * plain kernels (the nominal peaks are 8 TB/s and 157.3 TFLOP/s fp32 matrix):
 *   DBW_CAL_HBM_TRIAD  a = b + s c over three freshly allocated device arrays of `size` bytes
 *                      each (a multiple of 16, at most 16 GiB), streaming loads and stores;
 *                      *result = 3 size / time in GB/s
 *   DBW_CAL_MFMA_FP32  every wave of a grid that fills the chip runs `size` (<= 2^24) iterations
 *                      of four independent 32x32x2 fp32 matrix instructions on register
 *                      operands; *result in TFLOP/s
 * Timed over `repeats` (1..1000) launches with HIP events on `stream`; result [host].
 * Allocates and frees its own device memory and synchronises; not part of a round. */
enum { DBW_CAL_HBM_TRIAD = 0, DBW_CAL_MFMA_FP32 = 1 };
int dbw_calibrate(int32_t what, int64_t size, int32_t repeats, double *result, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* DBW_MEASURE_H */
