/*
 * llla_measure.h -- measurement aids of the LLA library.  NOT part of the method and NOT exported by the
 * production library libllla.so: these four symbols exist only in libllla_measure.so, which is the same sources
 * compiled with -DLLLA_MEASURE (every kernel launcher then records HIP events) plus csrc/measure.  It exports the
 * whole of llla.h as well, so a benchmark loads it in place of the production library for its per-kernel pass.
 * The state below is process-wide and not thread-safe, which is why it lives in a library of its own.
 */
#ifndef LLLA_MEASURE_H
#define LLLA_MEASURE_H

#include "llla.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * After llla_profile_enable(1) every call of an llla.h entry point records HIP events around each kernel it
 * enqueues, on the caller's stream.  llla_profile_last() waits for the events of the most recent call and writes
 * up to `max` stage durations in milliseconds to ms[] and pointers to static stage names to names[]; it returns
 * the number of stages (0 if profiling is off or nothing was recorded).
 */
void llla_profile_enable(int on);
int llla_profile_last(float *ms, const char **names, int max);

/*
 * Enqueues one launch of nothing but independent v_mfma_f32_16x16x32_f16 instructions on every compute unit,
 * `iters` x 8 per wavefront, and writes the number of floating-point operations of that launch to *flops (host).
 * Timing the launch on `stream` gives the 16-bit matrix-core rate the GPU sustains at the clock it settles to
 * under such a load, the practical ceiling beside the published peak.  `scratch` is a device buffer of >= 4 bytes
 * that is never written in practice (it only keeps the arithmetic alive).  1 <= iters <= 2^20.
 */
llla_status llla_probe_mfma_f16(int iters, void *scratch, double *flops, void *stream);

/*
 * Enqueues one plain copy of `bytes` bytes from src to dst (device pointers, 16-byte aligned, bytes a multiple of
 * 16, the two ranges disjoint): exactly `bytes` read and `bytes` written.  Run under a hardware counter it tells
 * what that counter reads per byte of HBM traffic, the scale for the traffic figures of the other kernels.
 */
llla_status llla_probe_copy(const void *src, void *dst, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LLLA_MEASURE_H */
