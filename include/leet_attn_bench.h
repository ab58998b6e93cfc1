/*
 * leet_attn_bench.h -- measurement aids of the MI355X (gfx950) decayed causal linear attention
 * library.  Not part of the attention boundary (that is leet_attn.h): the benchmark and the
 * profiling runs use them to time the kernels of one prefill separately and to calibrate the
 * profiler's byte counters.  Same conventions as leet_attn.h (device pointers, status codes).
 */
#ifndef LEET_ATTN_BENCH_H
#define LEET_ATTN_BENCH_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Computes what leet_attn_forward_ex computes (Alg. 2 with the decaying mask of Eq. "BCMV"), with
 * HIP events recorded on `stream` around each of the three kernels a prefill launches; the call
 * waits for them.  The pre-pass and the walk (which write the same values each time) are launched
 * five times back to back between their events and the time is divided by five; the scan runs once.
 *   kernel_ms  HOST pointer to 3 floats, filled with the milliseconds per launch of
 *              [0] the segment-state pre-pass, [1] the segment scan, [2] the chunk walk
 *              ([0] and [1] are 0 when the plan has a single segment).
 * state_out must not alias state_in here (LEET_ERR_INVALID_ARG): the repeated launches would
 * start from the state the first one left.
 * Synchronous (returns after the work has finished); not for use under graph capture.
 */
int leet_attn_forward_profile(const void *q, const void *k, const void *v, const float *gamma, float *out,
                              const float *state_in, float *state_out,
                              void *workspace, size_t workspace_bytes, int segments,
                              int B, int H, int N, int d, int dtype, void *stream,
                              float *kernel_ms);

/*
 * A plain streaming kernel of known traffic, used to calibrate the profiler's HBM byte counters
 * and to find the practical streaming rate of the device.
 *   mode 0  copy: reads `bytes` from src, writes `bytes` to dst
 *   mode 1  read: reads `bytes` from src; dst receives one float per workgroup
 *           (dst must hold `workgroups` floats)
 *   mode 2  fill: writes `bytes` to dst (src ignored)
 *   mode 3  copy, mode 4  fill, with nontemporal stores (how the library writes its outputs)
 *   bytes   multiple of 16; src, dst 16-byte aligned device pointers
 *   workgroups  grid size (256 threads each); each thread strides over the buffer
 * Asynchronous on `stream`.
 */
int leet_attn_calibration_stream(int mode, const void *src, void *dst, size_t bytes, int workgroups,
                                 void *stream);

#ifdef __cplusplus
}
#endif
#endif /* LEET_ATTN_BENCH_H */
