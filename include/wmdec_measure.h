/*
 * wmdec -- measurement hooks of libwmdec.so (not needed to decode frames).
 *
 * The benchmark prices every kernel of a decoder_run against its roofline; the
 * entry points below give it the steps of the graph, their algorithmic work
 * (the Eq. 9 accounting of Sec. IV-B-1: every input, residual, output and
 * weight tensor counted once) and HIP-event timings taken on the stream the
 * kernels run on.  Conventions as in wmdec.h.
 */
#ifndef WMDEC_MEASURE_H
#define WMDEC_MEASURE_H

#include "wmdec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-step timing for measurement.  With profiling enabled decoder_run records
 * a HIP event on `stream` before the first and after every step of the graph
 * (a step = one GroupNorm statistics pass, one convolution, the V transpose or
 * the attention core).  decoder_step_info gives, for step `index`, the name of
 * the kernel that executes it (for convolutions the template instantiation as
 * a profiler prints it; the string is valid until the thread's next call) and
 * its algorithmic FLOPs and HBM bytes per frame (every input, residual, output
 * and weight tensor counted once: the Eq. 9 accounting).  decoder_step_times
 * waits for the last profiled decoder_run and returns the elapsed milliseconds
 * of each step (count = decoder_num_steps); these intervals include the event
 * records themselves, several microseconds per step.
 * decoder_time_step measures one step without that overhead: after a
 * decoder_run with the same arguments has filled the workspace, it enqueues
 * step `step` `reps` times back to back between two HIP events on `stream`,
 * waits, and returns the mean milliseconds per launch.  The step runs on what
 * the workspace holds; steps timed in plan order see the tensors of a real
 * run, except that with separate_shortcut set the second convolution of a
 * channel-changing ResBlock accumulates onto its shortcut in place, once per
 * repetition.  Kernels branch on no tensor value; call decoder_run again before using the
 * frame or the workspace tensors. */
int decoder_set_profiling(wmdec_decoder* dec, int enable);
int decoder_num_steps(const wmdec_decoder* dec);
int decoder_step_info(const wmdec_decoder* dec, int index, const char** kernel, double* flops, double* bytes);
int decoder_step_times(const wmdec_decoder* dec, float* ms, int count);
int decoder_time_step(wmdec_decoder* dec, const void* latent, const void* packed, void* out, int batch,
                      int step, int reps, float* ms_per_launch, void* stream);

/* A plain copy of `bytes` bytes (a multiple of 16; both device pointers 16-byte
 * aligned, not overlapping) by one kernel, copy_u128_kernel, in which every
 * thread loads and stores 16 bytes: it reads and writes exactly `bytes` bytes
 * of HBM, which is what passes of hardware traffic counters over the benchmark
 * are scaled by (the counters' units differ between machines).  For callers
 * that measure; nothing in a decoder run uses it.  Asynchronous on `stream`. */
int wmdec_measure_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* WMDEC_MEASURE_H */
