/*
 * zr_debug.h - measuring and debugging aids of libzr.  NOT part of the product
 * boundary (zr.h): nothing on the hot path needs them.  Unlike the calls of zr.h
 * they keep state between calls: a flag, the last kernel's name and a pair of
 * event handles, all PER HOST THREAD (thread_local); a product call only looks at
 * them when zr_debug_record_kernel_names(1) or zr_debug_time_next_product armed
 * them on the same thread.
 */
#ifndef ZR_DEBUG_H
#define ZR_DEBUG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Switches the recording of GEMM kernel names on (non-zero) or off (0, the
 * default) for the calling thread.  While off, product calls format no name. */
void zr_debug_record_kernel_names(int on);

/* Name (as a profiler prints it, without namespaces) of the GEMM kernel
 * instantiation that the last forward / backward / accumulate product of this
 * thread launched while recording was on; "" if none. */
const char* zr_debug_last_kernel(void);

/* The NEXT forward / backward / accumulate product of this thread records the
 * two caller-owned HIP events (hipEvent_t, created with timing) on its stream
 * immediately before and after its own GEMM launch(es), leaving out an
 * extraction that precedes it and an imputation pass that follows, and records
 * the kernel's name.  One shot; a backward call that computes dX and dW times
 * the first of the two.  Errors: NULL. */
int zr_debug_time_next_product(void* start_event, void* stop_event);

/* Launches `blocks` workgroups of 4 wavefronts that each issue `iters` x 8
 * independent bf16 MFMAs (32 x 32 x 16, fp32 accumulate) on register operands,
 * with no memory traffic.  Timed by the caller, it gives the rate the matrix
 * cores sustain at the clock the chip holds under that load, to set beside the
 * published peak.  sink: device, at least `blocks` floats, overwritten.
 * Returns the FLOPs the launch performs through *flops (host, may be NULL).
 * Errors: NULL, SHAPE (blocks or iters < 1, or blocks > 2^20). */
int zr_debug_mfma_rate(int32_t blocks, int32_t iters, float* sink, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ZR_DEBUG_H */
