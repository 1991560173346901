/*
 * Measurement probes and one test hook of libfastar: NOT part of the method and not needed by any caller of fastar.h.
 * The benchmark uses them to report what this chip reaches on the two rooflines the kernels are priced
 * against, measured in the same process as the kernels.
 */
#ifndef FASTAR_PROBE_H
#define FASTAR_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 *   fastar_probe_mfma_bf16  register-resident bf16 32x32x16 matrix-instruction loop on every SIMD;
 *                           random_operands = 0: every operand element is 1.0 / 0.5; 1: operands drawn per lane, uniform
 *                           in (-2, 2).  The instruction stream is the same; the chip holds a lower clock under the
 *                           second (its power limit), so the two rates bracket what real data can reach;
 *                           *flops_out (host) receives the floating-point operations one launch performs;
 *                           sink is a device float the kernel may write (never does in practice).
 *   fastar_probe_copy       plain streaming copy of `bytes` (multiple of 16) from src to dst (device, 16-byte aligned).
 * Both enqueue one kernel on `stream`; the caller times them.
 */
int fastar_probe_mfma_bf16(int iters, int random_operands, float *sink, double *flops_out, void *stream);
int fastar_probe_copy(const void *src, void *dst, size_t bytes, void *stream);

/*
 * Test hook for the one place where workgroups of a launch wait for each other: the eviction plan of
 * tempcache_compress, whose waits are bounded.  Later calls of tempcache_compress (process-wide, all devices) bound
 * every such wait by `spin_limit` polls (negative: the built-in limit) and wait for `extra_arrivals` arrivals more than
 * will ever come (0: none), so a test can make the waits run out while every workgroup still finishes; the call then
 * reports status 1 for the heads concerned and leaves their cache untouched (see tempcache_compress).
 * fastar_debug_plan_wait(-1, 0) restores the normal behaviour.  Host state only; FASTAR_ERR_INVALID_ARG for a negative
 * extra_arrivals.
 */
int fastar_debug_plan_wait(int spin_limit, int extra_arrivals);

#ifdef __cplusplus
}
#endif
#endif /* FASTAR_PROBE_H */
