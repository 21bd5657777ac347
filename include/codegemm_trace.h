/*
 * codegemm_trace.h - the extra entry points of the DIAGNOSTIC build of the
 * library (libcodegemm_trace.so, compiled with -DCODEGEMM_TRACE).  That build
 * exports the whole ABI of codegemm.h with the same behaviour, except that the
 * gather kernels of codegemm_gemm record device clock stamps of their phases,
 * which costs registers and time; it is for measuring where a call's time
 * goes (the analogue of the paper's build/read phase study, Appendix A.1),
 * never for production.  libcodegemm.so does not export these symbols.
 */
#ifndef CODEGEMM_TRACE_H
#define CODEGEMM_TRACE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Sets (or, with NULL, clears) the device buffer the next codegemm_gemm calls
 * stamp into: uint64 stamps[workgroups of batch group 0][24], workgroup index
 * = row_block * k_splits + k_range, values of the 100 MHz constant device
 * clock, 0 = not reached.  The caller owns the buffer and zeroes it.  Slots:
 *    0 kernel entered                1 first Psumbook built
 *    2 prologue loads issued         3 output stored (single range, or the reducing workgroup)
 *    4 streaming loop done           5 partial sums issued
 *    6 partial sums acknowledged     7 ticket drawn
 *    8..15 unit (or tile) 0..7 done, slot 15 also for every later one
 *    16 row totals staged in LDS     17 staging barrier passed    18..23 unused
 * Process-wide state; not thread-safe.
 */
void codegemm_set_trace(uint64_t *stamps);

/*
 * Probe of how many vector loads a compute unit keeps outstanding (the fact the
 * depth of the gather kernels' code ring is chosen by).  Launches `workgroups`
 * workgroups of `waves` (1..16) wavefronts; every lane issues `loads_per_lane`
 * (1, 2, 4 or 8) coalesced 16-byte loads from its workgroup's own stretch of
 * `src` (device, 16-byte aligned, src_bytes >= workgroups * waves * 64 * 16 *
 * loads_per_lane + 16; read only) and then waits for them.  `out` (device,
 * caller-owned): uint64 [workgroups][waves][4] followed by 8 spare bytes; per
 * wavefront, shader-clock counts since its own start at which [0] its loads
 * were all issued, [1] its first datum was there, [2] all its data were there,
 * and [3] that last span in ticks of the constant 100 MHz clock.  Returns a
 * CODEGEMM_* status; enqueues on `stream`, does not synchronise.
 */
int codegemm_probe_load_issue(const void *src, size_t src_bytes, int workgroups, int waves,
                              int loads_per_lane, uint64_t *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CODEGEMM_TRACE_H */
