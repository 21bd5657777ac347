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
 *    16 row totals staged in LDS     17 staging barrier passed
 *    18 first pair add issued        19 first pair add returned   (calls that combine their K ranges
 *    20 last pair add returned           pairwise through 64-bit words instead of ticket and partial sums)
 *    21..23 unused
 * Process-wide state; not thread-safe.
 */
void codegemm_set_trace(uint64_t *stamps);

#ifdef __cplusplus
}
#endif
#endif /* CODEGEMM_TRACE_H */
