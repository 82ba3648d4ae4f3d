/*
 * maxsim_probe.h -- diagnostics for the benchmark of the fused MaxSim library (libmaxsim_probe.so).
 *
 * Not part of the operator and not ABI-stable: five kernels that show what an MI355X sustains, for roofline
 * context beside the library's own kernels.  Conventions (device pointers, `stream`, return codes) as in maxsim.h.
 *
 * maxsim_probe_mfma: a register-only loop of 32x32 MFMAs with four independent accumulators,
 *   512 workgroups x 4 wavefronts, `iters` rounds of 4 instructions per wavefront.
 *   kind 0 = fp16 (32x32x16), 1 = bf16 (32x32x16), 2 = int8 (32x32x32).  `operands` is >= 1 MiB of device memory
 *   whose bits are used as MFMA operands (random bits give the rate under realistic switching activity, zeros the
 *   rate at full clocks).  Operations per launch: 512 * 4 * iters * 4 * (2*32*32*16 for kinds 0/1, 2*32*32*32 for 2).
 * maxsim_probe_read: streams `bytes` (multiple of 16) from `buf` and discards them (a reference read rate);
 *   maxsim_probe_read_streaming does the same the way the streaming kernels read a corpus: every wavefront a
 *   contiguous run of its own, 1 KB per instruction, with non-temporal loads (the fastest read stream found).
 * maxsim_probe_copy: copies `bytes` (multiple of 16) from `src` to `dst`: a kernel of known HBM
 *   traffic for calibrating profiler byte counters.
 * maxsim_probe_gather: every wavefront (sixteen per CU) gathers iters x 16 pseudo-random whole rows of 256 bytes from
 *   `table` (`rows` rows, a power of two; rows * 256 bytes of device memory), sixteen loads in flight.  kind 0 = one row
 *   per load instruction (a dword per lane), kind 1 = four rows per load instruction (sixteen lanes x 16 bytes per
 *   row).  Returns the number of rows the launch gathers (> 0), or a negative error code.
 * `sink` is 4 bytes of device memory that is (practically) never written.
 */
#ifndef MAXSIM_PROBE_H
#define MAXSIM_PROBE_H

#include <stdint.h>

#include "maxsim.h"

#ifdef __cplusplus
extern "C" {
#endif

int maxsim_probe_mfma(int kind, const void *operands, int iters, float *sink, void *stream);
int maxsim_probe_read(const void *buf, int64_t bytes, float *sink, void *stream);
int maxsim_probe_read_streaming(const void *buf, int64_t bytes, float *sink, void *stream);
int maxsim_probe_copy(const void *src, void *dst, int64_t bytes, void *stream);
int64_t maxsim_probe_gather(int kind, const void *table, int64_t rows, int iters, float *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MAXSIM_PROBE_H */
