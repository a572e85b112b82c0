/*
 * tp_probe.h -- C ABI of libtpprobe, a measurement aid that ships beside libtplinear for bench.py only.
 */
#ifndef TP_PROBE_H
#define TP_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * tp_mfma_probe -- enqueues, on the HIP stream given (a hipStream_t cast to void*), a register-resident
 * loop of dense bf16 32x32x16 MFMAs on 256 workgroups of four waves, and reports in *flops (a HOST
 * pointer, written before the call returns) how many floating-point operations the launch performs.
 * Timed by the caller, it gives the dense-bf16 rate the chip sustains with nothing else running.
 * scratch: DEVICE buffer of at least 256 x 256 x 4 bytes, 16-byte aligned (receives checksums).
 * Returns 0, or the tp_status_t value of the failed check (1 null, 4 iters < 1, 7 scratch, 8 launch).
 */
int tp_mfma_probe(void* scratch, size_t scratch_bytes, int iters, double* flops, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* TP_PROBE_H */
