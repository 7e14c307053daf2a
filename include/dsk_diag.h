/*
 * dsk_diag - device measurements that benchmarks quote next to the product library's results.  A library of its
 * own (libdsk_diag.so): nothing in libdsk.so depends on it, and it implements no step of the method.
 */
#ifndef DSK_DIAG_H
#define DSK_DIAG_H

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define DSK_DIAG_API __attribute__((visibility("default")))
#else
#define DSK_DIAG_API
#endif

/* Matrix-core throughput this device sustains, in TFLOP/s: a register-only bf16 MFMA loop on every CU of the
 * current device, timed with HIP events on `stream` (a hipStream_t; blocks until done; allocates and frees a small
 * device buffer).  Returns 0, -1 for a null argument, -5 when a HIP call failed. */
DSK_DIAG_API int dsk_diag_mfma_peak(double* tflops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DSK_DIAG_H */
