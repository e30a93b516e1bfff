/*
 * affmae_timing.h - per-kernel timing of the INSTRUMENTED build (libaffmae_timed.so).
 *
 * libaffmae_timed.so is the same source as libaffmae.so compiled with -DAFFMAE_TIMING;
 * it exports everything include/affmae.h declares plus the three calls below.  It exists
 * for benchmarks that need the duration of the individual kernels inside one API call;
 * the product library has none of this and keeps no state.
 *
 * While enabled, every kernel the library launches is bracketed by two HIP events on the
 * launch stream (events are created on first use and reused).  The read and reset calls
 * synchronise the device.  Timing must stay disabled under HIP graph capture.  The
 * registry is process-wide and guarded by a mutex; it is not meant for concurrent launches.
 *   affmae_timing_read: fills the `index`-th entry (kernel name, total milliseconds,
 *   number of launches) if it exists; returns the entry count.
 */
#ifndef AFFMAE_TIMING_H_
#define AFFMAE_TIMING_H_

#ifdef __cplusplus
extern "C" {
#endif

void affmae_timing_enable(int on);
void affmae_timing_reset(void);
int affmae_timing_read(int index, char* name, int name_len, double* total_ms, int* count);

#ifdef __cplusplus
}
#endif
#endif /* AFFMAE_TIMING_H_ */
