/*
 * diffqkv -- experimental knobs and measurement aids.  Not part of the product interface of
 * diffqkv.h: tests and benchmarks use them to force a kernel variant or to time one kernel of a call.
 *
 * Everything set here is PER THREAD: it changes only later calls made by the thread that set it, so
 * the product entry points stay free of state shared between threads.
 */
#ifndef DIFFQKV_EXPERIMENTAL_H_
#define DIFFQKV_EXPERIMENTAL_H_

#include "diffqkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Optional knobs; zero fields mean "library default".  They apply to the calling thread's later
 * calls, the *_workspace_bytes queries included (a query and the call it sizes must see the same
 * knobs). */
typedef struct {
  int32_t decode_chunk_tokens; /* tokens per context split (multiple of 128)                      */
  int32_t force_generic;       /* 1: always take the portable kernels instead of the MFMA ones    */
  int32_t prefill_waves;       /* MFMA prefill variant: 0 choose; 8 or 4 wavefronts of 32 rows;  *
                                * 2 = 4 wavefronts of 64 rows (where that kernel exists)          */
  int32_t decode_ragged_mode;  /* work split of the MFMA decode kernel.  0: equal slices per
                                  wavefront when seqlens is given, fixed-size chunks otherwise;
                                  1: equal slices always; 2: fixed-size chunks always            */
  int32_t decode_workers;      /* wavefronts launched by the equal-slice split (multiple of 4)   */
  int32_t reserved[3];
} diffqkv_tuning;
void diffqkv_set_tuning(const diffqkv_tuning* t /* host; NULL resets */);

/*
 * Kernel timer.  While it is on, the main kernel of every call of this thread (the split kernel of a
 * decode call, the prefill kernel, the score kernel of a top-k call, the first product of the
 * augmented-Q call) and the kernel that follows it (combine, select, second product) are launched with
 * a pair of HIP events attached to their own dispatch, so that the pair reads that kernel's duration
 * and nothing else.  diffqkv_kernel_timer_read waits for every timed launch of this thread since the
 * last read and returns the average duration of the main kernel and of the second kernel in
 * microseconds (0 where none was launched) and the number of main-kernel launches; any pointer may
 * be NULL.  Both return a diffqkv_status.  Timed launches create HIP events, which are pooled and live
 * until the process ends: switch the timer on for measurements only.
 */
int diffqkv_kernel_timer(int on);
int diffqkv_kernel_timer_read(float* main_us /* host */, float* second_us /* host */,
                              int32_t* main_launches /* host */);

/*
 * Reads `bytes` (a multiple of 16) from `src` (device) with 128-bit loads, as fast as the memory
 * system allows, and writes one float per workgroup to `sink` (device, at least 4096 floats) so the
 * reads cannot be elided.  Measures the achievable HBM read rate beside the decode kernels.
 */
int diffqkv_probe_stream_read(const void* src, size_t bytes, float* sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DIFFQKV_EXPERIMENTAL_H_ */
