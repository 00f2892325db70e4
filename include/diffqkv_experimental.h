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
 * When `hip_event` (a hipEvent_t passed as void*) is not NULL, every later decode call of this
 * thread records it on its stream between the split kernel and the combine kernel, so a caller that
 * brackets the call with two events of its own can time the two kernels separately.  NULL turns it
 * off.
 */
void diffqkv_set_split_event(void* hip_event);

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
