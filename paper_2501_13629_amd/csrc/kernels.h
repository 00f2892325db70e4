// Internal declarations shared by the translation units of libdiffqkv (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <vector>

namespace diffqkv {

// Everything a decode launch needs; filled by the boundary after validation.
struct DecodeParams {
  const void* q;    // [B, n_q, d_qk]
  const void* k;    // contiguous cache or page pool
  const void* v;
  int64_t k_sb, k_sh, k_st;  // batch (or page) / head / token strides, in elements
  int64_t v_sb, v_sh, v_st;
  const int32_t* seqlens;      // device [B] or nullptr
  const int32_t* block_table;  // device [B, max_pages], paged only
  int32_t max_pages, page_size;
  int32_t T;  // uniform length, or upper bound when seqlens is given
  int32_t B, n_q, n_k, n_v, d_qk, d_v;
  int32_t n_groups;  // workgroup-owning heads per sequence: min(n_k, n_v)
  int32_t G;         // query rows per group: n_q / n_groups
  int32_t chunk;     // tokens per context split
  int32_t num_splits;
  float scale_log2;  // softmax scale * log2(e): scores live in the base-2 domain
  float* o_part;     // [B, n_q, num_splits, d_v] normalised partial outputs
  float* lse_part;   // [B, n_q, num_splits]      base-2 log-sum-exp of each split
  void* out;         // [B, n_q, d_v]
  float* lse_out;    // [B, n_q] or nullptr (natural log)
  // Ragged mode of the MFMA kernel (sk_cum != nullptr): equal slices of the unit space per
  // wavefront; num_splits then is the number of partial slots reserved per row.
  int32_t* sk_cum;     // workspace, [B + 1]: 32-token units of the sequences before b
  int32_t sk_workers;  // wavefronts launched (a multiple of 4)
  int32_t sk_lmin;     // smallest slice, in units
};

struct PrefillParams {
  const void* q;  // [B, n_q, S_q, d_qk]
  const void* k;  // [B, n_k, S_k, d_qk]
  const void* v;  // [B, n_v, S_k, d_v]
  void* out;      // [B, n_q, S_q, d_v]
  float* lse_out; // [B, n_q, S_q] or nullptr
  int32_t B, n_q, n_k, n_v, d_qk, d_v, S_q, S_k, causal;
  int32_t n_cu;  // compute units of the device (sizes the grid of the persistent kernel)
  float scale_log2;
};

// Strides here are in BYTES (the boundary converts).
struct AppendParams {
  const void* k_new;  // [B, n_k, d_qk]
  const void* v_new;  // [B, n_v, d_v]
  void* k;            // contiguous cache or page pool
  void* v;
  int64_t k_sb, k_sh, k_st;  // batch (or page) / head / token strides
  int64_t v_sb, v_sh, v_st;
  const int32_t* positions;    // device [B]: token index to write
  int32_t* seqlens_out;        // device [B] or nullptr: receives position + 1
  const int32_t* block_table;  // device [B, max_pages], paged only
  int32_t max_pages, page_size;
  int32_t capacity;            // positions >= capacity are skipped
  int32_t B, n_k, n_v;
  int32_t row_k_bytes, row_v_bytes;  // d_qk, d_v in bytes (multiples of 16)
};

// Decode with selective V fetching (top-k): strides in elements.
struct TopkParams {
  const void* q;
  const void* k;
  const void* v;
  int64_t k_sb, k_sh, k_st;
  int64_t v_sb, v_sh, v_st;
  const int32_t* seqlens;
  const int32_t* block_table;
  int32_t max_pages, page_size;
  int32_t T, T_pad;  // bound on the lengths; row length of the score workspace (multiple of 128)
  int32_t B, n_q, n_k, n_v, d_qk, d_v;
  int32_t top_k, renormalize;
  int32_t chunk;     // tokens per workgroup of the score kernel (multiple of 128)
  float scale_log2;
  float* scores;     // workspace [B, n_q, T_pad], base-2 domain
  void* out;
  float* lse_out;
  int32_t* sel_out;  // [B, n_q, top_k + 1] or nullptr
};

// dtype: 0 = fp32, 1 = bf16 (diffqkv_dtype).  All return a hipError_t from the launch.
hipError_t launch_decode_generic(const DecodeParams& p, int dtype, bool paged, hipStream_t s);
bool decode_mfma_supported(const DecodeParams& p, int dtype);
int decode_streamk_max_batch();
hipError_t launch_decode_mfma(const DecodeParams& p, bool paged, hipStream_t s);
hipError_t launch_combine(const DecodeParams& p, int dtype, hipStream_t s);
hipError_t launch_prefill_generic(const PrefillParams& p, int dtype, hipStream_t s);
bool prefill_mfma_supported(const PrefillParams& p, int dtype);
// variant: 0 choose; 8 / 4 wavefronts of 32 rows; 2 = the 64-row kernel where supported
hipError_t launch_prefill_mfma(const PrefillParams& p, int variant, hipStream_t s);
bool prefill_mfma64_supported(const PrefillParams& p, int dtype);       // d_v = 128, d_qk = 128 or 64
hipError_t launch_prefill_mfma64(const PrefillParams& p, hipStream_t s);  // 64 query rows per wavefront
int topk_max_k();
bool topk_scores_mfma_supported(const TopkParams& p, int dtype);
hipError_t launch_topk(const TopkParams& p, int dtype, bool paged, bool mfma, hipStream_t s);
hipError_t launch_append(const AppendParams& p, bool paged, hipStream_t s);

// One product of the augmented-Q feed-forward: out[M, N] = W0 x, or silu(W0 x) * (W1 x) when gated;
// x [M, K], W0 / W1 [N, K] row-major, everything in the I/O dtype.
struct AugqParams {
  const void* x;
  const void* w0;
  const void* w1;  // gated only
  void* out;
  int32_t M, K, N;
  int32_t n_cu;  // compute units of the device (chooses the tile height of the plain pass)
};
bool augq_mfma_supported(int dtype, int hidden, int inter);
hipError_t launch_augq(const AugqParams& p, int dtype, bool gated, bool mfma, hipStream_t s);
hipError_t launch_probe_stream_read(const void* src, size_t bytes, float* sink, hipStream_t s);

// ---- kernel timer (measurement aid of the experimental interface) ---------------------------------
// While the calling thread has the timer on, the main kernel of a call (which = 0: the decode split
// kernel, the prefill kernel, the top-k score kernel, the first augmented-Q product) and the kernel
// after it (which = 1: combine, select, second product) are launched with a pair of HIP events attached
// to their own dispatch: the difference of the pair is that kernel's duration, without the packets an
// event recorded around a launch adds.  Off (the normal state), a launch is the plain one.
struct KernelTimer {
  bool on;
  // event pairs handed to timed launches since the last read, and a pool they are taken from
  std::vector<hipEvent_t> start[2], stop[2], pool;
  bool next(int which, hipEvent_t* a, hipEvent_t* b);  // false if an event cannot be created
};
KernelTimer& kernel_timer();  // per thread; lives in api.hip
template <typename K, typename... A>
inline void launch_kernel(int which, K kernel, dim3 grid, dim3 block, size_t smem, hipStream_t s, A... args) {
  KernelTimer& t = kernel_timer();
  hipEvent_t a, b;
  if (t.on && t.next(which, &a, &b))
    hipExtLaunchKernelGGL(kernel, grid, block, smem, s, a, b, 0, args...);
  else
    kernel<<<grid, block, smem, s>>>(args...);
}

// ---- small device helpers -------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
// round-to-nearest-even fp32 -> bf16 bits (NaN stays NaN)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float load_as_float(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float load_as_float(const uint16_t* p, int64_t i) {
  return bf16_bits_to_float(p[i]);
}
__device__ __forceinline__ void store_from_float(float* p, int64_t i, float x) { p[i] = x; }
__device__ __forceinline__ void store_from_float(uint16_t* p, int64_t i, float x) {
  p[i] = float_to_bf16_bits(x);
}

constexpr float kLn2 = 0.69314718055994530942f;
constexpr float kLog2e = 1.44269504088896340736f;

}  // namespace diffqkv
