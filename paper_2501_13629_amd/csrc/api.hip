// The C ABI of libdiffqkv: argument validation, split planning and kernel dispatch.
// Declarations and their documentation live in include/diffqkv.h.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "../../include/diffqkv.h"
#include "../../include/diffqkv_experimental.h"
#include "kernels.h"

using namespace diffqkv;

// Scratch memory of diffqkv_decode_static: the partial results of the context splits live here instead
// of in a caller's workspace, so that the call allocates nothing.  One copy per GPU, at an address of
// its own on each; the name below is only a host-side handle for hipGetSymbolAddress, never an address
// to hand to a kernel.
static __device__ __align__(256) unsigned char scratch[DIFFQKV_STATIC_SCRATCH_BYTES];

namespace {

// Experimental knobs are per thread: they change only the calls of the thread that set them, and the
// product entry points share no mutable state between threads.
thread_local diffqkv_tuning t_tuning = {};
thread_local KernelTimer t_kernel_timer = {};

// Compute units of the current device, read once per device.  Without a device (validation-only use
// on a host without a GPU) the figure of the chip this library is built for stands in.
constexpr int kDefaultComputeUnits = 256;
constexpr int kMaxDevices = 64;
std::atomic<int> g_compute_units[kMaxDevices];
int compute_units() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return kDefaultComputeUnits;
  int cu = g_compute_units[dev].load(std::memory_order_relaxed);
  if (cu > 0) return cu;
  if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0)
    return kDefaultComputeUnits;
  g_compute_units[dev].store(cu, std::memory_order_relaxed);
  return cu;
}

// Device address of `scratch` on the current device, looked up on the first call there.
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};
int static_scratch(void** ptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return DIFFQKV_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return DIFFQKV_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return DIFFQKV_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return DIFFQKV_OK;
}

// Split plan, a pure function of the shapes and of the device's compute-unit count.  Measured on
// MI355X: the decode kernel streams fastest when the whole context fits one round of workgroups, one
// per compute unit, each as long as possible (every extra round exposes a prologue and an epilogue
// with no loads in flight).
constexpr int kChunkQuantum = 128;  // one workgroup step of the decode kernels
constexpr int kMinChunk = 128;
constexpr int kMaxChunk = 8192;
// With per-sequence lengths the work per (sequence, head) is uneven and unknown on the host:
// shorter chunks let the hardware dispatcher balance it.
constexpr int kMaxChunkRagged = 2048;

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_size(int dtype) { return dtype == DIFFQKV_F32 ? 4 : 2; }
inline bool stride_ok(int64_t stride, int dtype) { return stride >= 0 && (stride * (int64_t)elem_size(dtype)) % 16 == 0; }

int check_shape(const diffqkv_shape* s) {
  if (!s) return DIFFQKV_ERR_NULL;
  if (s->B < 0 || s->n_q <= 0 || s->n_k <= 0 || s->n_v <= 0) return DIFFQKV_ERR_SHAPE;
  if (s->d_qk < 8 || s->d_qk > 256 || s->d_qk % 8 || s->d_v < 8 || s->d_v > 256 || s->d_v % 8)
    return DIFFQKV_ERR_SHAPE;
  if (s->dtype != DIFFQKV_F32 && s->dtype != DIFFQKV_BF16) return DIFFQKV_ERR_SHAPE;
  if (!(s->softmax_scale >= 0.f) || isinf(s->softmax_scale)) return DIFFQKV_ERR_SHAPE;
  if (s->n_q % s->n_k || s->n_q % s->n_v) return DIFFQKV_ERR_HEADS;
  const int hi = s->n_k > s->n_v ? s->n_k : s->n_v, lo = s->n_k > s->n_v ? s->n_v : s->n_k;
  if (hi % lo) return DIFFQKV_ERR_HEADS;
  return DIFFQKV_OK;
}

float scale_log2(const diffqkv_shape* s) {
  const float scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / sqrtf((float)s->d_qk);
  return scale * kLog2e;
}

// Context split: a pure function of the shapes so that results are repeatable bit for bit.
void plan_decode(const diffqkv_shape* s, int32_t max_T, bool ragged, int32_t* chunk, int32_t* num_splits) {
  int c;
  if (t_tuning.decode_chunk_tokens > 0) {
    c = (t_tuning.decode_chunk_tokens + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
  } else {
    const int groups = (s->n_k < s->n_v ? s->n_k : s->n_v) * (s->B > 0 ? s->B : 1);
    const int64_t total = (int64_t)max_T * groups;
    const int target = compute_units();  // one workgroup per compute unit
    int64_t per = (total + target - 1) / target;
    per = (per + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum;
    const int hi = ragged ? kMaxChunkRagged : kMaxChunk;
    c = (int)(per < kMinChunk ? kMinChunk : (per > hi ? hi : per));
  }
  *chunk = c;
  int n = (int)(((int64_t)max_T + c - 1) / c);
  *num_splits = n < 1 ? 1 : n;
}

size_t workspace_for(const diffqkv_shape* s, int32_t num_splits) {
  if (num_splits <= 1) return 0;
  size_t rows = (size_t)s->B * s->n_q * num_splits;
  size_t bytes = rows * ((size_t)s->d_v + 1) * sizeof(float);
  return (bytes + 255) / 256 * 256;
}

// Ragged mode of the MFMA decode kernel: one worker per wavefront, two workgroups per compute unit,
// equal slices of the 32-token-unit space.  The smallest slice (and with it the number of partial
// slots a row can need) is fixed from the host-side bound on the work, so that small batches still
// spread over the whole chip while large ones keep the partial results few.
int streamk_workers() {
  return t_tuning.decode_workers > 0 ? (t_tuning.decode_workers + 3) / 4 * 4 : 2 * compute_units() * 4;
}
struct StreamKPlan {
  bool use;
  int32_t lmin, slots;
  size_t cum_bytes, bytes;
};
StreamKPlan plan_streamk(const diffqkv_shape* s, int32_t max_T) {
  StreamKPlan k = {};
  if (t_tuning.decode_ragged_mode == 2 || s->dtype != DIFFQKV_BF16 || s->B <= 0 || max_T <= 0) return k;
  if (s->B > decode_streamk_max_batch()) return k;
  int32_t chunk, splits;
  plan_decode(s, max_T, true, &chunk, &splits);
  if (splits <= 1) return k;  // a context this short runs in a single pass without partial results
  const int64_t u_max = (max_T + 31) / 32;
  int64_t lmin = ((int64_t)s->B * s->n_k * u_max + streamk_workers() - 1) / streamk_workers();
  lmin = lmin < 4 ? 4 : (lmin > 32 ? 32 : lmin);
  k.use = true;
  k.lmin = (int32_t)lmin;
  k.slots = (int32_t)((u_max + lmin - 1) / lmin) + 1;
  k.cum_bytes = ((size_t)(s->B + 1) * sizeof(int32_t) + 255) / 256 * 256;
  k.bytes = k.cum_bytes + workspace_for(s, k.slots < 2 ? 2 : k.slots);
  return k;
}

int run_decode(const diffqkv_shape* s, DecodeParams& p, bool paged, void* workspace,
               size_t workspace_bytes, hipStream_t stream) {
  p.B = s->B;
  p.n_q = s->n_q;
  p.n_k = s->n_k;
  p.n_v = s->n_v;
  p.d_qk = s->d_qk;
  p.d_v = s->d_v;
  p.n_groups = s->n_k < s->n_v ? s->n_k : s->n_v;
  p.G = s->n_q / p.n_groups;
  p.scale_log2 = scale_log2(s);
  const bool mfma = !t_tuning.force_generic && decode_mfma_supported(p, s->dtype);
  // ragged lengths on the MFMA kernel: equal slices per wavefront instead of fixed chunks
  StreamKPlan sk = {};
  if (mfma && (p.seqlens != nullptr || t_tuning.decode_ragged_mode == 1)) sk = plan_streamk(s, p.T);
  size_t need;
  if (sk.use) {
    p.chunk = 0;
    p.num_splits = sk.slots < 2 ? 2 : sk.slots;
    need = sk.bytes;
  } else {
    plan_decode(s, p.T, p.seqlens != nullptr, &p.chunk, &p.num_splits);
    need = workspace_for(s, p.num_splits);
  }
  if (need) {
    if (!workspace || workspace_bytes < need) return DIFFQKV_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DIFFQKV_ERR_ALIGN;
  }
  if (sk.use) {
    p.sk_cum = (int32_t*)workspace;
    p.sk_workers = streamk_workers();
    p.sk_lmin = sk.lmin;
    p.o_part = (float*)((char*)workspace + sk.cum_bytes);
  } else {
    p.o_part = (float*)workspace;
  }
  p.lse_part = need ? p.o_part + (size_t)s->B * s->n_q * p.num_splits * s->d_v : nullptr;
  if (s->B == 0) return DIFFQKV_OK;
  hipError_t e;
  if (mfma)
    e = launch_decode_mfma(p, paged, stream);
  else
    e = launch_decode_generic(p, s->dtype, paged, stream);
  if (e != hipSuccess) return DIFFQKV_ERR_HIP;
  if (p.num_splits > 1) {
    e = launch_combine(p, s->dtype, stream);
    if (e != hipSuccess) return DIFFQKV_ERR_HIP;
  }
  return DIFFQKV_OK;
}

}  // namespace

namespace diffqkv {
KernelTimer& kernel_timer() { return t_kernel_timer; }
bool KernelTimer::next(int which, hipEvent_t* a, hipEvent_t* b) {
  hipEvent_t e[2];
  for (int i = 0; i < 2; ++i) {
    if (!pool.empty()) {
      e[i] = pool.back();
      pool.pop_back();
    } else if (hipEventCreate(&e[i]) != hipSuccess) {
      if (i == 1) pool.push_back(e[0]);
      return false;
    }
  }
  start[which].push_back(e[0]);
  stop[which].push_back(e[1]);
  *a = e[0];
  *b = e[1];
  return true;
}
}  // namespace diffqkv

extern "C" {

void diffqkv_set_tuning(const diffqkv_tuning* t) {
  if (t)
    t_tuning = *t;
  else
    memset(&t_tuning, 0, sizeof t_tuning);
}

int diffqkv_kernel_timer(int on) {
  KernelTimer& t = t_kernel_timer;
  t.on = on != 0;
  return DIFFQKV_OK;
}

int diffqkv_kernel_timer_read(float* main_us, float* second_us, int32_t* main_launches) {
  KernelTimer& t = t_kernel_timer;
  float* dst[2] = {main_us, second_us};
  if (main_launches) *main_launches = (int32_t)t.start[0].size();
  int rc = DIFFQKV_OK;
  for (int w = 0; w < 2; ++w) {
    double sum_ms = 0.0;
    const size_t n = t.start[w].size();
    for (size_t i = 0; i < n; ++i) {
      float ms = 0.f;
      if (hipEventSynchronize(t.stop[w][i]) != hipSuccess ||
          hipEventElapsedTime(&ms, t.start[w][i], t.stop[w][i]) != hipSuccess)
        rc = DIFFQKV_ERR_HIP;
      sum_ms += ms;
      t.pool.push_back(t.start[w][i]);
      t.pool.push_back(t.stop[w][i]);
    }
    t.start[w].clear();
    t.stop[w].clear();
    if (dst[w]) *dst[w] = n ? (float)(sum_ms * 1e3 / (double)n) : 0.f;
  }
  return rc;
}

size_t diffqkv_decode_workspace_bytes(const diffqkv_shape* shape, int32_t max_T) {
  if (check_shape(shape) != DIFFQKV_OK || max_T < 0) return 0;
  // the fixed-chunk plan for ragged lengths never has fewer splits than the uniform one, and the
  // equal-slice plan of the MFMA kernel has a size of its own: the figure covers all three
  int32_t chunk, splits;
  plan_decode(shape, max_T, true, &chunk, &splits);
  size_t bytes = workspace_for(shape, splits);
  const StreamKPlan sk = plan_streamk(shape, max_T);
  if (sk.use && sk.bytes > bytes) bytes = sk.bytes;
  return bytes;
}

int diffqkv_decode(const diffqkv_shape* shape, const void* q, const void* k_cache,
                   const void* v_cache, int64_t k_stride_b, int64_t k_stride_h, int64_t k_stride_t,
                   int64_t v_stride_b, int64_t v_stride_h, int64_t v_stride_t,
                   const int32_t* seqlens, int32_t T, void* out, float* lse_out, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(shape);
  if (rc != DIFFQKV_OK) return rc;
  if (T < 0) return DIFFQKV_ERR_SHAPE;
  if (shape->B > 0) {
    if (!q || !out) return DIFFQKV_ERR_NULL;
    if (T > 0 && (!k_cache || !v_cache)) return DIFFQKV_ERR_NULL;
  }
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out))
    return DIFFQKV_ERR_ALIGN;
  const int dt = shape->dtype;
  if (!stride_ok(k_stride_b, dt) || !stride_ok(k_stride_h, dt) || !stride_ok(k_stride_t, dt) ||
      !stride_ok(v_stride_b, dt) || !stride_ok(v_stride_h, dt) || !stride_ok(v_stride_t, dt))
    return DIFFQKV_ERR_ALIGN;
  if (k_stride_t < shape->d_qk || v_stride_t < shape->d_v) return DIFFQKV_ERR_SHAPE;
  DecodeParams p = {};
  p.q = q;
  p.k = k_cache;
  p.v = v_cache;
  p.k_sb = k_stride_b;
  p.k_sh = k_stride_h;
  p.k_st = k_stride_t;
  p.v_sb = v_stride_b;
  p.v_sh = v_stride_h;
  p.v_st = v_stride_t;
  p.seqlens = seqlens;
  p.T = T;
  p.out = out;
  p.lse_out = lse_out;
  return run_decode(shape, p, false, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

int diffqkv_decode_static(const diffqkv_shape* shape, const void* q, const void* k_cache,
                          const void* v_cache, int64_t k_stride_b, int64_t k_stride_h, int64_t k_stride_t,
                          int64_t v_stride_b, int64_t v_stride_h, int64_t v_stride_t,
                          const int32_t* seqlens, int32_t T, void* out, float* lse_out, void* hip_stream) {
  // sizes first: a call whose partial results do not fit the static buffer is refused outright
  if (check_shape(shape) == DIFFQKV_OK && T >= 0 &&
      diffqkv_decode_workspace_bytes(shape, T) > (size_t)DIFFQKV_STATIC_SCRATCH_BYTES)
    return DIFFQKV_ERR_STATIC_LIMIT;
  void* ptr = nullptr;
  if (shape && shape->B > 0) {  // (the empty batch launches nothing and needs no device)
    const int rc = static_scratch(&ptr);
    if (rc != DIFFQKV_OK) return rc;
  }
  // Nothing in the buffer has to start at zero: a split's slot is written before the combine kernel
  // reads it, and slots of splits past the end of a sequence are never read.
  return diffqkv_decode(shape, q, k_cache, v_cache, k_stride_b, k_stride_h, k_stride_t, v_stride_b, v_stride_h,
                        v_stride_t, seqlens, T, out, lse_out, ptr, ptr ? (size_t)DIFFQKV_STATIC_SCRATCH_BYTES : 0,
                        hip_stream);
}

int diffqkv_decode_paged(const diffqkv_shape* shape, const void* q, const void* k_pool,
                         const void* v_pool, int64_t k_stride_page, int64_t k_stride_h,
                         int64_t k_stride_t, int64_t v_stride_page, int64_t v_stride_h,
                         int64_t v_stride_t, const int32_t* block_table, int32_t max_pages,
                         int32_t page_size, const int32_t* seqlens, void* out, float* lse_out,
                         void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(shape);
  if (rc != DIFFQKV_OK) return rc;
  if (max_pages < 0 || page_size <= 0) return DIFFQKV_ERR_SHAPE;
  if ((int64_t)max_pages * page_size > INT32_MAX) return DIFFQKV_ERR_SHAPE;
  if (shape->B > 0) {
    if (!q || !out || !seqlens) return DIFFQKV_ERR_NULL;
    if (max_pages > 0 && (!k_pool || !v_pool || !block_table)) return DIFFQKV_ERR_NULL;
  }
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(out))
    return DIFFQKV_ERR_ALIGN;
  const int dt = shape->dtype;
  if (!stride_ok(k_stride_page, dt) || !stride_ok(k_stride_h, dt) || !stride_ok(k_stride_t, dt) ||
      !stride_ok(v_stride_page, dt) || !stride_ok(v_stride_h, dt) || !stride_ok(v_stride_t, dt))
    return DIFFQKV_ERR_ALIGN;
  if (k_stride_t < shape->d_qk || v_stride_t < shape->d_v) return DIFFQKV_ERR_SHAPE;
  DecodeParams p = {};
  p.q = q;
  p.k = k_pool;
  p.v = v_pool;
  p.k_sb = k_stride_page;
  p.k_sh = k_stride_h;
  p.k_st = k_stride_t;
  p.v_sb = v_stride_page;
  p.v_sh = v_stride_h;
  p.v_st = v_stride_t;
  p.seqlens = seqlens;
  p.block_table = block_table;
  p.max_pages = max_pages;
  p.page_size = page_size;
  p.T = max_pages * page_size;
  p.out = out;
  p.lse_out = lse_out;
  return run_decode(shape, p, true, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

static int32_t topk_row(int32_t max_T) { return (max_T + 127) / 128 * 128; }

size_t diffqkv_decode_topk_workspace_bytes(const diffqkv_shape* shape, int32_t max_T) {
  if (check_shape(shape) != DIFFQKV_OK || max_T < 0) return 0;
  const size_t bytes = (size_t)shape->B * shape->n_q * topk_row(max_T) * sizeof(float);
  return (bytes + 255) / 256 * 256;
}

static int run_topk(const diffqkv_shape* shape, TopkParams& p, bool paged, int32_t top_k, int32_t renormalize,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (top_k < 0) return DIFFQKV_ERR_SHAPE;
  if (top_k > topk_max_k()) return DIFFQKV_ERR_UNSUPPORTED;  // more rows than the select kernel keeps on chip
  const size_t need = diffqkv_decode_topk_workspace_bytes(shape, p.T);
  if (need) {
    if (!workspace || workspace_bytes < need) return DIFFQKV_ERR_WORKSPACE;
    if (!aligned16(workspace)) return DIFFQKV_ERR_ALIGN;
  }
  p.T_pad = topk_row(p.T);
  p.B = shape->B;
  p.n_q = shape->n_q;
  p.n_k = shape->n_k;
  p.n_v = shape->n_v;
  p.d_qk = shape->d_qk;
  p.d_v = shape->d_v;
  p.top_k = top_k;
  p.renormalize = renormalize ? 1 : 0;
  p.chunk = t_tuning.decode_chunk_tokens > 0
                ? (t_tuning.decode_chunk_tokens + kChunkQuantum - 1) / kChunkQuantum * kChunkQuantum
                : 512;
  p.scale_log2 = scale_log2(shape);
  p.scores = (float*)workspace;
  if (shape->B == 0) return DIFFQKV_OK;
  const bool mfma = !t_tuning.force_generic && topk_scores_mfma_supported(p, shape->dtype);
  return launch_topk(p, shape->dtype, paged, mfma, (hipStream_t)hip_stream) == hipSuccess ? DIFFQKV_OK
                                                                                             : DIFFQKV_ERR_HIP;
}

int diffqkv_decode_topk(const diffqkv_shape* shape, const void* q, const void* k_cache, const void* v_cache,
                        int64_t k_stride_b, int64_t k_stride_h, int64_t k_stride_t, int64_t v_stride_b,
                        int64_t v_stride_h, int64_t v_stride_t, const int32_t* seqlens, int32_t T,
                        int32_t top_k, int32_t renormalize, void* out, float* lse_out, int32_t* sel_out,
                        void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_shape(shape);
  if (rc != DIFFQKV_OK) return rc;
  if (T < 0) return DIFFQKV_ERR_SHAPE;
  if (shape->B > 0) {
    if (!q || !out) return DIFFQKV_ERR_NULL;
    if (T > 0 && (!k_cache || !v_cache)) return DIFFQKV_ERR_NULL;
  }
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return DIFFQKV_ERR_ALIGN;
  const int dt = shape->dtype;
  if (!stride_ok(k_stride_b, dt) || !stride_ok(k_stride_h, dt) || !stride_ok(k_stride_t, dt) ||
      !stride_ok(v_stride_b, dt) || !stride_ok(v_stride_h, dt) || !stride_ok(v_stride_t, dt))
    return DIFFQKV_ERR_ALIGN;
  if (k_stride_t < shape->d_qk || v_stride_t < shape->d_v) return DIFFQKV_ERR_SHAPE;
  TopkParams p = {};
  p.q = q;
  p.k = k_cache;
  p.v = v_cache;
  p.k_sb = k_stride_b;
  p.k_sh = k_stride_h;
  p.k_st = k_stride_t;
  p.v_sb = v_stride_b;
  p.v_sh = v_stride_h;
  p.v_st = v_stride_t;
  p.seqlens = seqlens;
  p.T = T;
  p.out = out;
  p.lse_out = lse_out;
  p.sel_out = sel_out;
  return run_topk(shape, p, false, top_k, renormalize, workspace, workspace_bytes, hip_stream);
}

int diffqkv_decode_topk_paged(const diffqkv_shape* shape, const void* q, const void* k_pool, const void* v_pool,
                              int64_t k_stride_page, int64_t k_stride_h, int64_t k_stride_t,
                              int64_t v_stride_page, int64_t v_stride_h, int64_t v_stride_t,
                              const int32_t* block_table, int32_t max_pages, int32_t page_size,
                              const int32_t* seqlens, int32_t top_k, int32_t renormalize, void* out,
                              float* lse_out, int32_t* sel_out, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
  int rc = check_shape(shape);
  if (rc != DIFFQKV_OK) return rc;
  if (max_pages < 0 || page_size <= 0) return DIFFQKV_ERR_SHAPE;
  if ((int64_t)max_pages * page_size > INT32_MAX) return DIFFQKV_ERR_SHAPE;
  if (shape->B > 0) {
    if (!q || !out || !seqlens) return DIFFQKV_ERR_NULL;
    if (max_pages > 0 && (!k_pool || !v_pool || !block_table)) return DIFFQKV_ERR_NULL;
  }
  if (!aligned16(q) || !aligned16(k_pool) || !aligned16(v_pool) || !aligned16(out)) return DIFFQKV_ERR_ALIGN;
  const int dt = shape->dtype;
  if (!stride_ok(k_stride_page, dt) || !stride_ok(k_stride_h, dt) || !stride_ok(k_stride_t, dt) ||
      !stride_ok(v_stride_page, dt) || !stride_ok(v_stride_h, dt) || !stride_ok(v_stride_t, dt))
    return DIFFQKV_ERR_ALIGN;
  if (k_stride_t < shape->d_qk || v_stride_t < shape->d_v) return DIFFQKV_ERR_SHAPE;
  TopkParams p = {};
  p.q = q;
  p.k = k_pool;
  p.v = v_pool;
  p.k_sb = k_stride_page;
  p.k_sh = k_stride_h;
  p.k_st = k_stride_t;
  p.v_sb = v_stride_page;
  p.v_sh = v_stride_h;
  p.v_st = v_stride_t;
  p.seqlens = seqlens;
  p.block_table = block_table;
  p.max_pages = max_pages;
  p.page_size = page_size;
  p.T = max_pages * page_size;
  p.out = out;
  p.lse_out = lse_out;
  p.sel_out = sel_out;
  return run_topk(shape, p, true, top_k, renormalize, workspace, workspace_bytes, hip_stream);
}

static int run_append(const diffqkv_shape* shape, const void* k_new, const void* v_new, void* k, void* v,
                      int64_t k_s0, int64_t k_sh, int64_t k_st, int64_t v_s0, int64_t v_sh, int64_t v_st,
                      const int32_t* block_table, int32_t max_pages, int32_t page_size,
                      const int32_t* positions, int32_t capacity, int32_t* seqlens_out, bool paged,
                      void* hip_stream) {
  int rc = check_shape(shape);
  if (rc != DIFFQKV_OK) return rc;
  if (capacity < 0) return DIFFQKV_ERR_SHAPE;
  const int64_t es = (int64_t)elem_size(shape->dtype);
  if ((shape->d_qk * es) % 16 || (shape->d_v * es) % 16) return DIFFQKV_ERR_SHAPE;
  if (shape->B > 0) {
    if (!k_new || !v_new || !positions) return DIFFQKV_ERR_NULL;
    if (capacity > 0 && (!k || !v)) return DIFFQKV_ERR_NULL;
    if (paged && capacity > 0 && !block_table) return DIFFQKV_ERR_NULL;
  }
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k) || !aligned16(v)) return DIFFQKV_ERR_ALIGN;
  const int dt = shape->dtype;
  if (!stride_ok(k_s0, dt) || !stride_ok(k_sh, dt) || !stride_ok(k_st, dt) || !stride_ok(v_s0, dt) ||
      !stride_ok(v_sh, dt) || !stride_ok(v_st, dt))
    return DIFFQKV_ERR_ALIGN;
  if (k_st < shape->d_qk || v_st < shape->d_v) return DIFFQKV_ERR_SHAPE;
  AppendParams p = {};
  p.k_new = k_new;
  p.v_new = v_new;
  p.k = k;
  p.v = v;
  p.k_sb = k_s0 * es;
  p.k_sh = k_sh * es;
  p.k_st = k_st * es;
  p.v_sb = v_s0 * es;
  p.v_sh = v_sh * es;
  p.v_st = v_st * es;
  p.positions = positions;
  p.seqlens_out = seqlens_out;
  p.block_table = block_table;
  p.max_pages = max_pages;
  p.page_size = page_size;
  p.capacity = capacity;
  p.B = shape->B;
  p.n_k = shape->n_k;
  p.n_v = shape->n_v;
  p.row_k_bytes = (int32_t)(shape->d_qk * es);
  p.row_v_bytes = (int32_t)(shape->d_v * es);
  if (shape->B == 0 || capacity == 0) return DIFFQKV_OK;
  return launch_append(p, paged, (hipStream_t)hip_stream) == hipSuccess ? DIFFQKV_OK : DIFFQKV_ERR_HIP;
}

int diffqkv_append(const diffqkv_shape* shape, const void* k_new, const void* v_new, void* k_cache,
                   void* v_cache, int64_t k_stride_b, int64_t k_stride_h, int64_t k_stride_t,
                   int64_t v_stride_b, int64_t v_stride_h, int64_t v_stride_t,
                   const int32_t* positions, int32_t T_cap, int32_t* seqlens_out, void* hip_stream) {
  return run_append(shape, k_new, v_new, k_cache, v_cache, k_stride_b, k_stride_h, k_stride_t, v_stride_b,
                    v_stride_h, v_stride_t, nullptr, 0, 0, positions, T_cap, seqlens_out, false, hip_stream);
}

int diffqkv_append_paged(const diffqkv_shape* shape, const void* k_new, const void* v_new, void* k_pool,
                         void* v_pool, int64_t k_stride_page, int64_t k_stride_h, int64_t k_stride_t,
                         int64_t v_stride_page, int64_t v_stride_h, int64_t v_stride_t,
                         const int32_t* block_table, int32_t max_pages, int32_t page_size,
                         const int32_t* positions, int32_t* seqlens_out, void* hip_stream) {
  if (max_pages < 0 || page_size <= 0) return DIFFQKV_ERR_SHAPE;
  if ((int64_t)max_pages * page_size > INT32_MAX) return DIFFQKV_ERR_SHAPE;
  return run_append(shape, k_new, v_new, k_pool, v_pool, k_stride_page, k_stride_h, k_stride_t, v_stride_page,
                    v_stride_h, v_stride_t, block_table, max_pages, page_size, positions,
                    max_pages * page_size, seqlens_out, true, hip_stream);
}

size_t diffqkv_prefill_workspace_bytes(const diffqkv_shape* shape, int32_t S_q, int32_t S_k) {
  (void)shape;
  (void)S_q;
  (void)S_k;
  return 0;  // the prefill kernels keep all running state on chip
}

int diffqkv_prefill(const diffqkv_shape* shape, const void* q, const void* k, const void* v,
                    int32_t S_q, int32_t S_k, int32_t causal, void* out, float* lse_out,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  int rc = check_shape(shape);
  if (rc != DIFFQKV_OK) return rc;
  if (S_q <= 0 || S_k <= 0) return DIFFQKV_ERR_SHAPE;
  if (causal && S_k < S_q) return DIFFQKV_ERR_SHAPE;
  if (shape->B > 0 && (!q || !k || !v || !out)) return DIFFQKV_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return DIFFQKV_ERR_ALIGN;
  PrefillParams p = {};
  p.q = q;
  p.k = k;
  p.v = v;
  p.out = out;
  p.lse_out = lse_out;
  p.B = shape->B;
  p.n_q = shape->n_q;
  p.n_k = shape->n_k;
  p.n_v = shape->n_v;
  p.d_qk = shape->d_qk;
  p.d_v = shape->d_v;
  p.S_q = S_q;
  p.S_k = S_k;
  p.causal = causal ? 1 : 0;
  p.n_cu = compute_units();
  p.scale_log2 = scale_log2(shape);
  if (shape->B == 0) return DIFFQKV_OK;
  hipError_t e;
  if (!t_tuning.force_generic && prefill_mfma_supported(p, shape->dtype))
    e = launch_prefill_mfma(p, t_tuning.prefill_waves, (hipStream_t)hip_stream);
  else
    e = launch_prefill_generic(p, shape->dtype, (hipStream_t)hip_stream);
  return e == hipSuccess ? DIFFQKV_OK : DIFFQKV_ERR_HIP;
}

static int check_augq(const diffqkv_augq_shape* s) {
  if (!s) return DIFFQKV_ERR_NULL;
  if (s->M < 0 || s->hidden <= 0 || s->inter <= 0 || s->hidden % 8 || s->inter % 8) return DIFFQKV_ERR_SHAPE;
  if (s->dtype != DIFFQKV_F32 && s->dtype != DIFFQKV_BF16) return DIFFQKV_ERR_SHAPE;
  if ((int64_t)s->hidden * s->inter > (1ll << 40) || (int64_t)s->M * s->inter > (1ll << 40))
    return DIFFQKV_ERR_UNSUPPORTED;  // valid, but beyond the index range the kernels are built for
  return DIFFQKV_OK;
}

size_t diffqkv_augment_q_workspace_bytes(const diffqkv_augq_shape* shape) {
  if (check_augq(shape) != DIFFQKV_OK) return 0;
  const size_t elem = shape->dtype == DIFFQKV_F32 ? 4 : 2;
  // (whole blocks of 16 tokens: the matrix-core kernels keep the intermediate activations block by block)
  return ((size_t)((shape->M + 15) / 16 * 16) * shape->inter * elem + 255) / 256 * 256;
}

int diffqkv_augment_q(const diffqkv_augq_shape* shape, const void* q_in, const void* w_gate, const void* w_up,
                      const void* w_down, void* q_out, void* workspace, size_t workspace_bytes,
                      void* hip_stream) {
  int rc = check_augq(shape);
  if (rc != DIFFQKV_OK) return rc;
  if (shape->M == 0) return DIFFQKV_OK;
  if (!q_in || !w_gate || !w_up || !w_down || !q_out) return DIFFQKV_ERR_NULL;
  if (!aligned16(q_in) || !aligned16(w_gate) || !aligned16(w_up) || !aligned16(w_down) || !aligned16(q_out))
    return DIFFQKV_ERR_ALIGN;
  const size_t need = diffqkv_augment_q_workspace_bytes(shape);
  if (!workspace || workspace_bytes < need) return DIFFQKV_ERR_WORKSPACE;
  if (!aligned16(workspace)) return DIFFQKV_ERR_ALIGN;
  const bool mfma = !t_tuning.force_generic && augq_mfma_supported(shape->dtype, shape->hidden, shape->inter);
  AugqParams p = {};
  p.x = q_in;
  p.w0 = w_gate;
  p.w1 = w_up;
  p.out = workspace;
  p.M = shape->M;
  p.K = shape->hidden;
  p.N = shape->inter;
  p.n_cu = compute_units();
  if (launch_augq(p, shape->dtype, true, mfma, (hipStream_t)hip_stream) != hipSuccess) return DIFFQKV_ERR_HIP;
  p.x = workspace;
  p.w0 = w_down;
  p.w1 = nullptr;
  p.out = q_out;
  p.K = shape->inter;
  p.N = shape->hidden;
  return launch_augq(p, shape->dtype, false, mfma, (hipStream_t)hip_stream) == hipSuccess ? DIFFQKV_OK
                                                                                           : DIFFQKV_ERR_HIP;
}

int diffqkv_probe_stream_read(const void* src, size_t bytes, float* sink, void* hip_stream) {
  if (!src || !sink) return DIFFQKV_ERR_NULL;
  if (bytes % 16 || !aligned16(src)) return DIFFQKV_ERR_ALIGN;
  hipError_t e = launch_probe_stream_read(src, bytes, sink, (hipStream_t)hip_stream);
  return e == hipSuccess ? DIFFQKV_OK : DIFFQKV_ERR_HIP;
}

const char* diffqkv_strerror(int status) {
  switch (status) {
    case DIFFQKV_OK: return "ok";
    case DIFFQKV_ERR_NULL: return "a required pointer is NULL";
    case DIFFQKV_ERR_SHAPE: return "invalid shape, length or head width";
    case DIFFQKV_ERR_HEADS: return "head counts must divide n_q and one of n_k, n_v must divide the other";
    case DIFFQKV_ERR_ALIGN: return "pointer or stride breaks 16-byte row alignment";
    case DIFFQKV_ERR_WORKSPACE: return "workspace missing or too small";
    case DIFFQKV_ERR_UNSUPPORTED: return "no kernel for these arguments";
    case DIFFQKV_ERR_HIP: return "HIP launch failed";
    case DIFFQKV_ERR_STATIC_LIMIT: return "the call needs more scratch memory than the library's static buffer holds";
    default: return "unknown status";
  }
}

int diffqkv_version(void) { return 200; }

}  // extern "C"
