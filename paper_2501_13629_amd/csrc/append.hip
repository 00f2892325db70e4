// KV-cache append: store the current token's k_t [n_k, d_qk] and v_t [n_v, d_v] of every sequence
// at its write position, into a contiguous or a paged cache.  This is the store side of the cache of
// section 3.2 ("Differential Management of KV Cache"): K and V are kept as separate tensors with their
// own head counts, so one token costs (n_k d_qk + n_v d_v) elements (the cost model of section 3.1,
// "KV Cache") -- nothing is duplicated to a common head count.  Pure data movement: 16-byte vector copies, bit exact.
#include "kernels.h"

namespace diffqkv {

namespace {

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <bool PAGED>
__global__ __launch_bounds__(256) void append_kernel(AppendParams p) {
  const int b = blockIdx.x;
  const int pos = p.positions[b];
  if (pos < 0 || pos >= p.capacity) return;  // a full or invalid sequence is left untouched
  const int kvec = p.row_k_bytes / 16, vvec = p.row_v_bytes / 16;  // 16-byte pieces per head row
  int64_t k_off, v_off;  // byte offsets of (b, head 0, pos)
  if (PAGED) {
    const int page = p.block_table[(int64_t)b * p.max_pages + pos / p.page_size];
    const int slot = pos % p.page_size;
    k_off = (int64_t)page * p.k_sb + (int64_t)slot * p.k_st;
    v_off = (int64_t)page * p.v_sb + (int64_t)slot * p.v_st;
  } else {
    k_off = (int64_t)b * p.k_sb + (int64_t)pos * p.k_st;
    v_off = (int64_t)b * p.v_sb + (int64_t)pos * p.v_st;
  }
  const int total = p.n_k * kvec + p.n_v * vvec;
  for (int i = threadIdx.x; i < total; i += 256) {
    if (i < p.n_k * kvec) {
      const int h = i / kvec, c = i % kvec;
      const u32x4 x = *(const u32x4*)((const char*)p.k_new + ((int64_t)b * p.n_k + h) * p.row_k_bytes + c * 16);
      *(u32x4*)((char*)p.k + k_off + (int64_t)h * p.k_sh + c * 16) = x;
    } else {
      const int j = i - p.n_k * kvec;
      const int h = j / vvec, c = j % vvec;
      const u32x4 x = *(const u32x4*)((const char*)p.v_new + ((int64_t)b * p.n_v + h) * p.row_v_bytes + c * 16);
      *(u32x4*)((char*)p.v + v_off + (int64_t)h * p.v_sh + c * 16) = x;
    }
  }
  __syncthreads();  // seqlens_out may alias positions: every thread has read its position by now
  if (p.seqlens_out && threadIdx.x == 0) p.seqlens_out[b] = pos + 1;
}

}  // namespace

hipError_t launch_append(const AppendParams& p, bool paged, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  if (paged)
    append_kernel<true><<<p.B, 256, 0, s>>>(p);
  else
    append_kernel<false><<<p.B, 256, 0, s>>>(p);
  return hipGetLastError();
}

}  // namespace diffqkv
