// Shared pieces of the two bf16 causal-prefill kernels for gfx950 matrix cores: the LDS tile layout
// (K row-major with padded rows, V transposed and XOR-swizzled), buffer resources, the workgroup ->
// (sequence, query head, query tile) map, and small helpers.
#pragma once
#include <type_traits>

#include "kernels.h"

namespace diffqkv {
namespace prefill_tile {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kBN = 64;  // tokens per K/V tile
constexpr int kXcds = 8;
constexpr float kSlack = 8.f;  // log2 units a row maximum may exceed the softmax reference

// Compile-time loop: f(integral_constant<int, I>) for I = 0 .. N - 1, so that every register-array
// index in the body is a constant for the front end already.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// Transposed V tile in LDS: row = channel, 64 token positions (128 B, no padding).
// Position of token t (0..63): within each group of 16 tokens the quads are stored in the order
// 0, 2, 1, 3, so that the 8 tokens a lane needs for one k-step of the PV product (quads u and
// u + 2) form one 16-byte granule.  The granule index is XOR-swizzled with the channel so that
// both the 16-byte operand reads (32 consecutive channels) and the 8-byte transposed writes
// (channels 8 apart) spread over the banks (measured: no bank conflicts).
__device__ __forceinline__ int vt_pos(int t) {
  const int u = (t >> 2) & 3;
  return (t & ~15) + 8 * (u & 1) + 4 * (u >> 1) + (t & 3);
}
__device__ __forceinline__ int vt_swizzle(int ch) { return (ch ^ (ch >> 3)) & 7; }

template <int DQK, int DV>
struct Smem {
  static constexpr int kKPitch = DQK + 8;  // bf16 elements per K row (16 B of padding)
  uint16_t k[2][kBN][kKPitch];
  uint16_t vt[2][DV][kBN];
};

// Raw buffer resource over `bytes` bytes: a load whose per-lane offset (vector register plus
// immediate) falls past the end reads as zero.  The kernels rely on that for rows past the end of a
// head, so the tile start travels in the per-lane offset and the scalar offset stays zero: the
// per-lane part is the one the range check is documented to cover.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}


// Workgroup x -> (sequence b, query head h, query tile).  Heaviest (last) query tiles first.  With
// xcd_aware the (sequence, K head) groups are dealt round-robin to the XCDs and the query heads of a
// group sit side by side in one XCD's queue, so that its L2 serves their common K/V tiles.
__device__ __forceinline__ void locate_block(const PrefillParams& p, int x, int n_qtiles, int xcd_aware, int& b,
                                             int& h, int& qtile) {
  const int g_k = p.n_q / p.n_k;
  if (xcd_aware) {
    const int groups_per_xcd = p.B * p.n_k / kXcds;
    const int c = x % kXcds, j = x / kXcds;
    const int hq = j % g_k, t = j / g_k;
    const int group = (t % groups_per_xcd) * kXcds + c;
    qtile = n_qtiles - 1 - t / groups_per_xcd;
    b = group / p.n_k;
    h = (group % p.n_k) * g_k + hq;
  } else {
    h = x % p.n_q;
    b = (x / p.n_q) % p.B;
    qtile = n_qtiles - 1 - x / (p.n_q * p.B);
  }
}

}  // namespace prefill_tile
}  // namespace diffqkv
