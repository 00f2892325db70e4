// Stream-read probe: how fast can this GPU pull bytes out of HBM with plain 128-bit loads?
// Reported beside the decode kernels, whose roofline is that same read stream.
#include "kernels.h"

namespace diffqkv {

namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__global__ __launch_bounds__(kThreads) void stream_read_kernel(const u32x4* __restrict__ src, size_t n_vec,
                                                               float* __restrict__ sink) {
  // each workgroup walks its own contiguous slab, kUnroll independent 16-byte loads per lane in flight
  const size_t per_block = (n_vec + gridDim.x - 1) / gridDim.x;
  const size_t lo = per_block * blockIdx.x;
  size_t hi = lo + per_block;
  hi = hi < n_vec ? hi : n_vec;
  uint32_t acc = 0;
  size_t i = lo + threadIdx.x;
  for (; i + (size_t)(kUnroll - 1) * kThreads < hi; i += (size_t)kUnroll * kThreads) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + (size_t)u * kThreads);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
  }
  for (; i < hi; i += kThreads) {
    u32x4 v = src[i];
    acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o, 64);
  __shared__ uint32_t part[kThreads / 64];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = __uint_as_float((part[0] ^ part[1] ^ part[2] ^ part[3]) & 0x3fffffffu);
}

}  // namespace

hipError_t launch_probe_stream_read(const void* src, size_t bytes, float* sink, hipStream_t s) {
  const size_t n_vec = bytes / 16;
  if (n_vec == 0) return hipSuccess;
  int blocks = 4096;
  if ((size_t)blocks * kThreads > n_vec) blocks = (int)((n_vec + kThreads - 1) / kThreads);
  stream_read_kernel<<<blocks, kThreads, 0, s>>>((const u32x4*)src, n_vec, sink);
  return hipGetLastError();
}

}  // namespace diffqkv
