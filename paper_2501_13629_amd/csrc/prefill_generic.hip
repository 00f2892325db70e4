// Portable prefill kernel (fp32 and bf16, any supported shape): one wavefront per query position.
//
// Evaluates the attention of section 2 ("Formulation of DiffQKV Attention") for every query
// position i of a block, with K head floor(h n_k / n_q) and V head floor(h n_v / n_q) for query
// head h (the "idx" rule of section 3.2).  With the causal flag, query i attends to keys
// j <= i + (S_k - S_q): K_t holds the tokens up to and including the current one.
// This is the fp32 path and the fallback for shapes the MFMA prefill kernel does not take.
#include "kernels.h"

namespace diffqkv {

namespace {

constexpr int kWaves = 4;
constexpr int kMaxD = 256;

template <typename T>
__global__ __launch_bounds__(kWaves * 64) void prefill_generic_kernel(PrefillParams p) {
  __shared__ float qs[kWaves][kMaxD];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x * kWaves + wave;
  const int h = blockIdx.y, b = blockIdx.z;
  const bool live = i < p.S_q;
  const int kh = (int)(((int64_t)h * p.n_k) / p.n_q), vh = (int)(((int64_t)h * p.n_v) / p.n_q);
  const T* q = (const T*)p.q + (((int64_t)b * p.n_q + h) * p.S_q + (live ? i : 0)) * p.d_qk;
  const T* k = (const T*)p.k + ((int64_t)b * p.n_k + kh) * p.S_k * p.d_qk;
  const T* v = (const T*)p.v + ((int64_t)b * p.n_v + vh) * p.S_k * p.d_v;
  for (int c = lane; c < p.d_qk; c += 64) qs[wave][c] = load_as_float(q, c);
  __syncthreads();
  if (!live) return;
  const int Ti = p.causal ? i + 1 + (p.S_k - p.S_q) : p.S_k;

  float acc[kMaxD / 64];
#pragma unroll
  for (int a = 0; a < kMaxD / 64; ++a) acc[a] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  for (int t0 = 0; t0 < Ti; t0 += 64) {
    const int j = t0 + lane;
    float s = -INFINITY;
    if (j < Ti) {
      const T* kr = k + (int64_t)j * p.d_qk;
      float dot = 0.f;
      for (int c = 0; c < p.d_qk; ++c) dot = fmaf(qs[wave][c], load_as_float(kr, c), dot);
      s = dot * p.scale_log2;
    }
    float mt = s;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mt = fmaxf(mt, __shfl_xor(mt, o, 64));
    const float m_new = fmaxf(m_run, mt);
    const float pj = exp2f(s - m_new);
    float sum = pj;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    const float f = exp2f(m_run - m_new);
    l_run = l_run * f + sum;
    m_run = m_new;
    const int nt = (Ti - t0 < 64) ? Ti - t0 : 64;
#pragma unroll
    for (int a = 0; a < kMaxD / 64; ++a) {
      const int e = a * 64 + lane;
      float x = acc[a] * f;
      if (a * 64 < p.d_v) {  // wavefront-uniform, so every lane takes part in the shuffles
        const int ec = e < p.d_v ? e : 0;
        for (int jj = 0; jj < nt; ++jj)
          x = fmaf(__shfl(pj, jj, 64), load_as_float(v, (int64_t)(t0 + jj) * p.d_v + ec), x);
      }
      acc[a] = x;
    }
  }
  const int64_t row = ((int64_t)b * p.n_q + h) * p.S_q + i;
#pragma unroll
  for (int a = 0; a < kMaxD / 64; ++a) {
    const int e = a * 64 + lane;
    if (e < p.d_v) store_from_float((T*)p.out, row * p.d_v + e, acc[a] / l_run);
  }
  if (lane == 0 && p.lse_out) p.lse_out[row] = (m_run + log2f(l_run)) * kLn2;
}

}  // namespace

hipError_t launch_prefill_generic(const PrefillParams& p, int dtype, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  dim3 grid((p.S_q + kWaves - 1) / kWaves, p.n_q, p.B), block(kWaves * 64);
  if (dtype == 0)
    prefill_generic_kernel<float><<<grid, block, 0, s>>>(p);
  else
    prefill_generic_kernel<uint16_t><<<grid, block, 0, s>>>(p);
  return hipGetLastError();
}

}  // namespace diffqkv
