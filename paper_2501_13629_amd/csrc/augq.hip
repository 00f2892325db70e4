// Augmented Q (observations 3-4 of section 2; the appendix's attention listing): the output of the
// query projection passes through a gated feed-forward before the heads are formed,
//     q' = W_down ( silu(W_gate q) * (W_up q) ),
// with an intermediate width of 1.5 x the hidden width (3072 for 2048, 6144 for 4096).  During decode
// the token count M is the batch size, so the three products are matrix-vector shaped and bound by
// the one pass over the weights (37.7 MB at 2048 / 3072 in bf16).
//
// Matrix-core kernel: D^T[feature][token] = W x^T on v_mfma_f32_16x16x32_bf16 with the weight rows
// loaded from HBM straight into A-operand layout (each lane 16 contiguous bytes of one row) and up to
// 16 tokens of x as the B operand.  One workgroup = 16 wavefronts owns 16 output features (of both
// gate and up in the gated pass); the wavefronts split the input features sixteen ways, so every
// weight byte is read once and ~190 workgroups x 16 wavefronts have their loads in flight at
// once; partial sums meet in LDS, where the activation and the product are applied.  Two launches:
// gate + up -> intermediate (I/O dtype) in the workspace, then down.  More than 16 tokens repeat the
// pass per block of 16 (weights then come from L2): the entry point is meant for the decode step.
// A portable vector-ALU kernel serves fp32 and widths the matrix-core kernel leaves out.
#include "kernels.h"

namespace diffqkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kWavesMfma = 16;  // the k-steps (32 input features each) of a wavefront are loaded in batches of 4 or 6

__device__ __forceinline__ float silu(float z) { return z / (1.f + __expf(-z)); }

template <bool GATED, int kBatch>
__global__ __launch_bounds__(kWavesMfma * 64) void augq_mfma_kernel(AugqParams p) {
  __shared__ float red[kWavesMfma][GATED ? 2 : 1][16][16];  // [wavefront][matrix][token][feature]
  const int tile = blockIdx.x, tb = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, n = lane & 15;
  const int ksteps = p.K / (kWavesMfma * 32);  // per wavefront; a multiple of kBatch (checked on the host)
  const int k0 = wave * ksteps * 32 + g * 8;
  const uint16_t* w0 = (const uint16_t*)p.w0 + (int64_t)(tile * 16 + n) * p.K + k0;
  const uint16_t* w1 = GATED ? (const uint16_t*)p.w1 + (int64_t)(tile * 16 + n) * p.K + k0 : nullptr;
  const int token = tb * 16 + n;
  const bool live = token < p.M;
  const uint16_t* x = (const uint16_t*)p.x + (int64_t)(live ? token : 0) * p.K + k0;

  f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < ksteps; s0 += kBatch) {
    u32x4 a0[kBatch], a1[kBatch], bx[kBatch];
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      a0[i] = *(const u32x4*)(w0 + (s0 + i) * 32);
      if (GATED) a1[i] = *(const u32x4*)(w1 + (s0 + i) * 32);
      bx[i] = *(const u32x4*)(x + (s0 + i) * 32);
      if (!live) bx[i] = u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < kBatch; ++i) {
      const bf16x8 b = __builtin_bit_cast(bf16x8, bx[i]);
      acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a0[i]), b, acc0, 0, 0, 0);
      if (GATED) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a1[i]), b, acc1, 0, 0, 0);
    }
  }
  // lane (g, n): features 4 g .. 4 g + 3 of token n
  *(f32x4*)&red[wave][0][n][4 * g] = acc0;
  if (GATED) *(f32x4*)&red[wave][GATED ? 1 : 0][n][4 * g] = acc1;
  __syncthreads();
  if (threadIdx.x < 256) {
    const int t = threadIdx.x >> 4, f = threadIdx.x & 15;
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesMfma; ++w) {
      s0 += red[w][0][t][f];
      if (GATED) s1 += red[w][GATED ? 1 : 0][t][f];
    }
    const float y = GATED ? silu(s0) * s1 : s0;
    if (tb * 16 + t < p.M)
      ((uint16_t*)p.out)[(int64_t)(tb * 16 + t) * p.N + tile * 16 + f] = float_to_bf16_bits(y);
  }
}

// Portable: one wavefront per (token, output feature), lanes over the input features.
template <typename T, bool GATED>
__global__ __launch_bounds__(256) void augq_generic_kernel(AugqParams p) {
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + (threadIdx.x >> 6), m = blockIdx.y;
  if (j >= p.N) return;  // whole wavefronts
  const T* x = (const T*)p.x + (int64_t)m * p.K;
  const T* w0 = (const T*)p.w0 + (int64_t)j * p.K;
  const T* w1 = GATED ? (const T*)p.w1 + (int64_t)j * p.K : nullptr;
  float s0 = 0.f, s1 = 0.f;
  for (int c = lane; c < p.K; c += 64) {
    const float xv = load_as_float(x, c);
    s0 = fmaf(load_as_float(w0, c), xv, s0);
    if (GATED) s1 = fmaf(load_as_float(w1, c), xv, s1);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    s0 += __shfl_xor(s0, o, 64);
    if (GATED) s1 += __shfl_xor(s1, o, 64);
  }
  if (lane == 0) store_from_float((T*)p.out, (int64_t)m * p.N + j, GATED ? silu(s0) * s1 : s0);
}

}  // namespace

namespace {
int batch_for(int K) {  // k-steps per wavefront must come in whole batches
  if (K % (kWavesMfma * 32)) return 0;
  const int ksteps = K / (kWavesMfma * 32);
  return ksteps % 6 == 0 ? 6 : ksteps % 4 == 0 ? 4 : 0;
}
}  // namespace

bool augq_mfma_supported(int dtype, int hidden, int inter) {  // multiples of 2048 or 3072
  return dtype == 1 && batch_for(hidden) && batch_for(inter);
}

// One product: out[M, N] = act(W0 x)(* W1 x), x [M, K], W [N, K].
hipError_t launch_augq(const AugqParams& p, int dtype, bool gated, bool mfma, hipStream_t s) {
  if (p.M == 0) return hipSuccess;
  if (mfma) {
    dim3 grid(p.N / 16, (p.M + 15) / 16);
    const bool six = batch_for(p.K) == 6;
    if (gated) {
      if (six) launch_kernel(0, augq_mfma_kernel<true, 6>, dim3(grid), dim3(kWavesMfma * 64), 0, s, p);
      else launch_kernel(0, augq_mfma_kernel<true, 4>, dim3(grid), dim3(kWavesMfma * 64), 0, s, p);
    } else {
      if (six) launch_kernel(1, augq_mfma_kernel<false, 6>, dim3(grid), dim3(kWavesMfma * 64), 0, s, p);
      else launch_kernel(1, augq_mfma_kernel<false, 4>, dim3(grid), dim3(kWavesMfma * 64), 0, s, p);
    }
  } else {
    dim3 grid((p.N + 3) / 4, p.M);
    if (dtype == 0) {
      if (gated) augq_generic_kernel<float, true><<<grid, 256, 0, s>>>(p);
      else augq_generic_kernel<float, false><<<grid, 256, 0, s>>>(p);
    } else {
      if (gated) augq_generic_kernel<uint16_t, true><<<grid, 256, 0, s>>>(p);
      else augq_generic_kernel<uint16_t, false><<<grid, 256, 0, s>>>(p);
    }
  }
  return hipGetLastError();
}

}  // namespace diffqkv
