// Augmented Q (observations 3-4 of section 2; the appendix's attention listing): the output of the
// query projection passes through a gated feed-forward before the heads are formed,
//     q' = W_down ( silu(W_gate q) * (W_up q) ),
// with an intermediate width of 1.5 x the hidden width (3072 for 2048, 6144 for 4096).  During decode
// the token count M is the batch size, so the three products are matrix-vector shaped and bound by
// the one pass over the weights (37.7 MB at 2048 / 3072 in bf16).
//
// Matrix-core kernel: D^T[row][token] = W x^T on v_mfma_f32_16x16x32_bf16 with the weight rows loaded
// from HBM straight into A-operand layout (each lane 16 contiguous bytes of one row) and up to 16
// tokens of x as the B operand.  One workgroup = 16 wavefronts; a tile of work is 16 weight rows, and
// the wavefronts split the input features sixteen ways, so every weight byte is read once and all the
// loads of a tile are in flight together.  A wavefront keeps its share of x in registers and the
// workgroup walks over several tiles when there are more than the chip holds at once: measured, the
// activations of a tile cost as much as its weights when every tile fetches them again (16 tokens
// against 16 rows, and with 16 MB of loads in flight per XCD its 4 MB L2 does not keep them).  Partial
// sums meet in LDS, where the activation and the product are applied; the loads of the next tile are
// issued before that.  In the gated pass a tile is 8 rows of W_gate on top of the 8 rows of W_up for
// the same features, so that one matrix instruction serves both; the plain pass takes 16 rows per
// tile, or 8 (the tile's lower half repeats the upper: same cache lines, no further traffic) when 16
// would leave compute units without a workgroup.  Two launches: gate + up -> intermediate (I/O dtype)
// in the workspace, then down.  More than 16 tokens repeat the pass per block of 16 (weights then come
// from L2): the entry point is meant for the decode step.
// A portable vector-ALU kernel serves fp32 and widths the matrix-core kernel leaves out.
#include "kernels.h"

namespace diffqkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kWavesMfma = 16;

__device__ __forceinline__ float silu(float z) { return z / (1.f + __expf(-z)); }

// TILE: 0 = 16 rows of w0; 1 = 8 rows of w0 (twice); 2 = 8 rows of w0 over the same 8 rows of w1 (gated).
// KSTEPS: k-steps (32 input features each) of a wavefront: K = 16 wavefronts x KSTEPS x 32.
// Workgroup x of the grid's G takes tiles x, x + G, ... of n_tiles.
template <int TILE, int KSTEPS>
__global__ __launch_bounds__(kWavesMfma * 64) void augq_mfma_kernel(AugqParams p, int n_tiles) {
  constexpr bool GATED = TILE == 2;
  constexpr int kRows = TILE == 0 ? 16 : 8;  // output features per tile
  __shared__ float red[kWavesMfma][16][16];  // [wavefront][token][tile row]
  const int tb = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = lane >> 4, n = lane & 15;
  const int k0 = wave * KSTEPS * 32 + g * 8;
  const int row = TILE == 0 ? n : (n & 7);
  const uint16_t* wbase = (const uint16_t*)((GATED && n >= 8) ? p.w1 : p.w0) + (int64_t)row * p.K + k0;
  const int token = tb * 16 + n;
  const bool live = token < p.M;
  // The plain pass reads the intermediate activations as the gated pass leaves them: per block of 16
  // tokens, [K / 8][16 tokens][8 features], so that a wavefront's B operand of a k-step is one
  // contiguous KiB (row-major it is 16 pieces of 64 bytes, and such requests were measured to cost
  // as much per byte as the weights do).
  const uint16_t* x = GATED ? (const uint16_t*)p.x + (int64_t)(live ? token : 0) * p.K + k0
                            : (const uint16_t*)p.x + (int64_t)tb * 16 * p.K + (int64_t)(wave * KSTEPS * 4 + g) * 128 + n * 8;
  constexpr int kXStep = GATED ? 32 : 512;  // elements between the k-steps of a lane

  // Two tiles of weights in flight where the registers allow it (16 wavefronts on a compute unit have
  // 128 registers each): the loads of the tile after next are issued as soon as a tile's registers are free.
  constexpr int kDepth = KSTEPS <= 8 ? 2 : 1;
  u32x4 a[kDepth][KSTEPS], bx[KSTEPS];
  auto load_tile = [&](int tile, u32x4 (&dst)[KSTEPS]) {
    if (tile >= n_tiles) return;
    const uint16_t* w = wbase + (int64_t)tile * kRows * p.K;
#pragma unroll
    for (int i = 0; i < KSTEPS; ++i) dst[i] = *(const u32x4*)(w + i * 32);
  };
  const int G = gridDim.x;
  int tile = blockIdx.x;
  load_tile(tile, a[0]);
#pragma unroll
  for (int i = 0; i < KSTEPS; ++i) {
    bx[i] = *(const u32x4*)(x + i * kXStep);
    if (!live) bx[i] = u32x4{0u, 0u, 0u, 0u};
  }
  if (kDepth == 2) load_tile(tile + G, a[kDepth - 1]);
  auto one_tile = [&](int tile, u32x4 (&w)[KSTEPS]) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < KSTEPS; ++i)
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[i]), __builtin_bit_cast(bf16x8, bx[i]),
                                                    acc, 0, 0, 0);
    load_tile(tile + kDepth * G, w);
    // lane (g, n): tile rows 4 g .. 4 g + 3 of token n
    *(f32x4*)&red[wave][n][4 * g] = acc;
    __syncthreads();
    if (threadIdx.x < 256) {
      const int t = threadIdx.x >> 4, f = threadIdx.x & 15;
      float sum = 0.f;
#pragma unroll
      for (int wv = 0; wv < kWavesMfma; ++wv) sum += red[wv][t][f];
      float y = sum;
      if (GATED) y = silu(sum) * __shfl_down(sum, 8, 64);  // row f + 8 is the up projection of feature f
      if (f < kRows && tb * 16 + t < p.M) {
        const int64_t at = GATED ? (int64_t)tb * 16 * p.N + (int64_t)(tile * 16 + t) * 8 + f  // (a tile = 8 features)
                                 : (int64_t)(tb * 16 + t) * p.N + tile * kRows + f;
        ((uint16_t*)p.out)[at] = float_to_bf16_bits(y);
      }
    }
    __syncthreads();  // the sums are read: the next tile may overwrite them
  };
  for (; tile < n_tiles; tile += kDepth * G) {
    one_tile(tile, a[0]);
    if (kDepth == 2 && tile + G < n_tiles) one_tile(tile + G, a[kDepth - 1]);
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
int ksteps_for(int K) {  // k-steps per wavefront the matrix-core kernel is instantiated for; 0: none
  if (K % (kWavesMfma * 32)) return 0;
  const int ksteps = K / (kWavesMfma * 32);
  return (ksteps == 4 || ksteps == 6 || ksteps == 8 || ksteps == 12) ? ksteps : 0;
}

template <int TILE>
void launch_mfma(const AugqParams& p, int which, int n_tiles, hipStream_t s) {
  // As few workgroups as keep every compute unit busy, each with the same number of tiles: every
  // workgroup fetches the whole of x once, and that traffic costs as much per byte as the weights.
  const int per_wg = (n_tiles + p.n_cu - 1) / p.n_cu;
  const int n_wg = (n_tiles + per_wg - 1) / per_wg;
  const dim3 grid((unsigned)n_wg, (unsigned)((p.M + 15) / 16)), block(kWavesMfma * 64);
  switch (ksteps_for(p.K)) {
    case 12: launch_kernel(which, augq_mfma_kernel<TILE, 12>, grid, block, 0, s, p, n_tiles); break;
    case 8: launch_kernel(which, augq_mfma_kernel<TILE, 8>, grid, block, 0, s, p, n_tiles); break;
    case 6: launch_kernel(which, augq_mfma_kernel<TILE, 6>, grid, block, 0, s, p, n_tiles); break;
    default: launch_kernel(which, augq_mfma_kernel<TILE, 4>, grid, block, 0, s, p, n_tiles); break;
  }
}
}  // namespace

bool augq_mfma_supported(int dtype, int hidden, int inter) {  // 2048, 3072, 4096 or 6144 wide
  return dtype == 1 && ksteps_for(hidden) && ksteps_for(inter);
}

// One product: out[M, N] = act(W0 x)(* W1 x), x [M, K], W [N, K].
hipError_t launch_augq(const AugqParams& p, int dtype, bool gated, bool mfma, hipStream_t s) {
  if (p.M == 0) return hipSuccess;
  if (mfma) {
    if (gated) launch_mfma<2>(p, 0, p.N / 8, s);
    else if (p.N / 16 >= p.n_cu) launch_mfma<0>(p, 1, p.N / 16, s);
    else launch_mfma<1>(p, 1, p.N / 8, s);
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
