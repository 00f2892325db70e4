// Portable split-decode kernel (fp32 and bf16, any supported shape) and the log-sum-exp combine.
//
// The split kernel evaluates, for one (sequence, head group, context chunk), the attention of
// section 2 ("Formulation of DiffQKV Attention") restricted to the chunk's tokens, with the head
// map of the "idx" rule (section 3.2): query head h reads K head floor(h n_k / n_q) and V head
// floor(h n_v / n_q).  A head group is the set of query heads under one head of the coarser cache
// side, so every K row and V row of the chunk is fetched from HBM by exactly one workgroup.
// Partial results are normalised per chunk and carry their base-2 log-sum-exp; the combine kernel
// merges them (section 3.2, "combine kernel").
//
// This kernel is the fp32 path and the fallback for shapes the MFMA kernel does not take; it runs
// on the vector ALUs only.
#include "kernels.h"

namespace diffqkv {

namespace {

constexpr int kThreads = 256;
constexpr int kTile = 64;     // tokens per inner tile (= one wavefront wide)
constexpr int kAccPerThread = 8;
constexpr int kMaxRows = 32;  // query rows handled by one workgroup

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}

// rows handled per workgroup so that rows * d_v accumulators fit kThreads * kAccPerThread
__host__ __device__ inline int rows_per_block(int G, int d_v) {
  int r = (kThreads * kAccPerThread) / d_v;
  if (r > kMaxRows) r = kMaxRows;
  if (r > G) r = G;
  return r < 1 ? 1 : r;
}

template <typename T, bool PAGED>
__global__ __launch_bounds__(kThreads) void decode_generic_kernel(DecodeParams p) {
  extern __shared__ float smem[];
  const int split = blockIdx.x;
  const int GR = rows_per_block(p.G, p.d_v);
  const int row_blocks = (p.G + GR - 1) / GR;
  const int group = blockIdx.y / row_blocks;
  const int row0 = (blockIdx.y % row_blocks) * GR;  // first row of this block inside the group
  const int b = blockIdx.z;
  const int tid = threadIdx.x;

  int Tb = p.seqlens ? p.seqlens[b] : p.T;
  Tb = Tb < p.T ? Tb : p.T;
  const int c0 = split * p.chunk;
  if (c0 >= Tb) {
    // Nothing in this chunk; the combine kernel knows that from T_b.  With a single split there is
    // no combine pass, so an empty sequence gets its zeros (and lse = -inf) here.
    if (p.num_splits == 1) {
      const int rows_e = (p.G - row0 < GR) ? p.G - row0 : GR;
      const int h0_e = group * p.G + row0;
      for (int o = tid; o < rows_e * p.d_v; o += kThreads)
        store_from_float((T*)p.out, ((int64_t)b * p.n_q + h0_e + o / p.d_v) * p.d_v + o % p.d_v, 0.f);
      if (p.lse_out)
        for (int r = tid; r < rows_e; r += kThreads) p.lse_out[(int64_t)b * p.n_q + h0_e + r] = -INFINITY;
    }
    return;
  }
  const int c1 = (c0 + p.chunk < Tb) ? c0 + p.chunk : Tb;
  const int rows = (p.G - row0 < GR) ? p.G - row0 : GR;

  float* qs = smem;                       // [GR][d_qk]
  float* sc = qs + GR * p.d_qk;           // [GR][kTile]
  float* m_run = sc + GR * kTile;         // [GR]
  float* l_run = m_run + GR;              // [GR]
  float* fac = l_run + GR;                // [GR]

  const T* q = (const T*)p.q;
  const T* kbase = (const T*)p.k;
  const T* vbase = (const T*)p.v;
  const int h0 = group * p.G + row0;  // first query head of this block

  for (int i = tid; i < rows * p.d_qk; i += kThreads) {
    int r = i / p.d_qk, c = i % p.d_qk;
    qs[i] = load_as_float(q, ((int64_t)b * p.n_q + h0 + r) * p.d_qk + c);
  }
  for (int r = tid; r < rows; r += kThreads) {
    m_run[r] = -INFINITY;
    l_run[r] = 0.f;
  }
  float acc[kAccPerThread];
#pragma unroll
  for (int i = 0; i < kAccPerThread; ++i) acc[i] = 0.f;
  __syncthreads();

  const int32_t* bt = PAGED ? p.block_table + (int64_t)b * p.max_pages : nullptr;
  auto row_offset = [&](int j, int64_t sb, int64_t st) -> int64_t {
    if (PAGED) return (int64_t)bt[j / p.page_size] * sb + (int64_t)(j % p.page_size) * st;
    return (int64_t)b * sb + (int64_t)j * st;
  };

  for (int t0 = c0; t0 < c1; t0 += kTile) {
    // ---- scores: one (row, token) pair per thread --------------------------------------------
    for (int idx = tid; idx < rows * kTile; idx += kThreads) {
      int r = idx / kTile, jj = idx % kTile, j = t0 + jj;
      float s = -INFINITY;
      if (j < c1) {
        int kh = (int)(((int64_t)(h0 + r) * p.n_k) / p.n_q);
        const T* kr = kbase + row_offset(j, p.k_sb, p.k_st) + (int64_t)kh * p.k_sh;
        const float* qr = qs + r * p.d_qk;
        float dot = 0.f;
        for (int c = 0; c < p.d_qk; ++c) dot = fmaf(qr[c], load_as_float(kr, c), dot);
        s = dot * p.scale_log2;
      }
      sc[idx] = s;
    }
    __syncthreads();
    // ---- running softmax statistics: one wavefront per row -------------------------------------
    for (int r = tid / 64; r < rows; r += kThreads / 64) {
      float s = sc[r * kTile + (tid & 63)];
      float m_old = m_run[r];
      float m_new = fmaxf(m_old, wave_max(s));  // finite: the tile holds at least one live token
      float pj = exp2f(s - m_new);              // masked tokens: exp2(-inf) = 0
      float sum = wave_sum(pj);
      float f = exp2f(m_old - m_new);           // first tile: exp2(-inf) = 0
      sc[r * kTile + (tid & 63)] = pj;
      if ((tid & 63) == 0) {
        m_run[r] = m_new;
        l_run[r] = l_run[r] * f + sum;
        fac[r] = f;
      }
    }
    __syncthreads();
    // ---- weighted V sum: one (row, channel) accumulator per thread slot -----------------------
    const int nt = (c1 - t0 < kTile) ? c1 - t0 : kTile;
#pragma unroll
    for (int i = 0; i < kAccPerThread; ++i) {
      int o = i * kThreads + tid;
      if (o < rows * p.d_v) {
        int r = o / p.d_v, e = o % p.d_v;
        int vh = (int)(((int64_t)(h0 + r) * p.n_v) / p.n_q);
        float a = acc[i] * fac[r];
        const float* pr = sc + r * kTile;
        for (int jj = 0; jj < nt; ++jj) {
          const T* vr = vbase + row_offset(t0 + jj, p.v_sb, p.v_st) + (int64_t)vh * p.v_sh;
          a = fmaf(pr[jj], load_as_float(vr, e), a);
        }
        acc[i] = a;
      }
    }
    __syncthreads();
  }

  // ---- write the chunk's result ---------------------------------------------------------------
#pragma unroll
  for (int i = 0; i < kAccPerThread; ++i) {
    int o = i * kThreads + tid;
    if (o < rows * p.d_v) {
      int r = o / p.d_v, e = o % p.d_v;
      int h = h0 + r;
      float val = acc[i] / l_run[r];
      if (p.num_splits == 1) {
        store_from_float((T*)p.out, ((int64_t)b * p.n_q + h) * p.d_v + e, val);
      } else {
        p.o_part[(((int64_t)b * p.n_q + h) * p.num_splits + split) * p.d_v + e] = val;
      }
    }
  }
  for (int r = tid; r < rows; r += kThreads) {
    int h = h0 + r;
    float lse2 = m_run[r] + log2f(l_run[r]);
    if (p.num_splits == 1) {
      if (p.lse_out) p.lse_out[(int64_t)b * p.n_q + h] = lse2 * kLn2;
    } else {
      p.lse_part[((int64_t)b * p.n_q + h) * p.num_splits + split] = lse2;
    }
  }
}

// One workgroup per (sequence, query head): merges the live splits of that row.
//   lse = log2 sum_s 2^{lse_s},   out = sum_s 2^{lse_s - lse} o_s
// Sequences of length zero get out = 0, lse = -inf.  Only launched when num_splits > 1.
// Threads are laid out as (split lane, channel quad): each thread sums every nsl-th split of four
// channels with independent 16-byte loads, then the split lanes are added in a fixed order in LDS.
constexpr int kCombineThreads = 256;

template <typename T>
__global__ __launch_bounds__(kCombineThreads) void combine_kernel(DecodeParams p) {
  __shared__ float red[kCombineThreads * 4];
  __shared__ float stat[2];
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  int Tb = p.seqlens ? p.seqlens[b] : p.T;
  Tb = Tb < p.T ? Tb : p.T;
  const int64_t row = (int64_t)b * p.n_q + h;
  T* out = (T*)p.out + row * p.d_v;
  if (Tb <= 0) {
    for (int e = tid; e < p.d_v; e += kCombineThreads) store_from_float(out, e, 0.f);
    if (tid == 0 && p.lse_out) p.lse_out[row] = -INFINITY;
    return;
  }
  int live;
  if (p.sk_cum) {
    // ragged mode of the MFMA kernel: the stream (b, K head) occupies units [start, start + u_b) of
    // the unit space cut into slices of L units, one partial per slice that touches it
    const int64_t total = (int64_t)p.n_k * p.sk_cum[p.B];
    int64_t L = (total + p.sk_workers - 1) / p.sk_workers;
    L = L < p.sk_lmin ? p.sk_lmin : L;
    const int u_b = p.sk_cum[b + 1] - p.sk_cum[b];
    const int64_t start = (int64_t)p.n_k * p.sk_cum[b] + (int64_t)(h / p.G) * u_b;
    live = (int)((start + u_b - 1) / L - start / L) + 1;
  } else {
    live = (Tb + p.chunk - 1) / p.chunk;
  }
  const float* lp = p.lse_part + row * p.num_splits;
  const float* op = p.o_part + row * p.num_splits * p.d_v;

  // log-sum-exp of the live splits, by the first wavefront
  if (tid < 64) {
    float m = -INFINITY;
    for (int s = tid; s < live; s += 64) m = fmaxf(m, lp[s]);
    m = wave_max(m);
    float l = 0.f;
    for (int s = tid; s < live; s += 64) l += exp2f(lp[s] - m);
    l = wave_sum(l);
    if (tid == 0) {
      stat[0] = m;
      stat[1] = l;
    }
  }
  __syncthreads();
  const float m = stat[0], inv = 1.f / stat[1];

  const int nq = p.d_v / 4;               // channel quads
  const int nsl = kCombineThreads / nq;   // split lanes
  const int sl = tid / nq, cq = tid % nq;
  float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
  if (sl < nsl) {
    for (int s = sl; s < live; s += nsl) {
      const float w = exp2f(lp[s] - m) * inv;
      const float4 x = *(const float4*)(op + (int64_t)s * p.d_v + cq * 4);
      a.x = fmaf(w, x.x, a.x);
      a.y = fmaf(w, x.y, a.y);
      a.z = fmaf(w, x.z, a.z);
      a.w = fmaf(w, x.w, a.w);
    }
  }
  red[tid * 4 + 0] = a.x;
  red[tid * 4 + 1] = a.y;
  red[tid * 4 + 2] = a.z;
  red[tid * 4 + 3] = a.w;
  __syncthreads();
  for (int e = tid; e < p.d_v; e += kCombineThreads) {
    float v = 0.f;
    for (int j = 0; j < nsl; ++j) v += red[(j * nq + e / 4) * 4 + (e & 3)];
    store_from_float(out, e, v);
  }
  if (tid == 0 && p.lse_out) p.lse_out[row] = (m + log2f(stat[1])) * kLn2;
}

}  // namespace

hipError_t launch_decode_generic(const DecodeParams& p, int dtype, bool paged, hipStream_t s) {
  if (p.B == 0 || p.num_splits == 0) return hipSuccess;
  const int GR = rows_per_block(p.G, p.d_v);
  const int row_blocks = (p.G + GR - 1) / GR;
  dim3 grid(p.num_splits, p.n_groups * row_blocks, p.B), block(kThreads);
  size_t smem = sizeof(float) * ((size_t)GR * p.d_qk + (size_t)GR * kTile + 3 * (size_t)GR);
  if (dtype == 0) {
    if (paged)
      decode_generic_kernel<float, true><<<grid, block, smem, s>>>(p);
    else
      decode_generic_kernel<float, false><<<grid, block, smem, s>>>(p);
  } else {
    if (paged)
      decode_generic_kernel<uint16_t, true><<<grid, block, smem, s>>>(p);
    else
      decode_generic_kernel<uint16_t, false><<<grid, block, smem, s>>>(p);
  }
  return hipGetLastError();
}

hipError_t launch_combine(const DecodeParams& p, int dtype, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  dim3 grid(p.n_q, p.B), block(kCombineThreads);
  if (dtype == 0)
    launch_kernel(1, combine_kernel<float>, grid, block, 0, s, p);
  else
    launch_kernel(1, combine_kernel<uint16_t>, grid, block, 0, s, p);
  return hipGetLastError();
}

}  // namespace diffqkv
