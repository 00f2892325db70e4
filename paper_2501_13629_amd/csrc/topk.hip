// Decode with selective V-cache fetching (appendix "Selective V Cache Fetching"; LoadCacheV in the
// formulation of section 2): the attention weights are the softmax over ALL cached positions, so
// the whole K cache is streamed, but of the V cache only the rows of the top_k previous positions
// with the largest weights are fetched; the current token's row always takes part:
//     V_t = [LoadCacheV(V_cache, alpha); v_t],      o = sum over the loaded rows of alpha_j V_j.
// Ties go to the lower position.  The formula keeps alpha as it is; optionally the result is
// divided by the selected weights' sum.  K bytes are read once per K head (head map of the "idx"
// rule, section 3.2); V traffic drops from T rows to at most top_k + 1 rows per query head.
//
// Two kernels:
//   scores   one workgroup per (sequence, K head, chunk): S^T = K Q^T on the matrix cores exactly as
//            in the full decode kernel (K rows straight from HBM in operand layout, non-temporal),
//            scaled scores (base-2 domain) written as fp32 to the workspace, -inf beyond T_b.
//            A portable vector-ALU variant serves fp32 and the shapes the MFMA variant leaves out.
//   select   one workgroup per (sequence, query head): log-sum-exp of the row, an exact radix select
//            of the top_k-th largest score among the previous positions (4 rounds of 8 bits over a
//            monotone integer image of the floats; LDS histograms), in-order compaction of the
//            winners (ties in position order), then the weighted sum of the gathered V rows.
//            Integer counting only: the selection does not depend on thread scheduling.
#include "kernels.h"

namespace diffqkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __amdgpu_buffer_rsrc_t rsrc_t;

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kSub = 32;
constexpr int kNonTemporal = 2;

__device__ __forceinline__ rsrc_t make_rsrc(const void* base, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// ---- scores, matrix cores ------------------------------------------------------------------------
// Grid (chunks, n_k, B).  Wavefront w takes the 32-token sub-tiles w, w + 4, ... of the chunk.  Each
// 16-token block gets its own buffer resource whose size ends at the last live row, so rows past
// T_b read as zero (and are then written as -inf) without any per-lane clamping.
template <int DQK, bool PAGED>
__global__ __launch_bounds__(kThreads) void topk_scores_mfma_kernel(TopkParams p) {
  constexpr int KK = DQK / 32;
  const int chunk = blockIdx.x, kh = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane >> 4, n = lane & 15;
  const int G = p.n_q / p.n_k, h0 = kh * G;
  int Tb = p.seqlens ? p.seqlens[b] : p.T;
  Tb = Tb < 0 ? 0 : (Tb < p.T ? Tb : p.T);
  const int c0 = chunk * p.chunk;
  // the chunk is written up to the padded row end even past T_b: the select kernel never reads
  // beyond T_b, but whole sub-tiles keep the stores uniform
  const int c1 = (c0 + p.chunk < p.T_pad) ? c0 + p.chunk : p.T_pad;
  if (c0 >= Tb) return;  // nothing live here: the select kernel does not look past T_b

  const uint16_t* khead = (const uint16_t*)p.k + (int64_t)kh * p.k_sh;
  if (!PAGED) khead += (int64_t)b * p.k_sb;
  const int32_t* bt = PAGED ? p.block_table + (int64_t)b * p.max_pages : nullptr;
  const int k_row_bytes = (int)p.k_st * 2;

  bf16x8 qf[KK];
  {
    const uint16_t* qrow = (const uint16_t*)p.q + ((int64_t)b * p.n_q + h0 + (n < G ? n : 0)) * DQK;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      u32x4 w = *(const u32x4*)(qrow + kk * 32 + g * 8);
      if (n >= G) w = u32x4{0u, 0u, 0u, 0u};
      qf[kk] = __builtin_bit_cast(bf16x8, w);
    }
  }
  const int lane_off = n * k_row_bytes + g * 16;
  auto load_sub_tile = [&](int ts, u32x4 (&kw)[2][KK]) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int s0 = ts + 16 * blk;
      int live = Tb - s0;
      live = live < 0 ? 0 : (live > 16 ? 16 : live);
      const uint16_t* base = khead;
      if (live > 0) {
        if (PAGED)
          base += (int64_t)bt[s0 / p.page_size] * p.k_sb + (int64_t)(s0 % p.page_size) * p.k_st;
        else
          base += (int64_t)s0 * p.k_st;
      }
      const rsrc_t r = make_rsrc(base, live * k_row_bytes);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        kw[blk][kk] = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off + kk * 64, 0, kNonTemporal);
    }
  };
  float* srow = p.scores + ((int64_t)b * p.n_q + h0 + (n < G ? n : 0)) * p.T_pad;
  auto emit = [&](int ts, const u32x4 (&kw)[2][KK]) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kw[blk][kk]), qf[kk], s, 0, 0, 0);
      // lane (g, n): tokens ts + 16 blk + 4 g + x of query row n
      const int t0 = ts + 16 * blk + 4 * g;
      f32x4 o;
#pragma unroll
      for (int x = 0; x < 4; ++x) o[x] = (t0 + x) < Tb ? s[x] * p.scale_log2 : -INFINITY;
      if (n < G) *(f32x4*)(srow + t0) = o;
    }
  };
  int ts = c0 + wave * kSub;
  if (ts < c1) {
    u32x4 ka[2][KK], kb[2][KK];
    load_sub_tile(ts, ka);
    for (; ts < c1; ts += 2 * kWaves * kSub) {  // two sub-tiles per trip: loads of one under the other
      const int t2 = ts + kWaves * kSub;
      if (t2 < c1) load_sub_tile(t2, kb);
      emit(ts, ka);
      if (t2 < c1) {
        if (t2 + kWaves * kSub < c1) load_sub_tile(t2 + kWaves * kSub, ka);
        emit(t2, kb);
      }
    }
  }
}

// ---- scores, portable ------------------------------------------------------------------------------
// One thread per (query head, token); grid (token tiles of 256, n_q, B).
template <typename T, bool PAGED>
__global__ __launch_bounds__(kThreads) void topk_scores_generic_kernel(TopkParams p) {
  const int j = blockIdx.x * kThreads + threadIdx.x, h = blockIdx.y, b = blockIdx.z;
  int Tb = p.seqlens ? p.seqlens[b] : p.T;
  Tb = Tb < 0 ? 0 : (Tb < p.T ? Tb : p.T);
  if (j >= p.T_pad) return;
  float s = -INFINITY;
  if (j < Tb) {
    const int kh = (int)(((int64_t)h * p.n_k) / p.n_q);
    int64_t off = (int64_t)kh * p.k_sh;
    if (PAGED)
      off += (int64_t)p.block_table[(int64_t)b * p.max_pages + j / p.page_size] * p.k_sb +
             (int64_t)(j % p.page_size) * p.k_st;
    else
      off += (int64_t)b * p.k_sb + (int64_t)j * p.k_st;
    const T* kr = (const T*)p.k + off;
    const T* qr = (const T*)p.q + ((int64_t)b * p.n_q + h) * p.d_qk;
    float dot = 0.f;
    for (int c = 0; c < p.d_qk; ++c) dot = fmaf(load_as_float(qr, c), load_as_float(kr, c), dot);
    s = dot * p.scale_log2;
  }
  p.scores[((int64_t)b * p.n_q + h) * p.T_pad + j] = s;
}

// ---- select + gather ---------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t order_key(float f) {  // larger float <=> larger key
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float block_max(float x, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  x = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  return x;
}
__device__ __forceinline__ float block_sum(float x, float* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  x = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  return x;
}

constexpr int kMaxTopK = 512;

template <typename T, bool PAGED>
__global__ __launch_bounds__(kThreads) void topk_select_kernel(TopkParams p) {
  __shared__ float red[kWaves];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t sh_prefix, sh_need;
  __shared__ int32_t sel_gt[kWaves][kMaxTopK];   // winners above the threshold, per wavefront, in order
  __shared__ int32_t sel_eq[kWaves][kMaxTopK];   // the first ties of each wavefront's range, in order
  __shared__ int32_t n_gt[kWaves], n_eq[kWaves];
  __shared__ int32_t list_j[kMaxTopK + 1];
  __shared__ float list_w[kMaxTopK + 1];
  __shared__ float acc_red[16][260];

  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int Tb = p.seqlens ? p.seqlens[b] : p.T;
  Tb = Tb < 0 ? 0 : (Tb < p.T ? Tb : p.T);
  const int64_t row = (int64_t)b * p.n_q + h;
  T* out = (T*)p.out + row * p.d_v;
  int32_t* sel_out = p.sel_out ? p.sel_out + row * (p.top_k + 1) : nullptr;
  if (sel_out)
    for (int i = tid; i <= p.top_k; i += kThreads) sel_out[i] = -1;
  if (Tb <= 0) {
    for (int e = tid; e < p.d_v; e += kThreads) store_from_float(out, e, 0.f);
    if (tid == 0 && p.lse_out) p.lse_out[row] = -INFINITY;
    return;
  }
  const float* s = p.scores + row * p.T_pad;

  // ---- log-sum-exp over all T_b positions --------------------------------------------------------
  float m = -INFINITY;
  for (int j = tid; j < Tb; j += kThreads) m = fmaxf(m, s[j]);
  m = block_max(m, red);
  float l = 0.f;
  for (int j = tid; j < Tb; j += kThreads) l += exp2f(s[j] - m);
  l = block_sum(l, red);
  const float inv_l = 1.f / l;

  // ---- threshold: the top_k-th largest score among the previous positions 0 .. T_b - 2 -----------
  const int prev = Tb - 1;
  const bool all = prev <= p.top_k;
  uint32_t thr = 0;        // keys > thr are winners; of the keys == thr the first `need` in position order
  uint32_t need = 0;
  if (!all) {
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)p.top_k;
    for (int shift = 24; shift >= 0; shift -= 8) {
      for (int i = tid; i < 256; i += kThreads) hist[i] = 0;
      __syncthreads();
      for (int j = tid; j < prev; j += kThreads) {
        const uint32_t key = order_key(s[j]);
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (tid == 0) {
        uint32_t above = 0;
        int d = 255;
        for (; d > 0; --d) {
          if (above + hist[d] >= remaining) break;
          above += hist[d];
        }
        sh_prefix = prefix | ((uint32_t)d << shift);
        sh_need = remaining - above;  // still to take inside digit d
      }
      __syncthreads();
      prefix = sh_prefix;
      remaining = sh_need;
      mask |= 255u << shift;
      __syncthreads();
    }
    thr = prefix;
    need = remaining;
  }

  // ---- in-order compaction: every wavefront scans its own contiguous quarter of the positions -----
  const int per_wave = ((prev + kWaves - 1) / kWaves + 63) & ~63;
  const int w0 = wave * per_wave;
  int w1 = w0 + per_wave;
  w1 = w1 < prev ? w1 : prev;
  int cnt_gt = 0, cnt_eq = 0;  // wavefront-uniform running counts
  for (int base = w0; base < w1; base += 64) {
    const int j = base + lane;
    bool gt = false, eq = false;
    if (j < w1) {
      const uint32_t key = order_key(s[j]);
      gt = all || key > thr;
      eq = !all && key == thr;
    }
    const uint64_t bg = __ballot(gt), be = __ballot(eq);
    const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    if (gt) {
      const int pos = cnt_gt + __popcll(bg & below);
      if (pos < kMaxTopK) sel_gt[wave][pos] = j;
    }
    if (eq) {
      const int pos = cnt_eq + __popcll(be & below);
      if (pos < kMaxTopK) sel_eq[wave][pos] = j;
    }
    cnt_gt += __popcll(bg);
    cnt_eq += __popcll(be);
  }
  if (lane == 0) {
    n_gt[wave] = cnt_gt < kMaxTopK ? cnt_gt : kMaxTopK;
    n_eq[wave] = cnt_eq < kMaxTopK ? cnt_eq : kMaxTopK;
  }
  __syncthreads();
  // concatenate: winners of wavefront 0..3, then ties in position order up to `need`, then the
  // current token.  Thread 0 fixes the layout (counts are tiny), all threads fill it.
  __shared__ int32_t off_gt[kWaves + 1], off_eq[kWaves + 1], n_total;
  if (tid == 0) {
    int o = 0;
    for (int w = 0; w < kWaves; ++w) {
      off_gt[w] = o;
      o += n_gt[w];
    }
    off_gt[kWaves] = o;
    int left = (int)need;
    for (int w = 0; w < kWaves; ++w) {
      off_eq[w] = o;
      const int take = n_eq[w] < left ? n_eq[w] : left;
      o += take;
      left -= take;
    }
    off_eq[kWaves] = o;
    n_total = o + 1;
  }
  __syncthreads();
  for (int w = 0; w < kWaves; ++w) {
    for (int i = tid; i < off_gt[w + 1] - off_gt[w]; i += kThreads) list_j[off_gt[w] + i] = sel_gt[w][i];
    const int e_end = (w + 1 < kWaves) ? off_eq[w + 1] : off_eq[kWaves];
    for (int i = tid; i < e_end - off_eq[w]; i += kThreads) list_j[off_eq[w] + i] = sel_eq[w][i];
  }
  if (tid == 0) list_j[n_total - 1] = Tb - 1;
  __syncthreads();
  const int cnt = n_total;
  float mass = 0.f;
  for (int i = tid; i < cnt; i += kThreads) {
    const float w = exp2f(s[list_j[i]] - m) * inv_l;
    list_w[i] = w;
    mass += w;
    if (sel_out) sel_out[i] = list_j[i];
  }
  mass = block_sum(mass, red);  // (also orders the list_w writes before the reads below)
  const float norm = p.renormalize ? 1.f / mass : 1.f;

  // ---- weighted sum of the gathered V rows: thread (r, c) takes entries r, r + R, ... and 4 channels
  const int vh = (int)(((int64_t)h * p.n_v) / p.n_q);
  const int quads = p.d_v / 4;             // <= 64
  const int R = kThreads / quads;          // entries in flight per pass (>= 4)
  const int r = tid / quads, c = tid % quads;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  if (r < R && r < 16) {
    const int Ruse = R < 16 ? R : 16;
    for (int i = r; i < cnt; i += Ruse) {
      const int j = list_j[i];
      int64_t off = (int64_t)vh * p.v_sh + c * 4;
      if (PAGED)
        off += (int64_t)p.block_table[(int64_t)b * p.max_pages + j / p.page_size] * p.v_sb +
               (int64_t)(j % p.page_size) * p.v_st;
      else
        off += (int64_t)b * p.v_sb + (int64_t)j * p.v_st;
      const T* vr = (const T*)p.v + off;
      const float w = list_w[i];
      a0 = fmaf(w, load_as_float(vr, 0), a0);
      a1 = fmaf(w, load_as_float(vr, 1), a1);
      a2 = fmaf(w, load_as_float(vr, 2), a2);
      a3 = fmaf(w, load_as_float(vr, 3), a3);
    }
    acc_red[r][c * 4 + 0] = a0;
    acc_red[r][c * 4 + 1] = a1;
    acc_red[r][c * 4 + 2] = a2;
    acc_red[r][c * 4 + 3] = a3;
  }
  __syncthreads();
  const int Ruse = (R < 16 ? R : 16);
  for (int e = tid; e < p.d_v; e += kThreads) {
    float v = 0.f;
    for (int rr = 0; rr < Ruse; ++rr) v += acc_red[rr][e];
    store_from_float(out, e, v * norm);
  }
  if (tid == 0 && p.lse_out) p.lse_out[row] = (m + log2f(l)) * kLn2;
}

}  // namespace

int topk_max_k() { return kMaxTopK; }

bool topk_scores_mfma_supported(const TopkParams& p, int dtype) {
  if (dtype != 1) return false;
  if (p.n_q / p.n_k > 16) return false;
  if (p.d_qk != 64 && p.d_qk != 128) return false;
  if (p.block_table && (p.page_size % 16 != 0)) return false;
  return 16 * p.k_st * 2 + 512 < (1ll << 31);
}

hipError_t launch_topk(const TopkParams& p, int dtype, bool paged, bool mfma, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  if (p.T_pad > 0) {
    if (mfma) {
      dim3 grid((p.T_pad + p.chunk - 1) / p.chunk, p.n_k, p.B);
      if (p.d_qk == 128) {
        if (paged) topk_scores_mfma_kernel<128, true><<<grid, kThreads, 0, s>>>(p);
        else topk_scores_mfma_kernel<128, false><<<grid, kThreads, 0, s>>>(p);
      } else {
        if (paged) topk_scores_mfma_kernel<64, true><<<grid, kThreads, 0, s>>>(p);
        else topk_scores_mfma_kernel<64, false><<<grid, kThreads, 0, s>>>(p);
      }
    } else {
      dim3 grid((p.T_pad + kThreads - 1) / kThreads, p.n_q, p.B);
      if (dtype == 0) {
        if (paged) topk_scores_generic_kernel<float, true><<<grid, kThreads, 0, s>>>(p);
        else topk_scores_generic_kernel<float, false><<<grid, kThreads, 0, s>>>(p);
      } else {
        if (paged) topk_scores_generic_kernel<uint16_t, true><<<grid, kThreads, 0, s>>>(p);
        else topk_scores_generic_kernel<uint16_t, false><<<grid, kThreads, 0, s>>>(p);
      }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  dim3 grid2(p.n_q, p.B);
  if (dtype == 0) {
    if (paged) topk_select_kernel<float, true><<<grid2, kThreads, 0, s>>>(p);
    else topk_select_kernel<float, false><<<grid2, kThreads, 0, s>>>(p);
  } else {
    if (paged) topk_select_kernel<uint16_t, true><<<grid2, kThreads, 0, s>>>(p);
    else topk_select_kernel<uint16_t, false><<<grid2, kThreads, 0, s>>>(p);
  }
  return hipGetLastError();
}

}  // namespace diffqkv
