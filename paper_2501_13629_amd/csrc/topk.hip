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
//   select   one 1024-thread workgroup per (sequence, query head): maximum and a coarse histogram of
//            an order-preserving integer image of the scores locate the bin of the top_k-th largest
//            among the previous positions; the positions at or above it become candidates in LDS,
//            where three more radix rounds settle the threshold exactly; ties go by position; the
//            winners are put into position order, then their V rows are gathered and summed.
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
constexpr int kSelThreads = 1024;  // select kernel: one workgroup of 16 wavefronts per (sequence, head)
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kTile = kSelThreads * 4;  // positions covered by one workgroup-wide 16-byte load
constexpr int kRegTiles = 8;            // 32768 positions of a row stay in registers between the passes
constexpr int kCandMax = 4096;          // candidate slots of the fast selection path
constexpr int kCoarseBits = 12;         // sign + exponent + 3 mantissa bits decide the first radix round
constexpr int kCoarseBins = 1 << kCoarseBits;
constexpr int kMaxTopK = 512;

__device__ __forceinline__ float block_max(float x, float* red) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  if (lane == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  x = lane < kSelWaves ? red[lane] : -INFINITY;
#pragma unroll
  for (int o = kSelWaves / 2; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  x = __shfl(x, 0, 64);
  __syncthreads();
  return x;
}
__device__ __forceinline__ float block_sum(float x, float* red) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  if (lane == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  x = lane < kSelWaves ? red[lane] : 0.f;
#pragma unroll
  for (int o = kSelWaves / 2; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  x = __shfl(x, 0, 64);
  __syncthreads();
  return x;
}

// Among 256 counts in LDS (bin 255 = largest digit), the bin that holds the `remaining`-th element
// counted from the top, how many of that bin are still to take, and the bin's own count.  Called by
// one whole wavefront; lane i holds bins 4 i .. 4 i + 3, a suffix scan over lanes finds the lane,
// which then walks its four.  Requires 1 <= remaining <= total.  Every lane gets the result.
__device__ __forceinline__ void find_digit(const uint32_t* counts, uint32_t remaining, uint32_t& digit,
                                           uint32_t& need, uint32_t& in_bin) {
  const int lane = threadIdx.x & 63;
  uint32_t c[4];
#pragma unroll
  for (int x = 0; x < 4; ++x) c[x] = counts[4 * lane + x];
  const uint32_t tot = c[0] + c[1] + c[2] + c[3];
  uint32_t suf = tot;  // inclusive suffix sum over lanes >= lane
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t v = __shfl_down(suf, o, 64);
    if (lane + o < 64) suf += v;
  }
  uint32_t above = suf - tot;
  const bool here = suf >= remaining && above < remaining;
  int d = 3;
  for (; d > 0; --d) {
    if (above + c[d] >= remaining) break;
    above += c[d];
  }
  const uint64_t who = __ballot(here);
  const int src = who ? __builtin_ctzll(who) : 0;
  digit = (uint32_t)__shfl((int)(4 * lane + d), src, 64);
  need = (uint32_t)__shfl((int)(remaining - above), src, 64);
  in_bin = (uint32_t)__shfl((int)c[d], src, 64);
}

__device__ __forceinline__ void load4_as_float(const float* p, float (&x)[4]) {
  const f32x4 v = *(const f32x4*)p;
  x[0] = v[0], x[1] = v[1], x[2] = v[2], x[3] = v[3];
}
__device__ __forceinline__ void load4_as_float(const uint16_t* p, float (&x)[4]) {
  const uint2 v = *(const uint2*)p;
  x[0] = __uint_as_float(v.x << 16), x[1] = __uint_as_float(v.x & 0xffff0000u);
  x[2] = __uint_as_float(v.y << 16), x[3] = __uint_as_float(v.y & 0xffff0000u);
}

// Selection and gather.  The usual case takes two passes over the score row, the second out of
// registers for rows of up to 32768 positions:
//   1. maximum, and a 4096-bin histogram of the top 12 key bits of the previous positions, which
//      locates the bin that holds the top_k-th largest score;
//   2. sum of exponentials, and collection of every position at or above that bin into LDS.
// The exact threshold (remaining 20 key bits) and the tie rule are then settled on those few
// candidates, and the winners are put into position order by counting, so the order of the weighted
// sum never depends on scheduling.  If more than kCandMax candidates qualify (e.g. thousands of
// equal scores) an exact radix select over the row in global memory takes over, with an ordered
// two-step compaction.  Both produce the same list.
template <typename T, bool PAGED>
__global__ __launch_bounds__(kSelThreads) void topk_select_kernel(TopkParams p) {
  __shared__ float red[kSelWaves];
  __shared__ uint32_t hist[kCoarseBins];
  __shared__ uint32_t part[256];
  __shared__ uint32_t sh_prefix, sh_need, sh_inbin;
  __shared__ int32_t cand_j[kCandMax];
  __shared__ uint32_t cand_key[kCandMax];
  __shared__ int32_t n_cand_sh, n_sel_sh, n_total;
  __shared__ int32_t wave_gt[kSelWaves], wave_eq[kSelWaves];
  __shared__ int32_t sel_j[kMaxTopK + 1];
  __shared__ int32_t list_j[kMaxTopK + 1];
  __shared__ float list_w[kMaxTopK + 1];
  __shared__ float acc_red[kSelThreads * 4];

  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int Tb = p.seqlens ? p.seqlens[b] : p.T;
  Tb = Tb < 0 ? 0 : (Tb < p.T ? Tb : p.T);
  const int64_t row = (int64_t)b * p.n_q + h;
  T* out = (T*)p.out + row * p.d_v;
  int32_t* sel_out = p.sel_out ? p.sel_out + row * (p.top_k + 1) : nullptr;
  if (sel_out)
    for (int i = tid; i <= p.top_k; i += kSelThreads) sel_out[i] = -1;
  if (Tb <= 0) {
    for (int e = tid; e < p.d_v; e += kSelThreads) store_from_float(out, e, 0.f);
    if (tid == 0 && p.lse_out) p.lse_out[row] = -INFINITY;
    return;
  }
  const float* s = p.scores + row * p.T_pad;
  const int prev = Tb - 1;
  const bool all = prev <= p.top_k;             // everything is selected: no threshold needed
  const bool search = !all && p.top_k > 0;      // (top_k = 0: only the current token)
  const uint64_t below = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
  const int ntiles = (prev + kTile - 1) / kTile;
  const bool resident = ntiles <= kRegTiles;

  for (int i = tid; i < kCoarseBins; i += kSelThreads) hist[i] = 0;
  if (tid == 0) n_cand_sh = 0, n_sel_sh = 0;
  __syncthreads();

  // ---- pass 1: maximum over all T_b positions, coarse histogram over the previous ones -------------
  f32x4 v[kRegTiles];
  auto load_tiles = [&](int t0) {
#pragma unroll
    for (int u = 0; u < kRegTiles; ++u) {
      const int j = ((t0 + u) * kSelThreads + tid) * 4;  // j and the padded row length: multiples of 4
      v[u] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
      if (j < prev) v[u] = *(const f32x4*)(s + j);
    }
  };
  float m = -INFINITY;
  for (int t0 = 0; t0 < ntiles; t0 += kRegTiles) {
    load_tiles(t0);
#pragma unroll
    for (int u = 0; u < kRegTiles; ++u) {
      const int j = ((t0 + u) * kSelThreads + tid) * 4;
#pragma unroll
      for (int x = 0; x < 4; ++x)
        if (j + x < prev) {
          m = fmaxf(m, v[u][x]);
          if (search) atomicAdd(&hist[order_key(v[u][x]) >> (32 - kCoarseBits)], 1u);
        }
    }
  }
  if (tid == 0) m = fmaxf(m, s[Tb - 1]);  // the current token
  m = block_max(m, red);

  // bin of the top_k-th largest: 256 groups of 16 bins, then inside one group
  uint32_t coarse = 0, need = 0;  // candidates: top key bits >= coarse; `need` to take inside that bin
  bool fast = true;
  if (search) {
    if (tid < 256) {
      uint32_t mine = 0;
      for (int i = 0; i < kCoarseBins / 256; ++i) mine += hist[tid * (kCoarseBins / 256) + i];
      part[tid] = mine;
    }
    __syncthreads();
    if (wave == 0) {
      uint32_t grp, left, in_grp;
      find_digit(part, (uint32_t)p.top_k, grp, left, in_grp);
      if (lane == 0) {
        uint32_t above = 0;
        int d = kCoarseBins / 256 - 1;
        for (; d > 0; --d) {
          const uint32_t c = hist[grp * (kCoarseBins / 256) + d];
          if (above + c >= left) break;
          above += c;
        }
        const uint32_t bin = grp * (kCoarseBins / 256) + d;
        sh_prefix = bin;
        sh_need = left - above;
        sh_inbin = hist[bin];
      }
    }
    __syncthreads();
    coarse = sh_prefix;
    need = sh_need;
    // candidates = those above the bin (top_k - need of them) + the bin itself
    fast = (uint32_t)p.top_k - need + sh_inbin <= (uint32_t)kCandMax;
    __syncthreads();
  }

  // ---- pass 2: sum of exponentials; candidates into LDS (any order) --------------------------------------
  // (candidates are a few hundred of tens of thousands: one vote per quad decides whether to look closer)
  float l = 0.f;
  for (int t0 = 0; t0 < ntiles; t0 += kRegTiles) {
    if (!resident) load_tiles(t0);
#pragma unroll
    for (int u = 0; u < kRegTiles; ++u) {
      const int j = ((t0 + u) * kSelThreads + tid) * 4;
      bool c[4];
      uint32_t key[4];
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const bool live = j + x < prev;  // (a loaded quad may reach into the current token and the padding)
        const float e = __builtin_amdgcn_exp2f(v[u][x] - m);  // (arguments <= 0; results below the normal range count as zero)
        l += live ? e : 0.f;
        key[x] = order_key(v[u][x]);
        c[x] = fast && live && (all || (search && (key[x] >> (32 - kCoarseBits)) >= coarse));
      }
      if (__ballot(c[0] || c[1] || c[2] || c[3]) == 0) continue;
      const uint64_t b0 = __ballot(c[0]), b1 = __ballot(c[1]), b2 = __ballot(c[2]), b3 = __ballot(c[3]);
      int base = 0;
      if (lane == 0) base = atomicAdd(&n_cand_sh, __popcll(b0) + __popcll(b1) + __popcll(b2) + __popcll(b3));
      base = __shfl(base, 0, 64);
      int pos = base + __popcll(b0 & below) + __popcll(b1 & below) + __popcll(b2 & below) + __popcll(b3 & below);
#pragma unroll
      for (int x = 0; x < 4; ++x)
        if (c[x]) {
          cand_j[pos] = j + x;  // (the count was bounded above: pos < kCandMax)
          cand_key[pos] = key[x];
          ++pos;
        }
    }
  }
  if (tid == 0) l += __builtin_amdgcn_exp2f(s[Tb - 1] - m);
  l = block_sum(l, red);  // (its barriers also publish the candidates)
  const float inv_l = 1.f / l;

  if (fast) {
    const int n_cand = n_cand_sh;
    uint32_t thr = 0, n_ties = 0;
    if (search) {
      // ---- exact threshold among the candidates of the coarse bin: the remaining 20 key bits --------
      uint32_t prefix = coarse << (32 - kCoarseBits), mask = ~0u << (32 - kCoarseBits), remaining = need;
      for (int shift = 12; shift >= -4; shift -= 8) {  // digits at bits 19..12, 11..4, 3..0
        const int sh = shift < 0 ? 0 : shift;
        const uint32_t dmask = shift < 0 ? 15u : 255u;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n_cand; i += kSelThreads) {
          const uint32_t key = cand_key[i];
          if ((key & mask) == prefix) atomicAdd(&hist[(key >> sh) & dmask], 1u);
        }
        __syncthreads();
        if (wave == 0) {  // (with 16 digits the bins 16..255 stay zero)
          uint32_t d, left, in_bin;
          find_digit(hist, remaining, d, left, in_bin);
          if (lane == 0) {
            sh_prefix = prefix | (d << sh);
            sh_need = left;
            sh_inbin = in_bin;
          }
        }
        __syncthreads();
        prefix = sh_prefix;
        remaining = sh_need;
        n_ties = sh_inbin;
        mask |= dmask << sh;
        __syncthreads();
      }
      thr = prefix;
      need = remaining;
    }
    // ---- winners and the `need` lowest-positioned ties (any order), then into position order ------------
    for (int i = tid; i < n_cand; i += kSelThreads) {
      const uint32_t key = cand_key[i];
      const int j = cand_j[i];
      bool take = all || key > thr;
      if (!all && key == thr) {
        take = n_ties == need;  // every score equal to the threshold is in: the usual case
        if (!take) {            // real ties across the boundary: the lower positions win
          uint32_t rank = 0;
          for (int o = 0; o < n_cand; ++o) rank += (cand_key[o] == thr && cand_j[o] < j) ? 1u : 0u;
          take = rank < need;
        }
      }
      if (take) sel_j[atomicAdd(&n_sel_sh, 1)] = j;
    }
    __syncthreads();
    const int n_sel = n_sel_sh;
    for (int i = tid; i < n_sel; i += kSelThreads) {
      const int j = sel_j[i];
      int rank = 0;
      for (int o = 0; o < n_sel; ++o) rank += sel_j[o] < j ? 1 : 0;
      list_j[rank] = j;
    }
    if (tid == 0) {
      list_j[n_sel] = Tb - 1;
      n_total = n_sel + 1;
    }
    __syncthreads();
  } else {
    // ---- exact radix select straight from the score row (4 rounds of 8 bits) -------------------------
    uint32_t prefix = 0, mask = 0, remaining = (uint32_t)p.top_k;
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      for (int j = tid; j < prev; j += kSelThreads) {
        const uint32_t key = order_key(s[j]);
        if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (wave == 0) {
        uint32_t d, left, in_bin;
        find_digit(hist, remaining, d, left, in_bin);
        if (lane == 0) {
          sh_prefix = prefix | (d << shift);
          sh_need = left;
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      remaining = sh_need;
      mask |= 255u << shift;
      __syncthreads();
    }
    const uint32_t thr = prefix;
    need = remaining;
    // ordered compaction in two steps: every wavefront scans a contiguous share of the row; first the
    // counts of winners and ties per share, then -- knowing how many ties each share may still take
    // and where its output starts -- the positions themselves
    const int per_wave = ((prev + kSelWaves - 1) / kSelWaves + 63) & ~63;
    const int w0 = wave * per_wave;
    int w1 = w0 + per_wave;
    w1 = w1 < prev ? w1 : prev;
    int cnt_gt = 0, cnt_eq = 0;
    for (int base = w0; base < w1; base += 64) {
      const int j = base + lane;
      const uint32_t key = j < w1 ? order_key(s[j]) : 0u;
      cnt_gt += __popcll(__ballot(j < w1 && key > thr));
      cnt_eq += __popcll(__ballot(j < w1 && key == thr));
    }
    if (lane == 0) wave_gt[wave] = cnt_gt, wave_eq[wave] = cnt_eq;
    __syncthreads();
    int ties_before = 0, out_before = 0, quota = 0, total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      int q = (int)need - ties_before;
      q = q < 0 ? 0 : (q < wave_eq[w] ? q : wave_eq[w]);
      if (w == wave) quota = q, out_before = total;
      ties_before += wave_eq[w];
      total += wave_gt[w] + q;
    }
    int taken = 0, eq_seen = 0;
    for (int base = w0; base < w1; base += 64) {
      const int j = base + lane;
      const uint32_t key = j < w1 ? order_key(s[j]) : 0u;
      const bool gt = j < w1 && key > thr;
      bool eq = j < w1 && key == thr;
      const uint64_t be = __ballot(eq);
      eq = eq && (eq_seen + __popcll(be & below)) < quota;
      eq_seen += __popcll(be);
      const uint64_t bk = __ballot(gt || eq);
      if (gt || eq) list_j[out_before + taken + __popcll(bk & below)] = j;
      taken += __popcll(bk);
    }
    if (tid == 0) {
      list_j[total] = Tb - 1;
      n_total = total + 1;
    }
    __syncthreads();
  }

  const int cnt = n_total;
  float mass = 0.f;
  for (int i = tid; i < cnt; i += kSelThreads) {
    const float w = exp2f(s[list_j[i]] - m) * inv_l;
    list_w[i] = w;
    mass += w;
    if (sel_out) sel_out[i] = list_j[i];
  }
  mass = block_sum(mass, red);  // (also orders the list_w writes before the reads below)
  const float norm = p.renormalize ? 1.f / mass : 1.f;

  // ---- weighted sum of the gathered V rows: thread (r, c) takes entries r, r + R, ... and 4 channels
  const int vh = (int)(((int64_t)h * p.n_v) / p.n_q);
  const int quads = p.d_v / 4;        // <= 64
  const int R = kSelThreads / quads;  // rows in flight per pass (>= 16)
  const int r = tid / quads, c = tid % quads;
  if (r < R) {
    float a[4] = {0.f, 0.f, 0.f, 0.f};
    auto row_of = [&](int i) {
      const int j = list_j[i];
      int64_t off = (int64_t)vh * p.v_sh + c * 4;
      if (PAGED)
        off += (int64_t)p.block_table[(int64_t)b * p.max_pages + j / p.page_size] * p.v_sb +
               (int64_t)(j % p.page_size) * p.v_st;
      else
        off += (int64_t)b * p.v_sb + (int64_t)j * p.v_st;
      return (const T*)p.v + off;
    };
    int i = r;
    for (; i + R < cnt; i += 2 * R) {  // two rows per trip: both loads in flight together
      float x0[4], x1[4];
      load4_as_float(row_of(i), x0);
      load4_as_float(row_of(i + R), x1);
      const float w0 = list_w[i], w1 = list_w[i + R];
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] = fmaf(w1, x1[e], fmaf(w0, x0[e], a[e]));
    }
    if (i < cnt) {
      float x0[4];
      load4_as_float(row_of(i), x0);
      const float w0 = list_w[i];
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] = fmaf(w0, x0[e], a[e]);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) acc_red[r * p.d_v + c * 4 + e] = a[e];
  }
  __syncthreads();
  for (int e = tid; e < p.d_v; e += kSelThreads) {
    float acc = 0.f;
    for (int rr = 0; rr < R; ++rr) acc += acc_red[rr * p.d_v + e];
    store_from_float(out, e, acc * norm);
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
        if (paged) launch_kernel(0, topk_scores_mfma_kernel<128, true>, dim3(grid), dim3(kThreads), 0, s, p);
        else launch_kernel(0, topk_scores_mfma_kernel<128, false>, dim3(grid), dim3(kThreads), 0, s, p);
      } else {
        if (paged) launch_kernel(0, topk_scores_mfma_kernel<64, true>, dim3(grid), dim3(kThreads), 0, s, p);
        else launch_kernel(0, topk_scores_mfma_kernel<64, false>, dim3(grid), dim3(kThreads), 0, s, p);
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
    if (paged) launch_kernel(1, topk_select_kernel<float, true>, dim3(grid2), dim3(kSelThreads), 0, s, p);
    else launch_kernel(1, topk_select_kernel<float, false>, dim3(grid2), dim3(kSelThreads), 0, s, p);
  } else {
    if (paged) launch_kernel(1, topk_select_kernel<uint16_t, true>, dim3(grid2), dim3(kSelThreads), 0, s, p);
    else launch_kernel(1, topk_select_kernel<uint16_t, false>, dim3(grid2), dim3(kSelThreads), 0, s, p);
  }
  return hipGetLastError();
}

}  // namespace diffqkv
