// Split-decode kernel for bf16 caches on gfx950 matrix cores.
//
// One workgroup (4 wavefronts) owns one (sequence, K head, context chunk).  It streams the chunk's
// K rows once for all g_k = n_q / n_k query rows under that K head, and the rows of each of the
// R = n_v / n_k V heads under it once for their g_v = n_q / n_v query rows -- the byte count of the
// cost model in section 3.1 ("KV Cache"): (n_k d_qk + n_v d_v) elements per token.  The head map is
// the "idx" rule of section 3.2: query row r of the group reads V head  kh * R + r / g_v.
//
// Data path (per wavefront, 32 tokens at a time, no LDS in the loop):
//   S^T = K Q^T      v_mfma_f32_16x16x32_bf16, A = K rows straight from HBM (16 B per lane),
//                    B = Q^T held in registers.  Result: lane (g, n) holds the scores of query row
//                    n for tokens 4g..4g+3 of each 16-token block.
//   online softmax   in that layout: the running maximum is per query row = per lane column, so
//                    the rescale of the accumulators is lane-local; one cross-lane maximum (two
//                    shuffles) per 32 tokens.
//   O^T = V^T P^T    A = V^T: each lane loads 16 B (8 channels) of 8 different tokens and
//                    transposes the 8x8 block inside its own registers (v_perm_b32), giving the
//                    8 tokens of one channel per register quad; B = P^T is the softmax output as
//                    it stands, masked to the query rows of the V head being streamed, so all V
//                    heads accumulate into one 16 x d_v accumulator.
// Every global load is 16 B (d_v = 128) or 8 B (d_v = 64) per lane with each 16-lane group reading
// one contiguous row segment.
//
// The 4 wavefronts take interleaved 32-token sub-tiles of each 128-token tile and merge their
// running (max, sum, accumulator) through LDS at the end of the chunk.  The result is written as a
// normalised partial output with its base-2 log-sum-exp, or as the final row when there is a
// single split.
#include <type_traits>

#include "kernels.h"

namespace diffqkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kSub = 32;             // tokens per wavefront step
constexpr int kTile = kWaves * kSub; // tokens per workgroup step
constexpr int kStreamKMaxB = 4096;   // sequences whose unit prefix fits the LDS table of the ragged mode

// CW bf16 channels (CW * 2 bytes) from a 16-byte-aligned (CW = 8) or 8-byte-aligned (CW = 4) address
template <int CW>
struct ChunkLoad;
template <>
struct ChunkLoad<8> {
  static constexpr int kWords = 4;
  typedef u32x4 vec;
};
template <>
struct ChunkLoad<4> {
  static constexpr int kWords = 2;
  typedef u32x2 vec;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// Raw buffer resource over [base, base + 2 GiB): lets a load take a wavefront-uniform byte offset
// in a scalar register on top of the per-lane offset, so the loop carries no per-lane address
// arithmetic.  Every offset used below addresses a live cache row (checked on the host against the
// 2 GiB window; rows past the end of a sequence are redirected, never read).
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
// Cache rows are read exactly once: the loads carry the non-temporal hint (streaming, no reuse).
constexpr int kNonTemporal = 2;
template <int CW>
__device__ __forceinline__ typename ChunkLoad<CW>::vec buffer_load_chunk(rsrc_t r, int voff, int soff);
template <>
__device__ __forceinline__ u32x4 buffer_load_chunk<8>(rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, kNonTemporal);
}
template <>
__device__ __forceinline__ u32x2 buffer_load_chunk<4>(rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, kNonTemporal);
}

// RT: number of V heads per K head when it is one of the unrolled cases (1, 2, 4, 8); then the loop
// over V heads is unrolled and software-pipelined: while the matrix cores work on one unit (the K
// rows of a sub-tile, or the rows of one V head), the loads of the next unit are already in flight
// into a second set of registers.  RT = 0 takes any ratio with a plain loop.
//
// SK selects how the work is cut:
//   SK = false  grid (splits, n_k, B): one workgroup per (sequence, K head, fixed-size chunk); its 4
//               wavefronts take interleaved sub-tiles and merge through LDS.  Used for uniform lengths,
//               where one round of workgroups covers the whole cache.
//   SK = true   ragged lengths: every wavefront is a worker of its own.  All 32-token units of all
//               (sequence, K head) streams are laid end to end and cut into equal slices, one per
//               worker, so every worker streams the same number of bytes whatever the length mix.
//               A worker whose slice crosses from one (sequence, K head) to the next writes one
//               partial result per stream it touched; slot numbers follow from the slice length.
template <int DQK, int DV, bool PAGED, int RT, bool SK>
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(DecodeParams p) {
  constexpr int KK = DQK / 32;  // k-steps of the score product
  constexpr int CW = DV / 16;   // channels per lane in the V product
  typedef typename ChunkLoad<CW>::vec vvec;

  __shared__ float lds_ml[2][SK ? 1 : kWaves][16];
  __shared__ float lds_o[SK ? 1 : kWaves][16][DV + 4];
  __shared__ int32_t lds_cum[SK ? kStreamKMaxB + 1 : 1];  // units of the sequences before b
  __shared__ int32_t lds_scan[SK ? kThreads : 1];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, n = lane & 15;

  const int G = p.G;                           // query rows under a K head (<= 16)
  const int R = RT ? RT : p.n_v / p.n_k;       // V heads under a K head
  const int g_v = G / R;                       // query rows per V head
  const int k_row_bytes = (int)p.k_st * 2, v_row_bytes = (int)p.v_st * 2, v_head_bytes = (int)p.v_sh * 2;

  // The stream being read: set once (SK = false) or per segment of the worker's slice (SK = true).
  int b = 0, kh = 0, h0 = 0;
  int c1 = 0, last = 0;            // end of the live tokens this wavefront may read, and c1 - 1
  const uint16_t* khead = nullptr; // wavefront-uniform bases of the K head and of its first V head
  const uint16_t* vhead = nullptr;
  const int32_t* bt = nullptr;
  bf16x8 qf[KK];                   // Q^T as the B operand: lane (g, n): channels 32 kk + 8 g .. + 7 of row n
  auto select_stream = [&](int b_, int kh_) {
    b = b_;
    kh = kh_;
    h0 = kh * G;
    khead = (const uint16_t*)p.k + (int64_t)kh * p.k_sh;
    vhead = (const uint16_t*)p.v + (int64_t)(kh * R) * p.v_sh;
    if (!PAGED) {
      khead += (int64_t)b * p.k_sb;
      vhead += (int64_t)b * p.v_sb;
    }
    bt = PAGED ? p.block_table + (int64_t)b * p.max_pages : nullptr;
    const uint16_t* qrow = (const uint16_t*)p.q + ((int64_t)b * p.n_q + h0 + (n < G ? n : 0)) * DQK;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      u32x4 w = *(const u32x4*)(qrow + kk * 32 + g * 8);
      if (n >= G) w = u32x4{0u, 0u, 0u, 0u};
      qf[kk] = __builtin_bit_cast(bf16x8, w);
    }
  };

  // Where a sub-tile (two 16-token blocks starting at token ts) lives: one buffer resource per
  // block for K and for V (a block never straddles a page), plus this lane's byte offsets inside
  // the block.  In a full sub-tile the lane offsets are loop constants: K row n, V rows 4 g + x.
  // In the last, partial sub-tile of a sequence a block that starts beyond the last live token is
  // redirected to the block that holds it and a row beyond it to that token, so every address
  // stays inside live rows; the duplicates are masked out of the softmax.
  struct SubTile {
    rsrc_t k[2], v[2];
  };
  struct LaneOffsets {
    int k[2];
    int v[2][4];
  };
  auto block_start = [&](int ts, int blk, bool tail) {
    int s0 = ts + 16 * blk;
    if (tail) {
      const int lim = last & ~15;
      s0 = s0 < lim ? s0 : lim;
    }
    return s0;
  };
  auto locate = [&](int ts, bool tail) {
    SubTile t;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int s0 = block_start(ts, blk, tail);
      int64_t ko, vo;
      if (PAGED) {
        const int page = bt[s0 / p.page_size];
        const int slot = s0 % p.page_size;
        ko = (int64_t)page * p.k_sb + (int64_t)slot * p.k_st;
        vo = (int64_t)page * p.v_sb + (int64_t)slot * p.v_st;
      } else {
        ko = (int64_t)s0 * p.k_st;
        vo = (int64_t)s0 * p.v_st;
      }
      t.k[blk] = make_rsrc(khead + ko);
      t.v[blk] = make_rsrc(vhead + vo);
    }
    return t;
  };
  LaneOffsets full_off;
#pragma unroll
  for (int blk = 0; blk < 2; ++blk) {
    full_off.k[blk] = n * k_row_bytes + g * 16;
#pragma unroll
    for (int x = 0; x < 4; ++x) full_off.v[blk][x] = (4 * g + x) * v_row_bytes + n * (CW * 2);
  }
  auto tail_offsets = [&](int ts) {
    LaneOffsets o;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      const int maxr = last - block_start(ts, blk, true);
      o.k[blk] = (n < maxr ? n : maxr) * k_row_bytes + g * 16;
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int r = 4 * g + x;
        o.v[blk][x] = (r < maxr ? r : maxr) * v_row_bytes + n * (CW * 2);
      }
    }
    return o;
  };
  auto load_k = [&](const SubTile& t, const LaneOffsets& o, u32x4 (&kw)[2][KK]) {
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        kw[blk][kk] = __builtin_amdgcn_raw_buffer_load_b128(t.k[blk], o.k[blk] + kk * 64, 0, kNonTemporal);
  };
  auto load_v = [&](const SubTile& t, const LaneOffsets& o, int vv, vvec (&vr)[8]) {
    const int head = vv * v_head_bytes;  // wavefront-uniform: travels in a scalar register
#pragma unroll
    for (int e = 0; e < 8; ++e) vr[e] = buffer_load_chunk<CW>(t.v[e >> 2], o.v[e >> 2][e & 3], head);
  };

  f32x4 acc[CW];
  float m_run;   // running maximum of query row n (same in the 4 lanes of a column)
  float l_run;   // this lane's share of the running sum
  uint32_t pw[4];  // P^T as the B operand: k-slots 0..3 = block 0, 4..7 = block 1
  auto reset_state = [&]() {
#pragma unroll
    for (int c = 0; c < CW; ++c) acc[c] = f32x4{0.f, 0.f, 0.f, 0.f};
    m_run = -INFINITY;
    l_run = 0.f;
  };
  reset_state();

  // S^T = K Q^T, then the online softmax.  Lane (g, n): tokens ts + 16 blk + 4 g + x of row n.
  auto scores_and_softmax = [&](int ts, const u32x4 (&kw)[2][KK], bool tail) {
    float sv[8];
    float m_tile = -INFINITY;
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
      f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kk = 0; kk < KK; ++kk)
        s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kw[blk][kk]), qf[kk], s, 0, 0, 0);
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        float v = s[x] * p.scale_log2;
        if (tail) v = (ts + 16 * blk + 4 * g + x) < c1 ? v : -INFINITY;
        sv[blk * 4 + x] = v;
        m_tile = fmaxf(m_tile, v);
      }
    }
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 16, 64));
    m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
    const float m_new = fmaxf(m_run, m_tile);  // finite: token ts is live
    const float fac = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float p0 = __builtin_amdgcn_exp2f(sv[2 * i] - m_new);
      const float p1 = __builtin_amdgcn_exp2f(sv[2 * i + 1] - m_new);
      const uint32_t w = pack_bf16x2(p0, p1);
      pw[i] = w;
      // the sum runs over the rounded weights, so that they sum to one as used
      psum += __uint_as_float(w << 16) + __uint_as_float(w & 0xffff0000u);
    }
    l_run = l_run * fac + psum;
#pragma unroll
    for (int c = 0; c < CW; ++c) acc[c] *= fac;
  };

  // O^T += V^T P^T for one V head: transpose each lane's 8 tokens x CW channels in registers.
  auto accumulate_v = [&](int vv, const vvec (&vr)[8]) {
    const bool mine = (n / g_v) == vv;
    const u32x4 pb = {mine ? pw[0] : 0u, mine ? pw[1] : 0u, mine ? pw[2] : 0u, mine ? pw[3] : 0u};
#pragma unroll
    for (int c = 0; c < CW; ++c) {
      const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
      u32x4 a;
      a[0] = __builtin_amdgcn_perm(vr[1][c >> 1], vr[0][c >> 1], sel);
      a[1] = __builtin_amdgcn_perm(vr[3][c >> 1], vr[2][c >> 1], sel);
      a[2] = __builtin_amdgcn_perm(vr[5][c >> 1], vr[4][c >> 1], sel);
      a[3] = __builtin_amdgcn_perm(vr[7][c >> 1], vr[6][c >> 1], sel);
      acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, pb), acc[c], 0, 0, 0);
    }
  };

  // A sub-tile with no overlap of loads and arithmetic: the partial last sub-tile, and RT = 0.
  auto plain_sub_tile = [&](int ts, bool tail) {
    const SubTile t = locate(ts, tail);
    const LaneOffsets o = tail ? tail_offsets(ts) : full_off;
    u32x4 kw[2][KK];
    load_k(t, o, kw);
    scores_and_softmax(ts, kw, tail);
    for (int vv = 0; vv < R; ++vv) {
      vvec vr[8];
      load_v(t, o, vv, vr);
      accumulate_v(vv, vr);
    }
  };

  // Streams the sub-tiles ts, ts + step, ... below c1 of the selected stream into (m_run, l_run, acc).
  auto run_sub_tiles = [&](int ts, const int step) {
    if (RT) {
      if (ts + kSub <= c1) {  // at least one full sub-tile
        u32x4 kw[2][KK];
        vvec va[8], vb[8];
        SubTile cur = locate(ts, false);
        load_k(cur, full_off, kw);
        // MORE is a compile-time flag (a K prefetch for the next full sub-tile follows), so that the
        // number of loads in flight at every wait is known statically.
        auto sub_tile = [&](auto more_tag) {
          constexpr bool MORE = decltype(more_tag)::value;
          load_v(cur, full_off, 0, va);
          scores_and_softmax(ts, kw, false);
          SubTile nxt = cur;
          if (MORE) nxt = locate(ts + step, false);
#pragma unroll
          for (int vv = 0; vv < RT; ++vv) {
            // put the next unit's loads in flight, then consume the current V head
            if (vv + 1 < RT) {
              if (vv & 1)
                load_v(cur, full_off, vv + 1, va);
              else
                load_v(cur, full_off, vv + 1, vb);
            } else if (MORE) {
              load_k(nxt, full_off, kw);
            }
            if (vv & 1)
              accumulate_v(vv, vb);
            else
              accumulate_v(vv, va);
          }
          cur = nxt;
          ts += step;
        };
        while (ts + step + kSub <= c1) sub_tile(std::true_type{});
        sub_tile(std::false_type{});
      }
      if (ts < c1) plain_sub_tile(ts, true);
    } else {
      for (; ts + kSub <= c1; ts += step) plain_sub_tile(ts, false);
      if (ts < c1) plain_sub_tile(ts, true);
    }
  };

  if (SK) {
    // ---- prefix of 32-token units per sequence, in LDS (and, from workgroup 0, in the workspace
    //      for the combine kernel) ----------------------------------------------------------------
    const int B = p.B;
    const int per = (B + kThreads - 1) / kThreads;
    int mine_sum = 0;
    for (int i = 0; i < per; ++i) {
      const int bb = tid * per + i;
      if (bb < B) {
        int t = p.seqlens ? p.seqlens[bb] : p.T;
        t = t < 0 ? 0 : (t < p.T ? t : p.T);
        mine_sum += (t + kSub - 1) / kSub;
      }
    }
    lds_scan[tid] = mine_sum;
    __syncthreads();
    for (int d = 1; d < kThreads; d <<= 1) {  // inclusive scan of the per-thread sums
      const int v = tid >= d ? lds_scan[tid - d] : 0;
      __syncthreads();
      lds_scan[tid] += v;
      __syncthreads();
    }
    {
      int run = lds_scan[tid] - mine_sum;  // exclusive prefix of this thread's first sequence
      for (int i = 0; i < per; ++i) {
        const int bb = tid * per + i;
        if (bb < B) {
          lds_cum[bb] = run;
          int t = p.seqlens ? p.seqlens[bb] : p.T;
          t = t < 0 ? 0 : (t < p.T ? t : p.T);
          run += (t + kSub - 1) / kSub;
        }
      }
      if (tid == kThreads - 1) lds_cum[B] = lds_scan[kThreads - 1];
    }
    __syncthreads();
    if (blockIdx.x == 0)
      for (int i = tid; i <= B; i += kThreads) p.sk_cum[i] = lds_cum[i];

    // ---- this worker's slice of the unit space: stream (b, kh) starts at n_k cum[b] + kh u_b ----
    const int64_t total = (int64_t)p.n_k * lds_cum[B];
    const int workers = gridDim.x * kWaves;
    int64_t L = (total + workers - 1) / workers;
    L = L < p.sk_lmin ? p.sk_lmin : L;
    const int worker = blockIdx.x * kWaves + wave;
    int64_t pos = (int64_t)worker * L;
    const int64_t end = pos + L < total ? pos + L : total;
    while (pos < end) {
      // the sequence that holds unit `pos`: the last b with n_k cum[b] <= pos
      int lo = 0, hi = B - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int64_t)p.n_k * lds_cum[mid] <= pos) lo = mid; else hi = mid - 1;
      }
      const int bb = lo;
      const int u_b = lds_cum[bb + 1] - lds_cum[bb];  // > 0: empty sequences own no unit
      const int64_t rel = pos - (int64_t)p.n_k * lds_cum[bb];
      const int khh = (int)(rel / u_b), j0 = (int)(rel % u_b);
      const int64_t stream_start = pos - j0;
      int64_t seg_end = stream_start + u_b;
      seg_end = seg_end < end ? seg_end : end;
      const int j1 = (int)(seg_end - stream_start);  // units [j0, j1) of stream (bb, khh)
      int Tb = p.seqlens ? p.seqlens[bb] : p.T;
      Tb = Tb < p.T ? Tb : p.T;
      select_stream(bb, khh);
      c1 = j1 * kSub < Tb ? j1 * kSub : Tb;
      last = c1 - 1;
      reset_state();
      run_sub_tiles(j0 * kSub, kSub);
      // flush this stream's partial: slot = distance from the first worker that touches the stream
      l_run += __shfl_xor(l_run, 16, 64);
      l_run += __shfl_xor(l_run, 32, 64);
      const int slot = worker - (int)(stream_start / L);
      const float inv = 1.f / l_run;
      if (n < G) {
        const int64_t row = ((int64_t)b * p.n_q + h0 + n) * p.num_splits + slot;
        float* orow = p.o_part + row * DV;
        // lane (g, n), acc[c][x]: query row n, channel (4 g + x) * CW + c
#pragma unroll
        for (int x = 0; x < 4; ++x)
#pragma unroll
          for (int c4 = 0; c4 < CW; c4 += 4) {
            const f32x4 w = {acc[c4][x] * inv, acc[c4 + 1][x] * inv, acc[c4 + 2][x] * inv, acc[c4 + 3][x] * inv};
            *(f32x4*)(orow + (4 * g + x) * CW + c4) = w;
          }
        if (g == 0) p.lse_part[row] = m_run + log2f(l_run);
      }
      pos = seg_end;
    }
    return;
  }

  // ---- fixed-size chunks ---------------------------------------------------------------------------
  const int split = blockIdx.x;
  {
    const int kh_ = blockIdx.y, b_ = blockIdx.z;
    int Tb = p.seqlens ? p.seqlens[b_] : p.T;
    Tb = Tb < p.T ? Tb : p.T;
    const int c0 = split * p.chunk;
    if (c0 >= Tb) {
      if (p.num_splits == 1) {  // empty sequence and no combine pass: zeros, lse = -inf
        uint16_t* out = (uint16_t*)p.out + ((int64_t)b_ * p.n_q + kh_ * G) * DV;
        for (int o = tid; o < G * DV; o += kThreads) out[o] = 0;
        if (p.lse_out && tid < G) p.lse_out[(int64_t)b_ * p.n_q + kh_ * G + tid] = -INFINITY;
      }
      return;
    }
    select_stream(b_, kh_);
    c1 = (c0 + p.chunk < Tb) ? c0 + p.chunk : Tb;
    last = c1 - 1;
    run_sub_tiles(c0 + wave * kSub, kTile);
  }

  // ---- merge the 4 wavefronts --------------------------------------------------------------------
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (g == 0) {
    lds_ml[0][wave][n] = m_run;
    lds_ml[1][wave][n] = l_run;
  }
  __syncthreads();
  float m_all = -INFINITY;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, lds_ml[0][w][n]);
  // a wavefront that saw no token has m = -inf, l = 0, acc = 0: weight 0
  const float wgt = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m_all);
  // lane (g, n), acc[c][x]: query row n, channel (4 g + x) * CW + c
#pragma unroll
  for (int c = 0; c < CW; ++c)
#pragma unroll
    for (int x = 0; x < 4; ++x) lds_o[wave][n][(4 * g + x) * CW + c] = acc[c][x] * wgt;
  __syncthreads();

  for (int o = tid; o < G * DV; o += kThreads) {
    const int r = o / DV, e = o % DV;
    float l_all = 0.f, mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, lds_ml[0][w][r]);
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      float mw = lds_ml[0][w][r];
      l_all += (mw == -INFINITY) ? 0.f : lds_ml[1][w][r] * __builtin_amdgcn_exp2f(mw - mm);
    }
    float val = (lds_o[0][r][e] + lds_o[1][r][e]) + (lds_o[2][r][e] + lds_o[3][r][e]);
    val /= l_all;
    const int64_t row = (int64_t)b * p.n_q + h0 + r;
    if (p.num_splits == 1) {
      ((uint16_t*)p.out)[row * DV + e] = float_to_bf16_bits(val);
      if (e == 0 && p.lse_out) p.lse_out[row] = (mm + log2f(l_all)) * kLn2;
    } else {
      p.o_part[(row * p.num_splits + split) * DV + e] = val;
      if (e == 0) p.lse_part[row * p.num_splits + split] = mm + log2f(l_all);
    }
  }
}

template <int DQK, int DV, int RT>
hipError_t launch_ratio(const DecodeParams& p, bool paged, hipStream_t s) {
  dim3 block(kThreads);
  if (p.sk_cum) {  // equal slices of the ragged unit space, one per wavefront
    dim3 grid(p.sk_workers / kWaves);
    if (paged)
      launch_kernel(0, decode_mfma_kernel<DQK, DV, true, RT, true>, grid, block, 0, s, p);
    else
      launch_kernel(0, decode_mfma_kernel<DQK, DV, false, RT, true>, grid, block, 0, s, p);
  } else {
    dim3 grid(p.num_splits, p.n_k, p.B);
    if (paged)
      launch_kernel(0, decode_mfma_kernel<DQK, DV, true, RT, false>, grid, block, 0, s, p);
    else
      launch_kernel(0, decode_mfma_kernel<DQK, DV, false, RT, false>, grid, block, 0, s, p);
  }
  return hipGetLastError();
}

template <int DQK, int DV>
hipError_t launch_dims(const DecodeParams& p, bool paged, hipStream_t s) {
  switch (p.n_v / p.n_k) {
    case 1: return launch_ratio<DQK, DV, 1>(p, paged, s);
    case 2: return launch_ratio<DQK, DV, 2>(p, paged, s);
    case 4: return launch_ratio<DQK, DV, 4>(p, paged, s);
    case 8: return launch_ratio<DQK, DV, 8>(p, paged, s);
    default: return launch_ratio<DQK, DV, 0>(p, paged, s);
  }
}

}  // namespace

// bf16, K the coarser side, at most 16 query rows per K head, head widths 64 or 128.
int decode_streamk_max_batch() { return kStreamKMaxB; }

bool decode_mfma_supported(const DecodeParams& p, int dtype) {
  if (dtype != 1) return false;
  if (p.n_k > p.n_v || p.n_v % p.n_k != 0) return false;
  if (p.n_q / p.n_k > 16) return false;
  const bool dq = (p.d_qk == 64 || p.d_qk == 128), dv = (p.d_v == 64 || p.d_v == 128);
  if (!dq || !dv) return false;
  if (p.block_table && (p.page_size % 16 != 0)) return false;
  // every byte offset inside a 16-token block, V head offset included, must fit the 2 GiB window
  const int64_t R = p.n_v / p.n_k;
  if (16 * p.k_st * 2 + 512 >= (1ll << 31)) return false;
  if ((R * p.v_sh + 16 * p.v_st) * 2 + 512 >= (1ll << 31)) return false;
  return true;
}

hipError_t launch_decode_mfma(const DecodeParams& p, bool paged, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  if (p.d_qk == 128 && p.d_v == 128) return launch_dims<128, 128>(p, paged, s);
  if (p.d_qk == 64 && p.d_v == 64) return launch_dims<64, 64>(p, paged, s);
  if (p.d_qk == 64 && p.d_v == 128) return launch_dims<64, 128>(p, paged, s);
  return launch_dims<128, 64>(p, paged, s);
}

}  // namespace diffqkv
