// Causal prefill for bf16 on gfx950 matrix cores.
//
// The same attention as decode (section 2, "Formulation of DiffQKV Attention"), for a block of S_q
// query positions: query i attends to keys j <= i + (S_k - S_q) (K_t holds the tokens up to the
// current one).  Query head h reads K head floor(h n_k / n_q) and V head floor(h n_v / n_q) (the
// "idx" rule of section 3.2).  Prefill is a dense contraction, so both products run on
// v_mfma_f32_32x32x16_bf16.
//
// One workgroup = 4 wavefronts = 128 query rows of one (sequence, query head); each wavefront owns
// 32 rows.  K/V tiles of 64 tokens are staged through LDS, double-buffered: the global loads of
// tile i+1 are in flight while tile i is in the matrix cores.
//   S^T = K Q^T    A = K tile from LDS (row-major, padded rows), B = Q^T held in registers.
//                  In the result each lane column is one query row, so the online-softmax state
//                  and the accumulator rescale are lane-local (one cross-lane exchange per tile).
//   O^T = V^T P^T  B = P^T is the softmax output exactly as it sits in registers; A = V^T is read
//                  from an LDS copy of the tile that was transposed on the way in (each thread
//                  loads 4 tokens x 8 channels and transposes them in registers), stored with the
//                  token order that the score layout produces.
// Workgroups are ordered so that the query heads sharing a K head run side by side on one XCD
// (its L2 then serves their common K/V tiles), heaviest query tiles first.
#include <type_traits>

#include "kernels.h"

namespace diffqkv {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kBN = 64;  // tokens per K/V tile
constexpr int kXcds = 8;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// Transposed V tile in LDS: row = channel, 64 token positions (128 B, no padding).
// Position of token t (0..63): within each group of 16 tokens the quads are stored in the order
// 0, 2, 1, 3, so that the 8 tokens a lane needs for one k-step of the PV product (quads u and
// u + 2) form one 16-byte granule.  The granule index is XOR-swizzled with the channel so that
// both the 16-byte operand reads (32 consecutive channels) and the 8-byte transposed writes
// (channels 8 apart) spread over the banks.
__device__ __forceinline__ int vt_pos(int t) {
  const int u = (t >> 2) & 3;
  return (t & ~15) + 8 * (u & 1) + 4 * (u >> 1) + (t & 3);
}
__device__ __forceinline__ int vt_swizzle(int ch) { return (ch ^ (ch >> 3)) & 7; }

template <int D>
struct Smem {
  static constexpr int kKPitch = D + 8;  // bf16 elements per K row (16 B of padding)
  uint16_t k[2][kBN][kKPitch];
  uint16_t vt[2][D][kBN];
};

// QB: 32-row query blocks per wavefront (1 or 2).  With 2, every K / V^T operand read from LDS
// feeds two matrix instructions, halving LDS traffic per flop.
template <int D, int QB>
__global__ __launch_bounds__(kThreads, (QB == 1 ? 2 : 1)) void prefill_mfma_kernel(PrefillParams p, int n_qtiles,
                                                                                   int xcd_aware) {
  constexpr int KS = D / 16;  // k-steps of the score product (16 channels each)
  constexpr int CB = D / 32;  // 32-channel blocks of the output
  constexpr int kRowsPerWave = 32 * QB;
  constexpr int kBM = kWaves * kRowsPerWave;
  __shared__ Smem<D> sm;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, n = lane & 31;

  // ---- which (sequence, query head, query tile) ---------------------------------------------------
  const int g_k = p.n_q / p.n_k;
  int b, h, qtile;
  {
    const int x = blockIdx.x;
    if (xcd_aware) {
      // groups (sequence, K head) are dealt round-robin to the XCDs; inside an XCD's queue the query
      // heads of a group are adjacent, groups next, query tiles from the last (heaviest) down
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
  const int kh = (int)(((int64_t)h * p.n_k) / p.n_q), vh = (int)(((int64_t)h * p.n_v) / p.n_q);
  const int off = p.S_k - p.S_q;        // query i sees keys j <= i + off when causal
  const int q0 = qtile * kBM;           // first query row of the workgroup
  const int r0 = q0 + wave * kRowsPerWave;

  const uint16_t* qbase = (const uint16_t*)p.q + ((int64_t)b * p.n_q + h) * p.S_q * D;
  const uint16_t* kbase = (const uint16_t*)p.k + ((int64_t)b * p.n_k + kh) * p.S_k * D;
  const uint16_t* vbase = (const uint16_t*)p.v + ((int64_t)b * p.n_v + vh) * p.S_k * D;

  // tokens this workgroup / this wavefront can see
  int wg_limit = p.S_k, wave_limit = p.S_k;
  if (p.causal) {
    const int lastq = (q0 + kBM < p.S_q ? q0 + kBM : p.S_q) - 1;
    wg_limit = lastq + off + 1;
    int lastw = r0 + kRowsPerWave - 1;
    lastw = lastw < p.S_q ? lastw : p.S_q - 1;
    wave_limit = lastw + off + 1;
  }
  const int n_tiles = (wg_limit + kBN - 1) / kBN;

  // ---- Q^T as the B operand: lane (half, n) holds channels 16 ks + 8 half .. + 7 of its rows -----
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int row = r0 + 32 * qb + n;
    row = row < p.S_q ? row : p.S_q - 1;
    const uint16_t* qrow = qbase + (int64_t)row * D + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + ks * 16));
  }

  // ---- global -> register staging of one K/V tile --------------------------------------------------
  // K: thread t loads the 16-byte pieces (token, chunk) = ((i*256 + t) / (D/8), (i*256 + t) % (D/8))
  constexpr int KLD = kBN * (D / 8) / kThreads;
  // V: 16 token quads x D/8 channel chunks, one (quad, chunk) per thread (the first 128 threads at
  // D = 64).  Thread bits, low to high: chunk[2:0], quad-order bit 1, chunk[3] (D = 128 only),
  // quad-order bit 0, 16-token group: lanes that write the same channel rows in one instruction
  // then differ in the half-granule they write.
  constexpr int kChunkBits = (D == 128) ? 4 : 3;
  constexpr int kVItems = 16 * (D / 8);
  const bool v_active = tid < kVItems;
  const int v_c8 = (tid & 7) | ((kChunkBits == 4) ? ((tid >> 1) & 8) : 0);
  const int v_rest = tid >> (kChunkBits + 1);  // quad-order bit 0, then the 16-token group
  const int v_tq = ((v_rest >> 1) & 3) * 4 + ((v_rest & 1) | (((tid >> 3) & 1) << 1));
  u32x4 kst[KLD];
  u32x4 vst[4];
  auto load_tile = [&](int t0) {
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
      const int piece = i * kThreads + tid;
      int tok = t0 + piece / (D / 8);
      tok = tok < p.S_k ? tok : p.S_k - 1;
      kst[i] = *(const u32x4*)(kbase + (int64_t)tok * D + (piece % (D / 8)) * 8);
    }
    if (v_active) {
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        int tok = t0 + 4 * v_tq + x;
        tok = tok < p.S_k ? tok : p.S_k - 1;
        vst[x] = *(const u32x4*)(vbase + (int64_t)tok * D + v_c8 * 8);
      }
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < KLD; ++i) {
      const int piece = i * kThreads + tid;
      *(u32x4*)&sm.k[buf][piece / (D / 8)][(piece % (D / 8)) * 8] = kst[i];
    }
    if (v_active) {
      const int pos = vt_pos(4 * v_tq);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // channel e of the chunk: word e/2, low or high half, from the 4 tokens
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x2 w;
        w[0] = __builtin_amdgcn_perm(vst[1][e >> 1], vst[0][e >> 1], sel);
        w[1] = __builtin_amdgcn_perm(vst[3][e >> 1], vst[2][e >> 1], sel);
        const int ch = v_c8 * 8 + e;
        *(u32x2*)&sm.vt[buf][ch][(((pos >> 3) ^ vt_swizzle(ch)) << 3) + (pos & 7)] = w;
      }
    }
  };

  f32x16 acc[QB][CB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[qb][cb][r] = 0.f;
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
  }

  load_tile(0);
  store_tile(0);
  __syncthreads();

  // One tile step.  MASKED is a compile-time flag: tiles strictly below the diagonal of this
  // wavefront's rows (the vast majority) run straight-line code with no per-element selects; the
  // few tiles on or past the diagonal take the masked variant (or skip the arithmetic entirely and
  // only help with staging).  Every step has exactly one barrier, so wavefronts of a workgroup may
  // switch variants at different tiles.
  auto tile_step = [&](int it, auto masked_tag) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int t0 = it * kBN, buf = it & 1;
    const bool more = it + 1 < n_tiles;
    if (more) load_tile(t0 + kBN);

    if (!MASKED || t0 < wave_limit) {
      // ---- S^T = K Q^T: two 32-token blocks x QB query blocks; each K operand feeds QB products --
      f32x16 s[QB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[qb][blk][r] = 0.f;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)&sm.k[buf][32 * blk + n][16 * ks + 8 * half]);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            s[qb][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[qb][blk], 0, 0, 0);
        }
      // ---- online softmax; register r of block blk: token t0 + 32 blk + 8 (r/4) + 4 half + r%4 ---
      uint32_t pw[QB][2][8];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int row_limit = p.causal ? r0 + 32 * qb + n + off : p.S_k - 1;  // last visible token
        float m_tile = -INFINITY;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float v = s[qb][blk][r];
            if (MASKED) {
              const int tok = t0 + 32 * blk + 8 * (r >> 2) + 4 * half + (r & 3);
              v = (tok <= row_limit && tok < p.S_k) ? v : -INFINITY;
              s[qb][blk][r] = v;
            }
            m_tile = fmaxf(m_tile, v);
          }
        m_tile = fmaxf(m_tile, __shfl_xor(m_tile, 32, 64));
        // scores stay unscaled; the scale (> 0) is folded into the exponent: 2^(c s - c m)
        float m_new = fmaxf(m_run[qb], m_tile * p.scale_log2);
        // a row with nothing visible yet (only in a masked tile of a later query block) keeps a
        // finite reference so that exp2(-inf - m) stays 0 instead of NaN
        if (MASKED) m_new = (m_new == -INFINITY) ? 0.f : m_new;
        const float fac = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
        m_run[qb] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i], p.scale_log2, -m_new));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i + 1], p.scale_log2, -m_new));
            pw[qb][blk][i] = pack_bf16x2(p0, p1);
            psum += p0 + p1;
          }
        l_run[qb] = l_run[qb] * fac + psum;
        // the accumulator rescale is skipped when no row of the block raised its maximum
        if (__builtin_amdgcn_ballot_w64(fac != 1.0f)) {
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) acc[qb][cb] *= fac;
        }
      }
      // ---- O^T += V^T P^T: k-step kq covers tokens 16 kq .. 16 kq + 15 of the tile -----------------
#pragma unroll
      for (int kq = 0; kq < 4; ++kq) {
        const int blk = kq >> 1, sh = (kq & 1) * 4;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          const int ch = 32 * cb + n;
          const bf16x8 a = __builtin_bit_cast(
              bf16x8, *(const u32x4*)&sm.vt[buf][ch][((2 * kq + half) ^ vt_swizzle(ch)) << 3]);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            const u32x4 pb = {pw[qb][blk][sh], pw[qb][blk][sh + 1], pw[qb][blk][sh + 2], pw[qb][blk][sh + 3]};
            acc[qb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pb), acc[qb][cb], 0, 0, 0);
          }
        }
      }
    }
    if (more) store_tile(buf ^ 1);
    __syncthreads();
  };
  // tiles wholly visible to every row of this wavefront need no mask
  int n_plain = p.S_k / kBN;
  if (p.causal) {
    const int vis = (r0 + off + 1) / kBN;  // tiles entirely at or before the first row's limit
    n_plain = vis < n_plain ? vis : n_plain;
  }
  n_plain = n_plain < n_tiles ? n_plain : n_tiles;
  n_plain = n_plain < 0 ? 0 : n_plain;
  int it = 0;
  for (; it < n_plain; ++it) tile_step(it, std::false_type{});
  for (; it < n_tiles; ++it) tile_step(it, std::true_type{});

  // ---- write this wavefront's rows: lane (half, n), acc[qb][cb][r] = row 32 qb + n, channel
  //      32 cb + 8 (r/4) + 4 half + r%4.  Both halves hold the full row sum after the exchange.
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int my_row = r0 + 32 * qb + n;
    const float l = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
    if (my_row < p.S_q) {
      const float inv = 1.f / l;
      uint16_t* orow = (uint16_t*)p.out + (((int64_t)b * p.n_q + h) * p.S_q + my_row) * D;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16x2(acc[qb][cb][4 * q4] * inv, acc[qb][cb][4 * q4 + 1] * inv);
          w[1] = pack_bf16x2(acc[qb][cb][4 * q4 + 2] * inv, acc[qb][cb][4 * q4 + 3] * inv);
          *(u32x2*)(orow + 32 * cb + 8 * q4 + 4 * half) = w;
        }
      if (half == 0 && p.lse_out)
        p.lse_out[((int64_t)b * p.n_q + h) * p.S_q + my_row] = (m_run[qb] + log2f(l)) * kLn2;
    }
  }
}

}  // namespace

// bf16, equal head widths of 64 or 128.
bool prefill_mfma_supported(const PrefillParams& p, int dtype) {
  if (dtype != 1) return false;
  if (p.d_qk != p.d_v) return false;
  return p.d_qk == 128 || p.d_qk == 64;
}

namespace {
int g_prefill_query_blocks = 1;  // 32-row query blocks per wavefront
template <int D, int QB>
hipError_t launch_qb(const PrefillParams& p, hipStream_t s) {
  constexpr int kBM = kWaves * 32 * QB;
  const int n_qtiles = (p.S_q + kBM - 1) / kBM;
  const int64_t n_wg = (int64_t)n_qtiles * p.n_q * p.B;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  const int xcd_aware = ((p.B * p.n_k) % kXcds == 0) ? 1 : 0;
  prefill_mfma_kernel<D, QB><<<dim3((unsigned)n_wg), dim3(kThreads), 0, s>>>(p, n_qtiles, xcd_aware);
  return hipGetLastError();
}
}  // namespace

void set_prefill_query_blocks(int qb) { g_prefill_query_blocks = (qb == 2) ? 2 : 1; }

hipError_t launch_prefill_mfma(const PrefillParams& p, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  const bool two = g_prefill_query_blocks == 2;
  if (p.d_qk == 128) return two ? launch_qb<128, 2>(p, s) : launch_qb<128, 1>(p, s);
  return two ? launch_qb<64, 2>(p, s) : launch_qb<64, 1>(p, s);
}

}  // namespace diffqkv
