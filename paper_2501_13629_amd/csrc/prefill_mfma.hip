// Causal prefill for bf16 on gfx950 matrix cores, 32 query rows per wavefront.
//
// The same attention as decode (section 2, "Formulation of DiffQKV Attention"), for a block of S_q
// query positions: query i attends to keys j <= i + (S_k - S_q) (K_t holds the tokens up to the
// current one).  Query head h reads K head floor(h n_k / n_q) and V head floor(h n_v / n_q) (the
// "idx" rule of section 3.2).  Prefill is a dense contraction, so both products run on
// v_mfma_f32_32x32x16_bf16.
//
// One workgroup = 8 (or 4) wavefronts = 256 (128) query rows of one (sequence, query head); each
// wavefront owns 32 rows, two wavefronts share a SIMD.  K/V tiles of 64 tokens are staged through LDS,
// double-buffered: the global loads of tile i+1 are in flight while tile i is in the matrix cores.
//   S^T = K Q^T    A = K tile from LDS (row-major, padded rows), B = Q^T held in registers.
//                  In the result each lane column is one query row, so the online-softmax state
//                  and the accumulator rescale are lane-local.
//   O^T = V^T P^T  B = P^T is the softmax output exactly as it sits in registers; A = V^T is read
//                  from an LDS copy of the tile that was transposed on the way in (each thread
//                  loads 4 tokens x 8 channels and transposes them in registers), stored with the
//                  token order that the score layout produces.
// Workgroups are ordered so that the query heads sharing a K head run side by side on one XCD
// (its L2 then serves their common K/V tiles), heaviest query tiles first.
// This kernel serves the head widths (64, 64), (64, 128) and, on request, (128, 128); for (128, 128)
// the 64-rows-per-wavefront kernel of prefill_mfma64.hip is the default.
#include "prefill_tile.h"

namespace diffqkv {

namespace {

using namespace prefill_tile;

// NW wavefronts (4 or 8) of QB x 32 query rows each per workgroup (QB = 1 in every instantiation; two
// row blocks per wavefront need the whole register file and have a kernel of their own).  With 8
// wavefronts the K/V tile is staged once for 256 query rows, and half of the wavefronts stage K
// while the other half transpose V.
template <int DQK, int DV, int NW, int QB>
__global__ __launch_bounds__(NW * 64, QB == 2 ? 1 : 2) void prefill_mfma_kernel(PrefillParams p, int n_qtiles,
                                                                               int xcd_aware) {
  constexpr int KS = DQK / 16;  // k-steps of the score product (16 channels each)
  constexpr int CB = DV / 32;   // 32-channel blocks of the output
  constexpr int kThreads = NW * 64;
  constexpr int kWaveRows = 32 * QB;
  constexpr int kBM = NW * kWaveRows;
  __shared__ Smem<DQK, DV> sm;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, n = lane & 31;

  // ---- which (sequence, query head, query tile) ---------------------------------------------------
  int b, h, qtile;
  locate_block(p, blockIdx.x, n_qtiles, xcd_aware, b, h, qtile);
  const int kh = (int)(((int64_t)h * p.n_k) / p.n_q), vh = (int)(((int64_t)h * p.n_v) / p.n_q);
  const int off = p.S_k - p.S_q;        // query i sees keys j <= i + off when causal
  const int q0 = qtile * kBM;           // first query row of the workgroup
  const int r0 = q0 + wave * kWaveRows;  // first query row of this wavefront

  const uint16_t* qbase = (const uint16_t*)p.q + ((int64_t)b * p.n_q + h) * p.S_q * DQK;
  const rsrc_t k_rsrc = make_rsrc((const uint16_t*)p.k + ((int64_t)b * p.n_k + kh) * p.S_k * DQK, p.S_k * DQK * 2);
  const rsrc_t v_rsrc = make_rsrc((const uint16_t*)p.v + ((int64_t)b * p.n_v + vh) * p.S_k * DV, p.S_k * DV * 2);

  // tokens this workgroup / this wavefront can see
  int wg_limit = p.S_k, wave_limit = p.S_k;
  if (p.causal) {
    const int lastq = (q0 + kBM < p.S_q ? q0 + kBM : p.S_q) - 1;
    wg_limit = lastq + off + 1;
    int lastw = r0 + kWaveRows - 1;
    lastw = lastw < p.S_q ? lastw : p.S_q - 1;
    wave_limit = lastw + off + 1;
  }
  const int n_tiles = (wg_limit + kBN - 1) / kBN;

  // ---- Q^T as the B operand: lane (half, n) holds channels 16 ks + 8 half .. + 7 of its row ------
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    int row = r0 + 32 * qb + n;
    row = row < p.S_q ? row : p.S_q - 1;
    const uint16_t* qrow = qbase + (int64_t)row * DQK + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + ks * 16));
  }

  // ---- global -> register -> LDS staging of one K/V tile ---------------------------------------------
  // K tile = 64 rows x d_qk channels = one contiguous run of 16-byte pieces; K thread kt takes
  // pieces kt, kt + 256, ...  V tile: 16 token quads x d_v/8 channel chunks, one (quad, chunk) per V
  // thread: it loads 4 tokens x 8 channels and transposes them in registers.  V thread bits, low to
  // high: chunk[2:0], quad-order bit 1, chunk[3] (d_v = 128 only), quad-order bit 0, 16-token group --
  // lanes that write the same channel rows in one instruction differ in the half-granule they write.
  // With 8 wavefronts the first four are the V threads and the last four the K threads.
  constexpr int kKThreads = 256;
  constexpr int KLD = kBN * (DQK / 8) / kKThreads;
  constexpr int kChunkBits = (DV == 128) ? 4 : 3;
  constexpr int kVItems = 16 * (DV / 8);
  // both roles are whole wavefronts, so the branches below are scalar
  const bool k_role = (NW == 4) || wave >= 4;
  const bool v_role = wave < kVItems / 64;
  const int kt = tid & 255;
  const int v_c8 = (tid & 7) | ((kChunkBits == 4) ? ((tid >> 1) & 8) : 0);
  const int v_rest = tid >> (kChunkBits + 1);  // quad-order bit 0, then the 16-token group
  const int v_tq = ((v_rest >> 1) & 3) * 4 + ((v_rest & 1) | (((tid >> 3) & 1) << 1));
  const int v_voff = (4 * v_tq) * (DV * 2) + v_c8 * 16;
  constexpr int kStage = (NW == 4) ? 4 + KLD : 4;  // with 8 wavefronts the two roles share registers
  u32x4 st[kStage];
  u32x4* const kst = st + ((NW == 4) ? 4 : 0);
  auto load_tile = [&](int t0) {
    // (the tile start is part of the per-lane offset, which is what the bounds check that turns rows
    //  past the end of the head into zeros is documented to cover)
    // with 8 wavefronts the roles are exclusive (if / else), so sharing the registers is safe
    if (k_role) {
#pragma unroll
      for (int i = 0; i < KLD; ++i)
        kst[i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, (i * kKThreads + kt) * 16 + t0 * (DQK * 2), 0, 0);
    }
    if ((NW == 4 || !k_role) && v_role) {
#pragma unroll
      for (int x = 0; x < 4; ++x)
        st[x] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, v_voff + x * (DV * 2) + t0 * (DV * 2), 0, 0);
    }
  };
  auto store_tile = [&](int buf) {
    if (k_role) {
#pragma unroll
      for (int i = 0; i < KLD; ++i) {
        const int piece = i * kKThreads + kt;
        *(u32x4*)&sm.k[buf][piece / (DQK / 8)][(piece % (DQK / 8)) * 8] = kst[i];
      }
    }
    if ((NW == 4 || !k_role) && v_role) {
      const int pos = vt_pos(4 * v_tq);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // channel e of the chunk: word e/2, low or high half, from the 4 tokens
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        u32x2 w;
        w[0] = __builtin_amdgcn_perm(st[1][e >> 1], st[0][e >> 1], sel);
        w[1] = __builtin_amdgcn_perm(st[3][e >> 1], st[2][e >> 1], sel);
        const int ch = v_c8 * 8 + e;
        *(u32x2*)&sm.vt[buf][ch][(((pos >> 3) ^ vt_swizzle(ch)) << 3) + (pos & 7)] = w;
      }
    }
  };

  f32x16 acc[QB][CB];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[qb][cb][r] = 0.f;
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
  }

  load_tile(0);
  store_tile(0);
  // Pin the arrival of Q before the loop: otherwise the compiler, not knowing whether these loads
  // are still in flight when the loop is entered, makes every iteration wait on the vector-memory
  // counter -- and with it on the next tile's staging loads -- before each matrix instruction.
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qf[qb][ks]));
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
      // Each 32-token block is one online-softmax step of its own:
      //     S^T(blk) = K Q^T  ->  softmax(blk)  ->  O^T += V^T P^T(blk)
      // and the two blocks are written interleaved -- the score product of block 1 between the
      // softmax pieces of block 0, the softmax of block 1 between the output products of block 0 --
      // so that the vector ALU (exponentials) and the matrix cores work at the same time.
      int row_limit[QB];  // last visible token of this lane's row in each row block
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) row_limit[qb] = p.causal ? r0 + 32 * qb + n + off : p.S_k - 1;
      f32x16 s[QB][2];
      uint32_t pw[QB][2][8];
      // The operand fragments of the tile, in the order the matrix instructions consume them:
      //   K rows of block 0 (KS k-steps), K rows of block 1, V^T of block 0 (2 token halves x CB
      //   channel blocks), V^T of block 1.
      // They pass through a ring of kRing register slots: the LDS read of fragment f + kRing is issued
      // as soon as fragment f has been consumed, so LDS latency stays off the matrix pipeline.
      constexpr int kRing = 8;
      constexpr int kFrags = 2 * KS + 4 * CB;
      u32x4 fr[kRing];
      auto fetch = [&](auto fc) {
        constexpr int f = decltype(fc)::value;
        if constexpr (f < 2 * KS) {
          constexpr int blk = f / KS, ks = f % KS;
          fr[f % kRing] = *(const u32x4*)&sm.k[buf][32 * blk + n][16 * ks + 8 * half];
        } else {
          constexpr int j = f - 2 * KS, kq = j / CB, cb = j % CB;  // kq: 16-token step of the tile
          const int ch = 32 * cb + n;
          fr[f % kRing] = *(const u32x4*)&sm.vt[buf][ch][((2 * kq + half) ^ vt_swizzle(ch)) << 3];
        }
      };
      // softmax reference for one block; register r: token t0 + 32 blk + 8 (r/4) + 4 half + r%4.
      // Scores stay unscaled; the scale (> 0) is folded into the exponent: 2^(c s - m_ref).  The
      // reference m_ref only has to keep the exponentials in range, it need not be the exact
      // running maximum: it is raised (and the accumulators rescaled) only when some row's maximum
      // exceeds it by more than kSlack, so most blocks skip the rescale.  Weights are then at most
      // 2^kSlack, well inside bf16 / fp32 range; the final division by the row sum removes it.
      // Each lane first tests the 16 tokens it holds; the exchange with the lane that holds the
      // row's other 16 happens only when some lane of the wavefront needs a higher reference.
      auto reference = [&](int qb, int blk) {
        float m_blk = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = s[qb][blk][r];
          if (MASKED) {
            const int tok = t0 + 32 * blk + 8 * (r >> 2) + 4 * half + (r & 3);
            v = (tok <= row_limit[qb] && tok < p.S_k) ? v : -INFINITY;
            s[qb][blk][r] = v;
          }
          m_blk = fmaxf(m_blk, v);
        }
        float fac = 1.f;
        if (__builtin_amdgcn_ballot_w64(m_blk * p.scale_log2 > m_run[qb] + kSlack)) {
          m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32, 64));
          const float m_cand = m_blk * p.scale_log2;
          const float m_new = (m_cand > m_run[qb] + kSlack) ? m_cand : m_run[qb];
          fac = __builtin_amdgcn_exp2f(m_run[qb] - m_new);  // first block: exp2(-inf) = 0
          m_run[qb] = m_new;
          l_run[qb] *= fac;
        }
        return fac;  // the caller rescales the accumulators once they hold everything older
      };
      auto rescale = [&](int qb, float fac) {
        if (__builtin_amdgcn_ballot_w64(fac != 1.f)) {
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) acc[qb][cb] *= fac;
        }
      };
      auto weights_step = [&](int blk, int w) {  // w in [0, 8 QB): two of a row block's 16 weights
        const int qb = w / 8, i = w % 8;
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i], p.scale_log2, -m_run[qb]));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i + 1], p.scale_log2, -m_run[qb]));
        pw[qb][blk][i] = pack_bf16x2(p0, p1);
        l_run[qb] += p0 + p1;
      };
      constexpr int W = 8 * QB;  // weight pairs per block
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[qb][blk][r] = 0.f;
      static_for<0, kRing>(fetch);
      __builtin_amdgcn_sched_barrier(0);  // keep the first reads together, ahead of the matrix instructions
      float fac1[QB];
      static_for<0, kFrags>([&](auto fc) {
        constexpr int f = decltype(fc)::value;
        const bf16x8 a = __builtin_bit_cast(bf16x8, fr[f % kRing]);
        if constexpr (f < 2 * KS) {  // score product: block f / KS, k-step f % KS
          constexpr int blk = f / KS, ks = f % KS;
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            s[qb][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[qb][blk], 0, 0, 0);
        } else {           // output product: block blk, 16-token half kh2, channel block cb
          constexpr int j = f - 2 * KS, blk = j / (2 * CB), kh2 = (j / CB) % 2, cb = j % CB, sh = kh2 * 4;
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            const u32x4 pb = {pw[qb][blk][sh], pw[qb][blk][sh + 1], pw[qb][blk][sh + 2], pw[qb][blk][sh + 3]};
            acc[qb][cb] =
                __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pb), acc[qb][cb], 0, 0, 0);
          }
        }
        if constexpr (f + kRing < kFrags) fetch(std::integral_constant<int, f + kRing>{});
        // the softmax pieces, placed between the matrix instructions they can overlap with
        if constexpr (f == KS - 1) {
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) rescale(qb, reference(qb, 0));
        } else if constexpr (f >= KS && f < 2 * KS) {  // weights of block 0 under the score product of block 1
          constexpr int i = f - KS;
#pragma unroll
          for (int w = i * W / KS; w < (i + 1) * W / KS; ++w) weights_step(0, w);
          if constexpr (f == 2 * KS - 1) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) fac1[qb] = reference(qb, 1);
          }
        } else if constexpr (f >= 2 * KS && f < 2 * KS + 2 * CB) {  // weights of block 1 under block 0's output product
          constexpr int i = f - 2 * KS;
#pragma unroll
          for (int w = i * W / (2 * CB); w < (i + 1) * W / (2 * CB); ++w) weights_step(1, w);
          // block 0's weights were taken against the older reference: apply the new one after them
          if constexpr (f == 2 * KS + 2 * CB - 1) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) rescale(qb, fac1[qb]);
          }
        }
      });
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
      uint16_t* orow = (uint16_t*)p.out + (((int64_t)b * p.n_q + h) * p.S_q + my_row) * DV;
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

// bf16, head widths of 64 or 128 (d_qk <= d_v), and a K/V head -- plus the tiles the staging loads run
// past its end -- inside the 2 GiB window of 32-bit buffer offsets.
bool prefill_mfma_supported(const PrefillParams& p, int dtype) {
  if (dtype != 1) return false;
  const bool ok = (p.d_qk == 128 && p.d_v == 128) || (p.d_qk == 64 && p.d_v == 64) || (p.d_qk == 64 && p.d_v == 128);
  if (!ok) return false;
  return (int64_t)(p.S_k + 2 * kBN) * p.d_v * 2 < (1ll << 31);
}

namespace {
template <int DQK, int DV, int NW, int QB>
hipError_t launch_nw(const PrefillParams& p, hipStream_t s) {
  constexpr int kBM = NW * 32 * QB;
  const int n_qtiles = (p.S_q + kBM - 1) / kBM;
  const int64_t n_wg = (int64_t)n_qtiles * p.n_q * p.B;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  const int xcd_aware = ((p.B * p.n_k) % kXcds == 0) ? 1 : 0;
  launch_kernel(0, prefill_mfma_kernel<DQK, DV, NW, QB>, dim3((unsigned)n_wg), dim3(NW * 64), 0, s, p, n_qtiles, xcd_aware);
  return hipGetLastError();
}
// variant: 0 choose; 8 / 4 wavefronts of 32 rows; 2 = the 64-rows-per-wavefront kernel where supported
template <int DQK, int DV>
hipError_t launch_variant(const PrefillParams& p, int variant, hipStream_t s) {
  if ((variant == 0 || variant == 2) && prefill_mfma64_supported(p, 1)) return launch_prefill_mfma64(p, s);
  if (variant == 4) return launch_nw<DQK, DV, 4, 1>(p, s);
  return launch_nw<DQK, DV, 8, 1>(p, s);
}
}  // namespace

hipError_t launch_prefill_mfma(const PrefillParams& p, int variant, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  if (variant != 2 && variant != 4 && variant != 8) variant = 0;
  if (p.d_qk == 128) return launch_variant<128, 128>(p, variant, s);
  if (p.d_v == 128) return launch_variant<64, 128>(p, variant, s);
  return launch_variant<64, 64>(p, variant, s);
}

}  // namespace diffqkv
