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

constexpr int kBN = 64;  // tokens per K/V tile
constexpr int kXcds = 8;
constexpr float kSlack = 8.f;  // log2 units a row maximum may exceed the softmax reference

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 x = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
}

// Transposed V tile in LDS: row = channel, 64 token positions (128 B, no padding).
// Position of token t (0..63): within each group of 16 tokens the quads are stored in the order
// 0, 2, 1, 3, so that the 8 tokens a lane needs for one k-step of the PV product (quads u and
// u + 2) form one 16-byte granule.  The granule index is XOR-swizzled with the channel so that
// both the 16-byte operand reads (32 consecutive channels) and the 8-byte transposed writes
// (channels 8 apart) spread over the banks (measured: no bank conflicts).
__device__ __forceinline__ int vt_pos(int t) {
  const int u = (t >> 2) & 3;
  return (t & ~15) + 8 * (u & 1) + 4 * (u >> 1) + (t & 3);
}
__device__ __forceinline__ int vt_swizzle(int ch) { return (ch ^ (ch >> 3)) & 7; }

template <int DQK, int DV>
struct Smem {
  static constexpr int kKPitch = DQK + 8;  // bf16 elements per K row (16 B of padding)
  uint16_t k[2][kBN][kKPitch];
  uint16_t vt[2][DV][kBN];
};

// Raw buffer resource over `bytes` bytes: loads take a scalar byte offset (the tile start) on top
// of a loop-invariant per-lane offset, and rows past the end of the tensor read as zero.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// NW wavefronts of 32 query rows each per workgroup (4 or 8).  With 8 the K/V tile is staged once
// for 256 query rows, and half of the wavefronts stage K while the other half transpose V.
template <int DQK, int DV, int NW>
__global__ __launch_bounds__(NW * 64, 2) void prefill_mfma_kernel(PrefillParams p, int n_qtiles, int xcd_aware) {
  constexpr int KS = DQK / 16;  // k-steps of the score product (16 channels each)
  constexpr int CB = DV / 32;   // 32-channel blocks of the output
  constexpr int kThreads = NW * 64;
  constexpr int kBM = NW * 32;
  __shared__ Smem<DQK, DV> sm;

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
  const int r0 = q0 + wave * 32;        // first query row of this wavefront

  const uint16_t* qbase = (const uint16_t*)p.q + ((int64_t)b * p.n_q + h) * p.S_q * DQK;
  const rsrc_t k_rsrc = make_rsrc((const uint16_t*)p.k + ((int64_t)b * p.n_k + kh) * p.S_k * DQK, p.S_k * DQK * 2);
  const rsrc_t v_rsrc = make_rsrc((const uint16_t*)p.v + ((int64_t)b * p.n_v + vh) * p.S_k * DV, p.S_k * DV * 2);

  // tokens this workgroup / this wavefront can see
  int wg_limit = p.S_k, wave_limit = p.S_k;
  if (p.causal) {
    const int lastq = (q0 + kBM < p.S_q ? q0 + kBM : p.S_q) - 1;
    wg_limit = lastq + off + 1;
    int lastw = r0 + 31;
    lastw = lastw < p.S_q ? lastw : p.S_q - 1;
    wave_limit = lastw + off + 1;
  }
  const int n_tiles = (wg_limit + kBN - 1) / kBN;

  // ---- Q^T as the B operand: lane (half, n) holds channels 16 ks + 8 half .. + 7 of its row ------
  bf16x8 qf[KS];
  {
    int row = r0 + n;
    row = row < p.S_q ? row : p.S_q - 1;
    const uint16_t* qrow = qbase + (int64_t)row * DQK + half * 8;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qrow + ks * 16));
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
    // tile starts, wavefront-uniform: they travel in scalar registers
    // with 8 wavefronts the roles are exclusive (if / else), so sharing the registers is safe
    if (k_role) {
#pragma unroll
      for (int i = 0; i < KLD; ++i)
        kst[i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, (i * kKThreads + kt) * 16, t0 * (DQK * 2), 0);
    }
    if ((NW == 4 || !k_role) && v_role) {
#pragma unroll
      for (int x = 0; x < 4; ++x)
        st[x] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, v_voff + x * (DV * 2), t0 * (DV * 2), 0);
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

  f32x16 acc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[cb][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  load_tile(0);
  store_tile(0);
  // Pin the arrival of Q before the loop: otherwise the compiler, not knowing whether these loads
  // are still in flight when the loop is entered, makes every iteration wait on the vector-memory
  // counter -- and with it on the next tile's staging loads -- before each matrix instruction.
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) asm volatile("" ::"v"(qf[ks]));
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
      const int row_limit = p.causal ? r0 + n + off : p.S_k - 1;  // last visible token of this row
      f32x16 s[2];
      uint32_t pw[2][8];
      auto score_step = [&](int blk, int ks) {
        const bf16x8 a = __builtin_bit_cast(bf16x8, *(const u32x4*)&sm.k[buf][32 * blk + n][16 * ks + 8 * half]);
        s[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[ks], s[blk], 0, 0, 0);
      };
      // softmax reference for one block; register r: token t0 + 32 blk + 8 (r/4) + 4 half + r%4.
      // Scores stay unscaled; the scale (> 0) is folded into the exponent: 2^(c s - m_ref).  The
      // reference m_ref only has to keep the exponentials in range, it need not be the exact
      // running maximum: it is raised (and the accumulators rescaled) only when some row's maximum
      // exceeds it by more than kSlack, so most blocks skip the rescale.  Weights are then at most
      // 2^kSlack, well inside bf16 / fp32 range; the final division by the row sum removes it.
      auto reference = [&](int blk) {
        float m_blk = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = s[blk][r];
          if (MASKED) {
            const int tok = t0 + 32 * blk + 8 * (r >> 2) + 4 * half + (r & 3);
            v = (tok <= row_limit && tok < p.S_k) ? v : -INFINITY;
            s[blk][r] = v;
          }
          m_blk = fmaxf(m_blk, v);
        }
        m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32, 64));
        const float m_cand = m_blk * p.scale_log2;
        const bool raise = m_cand > m_run + kSlack;
        float fac = 1.f;
        if (__builtin_amdgcn_ballot_w64(raise)) {
          const float m_new = raise ? m_cand : m_run;
          fac = __builtin_amdgcn_exp2f(m_run - m_new);  // first block: exp2(-inf) = 0
          m_run = m_new;
          l_run *= fac;
        }
        return fac;  // the caller rescales the accumulators once they hold everything older
      };
      auto rescale = [&](float fac) {
        if (__builtin_amdgcn_ballot_w64(fac != 1.f)) {
#pragma unroll
          for (int cb = 0; cb < CB; ++cb) acc[cb] *= fac;
        }
      };
      auto weights_step = [&](int blk, int i) {  // two of the block's 16 weights
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[blk][2 * i], p.scale_log2, -m_run));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[blk][2 * i + 1], p.scale_log2, -m_run));
        pw[blk][i] = pack_bf16x2(p0, p1);
        l_run += p0 + p1;
      };
      auto output_step = [&](int blk, int kh2, int cb) {  // k-step kh2 (16 tokens) of block blk
        const int kq = 2 * blk + kh2, sh = kh2 * 4;
        const u32x4 pb = {pw[blk][sh], pw[blk][sh + 1], pw[blk][sh + 2], pw[blk][sh + 3]};
        const int ch = 32 * cb + n;
        const bf16x8 a = __builtin_bit_cast(
            bf16x8, *(const u32x4*)&sm.vt[buf][ch][((2 * kq + half) ^ vt_swizzle(ch)) << 3]);
        acc[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, pb), acc[cb], 0, 0, 0);
      };
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[blk][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) score_step(0, ks);
      rescale(reference(0));
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        score_step(1, ks);
        if (ks * 8 / KS != (ks + 1) * 8 / KS || KS == 8) {
#pragma unroll
          for (int i = ks * 8 / KS; i < (ks + 1) * 8 / KS; ++i) weights_step(0, i);
        }
      }
      const float fac1 = reference(1);
#pragma unroll
      for (int j = 0; j < 2 * CB; ++j) {
        output_step(0, j / CB, j % CB);
#pragma unroll
        for (int i = j * 8 / (2 * CB); i < (j + 1) * 8 / (2 * CB); ++i) weights_step(1, i);
      }
      rescale(fac1);  // block 0's weights were taken against the older reference: apply it after them
#pragma unroll
      for (int j = 0; j < 2 * CB; ++j) output_step(1, j / CB, j % CB);
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

  // ---- write this wavefront's rows: lane (half, n), acc[cb][r] = row n, channel
  //      32 cb + 8 (r/4) + 4 half + r%4.  Both halves hold the full row sum after the exchange.
  const int my_row = r0 + n;
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  if (my_row < p.S_q) {
    const float inv = 1.f / l;
    uint16_t* orow = (uint16_t*)p.out + (((int64_t)b * p.n_q + h) * p.S_q + my_row) * DV;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w;
        w[0] = pack_bf16x2(acc[cb][4 * q4] * inv, acc[cb][4 * q4 + 1] * inv);
        w[1] = pack_bf16x2(acc[cb][4 * q4 + 2] * inv, acc[cb][4 * q4 + 3] * inv);
        *(u32x2*)(orow + 32 * cb + 8 * q4 + 4 * half) = w;
      }
    if (half == 0 && p.lse_out)
      p.lse_out[((int64_t)b * p.n_q + h) * p.S_q + my_row] = (m_run + log2f(l)) * kLn2;
  }
}

}  // namespace

// bf16, head widths of 64 or 128 (d_qk <= d_v), and a K/V head no longer than the 2 GiB buffer window.
bool prefill_mfma_supported(const PrefillParams& p, int dtype) {
  if (dtype != 1) return false;
  const bool ok = (p.d_qk == 128 && p.d_v == 128) || (p.d_qk == 64 && p.d_v == 64) || (p.d_qk == 64 && p.d_v == 128);
  if (!ok) return false;
  return (int64_t)p.S_k * p.d_v * 2 < (1ll << 31);
}

namespace {
int g_prefill_waves = 8;
template <int DQK, int DV, int NW>
hipError_t launch_nw(const PrefillParams& p, hipStream_t s) {
  constexpr int kBM = NW * 32;
  const int n_qtiles = (p.S_q + kBM - 1) / kBM;
  const int64_t n_wg = (int64_t)n_qtiles * p.n_q * p.B;
  if (n_wg > 0x7fffffff) return hipErrorInvalidValue;
  const int xcd_aware = ((p.B * p.n_k) % kXcds == 0) ? 1 : 0;
  prefill_mfma_kernel<DQK, DV, NW><<<dim3((unsigned)n_wg), dim3(NW * 64), 0, s>>>(p, n_qtiles, xcd_aware);
  return hipGetLastError();
}
}  // namespace

void set_prefill_waves(int nw) { g_prefill_waves = (nw == 4) ? 4 : 8; }

hipError_t launch_prefill_mfma(const PrefillParams& p, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  const bool eight = g_prefill_waves == 8;
  if (p.d_qk == 128) return eight ? launch_nw<128, 128, 8>(p, s) : launch_nw<128, 128, 4>(p, s);
  if (p.d_v == 128) return eight ? launch_nw<64, 128, 8>(p, s) : launch_nw<64, 128, 4>(p, s);
  return eight ? launch_nw<64, 64, 8>(p, s) : launch_nw<64, 64, 4>(p, s);
}

}  // namespace diffqkv
