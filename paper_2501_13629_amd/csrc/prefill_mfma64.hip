// Causal prefill for bf16 on gfx950 matrix cores, 64 query rows per wavefront.
//
// Same attention and same tile layout in LDS as prefill_mfma.hip (section 2, "Formulation of DiffQKV
// Attention"; head map of the "idx" rule, section 3.2), organised for the other end of the register
// trade-off: one workgroup = 4 wavefronts = 256 query rows, one wavefront per SIMD with the whole
// register file.  Each wavefront owns two blocks of 32 rows, so every K or V^T fragment read from LDS
// feeds two matrix instructions -- half the LDS traffic per flop -- and the 64 x d_v output
// accumulators live in the accumulation registers, which the matrix instructions address directly.
//
// The workgroups are persistent: one per compute unit, each walking through its share of the work,
// which is dealt out in units of two query tiles of one (sequence, query head) -- tile k from the top
// with tile k from the bottom, so that under the causal mask every unit has the same number of
// K/V tile steps.  The K/V tiles of consecutive tiles of work form one continuous stream through
// the three LDS buffers and the staging registers: while the last steps of one query tile run, the
// first K/V tiles of the next are already being loaded and stored, and the next Q is loaded under the
// output epilogue, so that only the very first tile of a workgroup pays the latency of a cold start.
//
// With a single wavefront per SIMD nothing but the instruction stream itself overlaps the vector
// ALU (exponentials) with the matrix cores, so the loop is software-pipelined over 32-token blocks.
// For tile t (blocks 0 and 1) a step runs four phases of 16 matrix instructions each:
//     1  S0(t)   = K0 Q^T
//     2  O      += V1(t-1)^T P1      (the output product of a tile's second block runs one step
//     3  S1(t)   = K1 Q^T             late, from an LDS buffer the next step has not overwritten)
//     4  O      += V0(t)^T P0
// and every matrix instruction is followed by an even share of all the other work of the step: one
// half-piece of softmax weights (block 0 under phases 2-3, block 1 under phase 4 and phase 1 of the
// next step), an operand fetch from LDS, a piece of the staging of the next tile.  The softmax keeps
// no running maximum on this path: weights are taken against a reference that is only checked, per
// block, to have kept the block's sums in range (see close_block).  The matrix instructions are
// written as inline assembly to pin the score tiles to vector registers and the accumulators to
// accumulation registers; the wait states the hardware needs between a matrix instruction and a
// vector-ALU access to its result, which the compiler cannot insert for inline assembly, are spelled
// out (settle_*).  In the other direction -- a vector write needs two wait states before a matrix
// instruction may read the register -- no operand is produced right in front of its consumer:
// fragments arrive from LDS behind a wait, weights are packed at least a slot earlier
// (tests/test_prefill_codegen.py checks the compiled instruction stream for this).
#include "prefill_tile.h"

namespace diffqkv {

namespace {

using namespace prefill_tile;

constexpr float kMinRef = -1.0e30f;  // initial softmax reference: finite, so that exp2(-inf - ref) = 0

// d = a b^T (+ d): 32x32x16 bf16, results in vector registers (scores) or accumulation registers (output)
// (score product: the B operand, Q^T, is read from accumulation registers too -- Q stays there for the
// whole kernel and leaves the vector registers to the softmax)
__device__ __forceinline__ void mfma_first_v(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_v(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_a(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
// Wait states between the last matrix instruction writing these registers and the first vector-ALU
// instruction touching them (and the other way round).  16 + 4 covers the 8-pass instruction.
__device__ __forceinline__ void settle_v(f32x16& x, f32x16& y) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(x), "+v"(y));
}
template <int CB>
__device__ __forceinline__ void settle_a(f32x16 (&acc)[2][CB]) {
  if constexpr (CB == 4) {
    asm volatile("s_nop 15\n\ts_nop 3"
                 : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[0][2]), "+a"(acc[0][3]), "+a"(acc[1][0]),
                   "+a"(acc[1][1]), "+a"(acc[1][2]), "+a"(acc[1][3]));
  } else {
    asm volatile("s_nop 15\n\ts_nop 3" : "+a"(acc[0][0]), "+a"(acc[0][1]), "+a"(acc[1][0]), "+a"(acc[1][1]));
  }
}

// Tile t lives in buffer t % 3, K and V^T alike.  V^T needs three: the output product of a tile's
// second block runs during the next step, while the staging stores of the step after that are already
// being written.  K needs two and takes three so that both rotate together: the step body is compiled
// once per buffer index, which turns every LDS address in it into a loop-invariant register plus an
// immediate.
// A tile buffer index that is either a compile-time constant (std::integral_constant) or a plain int.
template <typename T>
__device__ __forceinline__ constexpr int buffer_index(T t) {
  if constexpr (std::is_integral_v<T>) return t;
  else return T::value;
}

typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) u32x2 lds_u32x2;

template <int DQK, int DV>
struct Smem64 {
  static constexpr int kKPitch = DQK + 8;  // bf16 elements per K row (16 B of padding)
  uint16_t k[3][kBN][kKPitch];
  // V tiles as they are in memory, token-major; the transposition that the output product's A operand
  // needs happens in the LDS read (ds_read_b64_tr_b16).  64 bytes of padding per row: the four rows a
  // half-wavefront reads in one such instruction then fall on four disjoint quarters of the banks.
  static constexpr int kVPitch = DV + 32;  // bf16 elements per V row
  uint16_t v[3][kBN][kVPitch];
  // one slice per wavefront through which a block of 32 output rows leaves (see the epilogue)
  static constexpr int kOutPitch = DV * 2 + 8;  // bytes per row; the 8 spread the rows over the banks
  char out[4][32 * kOutPitch];
};

// The work of a launch: units = pairs of query tiles (tile n-1-k and tile k of one (sequence, query
// head)); workgroup w of G takes the units w, w + G, w + 2 G, ...
struct Schedule64 {
  int n_qtiles;   // query tiles of 256 rows per (sequence, query head)
  int n_pairs;    // ceil(n_qtiles / 2)
  int n_units;    // n_pairs * n_q * B
  int xcd_aware;  // unit numbering that keeps the query heads of a K head on one XCD
};

template <int DQK, int DV>
__global__ __launch_bounds__(256, 1) void prefill_mfma64_kernel(PrefillParams p, Schedule64 sch) {
  static_assert((DQK == 128 || DQK == 64) && DV == 128, "head widths this kernel is laid out for");
  constexpr int KS = DQK / 16;  // k-steps of the score product (16 channels each)
  constexpr int CB = DV / 32;   // 32-channel blocks of the output
  constexpr int kThreads = 256;
  constexpr int kBM = 256;
  __shared__ Smem64<DQK, DV> sm;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5, n = lane & 31;
  const int off = p.S_k - p.S_q;   // query i sees keys j <= i + off when causal

  // ---- the tiles of work of this workgroup, in order: seq = 2 * round + part -----------------------
  // part 0 is the pair's tile from the bottom (the longer one under the causal mask), part 1 the
  // tile from the top; a pair whose two tiles coincide (the middle one of an odd count) has no part 1.
  struct Work {
    int b, h, qtile;
    int n_tiles;  // K/V tiles the workgroup walks through for it
  };
  const int n_seq = 2 * ((sch.n_units - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x);
  auto work_at = [&](int seq, Work& w) -> bool {  // false: no such tile of work
    if (seq >= n_seq) return false;
    const int x = (seq >> 1) * (int)gridDim.x + (int)blockIdx.x;
    int pair;
    const int g_k = p.n_q / p.n_k;
    if (sch.xcd_aware) {
      const int groups_per_xcd = p.B * p.n_k / kXcds;
      const int c = x % kXcds, j = x / kXcds;
      const int hq = j % g_k, t = j / g_k;
      const int group = (t % groups_per_xcd) * kXcds + c;
      pair = t / groups_per_xcd;
      w.b = group / p.n_k;
      w.h = (group % p.n_k) * g_k + hq;
    } else {
      w.h = x % p.n_q;
      w.b = (x / p.n_q) % p.B;
      pair = x / (p.n_q * p.B);
    }
    const int bottom = sch.n_qtiles - 1 - pair;
    if (seq & 1) {
      if (bottom == pair) return false;
      w.qtile = pair;
    } else {
      w.qtile = bottom;
    }
    int wg_limit = p.S_k;
    if (p.causal) {
      const int q0 = w.qtile * kBM;
      const int lastq = (q0 + kBM < p.S_q ? q0 + kBM : p.S_q) - 1;
      wg_limit = lastq + off + 1;
    }
    // (all of this is the same in every lane; saying so keeps it, and the buffer resources made from
    //  it, in scalar registers)
    w.n_tiles = __builtin_amdgcn_readfirstlane((wg_limit + kBN - 1) / kBN);
    w.b = __builtin_amdgcn_readfirstlane(w.b);
    w.h = __builtin_amdgcn_readfirstlane(w.h);
    w.qtile = __builtin_amdgcn_readfirstlane(w.qtile);
    return true;
  };
  auto next_work = [&](int seq, Work& w) -> int {  // the first tile of work after seq; n_seq if none
    for (++seq; seq < n_seq; ++seq)
      if (work_at(seq, w)) return seq;
    return n_seq;
  };
  auto uniform = [](const uint16_t* ptr) {
    const uint64_t a = (uint64_t)(uintptr_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    return (const uint16_t*)(uintptr_t)(((uint64_t)hi << 32) | lo);
  };
  auto k_head = [&](const Work& w) {
    const int kh = (int)(((int64_t)w.h * p.n_k) / p.n_q);
    return make_rsrc(uniform((const uint16_t*)p.k + ((int64_t)w.b * p.n_k + kh) * p.S_k * DQK), p.S_k * DQK * 2);
  };
  auto v_head = [&](const Work& w) {
    const int vh = (int)(((int64_t)w.h * p.n_v) / p.n_q);
    return make_rsrc(uniform((const uint16_t*)p.v + ((int64_t)w.b * p.n_v + vh) * p.S_k * DV), p.S_k * DV * 2);
  };

  // ---- Q^T as the B operand: lane (half, n) holds channels 16 ks + 8 half .. + 7 of its two rows ----
  u32x4 qf[2][KS];
  auto load_q = [&](const Work& w, u32x4 (&q)[2][KS]) {
    const uint16_t* qbase = (const uint16_t*)p.q + ((int64_t)w.b * p.n_q + w.h) * p.S_q * DQK;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      int row = w.qtile * kBM + wave * 64 + 32 * qb + n;
      row = row < p.S_q ? row : p.S_q - 1;
      const uint16_t* qrow = qbase + (int64_t)row * DQK + half * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) q[qb][ks] = *(const u32x4*)(qrow + ks * 16);
    }
  };

  // ---- global -> register -> LDS staging of one K/V tile (every thread takes part in both) ----------
  // K tile = 64 rows x d_qk channels: d_qk / 8 threads share a row (16 bytes each) and take KLD rows next
  // to each other, so one per-lane offset per tile serves all of a thread's loads through the
  // immediate field.  The V tile (64 rows x d_v channels) is staged the same way, VLD rows per thread.
  constexpr int KLD = kBN * (DQK / 8) / kThreads;
  constexpr int kRowThreads = DQK / 8;  // threads that share a K row
  static_assert(kThreads / kRowThreads * KLD == kBN, "whole rows per thread");
  const int k_row = (tid / kRowThreads) * KLD, k_chunk = tid % kRowThreads;
  const int k_voff = k_row * (DQK * 2) + k_chunk * 16;
  constexpr int VLD = kBN * (DV / 8) / kThreads;
  constexpr int kVRowThreads = DV / 8;
  static_assert(kThreads / kVRowThreads * VLD == kBN, "whole rows per thread");
  const int v_row = (tid / kVRowThreads) * VLD, v_chunk = tid % kVRowThreads;
  const int v_voff = v_row * (DV * 2) + v_chunk * 16;
  u32x4 kst[KLD], vst[VLD];
  // (t0: first token of the tile inside the head that the resource describes)
  auto load_k_tile = [&](rsrc_t k_rsrc, int t0) {
#pragma unroll
    for (int i = 0; i < KLD; ++i)
      kst[i] = __builtin_amdgcn_raw_buffer_load_b128(k_rsrc, k_voff + t0 * (DQK * 2) + i * (DQK * 2), 0, 0);
  };
  auto load_v_tile = [&](rsrc_t v_rsrc, int t0) {
#pragma unroll
    for (int i = 0; i < VLD; ++i)
      vst[i] = __builtin_amdgcn_raw_buffer_load_b128(v_rsrc, v_voff + t0 * (DV * 2) + i * (DV * 2), 0, 0);
  };
  // (LDS addresses as integers: a per-lane part that the step computes once from the buffer index --
  //  folded into the immediates where that index is a constant -- plus an immediate)
  constexpr uint32_t kKBuf = kBN * Smem64<DQK, DV>::kKPitch * 2;  // bytes of one K buffer
  constexpr uint32_t kVRow = Smem64<DQK, DV>::kVPitch * 2;
  constexpr uint32_t kVBuf = kBN * kVRow;                          // bytes of one V buffer
  constexpr uint32_t kKRow = Smem64<DQK, DV>::kKPitch * 2;
  const uint32_t k_base = (uint32_t)(uintptr_t)&sm.k[0][0][0];
  const uint32_t k_st = k_base + (uint32_t)(k_row * kKRow + k_chunk * 16);
  auto store_k_item = [&](int i, uint32_t k_st_buf) {  // i in [0, KLD); k_st_buf = k_st + buffer * kKBuf
    *(lds_u32x4*)(k_st_buf + (uint32_t)(i * kKRow)) = kst[i];
  };
  // (with the start of the V buffers folded into the per-lane part: the immediate field of an LDS
  //  instruction reaches 64 KiB from there, which covers all three buffers)
  const uint32_t v_base = (uint32_t)(uintptr_t)&sm.v[0][0][0];
  const uint32_t v_st = v_base + (uint32_t)(v_row * kVRow + v_chunk * 16);
  auto store_v_item = [&](int i, uint32_t v_st_buf) {  // i in [0, VLD); v_st_buf = v_st + buffer * kVBuf
    *(lds_u32x4*)(v_st_buf + (uint32_t)(i * kVRow)) = vst[i];
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < KLD; ++i) store_k_item(i, k_st + (uint32_t)buf * kKBuf);
#pragma unroll
    for (int i = 0; i < VLD; ++i) store_v_item(i, v_st + (uint32_t)buf * kVBuf);
  };

  // ---- state of the tile of work in hand ----------------------------------------------------------------
  int r0 = 0;           // first query row of this wavefront
  f32x16 acc[2][CB];     // accumulation registers
  f32x16 s[2][2];        // [row block][token block] scores
  uint32_t pw[2][2][8];  // [row block][token block] weights, bf16 pairs, as the B operand wants them
  float m_run[2], l_run[2];
  auto reset_state = [&]() {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      // (what the last tile of work left in the score and weight registers of block 0 is dead: say so,
      //  or the compiler keeps those registers alive through the epilogue and the next Q's arrival)
      asm volatile("" : "=v"(s[qb][0]));
#pragma unroll
      for (int i = 0; i < 8; ++i) asm volatile("" : "=v"(pw[qb][0][i]));
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[qb][cb][r] = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) s[qb][1][r] = -INFINITY;  // "previous tile": weights of zero
#pragma unroll
      for (int i = 0; i < 8; ++i) pw[qb][1][i] = 0u;
      m_run[qb] = kMinRef;
      l_run[qb] = 0.f;
    }
    settle_a<CB>(acc);
  };

  // Softmax without a running maximum on the hot path.  Scores stay unscaled; the scale (> 0) is
  // folded into the exponent: p = 2^(c s - m_ref).  The reference m_ref of a row only has to keep the
  // exponentials in range; it need not track the maximum.  So the weights of a block are computed
  // against the reference as it stands, their sum is kept apart (l_blk), and once the block is complete
  // -- before its output product starts -- one comparison per lane checks that no sum has left the
  // range [0, kBig].  Only then (the first block of a wavefront, where m_ref is still the initial
  // -1e30, and later if a score exceeds the reference by more than ~36 in log2 units) the block maximum
  // is taken, the reference raised, accumulators and row sums rescaled and the block's weights
  // computed again.  Weights stay below 2^40, inside bf16 / fp32 range with room for the sums; the final
  // division by the row sum removes the reference.
  constexpr float kBig = 1.0995116e12f;  // 2^40
  // Of the 32 half-pieces of a block's weights, how many run under the output-product phase of their
  // window (4 CB slots) and how many under the score phase (2 KS slots): in proportion, and even.
  constexpr int kHalvesA = 2 * ((16 * 4 * CB + (4 * CB + 2 * KS) / 2) / (4 * CB + 2 * KS));
  float l_blk[2][2] = {{0.f, 0.f}, {0.f, 0.f}};  // [token block][row block]: sum of the block's weights
  // two of a row block's 16 weights of a token block
  auto weights_piece = [&](int blk, int qb, int i) {
    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i], p.scale_log2, -m_run[qb]));
    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i + 1], p.scale_log2, -m_run[qb]));
    pw[qb][blk][i] = pack_bf16x2(p0, p1);
    l_blk[blk][qb] += p0 + p1;
  };
  // The same in two halves, numbered h = 0..31 per token block: groups of eight halves cover pieces
  // 0-3 of row block 0, 0-3 of row block 1, 4-7 of row block 0, 4-7 of row block 1; an even half
  // takes the two exponentials of its piece, the odd half after it packs and sums them.  Each half
  // is pinned where it is written, between the (volatile) matrix instructions around it; otherwise
  // the optimiser sinks the arithmetic towards its first use, out from under them.
  auto weights_half = [&](auto blkc, auto hc, float (&tp)[2]) {
    constexpr int blk = decltype(blkc)::value, h = decltype(hc)::value;
    constexpr int group = h / 8, qb = group & 1, i = (group >> 1) * 4 + (h % 8) / 2;
    if constexpr (h % 2 == 0) {
      tp[0] = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i], p.scale_log2, -m_run[qb]));
      tp[1] = __builtin_amdgcn_exp2f(fmaf(s[qb][blk][2 * i + 1], p.scale_log2, -m_run[qb]));
      asm volatile("" : "+v"(tp[0]), "+v"(tp[1]));
    } else {
      pw[qb][blk][i] = pack_bf16x2(tp[0], tp[1]);
      l_blk[blk][qb] += tp[0] + tp[1];
      asm volatile("" : "+v"(pw[qb][blk][i]), "+v"(l_blk[blk][qb]));
    }
  };
  // The block is complete: range check, then its sums join the row sums.
  auto close_block = [&](auto blkc) {
    constexpr int blk = decltype(blkc)::value;
    const float worst = fmaxf(l_blk[blk][0], l_blk[blk][1]);
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(!(worst <= kBig)) != 0, 0)) {  // (a NaN also lands here, and stays a NaN)
      settle_a<CB>(acc);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float m_blk = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) m_blk = fmaxf(m_blk, s[qb][blk][r]);
        m_blk = fmaxf(m_blk, __shfl_xor(m_blk, 32, 64));  // the lane holding the row's other 16 tokens
        const float m_new = fmaxf(m_run[qb], m_blk * p.scale_log2);
        const float fac = __builtin_amdgcn_exp2f(m_run[qb] - m_new);  // from the initial reference: 0
        m_run[qb] = m_new;
        l_run[qb] *= fac;
        // (one accumulator tile at a time: this rare path must not raise the register demand of the
        //  whole kernel, or the allocator spills hot-loop values to make room for it)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          acc[qb][cb] *= fac;
          asm volatile("" : "+a"(acc[qb][cb]));
        }
        l_blk[blk][qb] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) weights_piece(blk, qb, i);
      }
      settle_a<CB>(acc);
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      l_run[qb] += l_blk[blk][qb];
      l_blk[blk][qb] = 0.f;
    }
  };
  // V^T fragment of 16-token step kq (0..3 within the tile), channel block cb: lane (half, n) needs
  // channel 32 cb + n of the eight tokens 16 kq + 4 half + {0..3} and + 8 (the token order the score
  // layout produces).  A transposing LDS read hands each lane of a 16-lane group four values: element
  // e of lane l comes from the 8 bytes that lane (l / 4 + 4 e) of the group addressed, taking its
  // element l % 4.  So lane L of a group addresses token row (L / 4), channels 4 (L % 4) .. + 3 of the
  // group's 16 channels, and receives channel L of four consecutive tokens; two reads make a fragment.
  typedef __attribute__((ext_vector_type(4))) short s16x4;
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  const int tr_group = lane >> 4, tr_l = lane & 15;
  const uint32_t v_lane = v_base + (uint32_t)((4 * (tr_group >> 1) + (tr_l >> 2)) * kVRow + (16 * (tr_group & 1) + 4 * (tr_l & 3)) * 2);
  auto vt_frag = [&](uint32_t v_buf, auto kqc, auto cbc) {  // v_buf = v_lane + buffer * kVBuf
    constexpr int kq = decltype(kqc)::value, cb = decltype(cbc)::value;
    const uint32_t at = v_buf + (uint32_t)(16 * kq * kVRow + 32 * cb * 2);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)at);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(at + 8 * kVRow));
    const u32x2 l2 = __builtin_bit_cast(u32x2, lo), h2 = __builtin_bit_cast(u32x2, hi);
    return u32x4{l2[0], l2[1], h2[0], h2[1]};
  };
  const uint32_t k_lane = k_base + (uint32_t)(n * kKRow + 16 * half);  // this lane's K fragment of row block 0, k-step 0

  // One tile step; see the header for the phase order.  MASKED (compile time) adds the causal / length
  // select on the finished score blocks, the only place that looks at token positions.
  bool pending = false;  // the previous tile's second block still waits for its output product
  // A step of a wavefront that is past its last row: it only helps staging.  (ld_k, ld_v, ld_tok:
  // where the K/V stream stands two tiles ahead -- the tile whose loads this step issues.)
  auto staging_step = [&](int cur, rsrc_t ld_k, rsrc_t ld_v, int ld_tok) {
    const int next = cur == 2 ? 0 : cur + 1;
    store_tile(next);
    load_k_tile(ld_k, ld_tok);
    load_v_tile(ld_v, ld_tok);
    __syncthreads();
  };
  // curc = it % 3, the buffer of this step's tile: an int, or a std::integral_constant -- then every
  // LDS address of the step is a loop-invariant register plus an immediate.
  auto tile_step = [&](int it, auto masked_tag, auto curc, rsrc_t ld_k, rsrc_t ld_v, int ld_tok) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const int cur = buffer_index(curc), next = cur == 2 ? 0 : cur + 1, prev = cur == 0 ? 2 : cur - 1;
    const int t0 = it * kBN;
    // the step's LDS bases (constants folded into the immediates in the copies with a constant index)
    const uint32_t k_cur = k_lane + (uint32_t)cur * kKBuf;
    const uint32_t k_st_next = k_st + (uint32_t)next * kKBuf, v_st_next = v_st + (uint32_t)next * kVBuf;
    const uint32_t vt_cur = v_lane + (uint32_t)cur * kVBuf, vt_prev = v_lane + (uint32_t)prev * kVBuf;
    {
      // fragment order: K block 0 | V^T of the previous tile's block 1 | K block 1 | V^T block 0
      constexpr int G0 = KS, G1 = KS + 2 * CB, G2 = 2 * KS + 2 * CB, kFrags = 2 * KS + 4 * CB;
      constexpr int kRing = 8;
      u32x4 fr[kRing];
      auto fetch = [&](auto fc) {
        constexpr int f = decltype(fc)::value;
        if constexpr (f < G0) {
          fr[f % kRing] = *(const lds_u32x4*)(k_cur + (uint32_t)(32 * f));
        } else if constexpr (f < G1) {
          constexpr int j = f - G0;
          fr[f % kRing] = vt_frag(vt_prev, std::integral_constant<int, 2 + j / CB>{}, std::integral_constant<int, j % CB>{});
        } else if constexpr (f < G2) {
          constexpr int ks = f - G1;
          fr[f % kRing] = *(const lds_u32x4*)(k_cur + (uint32_t)(32 * kKRow + 32 * ks));
        } else {
          constexpr int j = f - G2;
          fr[f % kRing] = vt_frag(vt_cur, std::integral_constant<int, j / CB>{}, std::integral_constant<int, j % CB>{});
        }
      };
      static_for<0, kRing>(fetch);
      __builtin_amdgcn_sched_barrier(0);
      float tp[2];  // exponentials waiting to be packed by the next half

      // A wavefront issues in order; the matrix pipe takes one instruction per 32 cycles and holds
      // the vector ALU's operand ports for a good part of them, so two matrix instructions back to
      // back, or a long run of vector work, both leave one of the pipes idle.  Every matrix
      // instruction is therefore followed by a "slot" with an even share of all the other work of
      // the step.  Slots are numbered g = 0 .. 2 kFrags - 1, two per fragment; phase 1 (scores of block
      // 0) covers the first 2 KS of them, phase 2 (output product of the previous tile's block 1) the
      // next 4 CB, phase 3 (scores of block 1) 2 KS, phase 4 (output product of block 0) 4 CB:
      //   the weights of a token block as 32 half-pieces -- even: two exponentials, odd: pack and sum --
      //   spread evenly over the slots of two phases (one per slot at d_qk = 128, four per three slots
      //   at d_qk = 64): block 0 under phases 2-3 (its scores are complete after phase 1, its output
      //   product starts with phase 4), block 1 under phase 4 and on into phase 1 of the next step
      //   (an even number of them on each side: a pair of halves never straddles two steps);
      //   row block 0 / 1 alternate in groups of four pieces so that everything is ready when the
      //   output product asks for it; the range check that closes a block follows its last half;
      //   staging (LDS stores of the next tile, then the loads of the one after) on odd slots.
      // Register r of a score tile is token t0 + 32 blk + 8 (r/4) + 4 half + r%4.  On and past the
      // diagonal the scores of tokens a row may not see are replaced by -inf as soon as the block's
      // score product is complete (weight 0, and no part in a block maximum).
      auto mask_block = [&](auto blkc) {
        constexpr int blk = decltype(blkc)::value;
        settle_v(s[0][blk], s[1][blk]);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
          // register r is allowed iff 8 (r/4) + r%4 <= lim: one compare against a constant per register.
          // Whole blocks are decided first, from wavefront-uniform bounds on lim (rows n = 0..31, halves
          // 0..1): a block every lane sees in full is left alone -- the unmasked steps that run in this
          // body take that way out four times -- and one that no lane sees is overwritten without compares.
          const int tok0 = t0 + 32 * blk;                              // first token of the block
          const int row_last = p.causal ? r0 + 32 * qb + off : p.S_k;  // last token row n = 0 may see
          const int lim_lo = (row_last < p.S_k - 1 ? row_last : p.S_k - 1) - tok0 - 4;  // n = 0, half = 1
          const int lim_hi = (row_last + 31 < p.S_k - 1 ? row_last + 31 : p.S_k - 1) - tok0;  // n = 31, half = 0
          if (lim_lo >= 27) continue;  // every register of every lane is allowed
          if (lim_hi < 0) {            // none is
#pragma unroll
            for (int r = 0; r < 16; ++r) s[qb][blk][r] = -INFINITY;
            continue;
          }
          int last = p.causal ? r0 + 32 * qb + n + off : p.S_k - 1;  // last token this row may see
          last = last < p.S_k - 1 ? last : p.S_k - 1;
          const int lim = last - (tok0 + 4 * half);
#pragma unroll
          for (int r = 0; r < 16; ++r) s[qb][blk][r] = (8 * (r >> 2) + (r & 3) <= lim) ? s[qb][blk][r] : -INFINITY;
        }
      };
      auto stage_item = [&](auto ic) {
        constexpr int idx = decltype(ic)::value;
        // (unconditional: past the last tile of the last piece of work the stores park stale registers
        //  in a buffer nobody reads, and the loads go to an empty buffer resource and return zeros)
        if constexpr (idx < KLD) store_k_item(idx, k_st_next);
        else if constexpr (idx < KLD + VLD) store_v_item(idx - KLD, v_st_next);
        else if constexpr (idx == KLD + VLD) load_k_tile(ld_k, ld_tok);
        else load_v_tile(ld_v, ld_tok);
      };
      // halves [lo, hi) of a block's weights, in order
      auto halves = [&](auto blkc, auto loc, auto hic) {
        constexpr int lo = decltype(loc)::value, hi = decltype(hic)::value;
        static_for<lo, hi>([&](auto hc) { weights_half(blkc, hc, tp); });
      };
      auto slot = [&](auto gc) {
        constexpr int g = decltype(gc)::value;
        constexpr int P2 = 2 * G0, P3 = 2 * G1, P4 = 2 * G2;  // first slots of phases 2, 3, 4
        constexpr int nA = 4 * CB, nB = 2 * KS, HA = kHalvesA, HB = 32 - HA;
        if constexpr (MASKED && g == P2) mask_block(std::integral_constant<int, 0>{});
        if constexpr (MASKED && g == P4) mask_block(std::integral_constant<int, 1>{});
        if constexpr (g >= P2 && g < P3)
          halves(std::integral_constant<int, 0>{}, std::integral_constant<int, HA * (g - P2) / nA>{},
                 std::integral_constant<int, HA * (g - P2 + 1) / nA>{});
        if constexpr (g >= P3 && g < P4)
          halves(std::integral_constant<int, 0>{}, std::integral_constant<int, HA + HB * (g - P3) / nB>{},
                 std::integral_constant<int, HA + HB * (g - P3 + 1) / nB>{});
        if constexpr (g >= P4)
          halves(std::integral_constant<int, 1>{}, std::integral_constant<int, HA * (g - P4) / nA>{},
                 std::integral_constant<int, HA * (g - P4 + 1) / nA>{});
        if constexpr (g < P2)
          halves(std::integral_constant<int, 1>{}, std::integral_constant<int, HA + HB * g / nB>{},
                 std::integral_constant<int, HA + HB * (g + 1) / nB>{});
        if constexpr (g == P2 - 1) close_block(std::integral_constant<int, 1>{});  // the previous tile's second block
        if constexpr (g == P4 - 1) close_block(std::integral_constant<int, 0>{});
        // staging on odd slots: the K stores, then at once the K loads of the tile after (the longer a
        // load has before its store, a step later, the less that store waits), the V stores, the V loads
        if constexpr ((g & 1) && g < 2 * KLD) stage_item(std::integral_constant<int, g / 2>{});
        if constexpr (g == 2 * KLD + 1) stage_item(std::integral_constant<int, KLD + VLD>{});
        if constexpr ((g & 1) && g >= 2 * KLD + 3 && g < 2 * KLD + 3 + 2 * VLD) stage_item(std::integral_constant<int, KLD + (g - 2 * KLD - 3) / 2>{});
        if constexpr (g == 2 * KLD + 3 + 2 * VLD) stage_item(std::integral_constant<int, KLD + VLD + 1>{});
      };

      static_for<0, kFrags>([&](auto fc) {
        constexpr int f = decltype(fc)::value;
        constexpr int phase = f < G0 ? 1 : f < G1 ? 2 : f < G2 ? 3 : 4;
        constexpr int j = f - (phase == 1 ? 0 : phase == 2 ? G0 : phase == 3 ? G1 : G2);  // step inside the phase
        const u32x4 a = fr[f % kRing];
        auto matrix = [&](auto qc) {
          constexpr int qb = decltype(qc)::value;
          if constexpr (phase == 1 || phase == 3) {
            constexpr int blk = phase == 1 ? 0 : 1;
            if constexpr (j == 0) mfma_first_v(s[qb][blk], a, qf[qb][0]);
            else mfma_v(s[qb][blk], a, qf[qb][j]);
          } else {
            constexpr int blk = phase == 2 ? 1 : 0, sh = (j / CB) * 4, cb = j % CB;
            mfma_a(acc[qb][cb], a, u32x4{pw[qb][blk][sh], pw[qb][blk][sh + 1], pw[qb][blk][sh + 2], pw[qb][blk][sh + 3]});
          }
        };
        matrix(std::integral_constant<int, 0>{});
        __builtin_amdgcn_sched_barrier(0);
        slot(std::integral_constant<int, 2 * f>{});
        __builtin_amdgcn_sched_barrier(0);
        matrix(std::integral_constant<int, 1>{});
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (f + kRing < kFrags) fetch(std::integral_constant<int, f + kRing>{});
        slot(std::integral_constant<int, 2 * f + 1>{});
        __builtin_amdgcn_sched_barrier(0);
      });
      pending = true;
    }
    __syncthreads();
  };
  // The block that is still in flight after the last step a wavefront computes.
  auto drain = [&](int vprev) {  // vprev: buffer of the last tile computed
    const uint32_t vt_last = v_lane + (uint32_t)vprev * kVBuf;
    // the halves the next step would have taken: kHalvesA .. 31, whole pieces
    static_for<kHalvesA / 2, 16>([&](auto pc) {
      constexpr int h = 2 * decltype(pc)::value, group = h / 8;
      weights_piece(1, group & 1, (group >> 1) * 4 + (h % 8) / 2);
    });
    close_block(std::integral_constant<int, 1>{});
    static_for<0, 2 * CB>([&](auto jc) {
      constexpr int j = decltype(jc)::value, sh = (j / CB) * 4;
      const u32x4 a = vt_frag(vt_last, std::integral_constant<int, 2 + j / CB>{}, std::integral_constant<int, j % CB>{});
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
        mfma_a(acc[qb][j % CB], a, u32x4{pw[qb][1][sh], pw[qb][1][sh + 1], pw[qb][1][sh + 2], pw[qb][1][sh + 3]});
    });
    pending = false;
  };

  // ---- write this wavefront's rows.  Lane (half, n) holds row 32 qb + n in pieces of four channels
  //      (acc[qb][cb][r]: channel 32 cb + 8 (r/4) + 4 half + r%4); stored from there, one instruction
  //      would touch 32 rows.  So each row block passes through a slice of LDS that belongs to this
  //      wavefront alone and leaves in 16-byte pieces, 16 lanes to a row: whole 256-byte rows per
  //      store.  The LDS operations of one wavefront execute in order, so the slice needs no barrier.
  auto write_rows = [&](const Work& w) {
    settle_a<CB>(acc);
    constexpr int kOutPitch = Smem64<DQK, DV>::kOutPitch;
    const uint32_t slice = (uint32_t)(uintptr_t)&sm.out[wave][0];
    const int o_row = lane >> 4, o_chunk = lane & 15;
    // Rows at or past S_q are dropped by the range check of the buffer stores (no branches in here).
    const int64_t head = (int64_t)w.b * p.n_q + w.h;
    const rsrc_t o_rsrc = make_rsrc(uniform((const uint16_t*)p.out + head * p.S_q * DV), p.S_q * DV * 2);
    const rsrc_t lse_rsrc = make_rsrc(uniform((const uint16_t*)(p.lse_out ? p.lse_out + head * p.S_q : nullptr)),
                                      p.lse_out ? p.S_q * 4 : 0);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const float l = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);  // both halves hold the full row sum now
      const float inv = __builtin_amdgcn_rcpf(l);
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 x;
          x[0] = pack_bf16x2(acc[qb][cb][4 * q4] * inv, acc[qb][cb][4 * q4 + 1] * inv);
          x[1] = pack_bf16x2(acc[qb][cb][4 * q4 + 2] * inv, acc[qb][cb][4 * q4 + 3] * inv);
          *(lds_u32x2*)(slice + (uint32_t)(n * kOutPitch + (32 * cb + 8 * q4 + 4 * half) * 2)) = x;
        }
      // (the two halves of a row store the same value to the same place)
      __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, (m_run[qb] + __builtin_amdgcn_logf(l)) * kLn2),
                                            lse_rsrc, (r0 + 32 * qb + n) * 4, 0, 0);
      u32x4 piece[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) piece[i] = *(const lds_u32x4*)(slice + (uint32_t)((4 * i + o_row) * kOutPitch + o_chunk * 16));
#pragma unroll
      for (int i = 0; i < 8; ++i)
        __builtin_amdgcn_raw_buffer_store_b128(piece[i], o_rsrc, (r0 + 32 * qb + 4 * i + o_row) * (DV * 2) + o_chunk * 16, 0, 0);
    }
  };

  // ---- the K/V stream -------------------------------------------------------------------------------
  // The K/V tiles of this workgroup's tiles of work, laid end to end, form one stream; every tile of
  // work is padded to a multiple of three slots, so that each starts in LDS buffer 0 (the padding slots
  // cost a barrier and a round of staging stores each, no arithmetic).  At the start of the step that
  // takes stream slot g, LDS buffer g % 3 holds it, the staging registers hold slot g + 1 (stored into
  // buffer (g + 1) % 3 during the step) and the step issues the loads of slot g + 2.  The cursor below
  // is that slot g + 2: a head's buffer resources and a tile index inside the head.  On a padding slot,
  // and past the last tile of work, it points at an empty resource (loads return zeros).
  int ld_seq = -1, ld_tile = 0, ld_tiles = 0, ld_slots = 0;  // cursor: slot ld_tile of ld_slots, of which ld_tiles are tiles
  rsrc_t ld_k = make_rsrc(p.k, 0), ld_v = make_rsrc(p.v, 0);
  auto cursor_next_work = [&]() {
    Work ld_work;
    ld_seq = next_work(ld_seq, ld_work);
    ld_tile = 0;
    if (ld_seq < n_seq) {
      ld_tiles = ld_work.n_tiles;
      ld_slots = (ld_tiles + 2) / 3 * 3;
      ld_k = k_head(ld_work);
      ld_v = v_head(ld_work);
    } else {
      ld_tiles = ld_slots = 0x7ffffff0;
      ld_k = make_rsrc(p.k, 0);
      ld_v = make_rsrc(p.v, 0);
    }
  };
  auto cursor_advance = [&](int slots) {  // (never across more than one boundary)
    ld_tile += slots;
    if (ld_tile >= ld_slots) {
      cursor_next_work();
    } else if (ld_tile >= ld_tiles) {  // padding
      ld_k = make_rsrc(p.k, 0);
      ld_v = make_rsrc(p.v, 0);
    }
  };

  Work work;
  int seq = next_work(-1, work);
  if (seq >= n_seq) return;  // (a workgroup without work: the grid is never larger than the unit count)
  // cold start: Q and the first two tiles of the stream
  load_q(work, qf);
  cursor_next_work();  // -> tile 0 of the first tile of work
  load_k_tile(ld_k, ld_tile * kBN);
  load_v_tile(ld_v, ld_tile * kBN);
  cursor_advance(1);
  store_tile(0);
  load_k_tile(ld_k, ld_tile * kBN);  // staging registers always hold the tile after the one in LDS
  load_v_tile(ld_v, ld_tile * kBN);
  cursor_advance(1);
  // the first step runs the "previous tile" output product with weights of zero, from buffer 2: make
  // what it multiplies finite
  auto clear_vt = [&](int buf) {
    static_assert(kVBuf % (16 * kThreads) == 0, "whole rounds of 16-byte stores");
#pragma unroll
    for (int i = 0; i < (int)(kVBuf / (16 * kThreads)); ++i)
      *(lds_u32x4*)(v_base + (uint32_t)buf * kVBuf + (uint32_t)((i * kThreads + tid) * 16)) = u32x4{0u, 0u, 0u, 0u};
  };
  clear_vt(2);

  while (true) {
    // ---- one tile of work: 256 query rows of (work.b, work.h) against work.n_tiles K/V tiles --------
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[qb][ks]));  // Q has arrived, and sits in accumulation registers
    reset_state();
    __syncthreads();
    const int n_tiles = work.n_tiles;
    r0 = work.qtile * kBM + wave * 64;
    int wave_limit = p.S_k;  // tokens this wavefront can see
    if (p.causal) {
      int lastw = r0 + 63;
      lastw = lastw < p.S_q ? lastw : p.S_q - 1;
      wave_limit = lastw + off + 1;  // (<= 0 for a wavefront whose rows are all past S_q: it only stages)
    }
    // tiles wholly visible to every row of this wavefront need no mask; tiles past its last row are
    // staging only -- the pending block is finished before the first of those overwrites its buffer
    int n_plain = p.S_k / kBN;
    if (p.causal) {
      const int vis = (r0 + off + 1) / kBN;  // tiles entirely at or before the first row's limit
      n_plain = vis < n_plain ? vis : n_plain;
    }
    n_plain = n_plain < n_tiles ? n_plain : n_tiles;
    int n_compute = wave_limit > 0 ? (wave_limit + kBN - 1) / kBN : 0;
    n_compute = n_compute < n_tiles ? n_compute : n_tiles;
    n_plain = n_plain < n_compute ? n_plain : n_compute;

    // The bulk of the steps -- unmasked, three at a time, one per buffer -- run with constant buffer
    // indices; they stop two tiles short of the end of the tile of work, so that their loads never
    // leave its K/V head (the stream cursor stands in that head throughout, and is moved past those
    // steps in one go afterwards).  The steps after (the diagonal, and what the groups of three leave
    // over) run one more copy of the body, the masked one, which takes the buffer index as a value --
    // its LDS bases cost a dozen additions per step -- and its loads from the stream cursor.
    int hot_end = n_plain < n_tiles - 2 ? n_plain : n_tiles - 2;
    hot_end = hot_end > 0 ? hot_end / 3 * 3 : 0;
    int it = 0;
    for (; it < hot_end; it += 3) {
      tile_step(it, std::false_type{}, std::integral_constant<int, 0>{}, ld_k, ld_v, it * kBN + 2 * kBN);
      tile_step(it + 1, std::false_type{}, std::integral_constant<int, 1>{}, ld_k, ld_v, it * kBN + 3 * kBN);
      tile_step(it + 2, std::false_type{}, std::integral_constant<int, 2>{}, ld_k, ld_v, it * kBN + 4 * kBN);
    }
    cursor_advance(hot_end);
    int cur = 0;  // slot % 3: the LDS buffer of the tile the next step computes
    for (; it < n_compute; ++it, cur = cur == 2 ? 0 : cur + 1) {
      tile_step(it, std::true_type{}, cur, ld_k, ld_v, ld_tile * kBN);
      cursor_advance(1);
    }
    if (pending) drain(cur == 0 ? 2 : cur - 1);
    const int n_slots = (n_tiles + 2) / 3 * 3;
    for (; it < n_slots; ++it, cur = cur == 2 ? 0 : cur + 1) {  // (past this wavefront's last row, or padding)
      staging_step(cur, ld_k, ld_v, ld_tile * kBN);
      cursor_advance(1);
    }

    // ---- on to the next tile of work: its first K/V tile is in LDS already and its second in the
    //      staging registers; its Q is loaded under the output epilogue of this one ------------------
    Work next;
    const int next_seq = next_work(seq, next);
    __syncthreads();  // every wavefront is through its drain: the buffer of the last tile is free
    // (Q of this tile of work is dead: its registers take the next one, which arrives under the epilogue)
    if (next_seq < n_seq) {
      load_q(next, qf);
      // the first step of the next tile of work multiplies buffer 2 by weights of zero: whatever this
      // tile of work left there must not reach it (a zero times an infinity)
      clear_vt(2);
    }
    write_rows(work);
    if (next_seq >= n_seq) break;
    work = next;
    seq = next_seq;
  }
}

template <int DQK, int DV>
hipError_t launch64(const PrefillParams& p, hipStream_t s) {
  Schedule64 sch;
  sch.n_qtiles = (p.S_q + 255) / 256;
  sch.n_pairs = (sch.n_qtiles + 1) / 2;
  const int64_t n_units = (int64_t)sch.n_pairs * p.n_q * p.B;
  if (n_units > 0x3fffffff) return hipErrorInvalidValue;
  sch.n_units = (int)n_units;
  sch.xcd_aware = ((p.B * p.n_k) % kXcds == 0) ? 1 : 0;
  // one persistent workgroup per compute unit (a workgroup fills one: a wavefront per SIMD with the
  // whole register file), fewer if there is less work
  const int n_wg = sch.n_units < p.n_cu ? sch.n_units : p.n_cu;
  launch_kernel(0, prefill_mfma64_kernel<DQK, DV>, dim3((unsigned)n_wg), dim3(256), 0, s, p, sch);
  return hipGetLastError();
}

}  // namespace

bool prefill_mfma64_supported(const PrefillParams& p, int dtype) {
  // (the staging loads run up to two tiles past the end of a head: keep them inside the 32-bit offset)
  return dtype == 1 && (p.d_qk == 128 || p.d_qk == 64) && p.d_v == 128 &&
         (int64_t)(p.S_k + 2 * kBN) * 128 * 2 < (1ll << 31);
}

hipError_t launch_prefill_mfma64(const PrefillParams& p, hipStream_t s) {
  if (p.B == 0) return hipSuccess;
  return p.d_qk == 128 ? launch64<128, 128>(p, s) : launch64<64, 128>(p, s);
}

}  // namespace diffqkv
