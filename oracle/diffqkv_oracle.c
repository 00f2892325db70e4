/*
 * DiffQKV attention -- float64 CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked against.  Only the
 * test-suite, the smoke check and the cpu_baseline leg of the benchmark may load it; the product
 * (the HIP library and its Python binding) never calls into it and shares no code with it.
 *
 * What it computes (paper section 2, "Formulation of DiffQKV Attention"; head-index rule of the
 * equation labelled "idx" in section 3.2, "Flexible Attention Computation"):
 *
 *   for every sequence b and query head h:
 *       kh = floor(h * n_k / n_q)          the K head shared by h      (GroupSharing on K)
 *       vh = floor(h * n_v / n_q)          the V head shared by h      (GroupSharing on V)
 *       s_j   = scale * <q[b,h,:], K[b,kh,j,:]>          j = 0 .. T_b-1
 *       alpha = softmax_j(s)                              (over the cached positions)
 *       o[b,h,:] = sum_j alpha_j * V[b,vh,j,:]
 *       lse[b,h] = log sum_j exp(s_j)
 *
 * The softmax is evaluated in two passes (maximum first, then exponentials and their sum): there
 * is no tiling, no running rescale and no split/merge here.  All arithmetic is IEEE double; inputs
 * are fp32 or bf16 (as raw uint16 bit patterns) and are widened exactly, element by element, while
 * they are read -- no float64 copy of a cache is ever made.
 *
 * Parity pins (tests/test_oracle_pins.py): a context of one token returns V; constant V returns the
 * constant; q = 0 returns the mean of V; equality with grouped-query / multi-head / multi-query
 * attention from a library routine when the head counts coincide (appendix "Comparison with
 * Existing Attention Mechanisms"); equality with ordinary grouped attention on K expanded the way
 * the paper's "KV Group Sharing" workaround expands it; brute-force enumeration on tiny shapes;
 * shift and permutation invariances; the log-sum-exp split identity; prefill row i equals decode
 * on the first i+1 cache rows; head locality.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };

/* exact widening of one stored element */
static inline double load_elem(const void* base, int dtype, int64_t idx) {
  if (dtype == ORACLE_F32) return (double)((const float*)base)[idx];
  uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16; /* bf16 = upper half of an fp32 */
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/* head map: contiguous blocks of n_q/n_i query heads share head i (integer floor of the idx rule) */
static inline int shared_head(int h, int n_i, int n_q) { return (int)(((int64_t)h * n_i) / n_q); }

/*
 * Where the T rows of one (K head, V head) pair live.  Contiguous cache: row j at base + j*stride.
 * Paged cache (block_row set): row j at base + page(j)*page_stride + slot(j)*stride.
 */
typedef struct {
  const void* k;
  const void* v;
  int dtype;
  int d_qk, d_v;
  /* contiguous addressing */
  int64_t k_base, k_st, v_base, v_st;
  /* paged addressing (block_row != NULL) */
  const int32_t* block_row; /* page ids of this sequence */
  int page_size;
  int64_t k_sp, v_sp; /* page strides */
} kv_view;

static inline int64_t k_row_off(const kv_view* w, int64_t j) {
  if (!w->block_row) return w->k_base + j * w->k_st;
  return w->k_base + (int64_t)w->block_row[j / w->page_size] * w->k_sp + (j % w->page_size) * w->k_st;
}
static inline int64_t v_row_off(const kv_view* w, int64_t j) {
  if (!w->block_row) return w->v_base + j * w->v_st;
  return w->v_base + (int64_t)w->block_row[j / w->page_size] * w->v_sp + (j % w->page_size) * w->v_st;
}

/* q: d_qk doubles; s: scratch of T doubles; out: d_v doubles; returns lse (-inf, zeros if T == 0) */
static double attend_one(const double* q, double scale, const kv_view* w, int64_t T, double* s,
                         double* out) {
  for (int e = 0; e < w->d_v; ++e) out[e] = 0.0;
  if (T <= 0) return -INFINITY;
  double m = -INFINITY;
  for (int64_t j = 0; j < T; ++j) {
    int64_t off = k_row_off(w, j);
    double dot = 0.0;
    for (int c = 0; c < w->d_qk; ++c) dot += q[c] * load_elem(w->k, w->dtype, off + c);
    s[j] = scale * dot;
    if (s[j] > m) m = s[j];
  }
  double l = 0.0;
  for (int64_t j = 0; j < T; ++j) {
    s[j] = exp(s[j] - m);
    l += s[j];
  }
  for (int64_t j = 0; j < T; ++j) {
    int64_t off = v_row_off(w, j);
    double p = s[j];
    for (int e = 0; e < w->d_v; ++e) out[e] += p * load_elem(w->v, w->dtype, off + e);
  }
  for (int e = 0; e < w->d_v; ++e) out[e] /= l;
  return m + log(l);
}

/*
 * Decode over a contiguous cache.
 *   q        [B, n_q, d_qk]                     (dense)
 *   k_cache  element (b, kh, j, c) at  b*k_sb + kh*k_sh + j*k_st + c
 *   v_cache  element (b, vh, j, e) at  b*v_sb + vh*v_sh + j*v_st + e
 *   seqlens  [B] or NULL (then every T_b = T)
 *   out      [B, n_q, d_v] float64,  lse [B, n_q] float64
 * Returns 0, or -1 on a bad argument.
 */
int oracle_decode(int dtype, int B, int n_q, int n_k, int n_v, int d_qk, int d_v, double scale,
                  const void* q, const void* k_cache, const void* v_cache, int64_t k_sb,
                  int64_t k_sh, int64_t k_st, int64_t v_sb, int64_t v_sh, int64_t v_st,
                  const int32_t* seqlens, int T, double* out, double* lse) {
  if (B < 0 || n_q <= 0 || n_k <= 0 || n_v <= 0 || d_qk <= 0 || d_v <= 0 || T < 0) return -1;
  if (n_q % n_k || n_q % n_v) return -1;
  int err = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1));
    double* qd = (double*)malloc(sizeof(double) * (size_t)d_qk);
    if (!s || !qd) {
#pragma omp atomic write
      err = 1;
    } else {
#pragma omp for collapse(2) schedule(dynamic, 1)
      for (int b = 0; b < B; ++b)
        for (int h = 0; h < n_q; ++h) {
          int Tb = seqlens ? seqlens[b] : T;
          if (Tb > T) Tb = T;
          kv_view w;
          memset(&w, 0, sizeof w);
          w.k = k_cache;
          w.v = v_cache;
          w.dtype = dtype;
          w.d_qk = d_qk;
          w.d_v = d_v;
          w.k_base = (int64_t)b * k_sb + (int64_t)shared_head(h, n_k, n_q) * k_sh;
          w.v_base = (int64_t)b * v_sb + (int64_t)shared_head(h, n_v, n_q) * v_sh;
          w.k_st = k_st;
          w.v_st = v_st;
          for (int c = 0; c < d_qk; ++c)
            qd[c] = load_elem(q, dtype, ((int64_t)b * n_q + h) * d_qk + c);
          double r = attend_one(qd, scale, &w, Tb, s, out + ((int64_t)b * n_q + h) * d_v);
          if (lse) lse[(int64_t)b * n_q + h] = r;
        }
    }
    free(s);
    free(qd);
  }
  return err ? -1 : 0;
}

/*
 * Decode over a paged cache: logical token j of sequence b is slot j % page_size of physical page
 * block_table[b, j / page_size].
 *   k_pool   element (page, kh, slot, c) at  page*k_sp + kh*k_sh + slot*k_st + c
 *   v_pool   element (page, vh, slot, e) at  page*v_sp + vh*v_sh + slot*v_st + e
 *   block_table [B, max_pages] int32, seqlens [B] int32 (required)
 */
int oracle_decode_paged(int dtype, int B, int n_q, int n_k, int n_v, int d_qk, int d_v,
                        double scale, const void* q, const void* k_pool, const void* v_pool,
                        int64_t k_sp, int64_t k_sh, int64_t k_st, int64_t v_sp, int64_t v_sh,
                        int64_t v_st, const int32_t* block_table, int max_pages, int page_size,
                        const int32_t* seqlens, double* out, double* lse) {
  if (B < 0 || n_q <= 0 || n_k <= 0 || n_v <= 0 || d_qk <= 0 || d_v <= 0) return -1;
  if (n_q % n_k || n_q % n_v || page_size <= 0 || max_pages < 0 || !seqlens || !block_table)
    return -1;
  int Tmax = 1;
  for (int b = 0; b < B; ++b) {
    if (seqlens[b] < 0 || (int64_t)seqlens[b] > (int64_t)max_pages * page_size) return -1;
    if (seqlens[b] > Tmax) Tmax = seqlens[b];
  }
  int err = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)Tmax);
    double* qd = (double*)malloc(sizeof(double) * (size_t)d_qk);
    if (!s || !qd) {
#pragma omp atomic write
      err = 1;
    } else {
#pragma omp for collapse(2) schedule(dynamic, 1)
      for (int b = 0; b < B; ++b)
        for (int h = 0; h < n_q; ++h) {
          kv_view w;
          memset(&w, 0, sizeof w);
          w.k = k_pool;
          w.v = v_pool;
          w.dtype = dtype;
          w.d_qk = d_qk;
          w.d_v = d_v;
          w.k_base = (int64_t)shared_head(h, n_k, n_q) * k_sh;
          w.v_base = (int64_t)shared_head(h, n_v, n_q) * v_sh;
          w.k_st = k_st;
          w.v_st = v_st;
          w.block_row = block_table + (int64_t)b * max_pages;
          w.page_size = page_size;
          w.k_sp = k_sp;
          w.v_sp = v_sp;
          for (int c = 0; c < d_qk; ++c)
            qd[c] = load_elem(q, dtype, ((int64_t)b * n_q + h) * d_qk + c);
          double r = attend_one(qd, scale, &w, seqlens[b], s, out + ((int64_t)b * n_q + h) * d_v);
          if (lse) lse[(int64_t)b * n_q + h] = r;
        }
    }
    free(s);
    free(qd);
  }
  return err ? -1 : 0;
}

/*
 * Prefill: the same attention for every query position i of a block of S_q queries against S_k
 * keys.  With `causal` the query at position i sees keys j <= i + (S_k - S_q) (the newest query
 * sees the whole cache, so a single query is exactly the decode case).
 *   q [B, n_q, S_q, d_qk], k [B, n_k, S_k, d_qk], v [B, n_v, S_k, d_v]   (dense)
 *   rows: n_rows query positions to evaluate (NULL => all S_q positions, n_rows ignored)
 *   out [B, n_q, R, d_v] float64, lse [B, n_q, R] float64, R = n_rows or S_q
 */
int oracle_prefill(int dtype, int B, int n_q, int n_k, int n_v, int d_qk, int d_v, double scale,
                   const void* q, const void* k, const void* v, int S_q, int S_k, int causal,
                   const int32_t* rows, int n_rows, double* out, double* lse) {
  if (B < 0 || n_q <= 0 || n_k <= 0 || n_v <= 0 || d_qk <= 0 || d_v <= 0) return -1;
  if (n_q % n_k || n_q % n_v || S_q <= 0 || S_k <= 0) return -1;
  if (causal && S_k < S_q) return -1;
  int R = rows ? n_rows : S_q;
  if (rows)
    for (int r = 0; r < R; ++r)
      if (rows[r] < 0 || rows[r] >= S_q) return -1;
  int err = 0;
#pragma omp parallel
  {
    double* s = (double*)malloc(sizeof(double) * (size_t)S_k);
    double* qd = (double*)malloc(sizeof(double) * (size_t)d_qk);
    if (!s || !qd) {
#pragma omp atomic write
      err = 1;
    } else {
#pragma omp for collapse(3) schedule(dynamic, 4)
      for (int b = 0; b < B; ++b)
        for (int h = 0; h < n_q; ++h)
          for (int r = 0; r < R; ++r) {
            int i = rows ? rows[r] : r;
            int64_t Ti = causal ? (int64_t)i + 1 + (S_k - S_q) : S_k;
            kv_view w;
            memset(&w, 0, sizeof w);
            w.k = k;
            w.v = v;
            w.dtype = dtype;
            w.d_qk = d_qk;
            w.d_v = d_v;
            w.k_base = ((int64_t)b * n_k + shared_head(h, n_k, n_q)) * S_k * d_qk;
            w.v_base = ((int64_t)b * n_v + shared_head(h, n_v, n_q)) * S_k * d_v;
            w.k_st = d_qk;
            w.v_st = d_v;
            int64_t qoff = (((int64_t)b * n_q + h) * S_q + i) * d_qk;
            for (int c = 0; c < d_qk; ++c) qd[c] = load_elem(q, dtype, qoff + c);
            int64_t o = ((int64_t)b * n_q + h) * R + r;
            double x = attend_one(qd, scale, &w, Ti, s, out + o * d_v);
            if (lse) lse[o] = x;
          }
    }
    free(s);
    free(qd);
  }
  return err ? -1 : 0;
}

/*
 * Log-sum-exp merge of S partial results of one output row (the identity behind splitting the
 * context into chunks, section 3.2 "split kernel" / "combine kernel"): each part s carries a
 * normalised output o_s [d_v] and lse_s; the whole is
 *     lse = log sum_s exp(lse_s),   o = sum_s exp(lse_s - lse) * o_s.
 * Parts with lse_s = -inf (empty chunks) contribute nothing.
 */
int oracle_lse_merge(int S, int d_v, const double* o_parts, const double* lse_parts, double* out,
                     double* lse) {
  double m = -INFINITY;
  for (int s = 0; s < S; ++s)
    if (lse_parts[s] > m) m = lse_parts[s];
  for (int e = 0; e < d_v; ++e) out[e] = 0.0;
  if (m == -INFINITY) {
    if (lse) *lse = -INFINITY;
    return 0;
  }
  double l = 0.0;
  for (int s = 0; s < S; ++s) l += exp(lse_parts[s] - m);
  double tot = m + log(l);
  for (int s = 0; s < S; ++s) {
    if (lse_parts[s] == -INFINITY) continue;
    double w = exp(lse_parts[s] - tot);
    for (int e = 0; e < d_v; ++e) out[e] += w * o_parts[(int64_t)s * d_v + e];
  }
  if (lse) *lse = tot;
  return 0;
}


/*
 * Selective V-cache fetching (appendix "Selective V Cache Fetching"; LoadCacheV in section 2):
 * the attention weights alpha are the softmax over ALL T positions (the whole K cache is read);
 * of the V cache only the rows of the `top_k` previous positions with the largest weights are
 * loaded; the current token's row (position T-1, not yet "previous") always takes part:
 *     V_t = [LoadCacheV(V_cache, alpha); v_t],     o = sum over the loaded rows of alpha_j V_j.
 * Ties between equal weights go to the lower position.  The formula keeps alpha as it is
 * (renormalize = 0); with renormalize != 0 the result is divided by the sum of the selected
 * weights (softmax restricted to the selected set).  With top_k >= T-1 this is plain attention.
 *   sel_out: optional int32 [B, n_q, top_k + 1]: the selected positions in increasing order,
 *            padded with -1.
 */
typedef struct {
  double w;
  int32_t j;
} ranked;
static int ranked_cmp(const void* a, const void* b) {
  const ranked* x = (const ranked*)a;
  const ranked* y = (const ranked*)b;
  if (x->w > y->w) return -1;
  if (x->w < y->w) return 1;
  return (x->j > y->j) - (x->j < y->j);
}
static int int_cmp(const void* a, const void* b) {
  return (*(const int32_t*)a > *(const int32_t*)b) - (*(const int32_t*)a < *(const int32_t*)b);
}

int oracle_decode_topk(int dtype, int B, int n_q, int n_k, int n_v, int d_qk, int d_v, double scale,
                       const void* q, const void* k_cache, const void* v_cache, int64_t k_sb,
                       int64_t k_sh, int64_t k_st, int64_t v_sb, int64_t v_sh, int64_t v_st,
                       const int32_t* seqlens, int T, int top_k, int renormalize, double* out,
                       double* lse, int32_t* sel_out) {
  if (B < 0 || n_q <= 0 || n_k <= 0 || n_v <= 0 || d_qk <= 0 || d_v <= 0 || T < 0 || top_k < 0)
    return -1;
  if (n_q % n_k || n_q % n_v) return -1;
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < n_q; ++h) {
      int Tb = seqlens ? seqlens[b] : T;
      if (Tb > T) Tb = T;
      double* o = out + ((int64_t)b * n_q + h) * d_v;
      int32_t* sel = sel_out ? sel_out + ((int64_t)b * n_q + h) * (top_k + 1) : NULL;
      for (int e = 0; e < d_v; ++e) o[e] = 0.0;
      if (sel)
        for (int i = 0; i <= top_k; ++i) sel[i] = -1;
      if (Tb <= 0) {
        if (lse) lse[(int64_t)b * n_q + h] = -INFINITY;
        continue;
      }
      const int64_t kb = (int64_t)b * k_sb + (int64_t)shared_head(h, n_k, n_q) * k_sh;
      const int64_t vb = (int64_t)b * v_sb + (int64_t)shared_head(h, n_v, n_q) * v_sh;
      double* s = (double*)malloc(sizeof(double) * (size_t)Tb);
      ranked* r = (ranked*)malloc(sizeof(ranked) * (size_t)Tb);
      int32_t* chosen = (int32_t*)malloc(sizeof(int32_t) * (size_t)(top_k + 1));
      if (!s || !r || !chosen) return -1;
      double m = -INFINITY;
      for (int j = 0; j < Tb; ++j) {
        double dot = 0.0;
        for (int c = 0; c < d_qk; ++c)
          dot += load_elem(q, dtype, ((int64_t)b * n_q + h) * d_qk + c) *
                 load_elem(k_cache, dtype, kb + (int64_t)j * k_st + c);
        s[j] = scale * dot;
        if (s[j] > m) m = s[j];
      }
      double l = 0.0;
      for (int j = 0; j < Tb; ++j) {
        s[j] = exp(s[j] - m);
        l += s[j];
      }
      for (int j = 0; j < Tb; ++j) s[j] /= l; /* alpha */
      /* rank the previous positions 0 .. Tb-2 by weight, ties to the lower position */
      const int prev = Tb - 1;
      for (int j = 0; j < prev; ++j) {
        r[j].w = s[j];
        r[j].j = j;
      }
      qsort(r, (size_t)prev, sizeof(ranked), ranked_cmp);
      int n_sel = prev < top_k ? prev : top_k;
      for (int i = 0; i < n_sel; ++i) chosen[i] = r[i].j;
      chosen[n_sel++] = Tb - 1; /* the current token */
      qsort(chosen, (size_t)n_sel, sizeof(int32_t), int_cmp);
      double mass = 0.0;
      for (int i = 0; i < n_sel; ++i) {
        const int j = chosen[i];
        mass += s[j];
        for (int e = 0; e < d_v; ++e) o[e] += s[j] * load_elem(v_cache, dtype, vb + (int64_t)j * v_st + e);
        if (sel) sel[i] = j;
      }
      if (renormalize)
        for (int e = 0; e < d_v; ++e) o[e] /= mass;
      if (lse) lse[(int64_t)b * n_q + h] = m + log(l);
      free(s);
      free(r);
      free(chosen);
    }
  return 0;
}

/* Augmented Q (observations 3-4 of section 2; the appendix's attention listing): the output of the
 * query projection, one vector of `hidden` numbers per token, passes through a gated feed-forward
 * of intermediate width `inter` before the heads are formed:
 *     q' = W_down ( act(W_gate q) * (W_up q) ),    act = SiLU, z / (1 + exp(-z)), no biases.
 * Weights in the layout of a linear layer, [out features][in features]: w_gate, w_up [inter][hidden],
 * w_down [hidden][inter].  x [M][hidden]; out [M][hidden] in double.  Everything is evaluated in
 * double with no intermediate rounding. */
int oracle_augment_q(int dtype, int M, int hidden, int inter, const void* x, const void* w_gate,
                     const void* w_up, const void* w_down, double* out) {
  if (M < 0 || hidden <= 0 || inter <= 0) return -1;
#pragma omp parallel for schedule(dynamic)
  for (int m = 0; m < M; ++m) {
    double* xin = (double*)malloc(sizeof(double) * (size_t)hidden);
    double* mid = (double*)malloc(sizeof(double) * (size_t)inter);
    for (int c = 0; c < hidden; ++c) xin[c] = load_elem(x, dtype, (int64_t)m * hidden + c);
    for (int i = 0; i < inter; ++i) {
      double gate = 0.0, up = 0.0;
      for (int c = 0; c < hidden; ++c) {
        gate += load_elem(w_gate, dtype, (int64_t)i * hidden + c) * xin[c];
        up += load_elem(w_up, dtype, (int64_t)i * hidden + c) * xin[c];
      }
      mid[i] = gate / (1.0 + exp(-gate)) * up;
    }
    for (int j = 0; j < hidden; ++j) {
      double y = 0.0;
      for (int i = 0; i < inter; ++i) y += load_elem(w_down, dtype, (int64_t)j * inter + i) * mid[i];
      out[(int64_t)m * hidden + j] = y;
    }
    free(xin);
    free(mid);
  }
  return 0;
}

#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif
