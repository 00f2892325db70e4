/*
 * diffqkv -- DiffQKV attention over an asymmetric KV cache, for AMD MI355X (gfx950).
 *
 * C ABI of the library.  Every entry point takes plain pointers and sizes; there are no C++ or
 * framework types in any signature and no exception crosses this boundary.
 *
 * The operation (paper section 2, "Formulation of DiffQKV Attention"): queries have n_q heads, the
 * key cache n_k heads, the value cache n_v heads, with n_k and n_v both dividing n_q.  Query head h
 * reads K head  kh = floor(h * n_k / n_q)  and V head  vh = floor(h * n_v / n_q)  (GroupSharing;
 * head-index rule "idx" of section 3.2, "Flexible Attention Computation"), and
 *
 *     out[b,h,:] = sum_j softmax_j( scale * <q[b,h,:], K[b,kh,j,:]> ) * V[b,vh,j,:],   j < T_b.
 *
 * K is therefore streamed once per K head and V once per V head; nothing is ever expanded to n_q
 * (or to n_v) heads in memory, which is what the cost model of section 3.1 ("KV Cache") counts.
 *
 * Conventions common to all calls
 *   - All data pointers are DEVICE pointers unless a comment says "host".  The caller owns every
 *     buffer; the library never allocates, frees or synchronises: it validates on the host and
 *     enqueues kernels on `hip_stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Inputs are read-only.  `out` is fully overwritten.  `workspace` contents are undefined after
 *     the call.  Two calls may not share a workspace concurrently.
 *   - Strides are in ELEMENTS of the tensor's dtype.  The innermost (channel) stride is always 1.
 *     Base pointers and all strides must keep every row 16-byte aligned.
 *   - The current token's k_t, v_t are already in the cache when attention runs (the paper
 *     concatenates before attending), so a live sequence has T_b >= 1.  A sequence with T_b == 0
 *     produces out = 0 and lse = -inf.
 *   - Cache memory beyond T_b (the tail of the last page, unused capacity) may hold anything,
 *     including NaN; it never influences the result.
 *   - Return value: a diffqkv_status.  On any value other than DIFFQKV_OK nothing was enqueued.
 *     Errors raised asynchronously by the device surface at the caller's next synchronisation.
 *   - Results are a deterministic function of the arguments (no atomics in any reduction).
 *   - Thread safety: the entry points share no mutable state; calls from different threads are
 *     independent as long as they do not share output or workspace memory.  The only process-wide
 *     state is a cache of device properties (the compute-unit count, read once per device, which
 *     sizes the context split), so the *_workspace_bytes query and the call it sizes must run with
 *     the same device current.
 *
 * Experimental knobs and measurement aids live in diffqkv_experimental.h.
 */
#ifndef DIFFQKV_H_
#define DIFFQKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { DIFFQKV_F32 = 0, DIFFQKV_BF16 = 1 } diffqkv_dtype;

typedef enum {
  DIFFQKV_OK = 0,
  DIFFQKV_ERR_NULL = -1,        /* a required pointer is NULL                                      */
  DIFFQKV_ERR_SHAPE = -2,       /* a count is <= 0, a head width is unsupported, S_k < S_q, ...    */
  DIFFQKV_ERR_HEADS = -3,       /* n_k or n_v does not divide n_q, or neither of n_k, n_v divides
                                   the other                                                       */
  DIFFQKV_ERR_ALIGN = -4,       /* a base pointer or stride breaks 16-byte row alignment           */
  DIFFQKV_ERR_WORKSPACE = -5,   /* workspace is NULL or smaller than the *_workspace_bytes figure  */
  DIFFQKV_ERR_UNSUPPORTED = -6, /* valid arguments this build has no kernel for (top_k above 512,
                                   an augmented-Q product beyond 2^40 elements)                    */
  DIFFQKV_ERR_HIP = -7,         /* a HIP call failed at launch time                                */
  DIFFQKV_ERR_STATIC_LIMIT = -8 /* diffqkv_decode_static: the call needs more scratch memory than
                                   DIFFQKV_STATIC_SCRATCH_BYTES                                    */
} diffqkv_status;

/* Problem shape shared by all calls.  Supported head widths: multiples of 8 up to 256 (the tuned
 * kernels cover 64 and 128).  softmax_scale == 0 selects 1/sqrt(d_qk). */
typedef struct {
  int32_t B;     /* sequences in the batch                    */
  int32_t n_q;   /* query heads                               */
  int32_t n_k;   /* key heads   (divides n_q)                 */
  int32_t n_v;   /* value heads (divides n_q)                 */
  int32_t d_qk;  /* width of a query / key head               */
  int32_t d_v;   /* width of a value head (= output width)    */
  int32_t dtype; /* diffqkv_dtype of q, the caches and out    */
  float softmax_scale;
} diffqkv_shape;

/*
 * Split decode (section 3.2: "split kernel" producing per-chunk partial outputs, "combine kernel"
 * merging them by log-sum-exp).  One query token per sequence against a contiguous cache.
 *
 *   q        [B, n_q, d_qk]   dense
 *   k_cache  element (b, kh, j, c) at  b*k_stride_b + kh*k_stride_h + j*k_stride_t + c
 *   v_cache  element (b, vh, j, e) at  b*v_stride_b + vh*v_stride_h + j*v_stride_t + e
 *            (head-major [B, n, T_cap, d] and token-major [B, T_cap, n, d] are both expressible)
 *   seqlens  int32 [B] on the device, or NULL: then every sequence has T tokens
 *   T        with seqlens: an upper bound on every T_b (the cache capacity is a valid bound);
 *            T_b is clamped to it.  T >= 0.
 *   out      [B, n_q, d_v]   dtype of the inputs
 *   lse_out  float [B, n_q] natural-log sum of exp of the scaled scores, or NULL
 *   workspace/workspace_bytes  at least diffqkv_decode_workspace_bytes(shape, T) bytes (a figure
 *            that covers the call with and without seqlens), 16-byte aligned; holds the per-split
 *            partial outputs and their log-sum-exps
 */
size_t diffqkv_decode_workspace_bytes(const diffqkv_shape* shape /* host */, int32_t max_T);
int diffqkv_decode(const diffqkv_shape* shape /* host */, const void* q, const void* k_cache,
                   const void* v_cache, int64_t k_stride_b, int64_t k_stride_h, int64_t k_stride_t,
                   int64_t v_stride_b, int64_t v_stride_h, int64_t v_stride_t,
                   const int32_t* seqlens, int32_t T, void* out, float* lse_out, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/*
 * diffqkv_decode for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, same kernels
 * and bit-identical results as diffqkv_decode, minus the workspace: the partial results of the
 * context splits go to a buffer of DIFFQKV_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing.
 *
 *   - A call whose diffqkv_decode_workspace_bytes(shape, T) exceeds DIFFQKV_STATIC_SCRATCH_BYTES
 *     returns DIFFQKV_ERR_STATIC_LIMIT and enqueues nothing (32 MiB covers e.g. B = 8, n_q = 32,
 *     d_v = 128 at T = 32768 with or without seqlens: 2.1 MB / 17.0 MB).
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress, which may load
 *     the library's device image): make that first call outside any stream capture.
 *   - All calls on one GPU share that GPU's buffer.  Nothing in it has to start at zero and a call
 *     leaves nothing behind that a later call depends on, but two calls that overlap in time on one
 *     GPU (different streams, different threads) race on it: keep them on one stream or serialise
 *     them.  diffqkv_decode with separate workspaces has no such limit.
 */
#define DIFFQKV_STATIC_SCRATCH_BYTES (32u << 20)
int diffqkv_decode_static(const diffqkv_shape* shape /* host */, const void* q, const void* k_cache,
                          const void* v_cache, int64_t k_stride_b, int64_t k_stride_h,
                          int64_t k_stride_t, int64_t v_stride_b, int64_t v_stride_h,
                          int64_t v_stride_t, const int32_t* seqlens, int32_t T, void* out,
                          float* lse_out, void* hip_stream);

/*
 * Split decode over a paged cache (the paper only cites paged attention; the layout is this
 * library's).  Logical token j of sequence b is slot j % page_size of physical page
 * block_table[b * max_pages + j / page_size].  K and V share the block table.
 *
 *   k_pool   element (page, kh, slot, c) at  page*k_stride_page + kh*k_stride_h + slot*k_stride_t + c
 *   v_pool   element (page, vh, slot, e) at  page*v_stride_page + vh*v_stride_h + slot*v_stride_t + e
 *            (the tuned layout is head-major inside a page: [n_pages, n, page_size, d])
 *   block_table  int32 [B, max_pages] on the device; entries past ceil(T_b / page_size) are ignored
 *   page_size    tokens per page, > 0; multiples of 16 take the tuned kernel
 *   seqlens      int32 [B] on the device (required); 0 <= T_b <= max_pages * page_size
 *   workspace    at least diffqkv_decode_workspace_bytes(shape, max_pages * page_size) bytes
 * Page ids are not range-checked on the device: the caller guarantees they index the pools.
 */
int diffqkv_decode_paged(const diffqkv_shape* shape /* host */, const void* q, const void* k_pool,
                         const void* v_pool, int64_t k_stride_page, int64_t k_stride_h,
                         int64_t k_stride_t, int64_t v_stride_page, int64_t v_stride_h,
                         int64_t v_stride_t, const int32_t* block_table, int32_t max_pages,
                         int32_t page_size, const int32_t* seqlens, void* out, float* lse_out,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Prefill: the same attention for a block of S_q query positions against S_k keys (section 2: K_t
 * holds the t tokens up to the current one, so query i attends to positions <= i).  With
 * causal != 0 the mask is aligned to the newest token: query i sees keys j <= i + (S_k - S_q), so
 * S_q = 1 is exactly the decode case.  Requires S_k >= S_q when causal.
 *
 *   q   [B, n_q, S_q, d_qk]   k [B, n_k, S_k, d_qk]   v [B, n_v, S_k, d_v]   dense, head-major
 *   out [B, n_q, S_q, d_v]    lse_out float [B, n_q, S_q] or NULL
 *   workspace: diffqkv_prefill_workspace_bytes(...) bytes (may be 0, then NULL is accepted)
 */
size_t diffqkv_prefill_workspace_bytes(const diffqkv_shape* shape /* host */, int32_t S_q, int32_t S_k);
int diffqkv_prefill(const diffqkv_shape* shape /* host */, const void* q, const void* k,
                    const void* v, int32_t S_q, int32_t S_k, int32_t causal, void* out,
                    float* lse_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Decode with selective V-cache fetching (appendix "Selective V Cache Fetching"; LoadCacheV in the
 * formulation of section 2).  The attention weights alpha are the softmax over all T_b positions
 * (the whole K cache is read), but only the V rows of the `top_k` previous positions with the
 * largest weights are fetched; the current token's row (position T_b - 1) always takes part:
 *
 *     out[b,h,:] = sum over j in top_k(alpha[0 .. T_b-2]) and j = T_b-1 of alpha_j V[b,vh,j,:]
 *
 * Ties between equal scores go to the lower position.  The formula keeps alpha as it is; with
 * renormalize != 0 the result is divided by the sum of the selected weights.  With
 * top_k >= T_b - 1 the call equals diffqkv_decode.  An approximation by design: the paper reports
 * top_k = 100.
 *
 *   arguments as in diffqkv_decode / diffqkv_decode_paged, plus
 *   top_k        0 .. 512 (more: DIFFQKV_ERR_UNSUPPORTED)
 *   sel_out      int32 [B, n_q, top_k + 1] on the device or NULL: the selected positions of every
 *                query head (unordered, unused entries -1)
 *   workspace    at least diffqkv_decode_topk_workspace_bytes(shape, T) bytes (fp32 scores
 *                [B, n_q, T rounded up to 128]); for the paged call T = max_pages * page_size
 * The selection is made on the kernel's fp32 scores (bf16 products accumulated in fp32): two
 * positions whose scores differ by less than that arithmetic's rounding may swap places relative
 * to an exact evaluation.
 */
size_t diffqkv_decode_topk_workspace_bytes(const diffqkv_shape* shape /* host */, int32_t max_T);
int diffqkv_decode_topk(const diffqkv_shape* shape /* host */, const void* q, const void* k_cache,
                        const void* v_cache, int64_t k_stride_b, int64_t k_stride_h,
                        int64_t k_stride_t, int64_t v_stride_b, int64_t v_stride_h,
                        int64_t v_stride_t, const int32_t* seqlens, int32_t T, int32_t top_k,
                        int32_t renormalize, void* out, float* lse_out, int32_t* sel_out,
                        void* workspace, size_t workspace_bytes, void* hip_stream);
int diffqkv_decode_topk_paged(const diffqkv_shape* shape /* host */, const void* q, const void* k_pool,
                              const void* v_pool, int64_t k_stride_page, int64_t k_stride_h,
                              int64_t k_stride_t, int64_t v_stride_page, int64_t v_stride_h,
                              int64_t v_stride_t, const int32_t* block_table, int32_t max_pages,
                              int32_t page_size, const int32_t* seqlens, int32_t top_k,
                              int32_t renormalize, void* out, float* lse_out, int32_t* sel_out,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * KV-cache append (section 3.1, "KV Cache": the store side of the cache; K and V are separate
 * tensors with their own head counts -- "differential management of KV cache").  For every sequence
 * b, copies k_new[b] into token row positions[b] of the K cache and v_new[b] into the same row of
 * the V cache.  Call it before the attention of the same step: the paper concatenates the current
 * token first.  Bit exact.
 *
 *   k_new  [B, n_k, d_qk]   v_new [B, n_v, d_v]   dense, dtype of the cache
 *   k_cache / v_cache and their strides: as in diffqkv_decode (k_pool / v_pool and page strides as
 *            in diffqkv_decode_paged)
 *   positions    int32 [B] on the device: the row to write (the sequence length before the append)
 *   T_cap        rows per sequence in the contiguous cache; the paged capacity is
 *                max_pages * page_size.  A position outside [0, capacity) writes nothing.
 *   seqlens_out  int32 [B] on the device or NULL: receives positions[b] + 1 for every written row
 *                (it may alias `positions`)
 * Head widths must make every head row a multiple of 16 bytes.  shape->n_q and softmax_scale are
 * not used by these calls (n_q must still be a valid multiple of n_k and n_v).
 */
int diffqkv_append(const diffqkv_shape* shape /* host */, const void* k_new, const void* v_new,
                   void* k_cache, void* v_cache, int64_t k_stride_b, int64_t k_stride_h,
                   int64_t k_stride_t, int64_t v_stride_b, int64_t v_stride_h, int64_t v_stride_t,
                   const int32_t* positions, int32_t T_cap, int32_t* seqlens_out, void* hip_stream);
int diffqkv_append_paged(const diffqkv_shape* shape /* host */, const void* k_new, const void* v_new,
                         void* k_pool, void* v_pool, int64_t k_stride_page, int64_t k_stride_h,
                         int64_t k_stride_t, int64_t v_stride_page, int64_t v_stride_h,
                         int64_t v_stride_t, const int32_t* block_table, int32_t max_pages,
                         int32_t page_size, const int32_t* positions, int32_t* seqlens_out,
                         void* hip_stream);

/*
 * Augmented Q (observations 3-4 of section 2, "Formulation of DiffQKV Attention"; the attention
 * listing of the appendix): the output of the query projection, one vector of `hidden` numbers per
 * token, passes through a gated feed-forward of width `inter` before the heads are formed:
 *     q_out = W_down ( silu(W_gate q_in) * (W_up q_in) ),   silu(z) = z / (1 + exp(-z)),  no biases.
 * (Sigma: hidden 2048 / inter 3072 and 4096 / 6144.)  The attention kernels above are unaffected:
 * they receive q_out, reshaped to [n_q, d_qk] per token and rotated, as their q.
 *
 * Device pointers, all contiguous and 16-byte aligned, all of `dtype`:
 *   q_in [M, hidden], w_gate and w_up [inter, hidden], w_down [hidden, inter] (the layout of a linear
 *   layer: [out features][in features]), q_out [M, hidden] (may not alias q_in).
 * hidden and inter must be multiples of 8.  M is the number of tokens of the step (the batch size in
 * decode); the matrix-core path (bf16, widths of 2048, 3072, 4096 or 6144) is laid out for M <= 16 per
 * pass and repeats the pass for more.  Accumulation is fp32; the intermediate activations are rounded
 * once to `dtype` into the workspace (diffqkv_augment_q_workspace_bytes: M, rounded up to a multiple of 16,
 * x inter elements; the layout inside is the library's own).
 * Returns a diffqkv_status; on error nothing is enqueued.
 */
typedef struct diffqkv_augq_shape {
  int32_t M;      /* tokens */
  int32_t hidden; /* width of q_in and q_out */
  int32_t inter;  /* intermediate width */
  int32_t dtype;  /* DIFFQKV_F32 or DIFFQKV_BF16 */
} diffqkv_augq_shape;
size_t diffqkv_augment_q_workspace_bytes(const diffqkv_augq_shape* shape /* host */);
int diffqkv_augment_q(const diffqkv_augq_shape* shape /* host */, const void* q_in, const void* w_gate,
                      const void* w_up, const void* w_down, void* q_out, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/* Human-readable text for a diffqkv_status (static storage). */
const char* diffqkv_strerror(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int diffqkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DIFFQKV_H_ */
