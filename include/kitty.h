/*
 * kitty.h — C ABI of libkitty: page quantizer and decode attention over Kitty's page-centric
 * 2-bit KV cache (arXiv 2511.18643) for AMD MI355X (gfx950).
 *
 * Conventions shared by every entry point
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory.  The library never allocates, frees or retains device memory.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream) and
 *     the call returns without synchronising.  Structs are read during the call only.
 *   - Return value: KITTY_OK, or a negative KITTY_ERR_* code; when an error is returned nothing has
 *     been enqueued.  No exceptions cross the boundary.
 *   - Tensors are bf16 (1-8-7 bit patterns) with the channel index contiguous; cache metadata is
 *     IEEE fp16.  Inputs holding NaN/Inf or |x| > 65504 are outside the contract (fp16 metadata
 *     would saturate); this is not checked.
 *   - head_dim D = 128 and page_size G = 128 are the only supported sizes (the paper's models,
 *     Sec. 4.1 and Fig. 1 caption, use both).
 */
#ifndef KITTY_H_
#define KITTY_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KITTY_OK 0
#define KITTY_ERR_INVALID_ARG (-1) /* null pointer, bad alignment, inconsistent sizes          */
#define KITTY_ERR_UNSUPPORTED (-2) /* a size outside the supported set (D, G, R, GQA group)     */
#define KITTY_ERR_WORKSPACE (-3)   /* workspace smaller than kitty_decode_workspace_bytes()     */
#define KITTY_ERR_HIP (-4)         /* the HIP runtime rejected a launch                         */

/* Problem statement knobs (Fig. 1 caption: G, R; Sec. 3.2: boost fraction; Sec. 2.1: grouping). */
typedef struct kitty_layout {
  int32_t head_dim;        /* D: channels per head; must be 128                                          */
  int32_t page_size;       /* G: Key quantization group = tokens per page (Sec. 4.1); must be 128        */
  int32_t v_group;         /* Value quantization group along D (per-token, Sec. 2.1); must equal D       */
  int32_t n_boost;         /* boosted Key channels per page = boost fraction * D (Sec. 3.2): 0,16,..,128 */
  int32_t residual_window; /* R: full-precision tokens kept before a page forms (Sec. 4.3): 128, or 0    */
  int32_t n_q_heads;       /* query heads                                                                */
  int32_t n_kv_heads;      /* KV heads; n_q_heads / n_kv_heads must be an integer from 1 to 8           */
  int32_t rank_metric;     /* channel ranking: 0 = mean |x| over the page (Eq. 2), 1 = max - min         */
  int32_t sink_tokens;     /* S: initial tokens kept in full precision for K and V (Fig. 1, Sec. 3.1): 0..128.  The
                              paper leaves S free (default 32); this library stops at one page's worth and answers
                              KITTY_ERR_UNSUPPORTED beyond it                                              */
  int32_t v_local;         /* Value Local window (Fig. 1, Sec. 4.3 step 1): 0 = off, 128 = the Values of the newest
                              page are read in full precision until the next page forms; needs R = 128       */
  int32_t v_bits;          /* bits per Value code: 2 (the method; 0 means 2) or 4 (the K2V4 / K4V4-like points of the
                              design-space study, Table 2: a second Value plane holds the high bits)          */
} kitty_layout;

/* One batch's cache.  All pointers are device pointers.
 * The record of (physical page id p, kv-head h) starts at page_pool + (p*n_kv_heads + h)*kitty_page_bytes(). */
typedef struct kitty_cache {
  void*    page_pool;    /* n_pool_pages * n_kv_heads records, 128-byte aligned                          */
  int32_t* page_table;   /* [batch][max_pages] physical page ids in token order                          */
  int32_t* n_pages;      /* [batch] packed pages of each sequence, 0..max_pages                          */
  void*    resid_k;      /* bf16 [batch][n_kv_heads][R][D] newest tokens not yet in a page; NULL if R=0  */
  void*    resid_v;      /* same for Values; with v_local: bf16 [batch][n_kv_heads][2][R][D], the rows of page i
                            (and, before that, of the tokens that will form it) in half i & 1             */
  int32_t* n_resid;      /* [batch] valid rows of the window, 0..R; NULL if R=0                          */
  void*    sink_k;       /* bf16 [batch][n_kv_heads][S][D] first S tokens of every sequence; NULL if S=0 */
  void*    sink_v;       /* same for Values                                                              */
  int32_t* n_sink;       /* [batch] valid Sink rows, 0..S; NULL if S=0                                   */
  const int32_t* seq_order; /* optional [batch] permutation of 0..batch-1, or NULL (identity): the decode kernels
                            dispatch their workgroups sequence by sequence in this order, so listing the longest
                            sequences first shortens the tail of a variable-length batch.  Results do not depend on
                            it; entries outside [0, batch) are skipped, repeated entries are the caller's error,
                            and the output of a sequence the order does not name is unspecified                   */
  int32_t  batch;
  int32_t  max_pages;    /* row length of page_table                                                     */
  int32_t  n_pool_pages;
} kitty_cache;

/* Size in bytes of one (page, kv-head) record: a multiple of 128.  0 if the layout is unsupported.
 * Record contents (Sec. 4.1): dense 2-bit plane with the low bits of every Key channel, compact
 * 2-bit plane with the high bits of the boosted channels, fp16 scale and zero-point per channel,
 * ascending list of boosted channels, 2-bit Value plane (and the plane of the high bits with 4-bit Values),
 * fp16 scale and zero-point per token. */
size_t kitty_page_bytes(const kitty_layout* layout /*host*/);

/* Bytes of a record the method has to move (record minus the padding of the channel list): the sizes of the
 * tensors Sec. 4.1 lists, D*G/4 + n_boost*G/4 code bytes, fp16 scale and zero-point per channel and per token,
 * and one index byte per boosted channel.  This build's own accounting helper (used by the benchmark for the
 * algorithmic byte count); no passage of the paper defines it.  0 if unsupported. */
size_t kitty_page_payload_bytes(const kitty_layout* layout /*host*/);

/* Split plan used by the decode calls (this build's own: the paper runs one unsplit kernel per stage, Sec. 4.3
 * step 2; splitting the token axis is what fills 256 compute units when there are few (sequence, kv-head)
 * pairs).  n_splits_req = 0 picks a plan from the sizes and the
 * GPU's compute-unit count; otherwise n_splits_req ranges are used.  On return *n_splits is the
 * number of page ranges per (sequence, kv-head) and *min_pages the fewest pages a range covers:
 * a sequence with np pages uses min(n_splits, max(1, np / min_pages)) ranges of near-equal
 * length, each of which also takes an equal share of the rows held in full precision (Sink, window).
 * Host pointers. */
int kitty_decode_plan(const kitty_layout* layout, int32_t batch, int32_t max_pages,
                      int32_t n_splits_req, int32_t* n_splits, int32_t* min_pages);

/* Device workspace needed by the decode calls for the plan kitty_decode_plan() returns for the
 * same arguments.  0 if the arguments are invalid. */
size_t kitty_decode_workspace_bytes(const kitty_layout* layout, int32_t batch, int32_t max_pages,
                                    int32_t n_splits_req);

/* Page quantizer (Sec. 4.3 step 3; Sec. 3.2; Sec. 4.1): quantize and pack n_pages pages of
 * G tokens for every kv-head.
 *   k_src, v_src   device bf16.  Element (page i, head h, token t, channel c) is at
 *                  src + off_i + h*head_stride + t*token_stride + c   (all in elements), where
 *                  off_i = src_page_offsets[i] if that pointer is non-NULL, else i*page_stride.
 *                  Every row must be 16-byte aligned (strides and offsets multiples of 8).
 *   src_page_offsets device int64 [n_pages] or NULL.
 *   dst_page_ids   device int32 [n_pages]: physical page written by source page i; ids outside
 *                  [0, n_pool_pages) are skipped.
 *   page_pool      device, as in kitty_cache.
 * Per page and head: per-channel min/max of K over the G tokens, channel score, the n_boost
 * best channels (score descending, index ascending) get 4-bit codes and the rest 2-bit codes;
 * V gets 2-bit codes per token.  scale = fp16((max-min)/qmax), zero = fp16(min),
 * code = clamp(rint((x-zero) * inv), 0, qmax) with inv = fp32(1/scale) (0 for a zero scale), all in IEEE
 * fp32 against the stored fp16 values, ties to even. */
int kitty_quantize_pages(const kitty_layout* layout, const void* k_src, const void* v_src,
                         int64_t page_stride, int64_t head_stride, int64_t token_stride,
                         const int64_t* src_page_offsets, const int32_t* dst_page_ids,
                         int32_t n_pages, void* page_pool, int32_t n_pool_pages, void* hip_stream);

/* Prefill-side fusion of the page quantizer with the projection that produces its input (Sec. 4.3 step 3 applied
 * where the tokens of a page are produced; the system evaluation of Sec. 5.5 prefills prompts before decoding):
 * for every source page i and kv-head h
 *     K[t][c] = bf16( sum_j x[o_i + t][j] * w_k[h*D + c][j] ),   V likewise with w_v,      t < G, c < D, o_i = src_token_offsets[i]
 * on the bf16 matrix cores with fp32 accumulation (the order of the additions is not specified: results equal a
 * reference bit for bit whenever the sums are exact in fp32, else to the last bf16 digit), rounded to bf16 to
 * nearest even, and quantized into page dst_page_ids[i] exactly as kitty_quantize_pages would quantize those
 * bf16 values.  The bf16 K and V never reach device memory.
 *   x                  device bf16, token row t at x + t*x_token_stride (elements), `hidden` features per row,
 *                      16-byte aligned rows (x_token_stride a multiple of 8); hidden must be a multiple of 32.
 *   w_k, w_v           device bf16 [n_kv_heads*D][hidden], row-major (the layout of a linear layer's weight):
 *                      row h*D + c produces channel c of kv-head h.  No positional rotation or normalisation is
 *                      applied between the projection and the quantizer.
 *   src_token_offsets  device int64 [n_pages]; dst_page_ids, page_pool, n_pool_pages as in kitty_quantize_pages. */
int kitty_project_quantize_pages(const kitty_layout* layout, const void* x, int64_t x_token_stride, int32_t hidden,
                                 const void* w_k, const void* w_v, const int64_t* src_token_offsets,
                                 const int32_t* dst_page_ids, int32_t n_pages, void* page_pool, int32_t n_pool_pages,
                                 void* hip_stream);

/* Insert one new token per sequence (Sec. 4.3 steps 1 and 3, seen from the following step).
 *   k_new, v_new     device bf16 [batch][n_kv_heads][D].
 *   fresh_page_ids   device int32 [batch]; entry b is consumed only if sequence b flushes.
 * For each sequence b: while n_sink[b] < S the token is stored in the Sink and nothing else changes.
 * Otherwise: if n_resid[b] == R the window is first quantized into page
 * fresh_page_ids[b], that id is appended to the page table, and the window restarts empty; then the
 * new token is stored in the window.  Attention therefore always sees the newest token in full
 * precision, and a sequence flushes once every G appends.  If a flush is due but the page table
 * is full or the fresh id is outside the pool, that sequence is left unchanged.
 * With v_local the Value rows of the tokens that will form page i are stored in half i & 1 of resid_v; a
 * flush quantizes Keys and Values of the page together, and the bf16 Value rows stay in their half, where
 * attention reads them instead of the record's Value plane until page i+1 forms.  This holds the same tokens
 * in full precision as a Local window of the R newest tokens in front of a Value buffer of G tokens (Sec. 4.3
 * step 1), and per-token Value codes do not depend on when they are computed.
 * Requires residual_window == page_size. */
int kitty_append_token(const kitty_layout* layout, const kitty_cache* cache, const void* k_new,
                       const void* v_new, const int32_t* fresh_page_ids, void* hip_stream);

/* Decode attention for one new query token per sequence (Sec. 4.3 step 2; Eq. 1), read directly
 * from the packed records and the bf16 window:
 *   out[b][hq] = softmax(sm_scale * q[b][hq] . K^T) V   over the Sink rows 0..n_sink-1, the pages in
 * page-table order, then the window rows 0..n_resid-1, with kv-head = hq / (n_q_heads/n_kv_heads).  With
 * v_local the Values of the last page are taken from half (n_pages-1) & 1 of resid_v.
 *   q          device bf16 [batch][n_q_heads][D], 16-byte aligned.
 *   out        device, same shape; bf16 if out_dtype == 0, fp32 if out_dtype == 1.
 *   n_splits   0 = automatic; otherwise page ranges per (sequence, kv-head).
 *   workspace  device scratch of at least kitty_decode_workspace_bytes(..., n_splits) bytes,
 *              16-byte aligned; contents are overwritten.
 * A sequence with no tokens yields zeros.  Equivalent to kitty_decode_split + kitty_decode_merge. */
int kitty_decode_attention(const kitty_layout* layout, const kitty_cache* cache, const void* q,
                           void* out, float sm_scale, int32_t n_splits, int32_t out_dtype,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/* First half of kitty_decode_attention (Sec. 4.3 step 2: the logits, softmax and Value sum of Eq. 1 over the pages
 * of Sec. 4.1, dequantized as in Alg. 1): every page range (and the window) of every (sequence,
 * kv-head) is reduced to a partial (running max, sum of weights, weighted Value sum) in the
 * workspace.  This is the kernel that streams the cache. */
int kitty_decode_split(const kitty_layout* layout, const kitty_cache* cache, const void* q,
                       float sm_scale, int32_t n_splits, void* workspace, size_t workspace_bytes,
                       void* hip_stream);

/* Second half: log-sum-exp merge of the partials and the store of `out`.  The merge is the exact identity
 * softmax(x) = sum_i w_i softmax(x_i) over disjoint chunks x_i of the logits of Eq. 1 (this build's own step; the
 * paper does not split). */
int kitty_decode_merge(const kitty_layout* layout, const kitty_cache* cache, void* out,
                       int32_t n_splits, int32_t out_dtype, const void* workspace,
                       size_t workspace_bytes, void* hip_stream);

/* One decode step of one layer in a single call: kitty_append_token(k_new, v_new, fresh_page_ids) followed by
 * kitty_decode_attention(q -> out) (Sec. 4.3 steps 1-3), with the same arguments and results as those two
 * calls.  When the plan has one page range per (sequence, kv-head) both halves run in one kernel launch (each
 * block appends its own (sequence, kv-head) share, flushing a full window first, then attends).  With several
 * ranges there are two launches: the streaming kernel attends over the state the append will leave (the block of
 * a (sequence, kv-head)'s last range flushes a full window first; the new token is read from k_new / v_new), and
 * the merge launch then stores the token and advances the sequence state.  Requires residual_window ==
 * page_size. */
int kitty_decode_step(const kitty_layout* layout, const kitty_cache* cache, const void* k_new,
                      const void* v_new, const int32_t* fresh_page_ids, const void* q, void* out,
                      float sm_scale, int32_t n_splits, int32_t out_dtype, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/* kitty_decode_attention for callers that cannot allocate device memory or hand over a workspace: code running
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as kitty_decode_attention, except that the partial results of the page ranges go to a fixed array of
 * KITTY_STATIC_WORKSPACE_BYTES inside the library's device image instead of a caller buffer; every GPU the
 * library runs on holds its own copy of that array until the process ends.  The call allocates and frees nothing.
 *   - A plan that needs more than the array holds (kitty_decode_workspace_bytes(layout, batch, max_pages,
 *     n_splits) > KITTY_STATIC_WORKSPACE_BYTES) is refused with KITTY_ERR_WORKSPACE; nothing is enqueued.
 *   - All calls on one GPU share that GPU's array: calls that may run concurrently there (different streams,
 *     different host threads) race on it and must be serialised by the caller.  Nothing in the array needs to
 *     start at zero (every slot a merge reads was written by the same call), so a call may follow any other.
 *   - The array's address is looked up on the first call made on each device (not an allocation); if that lookup
 *     fails the call returns KITTY_ERR_HIP. */
#define KITTY_STATIC_WORKSPACE_BYTES (4 * 1024 * 1024)
int kitty_decode_attention_static(const kitty_layout* layout, const kitty_cache* cache, const void* q, void* out,
                                  float sm_scale, int32_t n_splits, int32_t out_dtype, void* hip_stream);

/* Static description of an error code (this build's own; no passage of the paper). */
const char* kitty_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* KITTY_H_ */
