/*
 * libcachecraft -- selective KV recomputation for reused RAG chunk-caches on MI355X (gfx950).
 *
 * C ABI of the data-parallel hot path of Cache-Craft for ONE attention layer and one batch of
 * prompts S = C_1 .. C_k U (cached chunks followed by the question, Sec. 2.2):
 *
 *   cc_rope_shift      re-position cached keys (Sec. 3.4.3, Sec. 4 "RPE Management")
 *   cc_rope_place      the same for a store that keeps keys without rotation (Sec. 4)
 *   cc_select          score chunk tokens by attention mass on prior chunks, keep the top N
 *                      (Eq. (2), Eq. (10), Sec. 3.2.1)
 *   cc_select_from_scores  keep the top N of scores the caller already has (Sec. 3.2.1)
 *   cc_gather_rows     compact the rows of the chosen tokens
 *   cc_qkv_project     Q, K, V of the chosen tokens only (Sec. 3.4.3)
 *   cc_rms_norm, cc_linear, cc_gated_linear  the rest of a decoder layer for the chosen tokens:
 *                      normalisation, output projection and feed-forward (Sec. 2.1, Sec. 3.4.3)
 *   cc_sparse_prefill  causal attention of the chosen tokens + question over the whole merged
 *                      paged KV, after writing their recomputed K, V into it
 *                      (Eq. (1), Sec. 3.4.3, Sec. 4 "Selective Token Recomputation")
 *                      (cc_shared_values: the values of reused chunks may stay in the chunk store
 *                      until one of their tokens is recomputed; cc_sparse_prefill_static: the same
 *                      call for callers that cannot allocate)
 *   cc_sparse_prefill_mass  cc_sparse_prefill that also returns the question's attention to every
 *                      chunk (Sec. 3.2.2), as a by-product of the attention kernel where it can
 *   cc_check_query_list  checks the row order the write of recomputed K, V relies on
 *   cc_scatter_kv      the write half of cc_sparse_prefill alone: K, V of chunks without a cache
 *                      (Sec. 3.4.1) go into the request's pages before the others are scored
 *   cc_question_mass   attention the question pays to every chunk in that layer, inter(C_i, U)
 *                      (Sec. 3.2.2); cc_focus_* turns it into the set of focused chunks (Algorithm 1)
 *   cc_preloader_*     layer-wise preloading of chunk-caches from host memory on a copy stream
 *                      (Sec. 3.4.2, Algorithm 2)
 *   cc_sparse_prefill_pairs  cc_sparse_prefill that also returns cc_chunk_attention's sums (the chunk-cache
 *                      metadata of Sec. 3.4.3) as a by-product of the attention kernel where it can
 *   cc_chunk_attention inter / intra attention sums between the segments of a prompt (Eq. (2), (3));
 *                      cc_chunk_ab / cc_chunk_cci / cc_chunk_reuse: CCI, beta, gamma, beta', CFO and
 *                      the token budget from them on the host (Sec. 3.1, 3.3)
 *
 * Conventions
 *   - Every tensor and every metadata array is DEVICE memory owned by the caller; the library
 *     never allocates, frees or synchronises.  Scratch comes from a caller-supplied workspace
 *     whose size the matching *_workspace_bytes() call returns (cc_sparse_prefill_static keeps
 *     its scratch in an array of the library's own).  Pointers must be 16-byte aligned.
 *   - Every call only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream) and returns.  Arguments that are visible from host scalars are checked
 *     before any launch; on error nothing is enqueued and nothing is written.
 *   - Return value: CC_OK (0) or a negative cc_status.  cc_last_error(ctx) gives a message.
 *   - Element type `dtype`: CC_F32 (float) or CC_BF16 (bfloat16 storage, fp32 accumulation).
 *   - Paged KV, 16-token blocks (Sec. 4 "Chunk Storage Management"); chunks are padded to whole
 *     blocks and the padding slots are never read as keys and never written:
 *         K pool  [n_blocks][Hkv][16][d]     token-major rows of d elements
 *         V pool  [n_blocks][Hkv][d][16]     dimension-major rows of 16 token slots
 *   - Rotary embedding: pair i of a head is (v[i], v[i + d/2]), i in [0, d/2), frequency
 *     theta^(-2i/d); a rotation by angle phi maps (x, y) to (x cos phi - y sin phi,
 *     y cos phi + x sin phi)  (Sec. 4 "RPE Management").
 *   - Grouped-query attention: query head h reads KV head h / (Hq / Hkv).
 *   - Logits are q.k / sqrt(d); a token at logical position p sees keys at positions <= p of its
 *     own request (per-token form of Eq. (1), Sec. 2.1).
 */
#ifndef CACHECRAFT_CC_H
#define CACHECRAFT_CC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cc_ctx cc_ctx;

typedef enum {
  CC_OK = 0,
  CC_ERR_INVALID_ARG = -1,          /* null / misaligned pointer, negative or inconsistent size */
  CC_ERR_UNSUPPORTED = -2,          /* dtype, head_dim, block size or head grouping not built    */
  CC_ERR_WORKSPACE_TOO_SMALL = -3,
  CC_ERR_HIP = -4                   /* a HIP runtime call failed; see cc_last_error              */
} cc_status;

enum { CC_F32 = 0, CC_BF16 = 1 };
enum { CC_SEG_CHUNK = 0, CC_SEG_QUESTION = 1 };
enum { CC_IMPL_AUTO = 0, CC_IMPL_SCALAR = 1, CC_IMPL_MFMA_NARROW = 2, CC_IMPL_MFMA_WIDE = 3 };   /* see cc_set_impl */

typedef struct {
  int32_t n_q_heads;     /* Hq                                   */
  int32_t n_kv_heads;    /* Hkv, divides Hq                      */
  int32_t head_dim;      /* d: 64 or 128                         */
  int32_t block_size;    /* tokens per KV block: 16              */
  int32_t dtype;         /* CC_F32 | CC_BF16                     */
  int32_t reserved;      /* 0                                    */
  double  rope_theta;    /* rotary base, e.g. 10000 or 500000    */
} cc_config;

/* One cached chunk placed into one request (a chunk *instance*).  Sec. 3: the chunk-cache is the
 * per-layer (K_C, V_C) of the chunk's tokens; Sec. 4: it maps to a list of 16-token blocks. */
typedef struct {
  int32_t src_tab_off;   /* index into src_block_tab of the instance's first block (shared store) */
  int32_t dst_tab_off;   /* index into dst_block_tab of its first request-owned block             */
  int32_t n_tokens;      /* chunk length |C|; occupies ceil(n_tokens/16) blocks                   */
  int32_t delta_pos;     /* new position of token 0 minus the position it was cached at           */
} cc_shift_desc;

/* One segment of a prompt, in prompt order: a cached chunk instance or the question. */
typedef struct {
  int32_t req;           /* request index                                                          */
  int32_t kind;          /* CC_SEG_CHUNK | CC_SEG_QUESTION                                         */
  int32_t logical_start; /* position of the segment's first token in its prompt (padding excluded) */
  int32_t n_tokens;
  int32_t tab_off;       /* index into block_tab of the segment's first request-owned block        */
  int32_t n_select;      /* chunk: N tokens to recompute (0..n_tokens); question: n_tokens         */
  int32_t tok_off;       /* row of the segment's first token in per-token tensors (q, scores)      */
  int32_t sel_off;       /* position of the segment's first entry in the compact query list        */
} cc_segment;

/* ---- context ----------------------------------------------------------------------------- */
/* Validates cfg and creates a context (host memory only).  *out is NULL on error. */
int cc_create(cc_ctx** out, const cc_config* cfg);
void cc_destroy(cc_ctx* ctx);
const char* cc_status_string(int status);
/* Message of the last failing call on this context (valid until the next call on it). */
const char* cc_last_error(const cc_ctx* ctx);
/* Kernel family used by cc_select / cc_sparse_prefill / cc_qkv_project: CC_IMPL_AUTO (default)
 * picks the fastest MFMA kernels built for the configuration (bf16, head_dim 128),
 * CC_IMPL_SCALAR forces the plain ones, CC_IMPL_MFMA_NARROW the MFMA kernels that give a
 * wavefront 32 query rows (64 tokens in the score stage; the only MFMA form for head groups of
 * 1 or 2), CC_IMPL_MFMA_WIDE the ones that give it 64 (128) even where AUTO would find the
 * launch of the score stage too small for them (head groups that are a multiple of 4; narrow
 * otherwise). */
int cc_set_impl(cc_ctx* ctx, int impl);

/* ---- (a) re-position cached keys ----------------------------------------------------------
 * For every instance i and token t < n_tokens, every KV head: read the key from the shared
 * store (block src_block_tab[src_tab_off + t/16], slot t%16), rotate every pair by
 * delta_pos * theta^(-2i/d), write it to block dst_block_tab[dst_tab_off + t/16], slot t%16 of
 * the destination pool.  If v_src_pool and v_dst_pool are non-NULL the instance's V blocks are
 * copied whole (values carry no position).  Source pools are never written.  Source and
 * destination may be the same allocation as long as the block ids differ.
 *   descs [n_instances] device; block tables device int32; max_tokens = max n_tokens (host).
 *   n_src_blocks / n_dst_blocks: pool sizes in blocks; a table entry outside them is skipped.
 *   v_map [n_dst_blocks] device int32 or NULL.  If given, both V pools must be NULL and no value is
 *   moved: for every page the call handles it records v_map[destination block] = source block,
 *   i.e. "the values that go with the keys now in this block are still those of that stored
 *   block" (values carry no position, so the stored ones are the right ones).  cc_sparse_prefill
 *   and its variants take the map through cc_shared_values and copy a page's values only when one
 *   of its tokens is recomputed (copy-on-write).  Entries of blocks the call does not handle are
 *   left alone: the caller sets the map to -1 once, before the first call.
 * Sec. 3.4.3, Sec. 4 "RPE Management". */
int cc_rope_shift(cc_ctx* ctx,
                  const void* k_src_pool, const void* v_src_pool, int32_t n_src_blocks,
                  void* k_dst_pool, void* v_dst_pool, int32_t n_dst_blocks,
                  const int32_t* src_block_tab, const int32_t* dst_block_tab,
                  const cc_shift_desc* descs, int32_t n_instances, int32_t max_tokens,
                  int32_t* v_map, void* stream);

/* ---- (a') place keys that were stored WITHOUT rotation ---------------------------------------
 * The store variant the paper describes (Sec. 4 "RPE Management": the rotation is taken off
 * before a chunk-cache is kept, and put on at run time with the positions of the new prompt).
 * Same arguments and layout as cc_rope_shift, but the source keys carry no rotation and token t of
 * instance i is rotated by (delta_pos + t) * theta^(-2i/d): delta_pos is read as the NEW position
 * of the instance's token 0.  Equivalent to cc_rope_shift on a store that was rotated at cached
 * positions c + t with delta_pos = new - c (the rotations compose).  V and v_map as in
 * cc_rope_shift. */
int cc_rope_place(cc_ctx* ctx,
                  const void* k_src_pool, const void* v_src_pool, int32_t n_src_blocks,
                  void* k_dst_pool, void* v_dst_pool, int32_t n_dst_blocks,
                  const int32_t* src_block_tab, const int32_t* dst_block_tab,
                  const cc_shift_desc* descs, int32_t n_instances, int32_t max_tokens,
                  int32_t* v_map, void* stream);

/* ---- (b) choose the tokens to recompute ---------------------------------------------------
 * For every chunk segment with logical_start > 0 and every token t (position p = start + t):
 *   mass_h(t) = sum over keys l < logical_start of softmax_{l <= p}(q_h(p).k_l / sqrt(d))
 *   score(t)  = mean over query heads of mass_h(t)
 * with q rotated to position p on load and k the (already shifted) keys of the request's pages.
 * A chunk at logical_start 0 scores 0.  Per chunk the n_select largest scores win (lower index
 * among equals) and are emitted in ascending index order.  Question segments emit all tokens.
 * Outputs, all [n_q_tot] int32 laid out by seg.sel_off (any of q_row/q_pos/slot_map may be NULL):
 *   sel_idx   index of the token inside its segment
 *   q_row     seg.tok_off + index        (row in per-token tensors)
 *   q_pos     seg.logical_start + index  (logical position)
 *   slot_map  block_tab[seg.tab_off + index/16] * 16 + index%16  (physical KV slot)
 * scores [n_tok] float (rows by tok_off; question rows untouched) or NULL.
 *   q [n_tok][Hq][d] pre-rotation, read-only.  segs [n_segs], req_seg_off [n_requests+1] device.
 *   max_seg_tokens: max n_tokens over segments (host scalar, sizes the launch).
 * Eq. (2), block matrix below Eq. (3), Eq. (10), Sec. 3.2.1. */
size_t cc_select_workspace_bytes(const cc_ctx* ctx, int32_t n_tok, int32_t n_segs);
int cc_select(cc_ctx* ctx, const void* q, int32_t n_tok,
              const void* k_pool, int32_t n_blocks, const int32_t* block_tab,
              const cc_segment* segs, int32_t n_segs,
              const int32_t* req_seg_off, int32_t n_requests, int32_t max_seg_tokens,
              int32_t* sel_idx, int32_t* q_row, int32_t* q_pos, int32_t* slot_map, int32_t n_q_tot,
              float* scores, void* workspace, size_t workspace_bytes, void* stream);

/* ---- (b') choose the tokens to recompute from given scores -----------------------------------
 * The selection half of cc_select alone: the per-token scores are an input, e.g. the ordered
 * token list a chunk's metadata keeps from cache time, when the attention weights came for free
 * (Sec. 3.2.1; Sec. 3.4.3 "metadata").  Per chunk segment the n_select largest scores win (lower
 * index among equals, ascending output); a chunk at logical_start 0 is treated like any other
 * (its given scores count); question segments emit all tokens.  Outputs as for cc_select.
 *   scores [n_tok] float, rows by tok_off (question rows ignored), read-only.
 *   workspace: at least cc_select_workspace_bytes(ctx, n_tok, n_segs) bytes. */
int cc_select_from_scores(cc_ctx* ctx, const float* scores, int32_t n_tok, const int32_t* block_tab,
                          const cc_segment* segs, int32_t n_segs,
                          int32_t* sel_idx, int32_t* q_row, int32_t* q_pos, int32_t* slot_map,
                          int32_t n_q_tot, void* workspace, size_t workspace_bytes, void* stream);

/* dst[i][:] = src[row_idx[i]][:] for i < n_rows; row_bytes a multiple of 16.  Compacts the rows
 * of the chosen tokens (hidden states before the projection, or given q / k / v rows). */
int cc_gather_rows(cc_ctx* ctx, const void* src, int32_t n_src_rows, const int32_t* row_idx,
                   int32_t n_rows, size_t row_bytes, void* dst, void* stream);

/* ---- Q, K, V of the chosen tokens ---------------------------------------------------------
 * [q | k | v] = x W^T with x [n_rows][hidden] and W [(Hq + 2 Hkv) d][hidden] row-major (one row
 * of `hidden` weights per output feature: q heads, then k heads, then v heads -- both operands
 * have the contraction index contiguous, which is what the matrix cores want); outputs
 * q [n_rows][Hq][d], k, v [n_rows][Hkv][d].  hidden must be a multiple of 64.  The projection is
 * restricted to the rows of the compact list (Sec. 3.4.3). */
int cc_qkv_project(cc_ctx* ctx, const void* x, const void* w_qkv, int32_t n_rows, int32_t hidden,
                   void* q, void* k, void* v, void* stream);

/* ---- (b'') the rest of a decoder layer, for the rows that are recomputed ----------------------
 * The hidden state of a recomputed token passes through the whole layer (Sec. 2.1: the next hidden
 * state is the token's own plus the feed-forward network of its attention output; Sec. 3.4.3: the
 * attention output goes through the FFN to give the layer output); the operators are those of the
 * models the paper runs (Llama-3): with h the hidden states of the chosen rows,
 *   x  = cc_rms_norm(h, gain_attn)               -> cc_qkv_project -> cc_sparse_prefill -> o
 *   h1 = cc_linear(o, W_o, residual = h)
 *   h2 = cc_linear(cc_gated_linear(cc_rms_norm(h1, gain_ffn), W_gate, W_up), W_down, residual = h1)
 * All tensors are row-major in the context's dtype, weights [out_features][in_features], 16-byte
 * aligned; sums are taken in fp32.
 *   cc_rms_norm:     y[r][c] = x[r][c] / sqrt(mean_c(x[r][c]^2) + eps) * gain[c]; x, y [n_rows][hidden]
 *                    (y may be x); hidden must be a multiple of 8 (bf16) / 4 (fp32).
 *   cc_linear:       y [n_rows][n_out] = x [n_rows][n_in] W^T (+ residual [n_rows][n_out], or NULL;
 *                    residual may be y itself, x may not).
 *   cc_gated_linear: y [n_rows][n_ffn] = silu(x W_gate^T) * (x W_up^T), silu(t) = t / (1 + exp(-t)).
 * bf16 with n_out (2 n_ffn for the gated form) a multiple of 256 and n_in a multiple of 64, at
 * least 128: MFMA GEMM with 128 x 128 outputs per wavefront; otherwise a plain tiled kernel. */
int cc_rms_norm(cc_ctx* ctx, const void* x, const void* gain, float eps, int32_t n_rows, int32_t hidden,
                void* y, void* stream);
int cc_linear(cc_ctx* ctx, const void* x, const void* w, const void* residual, int32_t n_rows,
              int32_t n_in, int32_t n_out, void* y, void* stream);
int cc_gated_linear(cc_ctx* ctx, const void* x, const void* w_gate, const void* w_up, int32_t n_rows,
                    int32_t n_in, int32_t n_ffn, void* y, void* stream);

/* ---- values that stay in the chunk store (copy-on-write) ------------------------------------
 * Optional argument of cc_sparse_prefill and its variants (NULL: every page's values are in
 * v_pool).  While v_map[b] >= 0, the values of the page whose KEYS sit in block b of k_pool are
 * those of block v_map[b] of v_shared (cc_rope_shift writes such entries instead of copying V);
 * otherwise they are in block b of v_pool.  Step 1 of the call (the write of the recomputed rows)
 * copies a page's values from v_shared into block b of v_pool the first time it writes a row of
 * that page, and sets v_map[b] = -1; step 2 reads every page's values from where the map says.
 * v_shared is never written.  A host struct; the arrays it points at are device memory.
 * Sec. 3.4.3 (only the recomputed tokens' K, V are new; Sec. 4: values need no re-positioning). */
typedef struct cc_shared_values {
  const void* v_shared;      /* pool of stored blocks, same block layout as v_pool               */
  int32_t n_shared_blocks;   /* its size in blocks; a map entry outside it counts as -1          */
  int32_t* v_map;            /* [n_blocks of k_pool / v_pool], read and updated by the call      */
} cc_shared_values;

/* ---- (c) partial prefill ------------------------------------------------------------------
 * For every row j < n_q_tot of the compact query list (requests delimited by cu_q):
 *   1. rotate k_new[j] to position q_pos[j] and write it, with v_new[j], into physical slot
 *      slot_map[j] of the request-owned pools (inputs are not modified);
 *   2. out[j][h] = softmax_{l <= q_pos[j]}(q'[j][h].k_l / sqrt(d)) v_l over all keys of the row's
 *      request (stale shifted rows, fixed rows, question rows), with q' = q[j] rotated to
 *      q_pos[j]; lse[j][h] = natural log of the softmax denominator.
 * Step 2 of every row sees step 1 of every row.  Keys are enumerated through segs/block_tab;
 * rows of one request must be contiguous, and rows whose slots lie in the same 16-token block
 * must be adjacent (the order cc_select emits); otherwise any order inside a request is accepted.
 *   q [n_q_tot][Hq][d], k_new, v_new [n_q_tot][Hkv][d]; out like q; lse [n_q_tot][Hq] or NULL.
 *   src_rows [n_q_tot] or NULL: if given, list row j reads row src_rows[j] of q, k_new and v_new
 *   (per-token tensors, e.g. cc_select's q_row output) instead of row j of compact ones, which
 *   saves the caller the gather; q_pos, slot_map, out and lse are always indexed by the list row.
 *   max_q_per_req: max rows of one request (host scalar, sizes the launch).
 *   n_ctx_tokens: sum of n_tokens over all segments, or any upper bound of it (host scalar; sizes
 *   the key-tile plan kept in the workspace).
 *   shared: see cc_shared_values (NULL: none).
 * Eq. (1), Sec. 3.4.3, Sec. 4 "Selective Token Recomputation". */
size_t cc_sparse_prefill_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs);
int cc_sparse_prefill(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                      const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                      const int32_t* cu_q, int32_t n_q_tot, int32_t max_q_per_req,
                      void* k_pool, void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                      const cc_segment* segs, int32_t n_segs,
                      const int32_t* req_seg_off, int32_t n_requests, int32_t n_ctx_tokens,
                      const cc_shared_values* shared, void* out, float* lse,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---- (c') cc_sparse_prefill for callers that cannot allocate ---------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the
 * same call (same kernels, same results bit for bit) without a workspace argument.  The key-tile
 * plan and the redo flags go into an array of CC_STATIC_SCRATCH_BYTES that is part of the
 * library's code object: every GPU the library runs on holds one copy until the process ends.
 * The call allocates nothing and frees nothing.  The array's address on a device is looked up
 * once, by cc_create for the device current then, else by the first call on that device (that
 * look-up, not the call, is what must stay outside a graph capture).
 *   Limit: cc_sparse_prefill_workspace_bytes(ctx, n_ctx_tokens, n_segs) <= CC_STATIC_SCRATCH_BYTES
 *   (about 30 000 key tiles: two million context tokens per call); larger batches return
 *   CC_ERR_WORKSPACE_TOO_SMALL before any launch.
 *   All calls on one GPU share that GPU's array, on every stream and from every context: two calls
 *   whose kernels may overlap on one GPU race.  Calls ordered on one stream are safe (each call
 *   rewrites all it reads, including the flags that must start at zero). */
#define CC_STATIC_SCRATCH_BYTES (1u << 20)
int cc_sparse_prefill_static(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                             const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                             const int32_t* cu_q, int32_t n_q_tot, int32_t max_q_per_req,
                             void* k_pool, void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                             const cc_segment* segs, int32_t n_segs,
                             const int32_t* req_seg_off, int32_t n_requests, int32_t n_ctx_tokens,
                             const cc_shared_values* shared, void* out, float* lse, void* stream);

/* ---- (c'') partial prefill that also returns the question's attention to every chunk --------
 * cc_sparse_prefill (same steps, same out and lse, bit for bit) plus seg_mass as cc_question_mass
 * defines it, in one call.  Where the attention kernel that runs can give the masses as a
 * by-product it does (the 64-row MFMA kernel: at the last key tile of every segment it stores the
 * log-sum-exp over all keys so far for the question rows; a row's weight on a segment is then
 * exp(cum_s - lse) - exp(cum_{s-1} - lse); rows it leaves to the other kernel because their
 * logits overflowed its fixed softmax reference are walked again, rarely, by a scalar kernel);
 * otherwise the masses come from cc_question_mass's pass after the attention.  The call is for
 * the per-layer loop of Sec. 3.2.2, where inter_l(C_i, U) is wanted in every layer.
 *   src_rows as for cc_sparse_prefill (NULL: q, k_new, v_new are compact); every pass of the call,
 *   the by-product path and the passes after the attention alike, reads q through it.
 *   lse is required.  max_question_rows as for cc_question_mass; max_segs_per_req: most segments
 *   of one request (host scalar).  seg_mass [n_segs] float.
 *   workspace: cc_sparse_prefill_mass_workspace_bytes(ctx, n_ctx_tokens, n_segs, n_requests,
 *   max_question_rows, max_segs_per_req). */
size_t cc_sparse_prefill_mass_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                              int32_t n_requests, int32_t max_question_rows,
                                              int32_t max_segs_per_req);
int cc_sparse_prefill_mass(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                           const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                           const int32_t* cu_q,
                           int32_t n_q_tot, int32_t max_q_per_req, int32_t max_question_rows,
                           void* k_pool, void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                           const cc_segment* segs, int32_t n_segs,
                           const int32_t* req_seg_off, int32_t n_requests, int32_t max_segs_per_req,
                           int32_t n_ctx_tokens, const cc_shared_values* shared,
                           void* out, float* lse, float* seg_mass,
                           void* workspace, size_t workspace_bytes, void* stream);

/* ---- (c3) partial prefill that also returns the segment-to-segment attention sums -----------
 * cc_sparse_prefill (same steps, same out and lse, bit for bit) plus pair_mass and self_mass as
 * cc_chunk_attention defines them and, if seg_mass is not NULL, seg_mass as cc_question_mass
 * defines it (it is the row of the pair matrix that belongs to the request's question segment),
 * in one call: the chunk-cache metadata of Sec. 3.4.3 at the cost of the prefill that produces
 * the cache.  Where the 64-row MFMA kernel runs, the sums come from the by-product of
 * cc_sparse_prefill_mass kept for EVERY row; otherwise from cc_chunk_attention's passes after the
 * attention.  The by-product path needs the rows of segment s at [sel_off, sel_off + n_select) of
 * the compact list, as cc_select lays them out.
 *   src_rows as for cc_sparse_prefill_mass.
 *   lse is required.  pair_mass [n_pairs] and self_mass [n_segs] float, both required; n_pairs as
 *   for cc_chunk_attention; max_segs_per_req: most segments of one request (host scalar).
 *   workspace: cc_sparse_prefill_pairs_workspace_bytes(ctx, n_ctx_tokens, n_segs, n_q_tot,
 *   max_q_per_req, max_segs_per_req); it holds max_segs_per_req floats per row and query head. */
size_t cc_sparse_prefill_pairs_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                               int32_t n_q_tot, int32_t max_q_per_req,
                                               int32_t max_segs_per_req);
int cc_sparse_prefill_pairs(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                            const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                            const int32_t* cu_q,
                            int32_t n_q_tot, int32_t max_q_per_req,
                            void* k_pool, void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                            const cc_segment* segs, int32_t n_segs,
                            const int32_t* req_seg_off, int32_t n_requests, int32_t max_segs_per_req,
                            int32_t n_ctx_tokens, int32_t n_pairs, const cc_shared_values* shared,
                            void* out, float* lse,
                            float* seg_mass, float* pair_mass, float* self_mass,
                            void* workspace, size_t workspace_bytes, void* stream);

/* ---- (c') step 1 of cc_sparse_prefill alone --------------------------------------------------
 * Rotates k_new[j] to position q_pos[j] and writes it, with v_new[j], into physical slot
 * slot_map[j] of the pools, for j < n_rows; nothing else.  For chunks that have NO chunk-cache
 * in a batch that also reuses caches (C_miss next to C_hit, Sec. 3.4.1): their K and V are
 * computed for every token and must be in the request's pages before cc_select scores the chunks
 * behind them.  Rows whose slots lie in the same 16-token block must be adjacent, as for
 * cc_sparse_prefill.  k_new, v_new [n_rows][Hkv][d]. */
/* Check of the order cc_sparse_prefill, its variants and cc_scatter_kv rely on (they do not check
 * it themselves: two separate runs of rows in one block would be written by two workgroups that
 * each rewrite whole value rows of the block).  *n_violations (device int32) receives the number
 * of runs of adjacent rows that name a block an earlier run has named already: 0 for a list in
 * cc_select's order, or any order that keeps the rows of a block together.  Rows with a slot
 * outside the pool are ignored here as they are by the scatter.  For callers that build the list
 * themselves; read the result when convenient (the call only enqueues).
 *   workspace: cc_check_query_list_workspace_bytes(ctx, n_blocks) (one int32 per block). */
size_t cc_check_query_list_workspace_bytes(const cc_ctx* ctx, int32_t n_blocks);
int cc_check_query_list(cc_ctx* ctx, const int32_t* slot_map, int32_t n_rows, int32_t n_blocks,
                        int32_t* n_violations, void* workspace, size_t workspace_bytes, void* stream);

int cc_scatter_kv(cc_ctx* ctx, const void* k_new, const void* v_new, const int32_t* q_pos,
                  const int32_t* slot_map, int32_t n_rows, void* k_pool, void* v_pool, int32_t n_blocks,
                  void* stream);

/* ---- (d) attention between the question and every chunk -----------------------------------
 * inter(C_i, U) of this layer (Sec. 3.2.2, with the weights of Eq. (1)): for every segment s of
 * the batch, of request r,
 *   seg_mass[s] = sum over the question rows u of r of
 *                 (1/Hq) sum over query heads h of  sum_{keys l of segment s, l <= q_pos[u]} a^h_{u,l}
 * where a^h_{u,.} are the softmax weights of step 2 of cc_sparse_prefill (same q, same pools, i.e.
 * the keys after the fix) and the question rows of r are the rows of its part of the compact list
 * with q_pos >= logical_start of r's CC_SEG_QUESTION segment (none: all its masses are 0).  For
 * the question segment itself this is the mass the question keeps on its own tokens, so the masses
 * of a request's segments add up to its number of question rows.
 * Call it after cc_sparse_prefill, on the same stream, with the same q, q_pos, cu_q, pools and
 * segment arrays, and with the lse that call wrote (required here).  The masses come from a pass
 * of their own over the question rows (the attention kernels run once per (segment, question
 * rows) pair and keep only the log-sum-exp); nothing but seg_mass and the workspace is written.
 *   max_question_rows: max question rows of one request (host scalar; a request with more has
 *   only its first max_question_rows counted).  seg_mass [n_segs] float.
 *   workspace: cc_question_mass_workspace_bytes(ctx, n_ctx_tokens, n_segs, max_question_rows). */
size_t cc_question_mass_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                        int32_t max_question_rows);
int cc_question_mass(cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                     int32_t n_q_tot, int32_t max_question_rows,
                     const void* k_pool, const void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                     const cc_segment* segs, int32_t n_segs,
                     const int32_t* req_seg_off, int32_t n_requests, int32_t n_ctx_tokens,
                     const float* lse, float* seg_mass, void* workspace, size_t workspace_bytes,
                     void* stream);

/* ---- (e) attention between segments: inter and intra of Eq. (2), Eq. (3) ---------------------
 * For every request r and every pair of its segments t >= s (indices inside the request):
 *   pair_mass[pair(r, t, s)] = sum over the rows u of the compact list whose position lies in
 *       segment t of (1/Hq) sum_h sum_{keys l of segment s, l <= q_pos[u]} a^h_{u,l}
 *   pair(r, t, s) = sum_{r' < r} n_{r'} (n_{r'} + 1) / 2  +  t (t + 1) / 2 + s,  n_r = segments of r
 * and, if self_mass is not NULL, for every segment s of the batch
 *   self_mass[s] = sum over the rows u in s of (1/Hq) sum_h a^h_{u,u}   (the row's own key)
 * with a the softmax weights of step 2 of cc_sparse_prefill.  With every token of the prompt in
 * the compact list (the full prefill that creates a chunk-cache, Sec. 3.4.3 "metadata") these are
 * inter(C_s, C_t) for s < t, and intra(C_t) = pair_mass[pair(r, t, t)] - self_mass[t] (Eq. (3)
 * sums strictly earlier tokens).  With fewer rows they are the same sums over the rows present.
 * Call it after cc_sparse_prefill like cc_question_mass (same arguments, its lse; slot_map is
 * needed for self_mass only).  The masses come from a pass of their own (the attention kernels
 * once per (segment, rows that see it) pair, log-sum-exp only): about one more attention pass.
 *   n_pairs: entries of pair_mass (host scalar, = sum_r n_r (n_r + 1) / 2); all are written
 *   (0 where no row falls).  max_q_per_req as for cc_sparse_prefill.
 *   workspace: cc_chunk_attention_workspace_bytes(ctx, n_ctx_tokens, n_segs, n_q_tot, max_q_per_req). */
size_t cc_chunk_attention_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                          int32_t n_q_tot, int32_t max_q_per_req);
int cc_chunk_attention(cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* slot_map,
                       const int32_t* cu_q, int32_t n_q_tot, int32_t max_q_per_req,
                       const void* k_pool, const void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                       const cc_segment* segs, int32_t n_segs,
                       const int32_t* req_seg_off, int32_t n_requests, int32_t n_ctx_tokens,
                       int32_t n_pairs, const float* lse, float* pair_mass, float* self_mass,
                       void* workspace, size_t workspace_bytes, void* stream);

/* ---- reuse scores of a chunk-cache (host only; no GPU work, HOST pointers) --------------------
 * cc_chunk_ab: one layer's a(C_i) = sum_{j<i} inter(C_j, C_i) / (|C_i| |C_j|) and
 *   b(C_i) = intra(C_i) / |C_i|^2 from the n_prefix inter sums of the chunk's prefix chunks, their
 *   lengths, the chunk's intra sum and its length (Sec. 3.1).
 * cc_chunk_cci: CCI = 1 / (1 + exp(-abar / bbar)) with abar, bbar the means of a and b over the
 *   layers given (Sec. 3.1).  abar = 0 gives ratio 0 (CCI 0.5), bbar = 0 < abar an infinite one (1).
 * cc_chunk_reuse: for a cache of chunk C_i made behind the ordered prefix old_prefix[n_old]
 *   (chunk ids, with inter(i, j) of each in old_inter) and now wanted behind new_prefix[n_new]:
 *     beta     = sum of old_inter over chunks also in the new prefix / sum of old_inter
 *                (1 when the old sum is 0: a cache that depended on nothing has lost nothing)
 *     gamma    = D / (m (m - 1) / 2): discordant pairs of the m common chunks between the two
 *                orders, i.e. the normalised Kendall tau distance (0 when m < 2)
 *     beta_adj = beta (1 - gamma)
 *     cfo      = alpha * cci * (1 - beta_adj), clipped to [0, 1]              (Sec. 3.3)
 *     n_recompute = ceil(cfo * chunk_len) (guarded against representation noise), clipped to
 *                [0, chunk_len]                                                (Sec. 3.2.1)
 * All return CC_OK or CC_ERR_INVALID_ARG (null pointer, non-finite or negative score). */
typedef struct {
  double beta, gamma, beta_adj, cfo;
  int32_t n_recompute;
  int32_t reserved;
} cc_reuse;
int cc_chunk_ab(const double* inter, const int32_t* prefix_len, int32_t n_prefix, double intra,
                int32_t chunk_len, double* a, double* b);
int cc_chunk_cci(const double* a, const double* b, int32_t n_layers, double* cci);
int cc_chunk_reuse(const int64_t* old_prefix, const double* old_inter, int32_t n_old,
                   const int64_t* new_prefix, int32_t n_new, double cci, double alpha,
                   int32_t chunk_len, cc_reuse* out);

/* ---- layer-wise preloading of chunk-caches (Sec. 3.4.2, Eq. (12), Algorithm 2) ---------------
 * Host-side runtime: copies each layer's chunk-caches from PINNED HOST memory into a device read
 * buffer on a copy stream of the library's own (default priority), ahead of the compute stream.
 *   cc_preload_depth: L_p = max(1, ceil((L - 1) (1 - T_prefill / T_load) + 1)), at most L; 1 when
 *     T_prefill >= T_load (times in any common unit).  Negative on invalid arguments.
 *   cc_preloader_create: L layers, preloading depth L_p, and a ring of n_slots >= min(L_p + 1, L)
 *     slots in the caller's device read buffer: layer j is expected in slot j mod n_slots, and its
 *     copy waits (on the GPU) until layer j - n_slots has been released.
 *   cc_preloader_set_layer: where layer j comes from (pinned host pointer), where it goes (device
 *     pointer: the caller's slot for it) and how many bytes; before the layer's copy is enqueued.
 *   cc_preloader_acquire(layer, compute_stream): Algorithm 2's inner loop - enqueues, in layer
 *     order, every copy up to layer + L_p that is not enqueued yet - then makes compute_stream wait
 *     (hipStreamWaitEvent; the host does not block) until the layer's data has landed.
 *   cc_preloader_release(layer, compute_stream): the layer's kernels have been enqueued; its slot
 *     may be overwritten once compute_stream reaches this point.
 *   cc_preloader_issued: number of copies enqueued so far; their layer order into order[] if given.
 * Call acquire(i), enqueue layer i's work, release(i), for i = 0 .. L-1.  Nothing here allocates
 * device or pinned memory; create makes one stream and 2 L events, destroy waits for the copy
 * stream and frees them. */
typedef struct cc_preloader cc_preloader;
int32_t cc_preload_depth(int32_t n_layers, double t_prefill, double t_load);
int cc_preloader_create(cc_preloader** out, int32_t n_layers, int32_t depth, int32_t n_slots);
void cc_preloader_destroy(cc_preloader* p);
int cc_preloader_set_layer(cc_preloader* p, int32_t layer, const void* host_src, void* dev_dst, size_t bytes);
int cc_preloader_acquire(cc_preloader* p, int32_t layer, void* compute_stream);
int cc_preloader_release(cc_preloader* p, int32_t layer, void* compute_stream);
int32_t cc_preloader_issued(const cc_preloader* p, int32_t* order, int32_t capacity);

/* ---- focused chunks (host only; no GPU work, HOST pointers) --------------------------------
 * Algorithm 1 for ONE request with k chunks, fed once per layer l = 1, 2, ... with that layer's
 * inter_l(C_i, U), i < k (e.g. the request's chunk entries of cc_question_mass's seg_mass, copied
 * to the host): adds them to the cumulative scores, sorts the scores in descending order, turns
 * the k-1 gaps between neighbours into a distribution p, and keeps the top i* chunks, where i* in
 * 1..k-2 is the index that maximises h_{i+1} - h_i of the cumulative entropy h_i = -sum_{j<=i}
 * p_j log p_j (first maximum; 0 log 0 = 0; with fewer than 3 chunks, or all scores equal, every
 * chunk is kept).  focused[i] = 1 if chunk i is kept this layer, else 0; *n_focused (may be NULL)
 * their number.  Returns 1 once the kept set has been the same for the last `window` layers
 * (the caller stops recomputing the other chunks from here on: this layer is L*), 0 otherwise,
 * negative cc_status on error (null pointer, non-finite score). */
typedef struct cc_focus cc_focus;
int cc_focus_create(cc_focus** out, int32_t n_chunks, int32_t window);
void cc_focus_destroy(cc_focus* f);
int cc_focus_update(cc_focus* f, const float* inter, int32_t* focused, int32_t* n_focused);
/* number of layers fed so far (-1 for NULL) */
int32_t cc_focus_layer(const cc_focus* f);

#ifdef __cplusplus
}
#endif
#endif /* CACHECRAFT_CC_H */
