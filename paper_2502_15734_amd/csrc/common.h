// Shared declarations of libcachecraft's translation units (host + gfx950 device code).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>

#include "cc.h"

namespace cc {

constexpr int kBlock = 16;        // tokens per KV block (Sec. 4, chunk storage management)
constexpr int kMaxHalf = 64;      // d/2 for the largest supported head_dim (128)

// Rotation frequencies theta^(-2i/d), computed once on the host in fp64 and passed by value
// as a kernel argument (512 bytes), so no device table has to be allocated.
struct InvFreq {
  double f[kMaxHalf];
};

}  // namespace cc

struct cc_ctx {
  cc_config cfg;
  cc::InvFreq inv_freq;
  int impl;
  std::string last_error;
};

namespace cc {

int fail(cc_ctx* ctx, int status, const std::string& msg);
int check_launch(cc_ctx* ctx, const char* what);
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Values that were not copied into the request's pages (copy-on-write, cc_shared_values): while
// v_map[b] >= 0 the values of the page whose keys sit in block b of k_pool are those of block
// v_map[b] of v_shared; otherwise they are in block b of v_pool.  v_map == NULL: always v_pool.
struct ValueSource {
  const void* v_shared = nullptr;
  int n_shared_blocks = 0;
  int32_t* v_map = nullptr;
};

// ---- launchers implemented in the .hip files -------------------------------------------------
void launch_rope_shift(const cc_ctx* ctx, const void* k_src, const void* v_src, int n_src_blocks,
                       void* k_dst, void* v_dst, int n_dst_blocks, const int32_t* src_tab,
                       const int32_t* dst_tab, const cc_shift_desc* descs, int n_instances,
                       int max_tokens, bool absolute, int32_t* v_map, hipStream_t stream);

void launch_gather_rows(const void* src, int n_src_rows, const int32_t* row_idx, int n_rows,
                        size_t row_bytes, void* dst, hipStream_t stream);

// scores: per (token, query head) prior-chunk mass -> mass [n_tok][Hq] fp32
void launch_score_scalar(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks,
                         const int32_t* block_tab, const cc_segment* segs, int n_segs,
                         const int32_t* req_seg_off, int max_seg_tokens, float* mass,
                         hipStream_t stream);
bool score_mfma_supported(const cc_ctx* ctx);
// bytes of the tile plan (per-segment tile offsets + tile descriptors, and the redo flags of up to
// n_q_max query rows) the MFMA kernels need
size_t mfma_plan_bytes(int n_segs, int max_tiles, int n_q_max);
void launch_score_mfma(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks,
                       const int32_t* block_tab, const cc_segment* segs, int n_segs,
                       const int32_t* req_seg_off, int max_seg_tokens, float* mass,
                       void* plan_ws, int max_tiles, int n_tok, hipStream_t stream);
// given = false: mass [n_tok][Hq], score = mean over heads (0 for a chunk at position 0);
// given = true: mass [n_tok] are the scores themselves
void launch_topn(const cc_ctx* ctx, const float* mass, const int32_t* block_tab,
                 const cc_segment* segs, int n_segs, int32_t* sel_idx, int32_t* q_row,
                 int32_t* q_pos, int32_t* slot_map, float* scores, uint32_t* key_buf,
                 bool given, hipStream_t stream);

void launch_rope_scatter(const cc_ctx* ctx, const void* k_new, const void* v_new,
                         const int32_t* q_pos, const int32_t* slot_map, int n_q_tot, void* k_pool,
                         void* v_pool, int n_blocks, const int32_t* src_rows, hipStream_t stream,
                         const ValueSource& vs = ValueSource());
void launch_list_order_check(const int32_t* slot_map, int n_rows, int n_blocks, int32_t* mark,
                             int32_t* n_violations, hipStream_t stream);
void launch_attn_scalar(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                        int n_q_tot, int max_q_per_req, const void* k_pool, const void* v_pool,
                        int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                        const int32_t* req_seg_off, int n_requests, void* out, float* lse,
                        const int32_t* q_map, int map_pos, hipStream_t stream,
                        const ValueSource& vs = ValueSource());
bool attn_mfma_supported(const cc_ctx* ctx);
// By-product of the attention launch (optional): for rows with snap_index >= 0 the wide kernel
// writes cum[snap row][head][segment's index in its request] = log-sum-exp over all keys up to the
// end of that segment.  On return `wide` says whether the wide kernel ran at all (else nothing was
// written) and `redo` points at its per-tile flags (rows it left to the narrow kernel).
struct AttnByProduct {
  const int32_t* snap_index;
  float* cum;
  int s_max;
  mutable bool wide;
  mutable const int32_t* redo;
};
void launch_attn_mfma(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                      int n_q_tot, int max_q_per_req, const void* k_pool, const void* v_pool,
                      int n_blocks, const int32_t* block_tab, const cc_segment* segs, int n_segs,
                      const int32_t* req_seg_off, int n_requests, void* out, float* lse,
                      void* plan_ws, int max_tiles, const int32_t* q_map, int map_pos, hipStream_t stream,
                      const AttnByProduct* by = nullptr, const ValueSource& vs = ValueSource());

// attention mass of the question rows on every segment (focus.hip)
void launch_fill_zero(float* p, int n, hipStream_t stream);
// n_q_tot_self: rows of the compact list when the self weights are wanted too (else 0)
size_t segment_mass_bytes(const cc_ctx* ctx, int n_segs, int max_tiles, int max_rows, int n_q_tot_self);
// (src_rows, where given: list row j reads row src_rows[j] of q; NULL: q is compact)
void launch_chunk_attention(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                            const int32_t* cu_q, int n_q_tot, int max_q_per_req, const void* k_pool,
                            const void* v_pool, int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                            int n_segs, const int32_t* req_seg_off, int n_requests, const float* lse,
                            float* pair_mass, int n_pairs, float* self_mass, void* workspace, int max_tiles,
                            hipStream_t stream);
void launch_question_mass(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* cu_q,
                          int max_question_rows, const void* k_pool, const void* v_pool, int n_blocks,
                          const int32_t* block_tab, const cc_segment* segs, int n_segs,
                          const int32_t* req_seg_off, int n_requests, const float* lse, float* seg_mass,
                          void* workspace, int max_tiles, hipStream_t stream);

// cc_sparse_prefill's attention with the question's per-segment masses as a by-product where the
// kernels can give it (focus.hip)
size_t prefill_mass_bytes(const cc_ctx* ctx, int n_ctx_tokens, int n_segs, int n_requests, int max_tiles,
                          int max_question_rows, int s_max);
void launch_prefill_mass(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* cu_q,
                         int n_q_tot, int max_q_per_req, int max_question_rows, int s_max, const void* k_pool,
                         const void* v_pool, int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                         int n_segs, const int32_t* req_seg_off, int n_requests, int n_ctx_tokens, void* out,
                         float* lse, float* seg_mass, void* workspace, int max_tiles, hipStream_t stream,
                         const ValueSource& vs = ValueSource());

// ... and with the whole segment-to-segment matrix (every row's cumulative sums are kept)
size_t prefill_pairs_bytes(const cc_ctx* ctx, int n_ctx_tokens, int n_segs, int max_tiles, int n_q_tot,
                           int max_q_per_req, int s_max);
void launch_prefill_pairs(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                          const int32_t* cu_q, int n_q_tot, int max_q_per_req, int s_max, const void* k_pool,
                          const void* v_pool, int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                          int n_segs, const int32_t* req_seg_off, int n_requests, int n_ctx_tokens, void* out,
                          float* lse, float* seg_mass, float* pair_mass, int n_pairs, float* self_mass,
                          void* workspace, int max_tiles, hipStream_t stream,
                          const ValueSource& vs = ValueSource());

// attention for head groups that are a multiple of 4: 64 query rows per wavefront (attn_mfma2.hip)
bool attn_v2_supported(const cc_ctx* ctx);
// score stage for the same head groups: 128 tokens per wavefront (score_mfma2.hip)
bool score_v2_supported(const cc_ctx* ctx);

void launch_qkv_project(const cc_ctx* ctx, const void* x, const void* w, int n_rows, int hidden,
                        void* q, void* k, void* v, hipStream_t stream);
// the other dense products of a decoder layer, for the recomputed rows (Sec. 2.1, Sec. 3.4.3)
void launch_linear(const cc_ctx* ctx, const void* x, const void* w, const void* residual, int n_rows, int n_in,
                   int n_out, void* y, hipStream_t stream);
void launch_gated_linear(const cc_ctx* ctx, const void* x, const void* w_gate, const void* w_up, int n_rows,
                         int n_in, int n_ffn, void* y, hipStream_t stream);
void launch_rms_norm(const cc_ctx* ctx, const void* x, const void* gain, float eps, int n_rows, int hidden, void* y,
                     hipStream_t stream);

}  // namespace cc
