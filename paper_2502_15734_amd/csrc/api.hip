// C ABI of libcachecraft: argument checks and kernel dispatch.  See include/cc.h.
#include <cmath>
#include <cstdio>
#include <mutex>
#include <new>

#include "common.h"

namespace cc {

int fail(cc_ctx* ctx, int status, const std::string& msg) {
  if (ctx) ctx->last_error = msg;
  return status;
}

int check_launch(cc_ctx* ctx, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess)
    return fail(ctx, CC_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
  return CC_OK;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- scratch of cc_sparse_prefill_static --------------------------------------------------------
// A device array that lives in the library's code object: every GPU the library runs on holds its
// own copy, at its own address, until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; kernels and copies get the address that call returned.
static __device__ __align__(256) unsigned char scratch[CC_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void* scratch_of_device[kMaxDevices];      // resolved once per device, with that device current

// Address of the current device's scratch array (nullptr + *err set if it cannot be resolved).
static void* static_scratch(hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_of_device[dev] == nullptr) {
    void* p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess) return nullptr;
    scratch_of_device[dev] = p;
  }
  return scratch_of_device[dev];
}

}  // namespace cc

using cc::aligned16;
using cc::fail;

#define CC_REQUIRE(cond, msg)                                         \
  do {                                                                \
    if (!(cond)) return fail(ctx, CC_ERR_INVALID_ARG, std::string(fn) + ": " + (msg)); \
  } while (0)

extern "C" {

const char* cc_status_string(int status) {
  switch (status) {
    case CC_OK: return "ok";
    case CC_ERR_INVALID_ARG: return "invalid argument";
    case CC_ERR_UNSUPPORTED: return "unsupported configuration";
    case CC_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case CC_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int cc_create(cc_ctx** out, const cc_config* cfg) {
  if (out == nullptr) return CC_ERR_INVALID_ARG;
  *out = nullptr;
  if (cfg == nullptr) return CC_ERR_INVALID_ARG;
  if (cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->n_q_heads % cfg->n_kv_heads != 0 ||
      !(cfg->rope_theta > 0.0) || !std::isfinite(cfg->rope_theta))
    return CC_ERR_INVALID_ARG;
  if ((cfg->head_dim != 64 && cfg->head_dim != 128) || cfg->block_size != cc::kBlock ||
      (cfg->dtype != CC_F32 && cfg->dtype != CC_BF16) || cfg->n_q_heads > 1024)
    return CC_ERR_UNSUPPORTED;
  cc_ctx* ctx = new (std::nothrow) cc_ctx();
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  ctx->cfg = *cfg;
  ctx->impl = CC_IMPL_AUTO;
  const int half = cfg->head_dim / 2;
  for (int i = 0; i < cc::kMaxHalf; ++i)
    ctx->inv_freq.f[i] = i < half ? std::pow(cfg->rope_theta, -2.0 * i / cfg->head_dim) : 0.0;
  // The scratch array of cc_sparse_prefill_static is looked up here for the device that is current
  // now, so that the call itself finds it ready (a process without a GPU simply has none; the call
  // looks again on its first use on any other device).
  hipError_t scratch_err;
  (void)cc::static_scratch(&scratch_err);
  (void)hipGetLastError();
  *out = ctx;
  return CC_OK;
}

void cc_destroy(cc_ctx* ctx) { delete ctx; }

const char* cc_last_error(const cc_ctx* ctx) { return ctx ? ctx->last_error.c_str() : "null context"; }

int cc_set_impl(cc_ctx* ctx, int impl) {
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  if (impl != CC_IMPL_AUTO && impl != CC_IMPL_SCALAR && impl != CC_IMPL_MFMA_NARROW && impl != CC_IMPL_MFMA_WIDE)
    return fail(ctx, CC_ERR_INVALID_ARG, "cc_set_impl: unknown implementation id");
  ctx->impl = impl;
  return CC_OK;
}

static int rope_move(cc_ctx* ctx, const char* fn, bool absolute, const void* k_src_pool,
                     const void* v_src_pool, int32_t n_src_blocks, void* k_dst_pool, void* v_dst_pool,
                     int32_t n_dst_blocks, const int32_t* src_block_tab, const int32_t* dst_block_tab,
                     const cc_shift_desc* descs, int32_t n_instances, int32_t max_tokens, int32_t* v_map,
                     void* stream) {
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_instances >= 0 && max_tokens >= 0, "negative count");
  CC_REQUIRE(n_instances <= 65535, "more than 65535 chunk instances in one call");
  if (n_instances == 0 || max_tokens == 0) return CC_OK;
  CC_REQUIRE(k_src_pool && k_dst_pool && src_block_tab && dst_block_tab && descs, "null pointer");
  CC_REQUIRE((v_src_pool == nullptr) == (v_dst_pool == nullptr), "v_src_pool and v_dst_pool must both be given or both be NULL");
  CC_REQUIRE(aligned16(k_src_pool) && aligned16(k_dst_pool) && aligned16(v_src_pool) && aligned16(v_dst_pool),
             "pools must be 16-byte aligned");
  CC_REQUIRE(n_src_blocks > 0 && n_dst_blocks > 0, "pool sizes must be positive");
  CC_REQUIRE(v_map == nullptr || v_dst_pool == nullptr, "with a value map the values are not copied: pass no V pools");
  cc::launch_rope_shift(ctx, k_src_pool, v_src_pool, n_src_blocks, k_dst_pool, v_dst_pool,
                        n_dst_blocks, src_block_tab, dst_block_tab, descs, n_instances, max_tokens,
                        absolute, v_map, static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

int cc_rope_shift(cc_ctx* ctx, const void* k_src_pool, const void* v_src_pool, int32_t n_src_blocks,
                  void* k_dst_pool, void* v_dst_pool, int32_t n_dst_blocks,
                  const int32_t* src_block_tab, const int32_t* dst_block_tab,
                  const cc_shift_desc* descs, int32_t n_instances, int32_t max_tokens,
                  int32_t* v_map, void* stream) {
  return rope_move(ctx, "cc_rope_shift", false, k_src_pool, v_src_pool, n_src_blocks, k_dst_pool, v_dst_pool,
                   n_dst_blocks, src_block_tab, dst_block_tab, descs, n_instances, max_tokens, v_map, stream);
}

int cc_rope_place(cc_ctx* ctx, const void* k_src_pool, const void* v_src_pool, int32_t n_src_blocks,
                  void* k_dst_pool, void* v_dst_pool, int32_t n_dst_blocks,
                  const int32_t* src_block_tab, const int32_t* dst_block_tab,
                  const cc_shift_desc* descs, int32_t n_instances, int32_t max_tokens,
                  int32_t* v_map, void* stream) {
  return rope_move(ctx, "cc_rope_place", true, k_src_pool, v_src_pool, n_src_blocks, k_dst_pool, v_dst_pool,
                   n_dst_blocks, src_block_tab, dst_block_tab, descs, n_instances, max_tokens, v_map, stream);
}

// upper bound on the number of 64-key tiles of n_tok tokens spread over n_segs segments
static int max_tiles_for(int32_t n_tok, int32_t n_segs) { return n_tok / 64 + n_segs + 1; }

// workspace of cc_select: [mass: n_tok * Hq floats][keys: n_tok uint32][tile plan]
size_t cc_select_workspace_bytes(const cc_ctx* ctx, int32_t n_tok, int32_t n_segs) {
  if (ctx == nullptr || n_tok < 0 || n_segs < 0) return 0;
  return cc::align_up(static_cast<size_t>(n_tok) * ctx->cfg.n_q_heads * sizeof(float), 256) +
         cc::align_up(static_cast<size_t>(n_tok) * sizeof(uint32_t), 256) +
         cc::align_up(cc::mfma_plan_bytes(n_segs, max_tiles_for(n_tok, n_segs), n_tok), 256) + 256;
}

int cc_select(cc_ctx* ctx, const void* q, int32_t n_tok, const void* k_pool, int32_t n_blocks,
              const int32_t* block_tab, const cc_segment* segs, int32_t n_segs,
              const int32_t* req_seg_off, int32_t n_requests, int32_t max_seg_tokens,
              int32_t* sel_idx, int32_t* q_row, int32_t* q_pos, int32_t* slot_map, int32_t n_q_tot,
              float* scores, void* workspace, size_t workspace_bytes, void* stream) {
  static const char* fn = "cc_select";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_tok >= 0 && n_segs >= 0 && n_requests >= 0 && max_seg_tokens >= 0 && n_q_tot >= 0,
             "negative count");
  CC_REQUIRE(n_segs <= 65535, "more than 65535 segments in one call");
  if (n_segs == 0 || max_seg_tokens == 0) return CC_OK;
  CC_REQUIRE(q && k_pool && block_tab && segs && req_seg_off && sel_idx, "null pointer");
  CC_REQUIRE(n_blocks > 0 && n_requests > 0, "pool size and request count must be positive");
  CC_REQUIRE(aligned16(q) && aligned16(k_pool), "tensors must be 16-byte aligned");
  CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
  if (workspace_bytes < cc_select_workspace_bytes(ctx, n_tok, n_segs))
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL, "cc_select: workspace smaller than cc_select_workspace_bytes()");
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* mass = static_cast<float*>(workspace);
  uint32_t* keys = reinterpret_cast<uint32_t*>(
      static_cast<char*>(workspace) +
      cc::align_up(static_cast<size_t>(n_tok) * ctx->cfg.n_q_heads * sizeof(float), 256));
  void* plan_ws = reinterpret_cast<char*>(keys) + cc::align_up(static_cast<size_t>(n_tok) * sizeof(uint32_t), 256);
  if (ctx->impl != CC_IMPL_SCALAR && cc::score_mfma_supported(ctx))
    cc::launch_score_mfma(ctx, q, k_pool, n_blocks, block_tab, segs, n_segs, req_seg_off,
                          max_seg_tokens, mass, plan_ws, max_tiles_for(n_tok, n_segs), n_tok, st);
  else
    cc::launch_score_scalar(ctx, q, k_pool, n_blocks, block_tab, segs, n_segs, req_seg_off,
                            max_seg_tokens, mass, st);
  cc::launch_topn(ctx, mass, block_tab, segs, n_segs, sel_idx, q_row, q_pos, slot_map, scores, keys, false, st);
  return cc::check_launch(ctx, fn);
}

int cc_select_from_scores(cc_ctx* ctx, const float* scores, int32_t n_tok, const int32_t* block_tab,
                          const cc_segment* segs, int32_t n_segs, int32_t* sel_idx, int32_t* q_row,
                          int32_t* q_pos, int32_t* slot_map, int32_t n_q_tot, void* workspace,
                          size_t workspace_bytes, void* stream) {
  static const char* fn = "cc_select_from_scores";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_tok >= 0 && n_segs >= 0 && n_q_tot >= 0, "negative count");
  CC_REQUIRE(n_segs <= 65535, "more than 65535 segments in one call");
  if (n_segs == 0) return CC_OK;
  CC_REQUIRE(scores && block_tab && segs && sel_idx, "null pointer");
  CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
  if (workspace_bytes < cc_select_workspace_bytes(ctx, n_tok, n_segs))
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                "cc_select_from_scores: workspace smaller than cc_select_workspace_bytes()");
  // same workspace layout as cc_select: only the key buffer (chunks too long for LDS) is used
  uint32_t* keys = reinterpret_cast<uint32_t*>(
      static_cast<char*>(workspace) +
      cc::align_up(static_cast<size_t>(n_tok) * ctx->cfg.n_q_heads * sizeof(float), 256));
  cc::launch_topn(ctx, scores, block_tab, segs, n_segs, sel_idx, q_row, q_pos, slot_map, nullptr, keys, true,
                  static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

int cc_gather_rows(cc_ctx* ctx, const void* src, int32_t n_src_rows, const int32_t* row_idx,
                   int32_t n_rows, size_t row_bytes, void* dst, void* stream) {
  static const char* fn = "cc_gather_rows";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_rows >= 0 && n_src_rows >= 0, "negative count");
  if (n_rows == 0) return CC_OK;
  CC_REQUIRE(src && row_idx && dst, "null pointer");
  CC_REQUIRE(row_bytes > 0 && row_bytes % 16 == 0, "row_bytes must be a positive multiple of 16");
  CC_REQUIRE(aligned16(src) && aligned16(dst), "tensors must be 16-byte aligned");
  cc::launch_gather_rows(src, n_src_rows, row_idx, n_rows, row_bytes, dst,
                         static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

int cc_qkv_project(cc_ctx* ctx, const void* x, const void* w_qkv, int32_t n_rows, int32_t hidden,
                   void* q, void* k, void* v, void* stream) {
  static const char* fn = "cc_qkv_project";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_rows >= 0 && hidden > 0, "bad sizes");
  CC_REQUIRE(hidden % 64 == 0, "hidden must be a multiple of 64");
  if (n_rows == 0) return CC_OK;
  CC_REQUIRE(x && w_qkv && q && k && v, "null pointer");
  CC_REQUIRE(aligned16(x) && aligned16(w_qkv) && aligned16(q) && aligned16(k) && aligned16(v),
             "tensors must be 16-byte aligned");
  cc::launch_qkv_project(ctx, x, w_qkv, n_rows, hidden, q, k, v, static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

int cc_rms_norm(cc_ctx* ctx, const void* x, const void* gain, float eps, int32_t n_rows, int32_t hidden,
                void* y, void* stream) {
  static const char* fn = "cc_rms_norm";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_rows >= 0 && hidden > 0, "bad sizes");
  CC_REQUIRE(eps >= 0.f && eps == eps, "eps must not be negative");
  CC_REQUIRE(hidden % (ctx->cfg.dtype == CC_BF16 ? 8 : 4) == 0, "hidden must be a multiple of 16 bytes of elements");
  if (n_rows == 0) return CC_OK;
  CC_REQUIRE(x && gain && y, "null pointer");
  CC_REQUIRE(aligned16(x) && aligned16(gain) && aligned16(y), "tensors must be 16-byte aligned");
  cc::launch_rms_norm(ctx, x, gain, eps, n_rows, hidden, y, static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

int cc_linear(cc_ctx* ctx, const void* x, const void* w, const void* residual, int32_t n_rows,
              int32_t n_in, int32_t n_out, void* y, void* stream) {
  static const char* fn = "cc_linear";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_rows >= 0 && n_in > 0 && n_out > 0, "bad sizes");
  if (n_rows == 0) return CC_OK;
  CC_REQUIRE(x && w && y, "null pointer");
  CC_REQUIRE(x != y, "x and y must not be the same tensor");
  CC_REQUIRE(aligned16(x) && aligned16(w) && aligned16(y) && aligned16(residual), "tensors must be 16-byte aligned");
  cc::launch_linear(ctx, x, w, residual, n_rows, n_in, n_out, y, static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

int cc_gated_linear(cc_ctx* ctx, const void* x, const void* w_gate, const void* w_up, int32_t n_rows,
                    int32_t n_in, int32_t n_ffn, void* y, void* stream) {
  static const char* fn = "cc_gated_linear";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_rows >= 0 && n_in > 0 && n_ffn > 0, "bad sizes");
  if (n_rows == 0) return CC_OK;
  CC_REQUIRE(x && w_gate && w_up && y, "null pointer");
  CC_REQUIRE(x != y, "x and y must not be the same tensor");
  CC_REQUIRE(aligned16(x) && aligned16(w_gate) && aligned16(w_up) && aligned16(y), "tensors must be 16-byte aligned");
  cc::launch_gated_linear(ctx, x, w_gate, w_up, n_rows, n_in, n_ffn, y, static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

// the caller's cc_shared_values (or NULL) as the launchers take it; false (error recorded) if it is malformed
static bool value_source(cc_ctx* ctx, const char* fn, const cc_shared_values* shared, cc::ValueSource* vs) {
  *vs = cc::ValueSource();
  if (shared == nullptr) return true;
  if (shared->v_shared == nullptr || shared->v_map == nullptr || shared->n_shared_blocks <= 0 ||
      !aligned16(shared->v_shared)) {
    fail(ctx, CC_ERR_INVALID_ARG, std::string(fn) + ": shared values need a 16-byte aligned pool, its size in blocks and a value map");
    return false;
  }
  vs->v_shared = shared->v_shared;
  vs->n_shared_blocks = shared->n_shared_blocks;
  vs->v_map = shared->v_map;
  return true;
}

size_t cc_sparse_prefill_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs) {
  if (ctx == nullptr || n_ctx_tokens < 0 || n_segs < 0) return 0;
  // queries are a subset of the context tokens, so n_ctx_tokens bounds the rows of the compact list
  return cc::align_up(cc::mfma_plan_bytes(n_segs, max_tiles_for(n_ctx_tokens, n_segs), n_ctx_tokens), 256) + 256;
}

int cc_sparse_prefill(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                      const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                      const int32_t* cu_q, int32_t n_q_tot, int32_t max_q_per_req, void* k_pool, void* v_pool,
                      int32_t n_blocks, const int32_t* block_tab, const cc_segment* segs,
                      int32_t n_segs, const int32_t* req_seg_off, int32_t n_requests,
                      int32_t n_ctx_tokens, const cc_shared_values* shared, void* out, float* lse,
                      void* workspace, size_t workspace_bytes, void* stream) {
  static const char* fn = "cc_sparse_prefill";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_q_tot >= 0 && max_q_per_req >= 0 && n_segs >= 0 && n_requests >= 0 && n_ctx_tokens >= 0,
             "negative count");
  CC_REQUIRE(max_q_per_req <= n_q_tot, "max_q_per_req exceeds n_q_tot");
  if (n_q_tot == 0) return CC_OK;
  CC_REQUIRE(n_q_tot <= n_ctx_tokens, "n_ctx_tokens must bound the rows of the compact list");
  CC_REQUIRE(q && k_new && v_new && q_pos && slot_map && cu_q && k_pool && v_pool && block_tab &&
                 segs && req_seg_off && out, "null pointer");
  CC_REQUIRE(n_blocks > 0 && n_requests > 0 && n_segs > 0 && max_q_per_req > 0, "sizes must be positive");
  CC_REQUIRE(n_requests <= 65535, "more than 65535 requests in one call");
  CC_REQUIRE(n_requests <= n_segs, "every request needs at least one segment");
  CC_REQUIRE(aligned16(q) && aligned16(k_new) && aligned16(v_new) && aligned16(k_pool) &&
                 aligned16(v_pool) && aligned16(out), "tensors must be 16-byte aligned");
  CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
  if (workspace_bytes < cc_sparse_prefill_workspace_bytes(ctx, n_ctx_tokens, n_segs))
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                "cc_sparse_prefill: workspace smaller than cc_sparse_prefill_workspace_bytes()");
  cc::ValueSource vs;
  if (!value_source(ctx, fn, shared, &vs)) return CC_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  cc::launch_rope_scatter(ctx, k_new, v_new, q_pos, slot_map, n_q_tot, k_pool, v_pool, n_blocks, src_rows, st, vs);
  if (ctx->impl != CC_IMPL_SCALAR && cc::attn_mfma_supported(ctx))
    cc::launch_attn_mfma(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks,
                         block_tab, segs, n_segs, req_seg_off, n_requests, out, lse, workspace,
                         max_tiles_for(n_ctx_tokens, n_segs), src_rows, 0, st, nullptr, vs);
  else
    cc::launch_attn_scalar(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks,
                           block_tab, segs, req_seg_off, n_requests, out, lse, src_rows, 0, st, vs);
  return cc::check_launch(ctx, fn);
}

int cc_sparse_prefill_static(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                             const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                             const int32_t* cu_q, int32_t n_q_tot, int32_t max_q_per_req, void* k_pool,
                             void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                             const cc_segment* segs, int32_t n_segs, const int32_t* req_seg_off,
                             int32_t n_requests, int32_t n_ctx_tokens, const cc_shared_values* shared,
                             void* out, float* lse, void* stream) {
  static const char* fn = "cc_sparse_prefill_static";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_ctx_tokens >= 0 && n_segs >= 0, "negative count");
  const size_t need = cc_sparse_prefill_workspace_bytes(ctx, n_ctx_tokens, n_segs);
  if (need > CC_STATIC_SCRATCH_BYTES)
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                "cc_sparse_prefill_static: the key-tile plan of this batch needs " + std::to_string(need) +
                    " bytes, the built-in scratch holds " + std::to_string(CC_STATIC_SCRATCH_BYTES) +
                    " (use cc_sparse_prefill with a workspace)");
  if (n_q_tot == 0) return CC_OK;
  hipError_t err = hipSuccess;
  void* ws = cc::static_scratch(&err);
  if (ws == nullptr)
    return fail(ctx, CC_ERR_HIP, std::string("cc_sparse_prefill_static: scratch array not available: ") +
                                     hipGetErrorString(err));
  // (the plan kernels rewrite every part of the scratch the attention kernels read, including the
  // flags that must start at zero, so nothing of an earlier call survives into this one)
  return cc_sparse_prefill(ctx, q, k_new, v_new, src_rows, q_pos, slot_map, cu_q, n_q_tot, max_q_per_req, k_pool,
                           v_pool, n_blocks, block_tab, segs, n_segs, req_seg_off, n_requests, n_ctx_tokens, shared,
                           out, lse, ws, CC_STATIC_SCRATCH_BYTES, stream);
}

size_t cc_sparse_prefill_mass_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                              int32_t n_requests, int32_t max_question_rows,
                                              int32_t max_segs_per_req) {
  if (ctx == nullptr || n_ctx_tokens < 0 || n_segs < 0 || n_requests < 0 || max_question_rows < 0 ||
      max_segs_per_req < 0)
    return 0;
  return cc::prefill_mass_bytes(ctx, n_ctx_tokens, n_segs, n_requests, max_tiles_for(n_ctx_tokens, n_segs),
                                max_question_rows, max_segs_per_req) + 256;
}

int cc_sparse_prefill_mass(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                           const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map, const int32_t* cu_q,
                           int32_t n_q_tot, int32_t max_q_per_req, int32_t max_question_rows,
                           void* k_pool, void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                           const cc_segment* segs, int32_t n_segs, const int32_t* req_seg_off,
                           int32_t n_requests, int32_t max_segs_per_req, int32_t n_ctx_tokens,
                           const cc_shared_values* shared, void* out,
                           float* lse, float* seg_mass, void* workspace, size_t workspace_bytes,
                           void* stream) {
  static const char* fn = "cc_sparse_prefill_mass";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_q_tot >= 0 && max_q_per_req >= 0 && n_segs >= 0 && n_requests >= 0 && n_ctx_tokens >= 0 &&
                 max_question_rows >= 0 && max_segs_per_req >= 0, "negative count");
  CC_REQUIRE(max_q_per_req <= n_q_tot && max_question_rows <= max_q_per_req, "row bounds are inconsistent");
  if (n_segs == 0) return CC_OK;
  CC_REQUIRE(seg_mass != nullptr, "null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (n_q_tot == 0) {
    cc::launch_fill_zero(seg_mass, n_segs, st);
    return cc::check_launch(ctx, fn);
  }
  CC_REQUIRE(q && k_new && v_new && q_pos && slot_map && cu_q && k_pool && v_pool && block_tab &&
                 segs && req_seg_off && out && lse, "null pointer (lse is required here)");
  CC_REQUIRE(n_blocks > 0 && n_requests > 0 && max_q_per_req > 0 && max_segs_per_req > 0, "sizes must be positive");
  CC_REQUIRE(n_requests <= 65535 && n_segs <= 65535, "more than 65535 requests or segments in one call");
  CC_REQUIRE(n_requests <= n_segs, "every request needs at least one segment");
  CC_REQUIRE(n_q_tot <= n_ctx_tokens, "n_ctx_tokens must bound the rows of the compact list");
  CC_REQUIRE(static_cast<int64_t>(n_segs) * max_question_rows <= 0x3fffffff, "n_segs * max_question_rows too large");
  CC_REQUIRE(aligned16(q) && aligned16(k_new) && aligned16(v_new) && aligned16(k_pool) &&
                 aligned16(v_pool) && aligned16(out), "tensors must be 16-byte aligned");
  CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
  if (workspace_bytes < cc_sparse_prefill_mass_workspace_bytes(ctx, n_ctx_tokens, n_segs, n_requests,
                                                               max_question_rows, max_segs_per_req))
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                "cc_sparse_prefill_mass: workspace smaller than cc_sparse_prefill_mass_workspace_bytes()");
  cc::ValueSource vs;
  if (!value_source(ctx, fn, shared, &vs)) return CC_ERR_INVALID_ARG;
  cc::launch_rope_scatter(ctx, k_new, v_new, q_pos, slot_map, n_q_tot, k_pool, v_pool, n_blocks, src_rows, st, vs);
  if (max_question_rows == 0) {                               // no question rows: plain attention, zero masses
    if (ctx->impl != CC_IMPL_SCALAR && cc::attn_mfma_supported(ctx))
      cc::launch_attn_mfma(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks, block_tab,
                           segs, n_segs, req_seg_off, n_requests, out, lse, workspace,
                           max_tiles_for(n_ctx_tokens, n_segs), src_rows, 0, st, nullptr, vs);
    else
      cc::launch_attn_scalar(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks, block_tab,
                             segs, req_seg_off, n_requests, out, lse, src_rows, 0, st, vs);
    cc::launch_fill_zero(seg_mass, n_segs, st);
    return cc::check_launch(ctx, fn);
  }
  cc::launch_prefill_mass(ctx, q, src_rows, q_pos, cu_q, n_q_tot, max_q_per_req, max_question_rows, max_segs_per_req,
                          k_pool, v_pool, n_blocks, block_tab, segs, n_segs, req_seg_off, n_requests,
                          n_ctx_tokens, out, lse, seg_mass, workspace, max_tiles_for(n_ctx_tokens, n_segs), st, vs);
  return cc::check_launch(ctx, fn);
}

size_t cc_sparse_prefill_pairs_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                               int32_t n_q_tot, int32_t max_q_per_req,
                                               int32_t max_segs_per_req) {
  if (ctx == nullptr || n_ctx_tokens < 0 || n_segs < 0 || n_q_tot < 0 || max_q_per_req < 0 || max_segs_per_req < 0)
    return 0;
  return cc::prefill_pairs_bytes(ctx, n_ctx_tokens, n_segs, max_tiles_for(n_ctx_tokens, n_segs), n_q_tot,
                                 max_q_per_req, max_segs_per_req) + 256;
}

int cc_sparse_prefill_pairs(cc_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                            const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map, const int32_t* cu_q,
                            int32_t n_q_tot, int32_t max_q_per_req, void* k_pool, void* v_pool,
                            int32_t n_blocks, const int32_t* block_tab, const cc_segment* segs,
                            int32_t n_segs, const int32_t* req_seg_off, int32_t n_requests,
                            int32_t max_segs_per_req, int32_t n_ctx_tokens, int32_t n_pairs,
                            const cc_shared_values* shared, void* out,
                            float* lse, float* seg_mass, float* pair_mass, float* self_mass,
                            void* workspace, size_t workspace_bytes, void* stream) {
  static const char* fn = "cc_sparse_prefill_pairs";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_q_tot >= 0 && max_q_per_req >= 0 && n_segs >= 0 && n_requests >= 0 && n_ctx_tokens >= 0 &&
                 max_segs_per_req >= 0 && n_pairs >= 0, "negative count");
  CC_REQUIRE(max_q_per_req <= n_q_tot, "row bounds are inconsistent");
  if (n_segs == 0) return CC_OK;
  CC_REQUIRE(pair_mass != nullptr && self_mass != nullptr, "null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (n_q_tot == 0) {
    if (n_pairs > 0) cc::launch_fill_zero(pair_mass, n_pairs, st);
    cc::launch_fill_zero(self_mass, n_segs, st);
    if (seg_mass != nullptr) cc::launch_fill_zero(seg_mass, n_segs, st);
    return cc::check_launch(ctx, fn);
  }
  CC_REQUIRE(q && k_new && v_new && q_pos && slot_map && cu_q && k_pool && v_pool && block_tab &&
                 segs && req_seg_off && out && lse, "null pointer (lse is required here)");
  CC_REQUIRE(n_blocks > 0 && n_requests > 0 && max_q_per_req > 0 && max_segs_per_req > 0 && n_pairs > 0,
             "sizes must be positive");
  CC_REQUIRE(n_requests <= 65535 && n_segs <= 65535, "more than 65535 requests or segments in one call");
  CC_REQUIRE(n_requests <= n_segs, "every request needs at least one segment");
  CC_REQUIRE(n_q_tot <= n_ctx_tokens, "n_ctx_tokens must bound the rows of the compact list");
  CC_REQUIRE(static_cast<int64_t>(n_segs) * max_q_per_req <= 0x3fffffff, "n_segs * max_q_per_req too large");
  CC_REQUIRE(n_pairs >= n_segs, "n_pairs is smaller than the number of segments");
  CC_REQUIRE(aligned16(q) && aligned16(k_new) && aligned16(v_new) && aligned16(k_pool) &&
                 aligned16(v_pool) && aligned16(out), "tensors must be 16-byte aligned");
  CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
  if (workspace_bytes < cc_sparse_prefill_pairs_workspace_bytes(ctx, n_ctx_tokens, n_segs, n_q_tot,
                                                                max_q_per_req, max_segs_per_req))
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                "cc_sparse_prefill_pairs: workspace smaller than cc_sparse_prefill_pairs_workspace_bytes()");
  cc::ValueSource vs;
  if (!value_source(ctx, fn, shared, &vs)) return CC_ERR_INVALID_ARG;
  cc::launch_rope_scatter(ctx, k_new, v_new, q_pos, slot_map, n_q_tot, k_pool, v_pool, n_blocks, src_rows, st, vs);
  cc::launch_fill_zero(pair_mass, n_pairs, st);               // pairs no row of the list falls into stay 0
  cc::launch_prefill_pairs(ctx, q, src_rows, q_pos, slot_map, cu_q, n_q_tot, max_q_per_req, max_segs_per_req, k_pool,
                           v_pool, n_blocks, block_tab, segs, n_segs, req_seg_off, n_requests, n_ctx_tokens,
                           out, lse, seg_mass, pair_mass, n_pairs, self_mass, workspace,
                           max_tiles_for(n_ctx_tokens, n_segs), st, vs);
  return cc::check_launch(ctx, fn);
}

int cc_scatter_kv(cc_ctx* ctx, const void* k_new, const void* v_new, const int32_t* q_pos,
                  const int32_t* slot_map, int32_t n_rows, void* k_pool, void* v_pool, int32_t n_blocks,
                  void* stream) {
  static const char* fn = "cc_scatter_kv";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_rows >= 0, "negative count");
  if (n_rows == 0) return CC_OK;
  CC_REQUIRE(k_new && v_new && q_pos && slot_map && k_pool && v_pool, "null pointer");
  CC_REQUIRE(n_blocks > 0, "sizes must be positive");
  CC_REQUIRE(aligned16(k_new) && aligned16(v_new) && aligned16(k_pool) && aligned16(v_pool),
             "tensors must be 16-byte aligned");
  cc::launch_rope_scatter(ctx, k_new, v_new, q_pos, slot_map, n_rows, k_pool, v_pool, n_blocks, nullptr,
                          static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

size_t cc_check_query_list_workspace_bytes(const cc_ctx* ctx, int32_t n_blocks) {
  if (ctx == nullptr || n_blocks < 0) return 0;
  return cc::align_up(static_cast<size_t>(n_blocks) * sizeof(int32_t), 256) + 256;
}

int cc_check_query_list(cc_ctx* ctx, const int32_t* slot_map, int32_t n_rows, int32_t n_blocks,
                        int32_t* n_violations, void* workspace, size_t workspace_bytes, void* stream) {
  static const char* fn = "cc_check_query_list";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_rows >= 0 && n_blocks > 0, "negative count or empty pool");
  CC_REQUIRE(n_violations != nullptr && (slot_map != nullptr || n_rows == 0), "null pointer");
  CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
  if (workspace_bytes < cc_check_query_list_workspace_bytes(ctx, n_blocks))
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                "cc_check_query_list: workspace smaller than cc_check_query_list_workspace_bytes()");
  cc::launch_list_order_check(slot_map, n_rows, n_blocks, static_cast<int32_t*>(workspace), n_violations,
                              static_cast<hipStream_t>(stream));
  return cc::check_launch(ctx, fn);
}

size_t cc_question_mass_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                        int32_t max_question_rows) {
  if (ctx == nullptr || n_ctx_tokens < 0 || n_segs < 0 || max_question_rows < 0) return 0;
  return cc::segment_mass_bytes(ctx, n_segs, max_tiles_for(n_ctx_tokens, n_segs), max_question_rows, 0) + 256;
}

int cc_question_mass(cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                     int32_t n_q_tot, int32_t max_question_rows, const void* k_pool, const void* v_pool,
                     int32_t n_blocks, const int32_t* block_tab, const cc_segment* segs, int32_t n_segs,
                     const int32_t* req_seg_off, int32_t n_requests, int32_t n_ctx_tokens,
                     const float* lse, float* seg_mass, void* workspace, size_t workspace_bytes,
                     void* stream) {
  static const char* fn = "cc_question_mass";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_q_tot >= 0 && max_question_rows >= 0 && n_segs >= 0 && n_requests >= 0 && n_ctx_tokens >= 0,
             "negative count");
  CC_REQUIRE(max_question_rows <= n_q_tot, "max_question_rows exceeds n_q_tot");
  if (n_segs == 0) return CC_OK;
  CC_REQUIRE(seg_mass != nullptr, "null pointer");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (n_q_tot == 0 || max_question_rows == 0) {          // no question rows: every mass is zero
    cc::launch_fill_zero(seg_mass, n_segs, st);
    return cc::check_launch(ctx, fn);
  }
  CC_REQUIRE(q && q_pos && cu_q && k_pool && v_pool && block_tab && segs && req_seg_off && lse, "null pointer");
  CC_REQUIRE(n_blocks > 0 && n_requests > 0, "sizes must be positive");
  CC_REQUIRE(n_segs <= 65535, "more than 65535 segments in one call");
  CC_REQUIRE(n_requests <= n_segs, "every request needs at least one segment");
  CC_REQUIRE(static_cast<int64_t>(n_segs) * max_question_rows <= 0x3fffffff, "n_segs * max_question_rows too large");
  CC_REQUIRE(aligned16(q) && aligned16(k_pool) && aligned16(v_pool), "tensors must be 16-byte aligned");
  CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
  if (workspace_bytes < cc_question_mass_workspace_bytes(ctx, n_ctx_tokens, n_segs, max_question_rows))
    return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                "cc_question_mass: workspace smaller than cc_question_mass_workspace_bytes()");
  cc::launch_question_mass(ctx, q, nullptr, q_pos, cu_q, max_question_rows, k_pool, v_pool, n_blocks, block_tab, segs,
                           n_segs, req_seg_off, n_requests, lse, seg_mass, workspace,
                           max_tiles_for(n_ctx_tokens, n_segs), st);
  return cc::check_launch(ctx, fn);
}

size_t cc_chunk_attention_workspace_bytes(const cc_ctx* ctx, int32_t n_ctx_tokens, int32_t n_segs,
                                          int32_t n_q_tot, int32_t max_q_per_req) {
  if (ctx == nullptr || n_ctx_tokens < 0 || n_segs < 0 || n_q_tot < 0 || max_q_per_req < 0) return 0;
  return cc::segment_mass_bytes(ctx, n_segs, max_tiles_for(n_ctx_tokens, n_segs), max_q_per_req, n_q_tot) + 256;
}

int cc_chunk_attention(cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* slot_map,
                       const int32_t* cu_q, int32_t n_q_tot, int32_t max_q_per_req, const void* k_pool,
                       const void* v_pool, int32_t n_blocks, const int32_t* block_tab,
                       const cc_segment* segs, int32_t n_segs, const int32_t* req_seg_off,
                       int32_t n_requests, int32_t n_ctx_tokens, int32_t n_pairs, const float* lse,
                       float* pair_mass, float* self_mass, void* workspace, size_t workspace_bytes,
                       void* stream) {
  static const char* fn = "cc_chunk_attention";
  if (ctx == nullptr) return CC_ERR_INVALID_ARG;
  CC_REQUIRE(n_q_tot >= 0 && max_q_per_req >= 0 && n_segs >= 0 && n_requests >= 0 && n_ctx_tokens >= 0 &&
                 n_pairs >= 0, "negative count");
  CC_REQUIRE(max_q_per_req <= n_q_tot, "max_q_per_req exceeds n_q_tot");
  if (n_segs == 0 || n_pairs == 0) return CC_OK;
  CC_REQUIRE(pair_mass != nullptr, "null pointer");
  CC_REQUIRE(n_pairs >= n_segs, "n_pairs is smaller than the number of segments");
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (n_q_tot > 0) {
    CC_REQUIRE(q && q_pos && cu_q && k_pool && v_pool && block_tab && segs && req_seg_off && lse, "null pointer");
    CC_REQUIRE(self_mass == nullptr || slot_map != nullptr, "self_mass needs slot_map");
    CC_REQUIRE(n_blocks > 0 && n_requests > 0 && max_q_per_req > 0, "sizes must be positive");
    CC_REQUIRE(n_segs <= 65535, "more than 65535 segments in one call");
    CC_REQUIRE(n_requests <= n_segs, "every request needs at least one segment");
    CC_REQUIRE(static_cast<int64_t>(n_segs) * max_q_per_req <= 0x3fffffff, "n_segs * max_q_per_req too large");
    CC_REQUIRE(aligned16(q) && aligned16(k_pool) && aligned16(v_pool), "tensors must be 16-byte aligned");
    CC_REQUIRE(workspace != nullptr && aligned16(workspace), "workspace missing or misaligned");
    if (workspace_bytes < cc_chunk_attention_workspace_bytes(ctx, n_ctx_tokens, n_segs, n_q_tot, max_q_per_req))
      return fail(ctx, CC_ERR_WORKSPACE_TOO_SMALL,
                  "cc_chunk_attention: workspace smaller than cc_chunk_attention_workspace_bytes()");
  }
  cc::launch_fill_zero(pair_mass, n_pairs, st);             // pairs no row of the list falls into stay 0
  if (self_mass != nullptr) cc::launch_fill_zero(self_mass, n_segs, st);
  if (n_q_tot == 0) return cc::check_launch(ctx, fn);
  cc::launch_chunk_attention(ctx, q, nullptr, q_pos, slot_map, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks,
                             block_tab, segs, n_segs, req_seg_off, n_requests, lse, pair_mass, n_pairs, self_mass,
                             workspace, max_tiles_for(n_ctx_tokens, n_segs), st);
  return cc::check_launch(ctx, fn);
}

}  // extern "C"
