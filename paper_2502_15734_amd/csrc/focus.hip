// Attention the question pays to each chunk, inter(C_i, U) of one layer, and the prediction of the
// "focused" chunks from it (Sec. 3.2.2, Algorithm 1).
//
// Device part.  The mass a question row u puts on segment s is exp(lse_s(u) - lse(u)): lse(u) is
// the log-sum-exp over every key the row sees (cc_sparse_prefill's output), lse_s(u) the one over
// the keys of segment s alone.  lse_s comes from the same attention kernels run on a list of
// "one-segment requests": entry s of the list is segment s of the batch with the question rows
// of its request as queries.  A row map tells the kernels which row of q each list row reads, so
// nothing is copied; they are given no output tensor, only the log-sum-exp.  Three small kernels
// build the list (question rows per request, offsets per segment, the row map), one reduces
// exp(lse_s - lse) over rows and heads in a fixed order.
//
// Host part.  Algorithm 1: per-chunk cumulative scores over the layers, a split of the sorted
// scores at the gap with the largest entropy term, and a stop once the chosen set has not changed
// for w layers.
#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "device_util.h"

namespace cc {

namespace {

constexpr int kNoQuestion = 0x7fffffff;

// logical position of the first question token of request r (kNoQuestion if it has none)
__device__ __forceinline__ int question_start(const cc_segment* __restrict__ segs,
                                              const int32_t* __restrict__ req_seg_off, int r) {
  int qs = kNoQuestion;
  for (int s = req_seg_off[r]; s < req_seg_off[r + 1]; ++s)
    if (segs[s].kind == CC_SEG_QUESTION) qs = min(qs, segs[s].logical_start);
  return qs;
}

// inclusive scan of one int per thread over a 256-thread workgroup; *total gets the sum
__device__ __forceinline__ int block_scan_256(int v, int* total) {
  __shared__ int wsum[4];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int t = __shfl_up(incl, o, 64);
    if (lane >= o) incl += t;
  }
  __syncthreads();                       // (wsum may still be read from the previous call)
  if (lane == 63) wsum[w] = incl;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (i < w) before += wsum[i];
    all += wsum[i];
  }
  *total = all;
  return incl + before;
}

// m_req[r] = number of rows of request r at question positions (at most max_rows are kept)
__global__ __launch_bounds__(256) void question_count_kernel(
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int max_rows,
    int32_t* __restrict__ m_req) {
  const int r = blockIdx.x;
  const int qs = question_start(segs, req_seg_off, r);
  int cnt = 0;
  for (int j0 = cu_q[r]; j0 < cu_q[r + 1]; j0 += 256) {
    const int j = j0 + threadIdx.x;
    cnt += __syncthreads_count(j < cu_q[r + 1] && q_pos[j] >= qs);
  }
  if (threadIdx.x == 0) m_req[r] = min(cnt, max_rows);
}

// cu_v[s] = list rows before entry s (exclusive scan of m_req[segs[s].req]); seg_iota[s] = s
__global__ __launch_bounds__(256) void list_scan_kernel(
    const cc_segment* __restrict__ segs, int n_segs, int n_requests, const int32_t* __restrict__ m_req,
    int32_t* __restrict__ cu_v, int32_t* __restrict__ seg_iota) {
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int s0 = 0; s0 < n_segs; s0 += 256) {
    const int s = s0 + threadIdx.x;
    int m = 0;
    if (s < n_segs) {
      const int r = segs[s].req;
      m = (r >= 0 && r < n_requests) ? m_req[r] : 0;
    }
    int total;
    const int incl = block_scan_256(m, &total);
    const int carry = carry_s;
    if (s < n_segs) {
      cu_v[s] = carry + incl - m;
      seg_iota[s] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) carry_s = carry + total;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    cu_v[n_segs] = carry_s;
    seg_iota[n_segs] = n_segs;
  }
}

// q_map[cu_v[s] + i] = i-th question row of segment s's request (rows in list order);
// lse_seg of those rows starts at -inf (a row tile that sees no key of the segment writes nothing)
__global__ __launch_bounds__(256) void row_map_kernel(
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int n_requests,
    const int32_t* __restrict__ cu_v, int hq, int32_t* __restrict__ q_map, float* __restrict__ lse_seg) {
  const int s = blockIdx.x;
  const int r = segs[s].req;
  if (r < 0 || r >= n_requests) return;
  const int base = cu_v[s], m = cu_v[s + 1] - base;
  if (m <= 0) return;
  const int qs = question_start(segs, req_seg_off, r);
  int done = 0;
  for (int j0 = cu_q[r]; j0 < cu_q[r + 1]; j0 += 256) {      // (uniform trip count)
    const int j = j0 + threadIdx.x;
    const int is_q = (j < cu_q[r + 1] && q_pos[j] >= qs) ? 1 : 0;
    int total;
    const int ord = done + block_scan_256(is_q, &total) - is_q;
    if (is_q && ord < m) q_map[base + ord] = j;
    done += total;
  }
  for (int i = threadIdx.x; i < m * hq; i += 256) lse_seg[static_cast<size_t>(base) * hq + i] = -INFINITY;
}

// seg_mass[s] = (1/Hq) sum over the entry's rows and heads of exp(lse_seg - lse)
__global__ __launch_bounds__(256) void seg_mass_kernel(
    const int32_t* __restrict__ cu_v, const int32_t* __restrict__ q_map, int hq,
    const float* __restrict__ lse_seg, const float* __restrict__ lse, float* __restrict__ seg_mass) {
  __shared__ float part[256];
  const int s = blockIdx.x;
  const int base = cu_v[s], m = cu_v[s + 1] - base;
  float acc = 0.f;
  for (int i = threadIdx.x; i < m * hq; i += 256) {
    const int u = i / hq, h = i - u * hq;
    const float a = lse_seg[static_cast<size_t>(base + u) * hq + h];
    const float b = lse[static_cast<size_t>(q_map[base + u]) * hq + h];
    acc += a == -INFINITY ? 0.f : __expf(a - b);
  }
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {                        // fixed tree: the same sum every run
    if (threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) seg_mass[s] = part[0] / static_cast<float>(hq);
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0.f;
}

size_t up256(size_t v) { return (v + 255) / 256 * 256; }

}  // namespace

void launch_fill_zero(float* p, int n, hipStream_t stream) {
  if (n > 0) hipLaunchKernelGGL(fill_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
}

// workspace: tile plan | m_req[n_segs] | cu_v[n_segs+1] | seg_iota[n_segs+1] | q_map[cap] | lse_seg[cap][Hq]
size_t question_mass_bytes(const cc_ctx* ctx, int n_segs, int max_tiles, int max_question_rows) {
  const size_t cap = static_cast<size_t>(n_segs) * max_question_rows;
  return up256(mfma_plan_bytes(n_segs, max_tiles, static_cast<int>(cap))) +
         3 * up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t)) + up256(cap * sizeof(int32_t)) +
         up256(cap * ctx->cfg.n_q_heads * sizeof(float));
}

void launch_question_mass(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                          int max_question_rows, const void* k_pool, const void* v_pool, int n_blocks,
                          const int32_t* block_tab, const cc_segment* segs, int n_segs,
                          const int32_t* req_seg_off, int n_requests, const float* lse, float* seg_mass,
                          void* workspace, int max_tiles, hipStream_t stream) {
  const int hq = ctx->cfg.n_q_heads;
  const size_t cap = static_cast<size_t>(n_segs) * max_question_rows;
  char* w = static_cast<char*>(workspace);
  void* plan_ws = w;
  w += up256(mfma_plan_bytes(n_segs, max_tiles, static_cast<int>(cap)));
  int32_t* m_req = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t));
  int32_t* cu_v = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t));
  int32_t* seg_iota = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t));
  int32_t* q_map = reinterpret_cast<int32_t*>(w);
  w += up256(cap * sizeof(int32_t));
  float* lse_seg = reinterpret_cast<float*>(w);

  hipLaunchKernelGGL(question_count_kernel, dim3(n_requests), dim3(256), 0, stream, q_pos, cu_q, segs,
                     req_seg_off, max_question_rows, m_req);
  hipLaunchKernelGGL(list_scan_kernel, dim3(1), dim3(256), 0, stream, segs, n_segs, n_requests, m_req, cu_v,
                     seg_iota);
  hipLaunchKernelGGL(row_map_kernel, dim3(n_segs), dim3(256), 0, stream, q_pos, cu_q, segs, req_seg_off,
                     n_requests, cu_v, hq, q_map, lse_seg);
  // the attention kernels over the list: request = one segment, queries = its question rows
  if (ctx->impl != CC_IMPL_SCALAR && attn_mfma_supported(ctx))
    launch_attn_mfma(ctx, q, q_pos, cu_v, static_cast<int>(cap), max_question_rows, k_pool, v_pool, n_blocks,
                     block_tab, segs, n_segs, seg_iota, n_segs, nullptr, lse_seg, plan_ws, max_tiles, q_map,
                     stream);
  else
    launch_attn_scalar(ctx, q, q_pos, cu_v, static_cast<int>(cap), max_question_rows, k_pool, v_pool,
                       n_blocks, block_tab, segs, seg_iota, n_segs, nullptr, lse_seg, q_map, stream);
  hipLaunchKernelGGL(seg_mass_kernel, dim3(n_segs), dim3(256), 0, stream, cu_v, q_map, hq, lse_seg, lse,
                     seg_mass);
}

}  // namespace cc

// ---- Algorithm 1 (host) -----------------------------------------------------------------------------
struct cc_focus {
  int k = 0, window = 0, layer = 0;
  std::vector<double> cinter;                 // cumulative inter-attention per chunk
  std::vector<std::vector<int32_t>> history;  // chosen set of every layer so far (as 0/1 flags)
};

extern "C" {

int cc_focus_create(cc_focus** out, int32_t n_chunks, int32_t window) {
  if (out == nullptr) return CC_ERR_INVALID_ARG;
  *out = nullptr;
  if (n_chunks <= 0 || window <= 0) return CC_ERR_INVALID_ARG;
  cc_focus* f = new (std::nothrow) cc_focus();
  if (f == nullptr) return CC_ERR_INVALID_ARG;
  f->k = n_chunks;
  f->window = window;
  f->cinter.assign(n_chunks, 0.0);
  *out = f;
  return CC_OK;
}

void cc_focus_destroy(cc_focus* f) { delete f; }

int cc_focus_update(cc_focus* f, const float* inter, int32_t* focused, int32_t* n_focused) {
  if (f == nullptr || inter == nullptr || focused == nullptr) return CC_ERR_INVALID_ARG;
  const int k = f->k;
  for (int i = 0; i < k; ++i) {
    if (!std::isfinite(inter[i])) return CC_ERR_INVALID_ARG;
    f->cinter[i] += static_cast<double>(inter[i]);
  }
  f->layer += 1;
  // chunks by cumulative score, descending (earlier chunk first among equals)
  std::vector<int> order(k);
  for (int i = 0; i < k; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return f->cinter[a] > f->cinter[b]; });
  // gaps between neighbours, as a distribution; entropy term of every gap
  int n_top = k;                              // fewer than three chunks, or no gap at all: keep all
  if (k >= 3) {
    std::vector<double> term(k - 1, 0.0);
    double total = 0.0;
    for (int i = 0; i + 1 < k; ++i) total += f->cinter[order[i]] - f->cinter[order[i + 1]];
    if (total > 0.0) {
      for (int i = 0; i + 1 < k; ++i) {
        const double p = (f->cinter[order[i]] - f->cinter[order[i + 1]]) / total;
        term[i] = p > 0.0 ? -p * std::log(p) : 0.0;
      }
      // h_{i+1} - h_i is the entropy term of gap i+1; i runs over 1..k-2 (1-based), so the first
      // gap is never the one chosen; the top i* chunks are kept
      int best = 1;
      for (int i = 2; i <= k - 2; ++i)
        if (term[i] > term[best]) best = i;   // term[] is 0-based: term[i] is gap i+1
      n_top = best;
    }
  }
  std::vector<int32_t> flags(k, 0);
  for (int i = 0; i < n_top; ++i) flags[order[i]] = 1;
  for (int i = 0; i < k; ++i) focused[i] = flags[i];
  if (n_focused != nullptr) *n_focused = n_top;
  f->history.push_back(flags);
  // stop once the last `window` layers chose the same set
  if (f->layer < f->window) return 0;
  for (int l = f->layer - f->window; l < f->layer; ++l)
    if (f->history[l] != flags) return 0;
  return 1;
}

int32_t cc_focus_layer(const cc_focus* f) { return f == nullptr ? -1 : f->layer; }

}  // extern "C"
