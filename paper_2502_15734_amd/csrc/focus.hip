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
// The same list with every row of the compact query list (each from the first segment it can see
// on) gives the whole lower-triangular matrix of segment-to-segment attention: inter(C_j, C_i) of
// Eq. (2) off the diagonal, intra(C_i) of Eq. (3) on it once the weight every row puts on its own
// key is taken off (a small kernel of its own).
//
// Host part.  Algorithm 1: per-chunk cumulative scores over the layers, a split of the sorted
// scores at the gap with the largest entropy term, and a stop once the chosen set has not changed
// for w layers.  Reuse scores of Sec. 3.1 / 3.3: a, b, CCI, prefix overlap beta, order penalty
// gamma (normalised Kendall tau distance), beta', CFO and the token budget N.
#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

#include "device_util.h"
#include "mfma_tile.h"

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

// Rows of list entry s (= segment s as the only keys): the rows of its request at positions
// >= this threshold.  question_only: the request's question rows; else every row that can see the
// segment at all, i.e. from the segment's first position on.
__device__ __forceinline__ int entry_threshold(const cc_segment* __restrict__ segs,
                                               const int32_t* __restrict__ req_seg_off, int s, int r,
                                               bool question_only) {
  return question_only ? question_start(segs, req_seg_off, r) : segs[s].logical_start;
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

// sum of one float per thread over a 256-thread workgroup, fixed tree (the same sum every run);
// valid in thread 0
__device__ __forceinline__ float block_sum_256(float v) {
  __shared__ float part[256];
  __syncthreads();
  part[threadIdx.x] = v;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  return part[0];
}

// m_seg[s] = number of rows of entry s (at most max_rows are kept)
__global__ __launch_bounds__(256) void entry_count_kernel(
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int n_requests,
    int max_rows, bool question_only, int32_t* __restrict__ m_seg) {
  const int s = blockIdx.x;
  const int r = segs[s].req;
  if (r < 0 || r >= n_requests) {
    if (threadIdx.x == 0) m_seg[s] = 0;
    return;
  }
  const int thr = entry_threshold(segs, req_seg_off, s, r, question_only);
  int cnt = 0;
  for (int j0 = cu_q[r]; j0 < cu_q[r + 1]; j0 += 256) {
    const int j = j0 + threadIdx.x;
    cnt += __syncthreads_count(j < cu_q[r + 1] && q_pos[j] >= thr);
  }
  if (threadIdx.x == 0) m_seg[s] = min(cnt, max_rows);
}

// cu_v[s] = list rows before entry s (exclusive scan of m_seg); seg_iota[s] = s
__global__ __launch_bounds__(256) void list_scan_kernel(
    int n_segs, const int32_t* __restrict__ m_seg, int32_t* __restrict__ cu_v, int32_t* __restrict__ seg_iota) {
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int s0 = 0; s0 < n_segs; s0 += 256) {
    const int s = s0 + threadIdx.x;
    const int m = s < n_segs ? m_seg[s] : 0;
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

// q_map[cu_v[s] + i] = i-th row of entry s (rows in list order); row_seg (optional) = the segment
// that row's own position lies in; lse_seg of the entry's rows starts at -inf (a row tile that
// sees no key of the segment writes nothing)
__global__ __launch_bounds__(256) void row_map_kernel(
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int n_requests,
    const int32_t* __restrict__ cu_v, int hq, bool question_only, int32_t* __restrict__ q_map,
    int32_t* __restrict__ row_seg, float* __restrict__ lse_seg) {
  const int s = blockIdx.x;
  const int r = segs[s].req;
  if (r < 0 || r >= n_requests) return;
  const int base = cu_v[s], m = cu_v[s + 1] - base;
  if (m <= 0) return;
  const int thr = entry_threshold(segs, req_seg_off, s, r, question_only);
  int done = 0;
  for (int j0 = cu_q[r]; j0 < cu_q[r + 1]; j0 += 256) {      // (uniform trip count)
    const int j = j0 + threadIdx.x;
    const int pos = j < cu_q[r + 1] ? q_pos[j] : -1;
    const int take = pos >= thr ? 1 : 0;
    int total;
    const int ord = done + block_scan_256(take, &total) - take;
    if (take && ord < m) {
      q_map[base + ord] = j;
      if (row_seg != nullptr) {
        int own = -1;
        for (int t = req_seg_off[r]; t < req_seg_off[r + 1]; ++t)
          if (pos >= segs[t].logical_start && pos < segs[t].logical_start + segs[t].n_tokens) own = t;
        row_seg[base + ord] = own;
      }
    }
    done += total;
  }
  for (int i = threadIdx.x; i < m * hq; i += 256) lse_seg[static_cast<size_t>(base) * hq + i] = -INFINITY;
}

// weight a list row's head puts on the entry's segment
__device__ __forceinline__ float entry_weight(const float* __restrict__ lse_seg, const float* __restrict__ lse,
                                              const int32_t* __restrict__ q_map, int list_row, int h, int hq) {
  const float a = lse_seg[static_cast<size_t>(list_row) * hq + h];
  const float b = lse[static_cast<size_t>(q_map[list_row]) * hq + h];
  return a == -INFINITY ? 0.f : __expf(a - b);
}

// seg_mass[s] = (1/Hq) sum over the entry's rows and heads of exp(lse_seg - lse)
__global__ __launch_bounds__(256) void seg_mass_kernel(
    const int32_t* __restrict__ cu_v, const int32_t* __restrict__ q_map, int hq,
    const float* __restrict__ lse_seg, const float* __restrict__ lse, float* __restrict__ seg_mass) {
  const int s = blockIdx.x;
  const int base = cu_v[s], m = cu_v[s + 1] - base;
  float acc = 0.f;
  for (int i = threadIdx.x; i < m * hq; i += 256) {
    const int u = i / hq;
    acc += entry_weight(lse_seg, lse, q_map, base + u, i - u * hq, hq);
  }
  const float tot = block_sum_256(acc);
  if (threadIdx.x == 0) seg_mass[s] = tot / static_cast<float>(hq);
}

// pair_mass[pair(t, s)] for every segment t >= s of entry s's request: the entry's rows whose own
// position lies in t.  pair(t, s) = pairs of earlier requests + tl (tl + 1) / 2 + sl with tl, sl
// the segments' indices inside their request.
__global__ __launch_bounds__(256) void pair_mass_kernel(
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int n_requests,
    const int32_t* __restrict__ cu_v, const int32_t* __restrict__ q_map, const int32_t* __restrict__ row_seg,
    int hq, const float* __restrict__ lse_seg, const float* __restrict__ lse, float* __restrict__ pair_mass,
    int n_pairs) {
  const int s = blockIdx.x;
  const int r = segs[s].req;
  if (r < 0 || r >= n_requests) return;
  int pair_base = 0;
  for (int r2 = 0; r2 < r; ++r2) {
    const int n2 = req_seg_off[r2 + 1] - req_seg_off[r2];
    pair_base += n2 * (n2 + 1) / 2;
  }
  const int s_first = req_seg_off[r], sl = s - s_first;
  const int base = cu_v[s], m = cu_v[s + 1] - base;
  for (int t = s; t < req_seg_off[r + 1]; ++t) {
    float acc = 0.f;
    for (int i = threadIdx.x; i < m * hq; i += 256) {
      const int u = i / hq;
      if (row_seg[base + u] == t) acc += entry_weight(lse_seg, lse, q_map, base + u, i - u * hq, hq);
    }
    const float tot = block_sum_256(acc);
    const int tl = t - s_first;
    const int pi = pair_base + tl * (tl + 1) / 2 + sl;
    if (threadIdx.x == 0 && pi < n_pairs) pair_mass[pi] = tot / static_cast<float>(hq);
  }
}

// self_mass[s] = (1/Hq) sum over the rows of the compact list that lie in segment s and over heads
// of the weight the row puts on its own key: exp(q'.k_own / sqrt(d) - lse).  One wavefront per
// row walks the heads; lane i owns rotation pair (i, i + d/2), whose angle it needs once per row.
// The sum over heads is written per row into row_self, then summed per segment in a fixed order
// by self_sum_kernel.
template <typename T, int D>
__global__ __launch_bounds__(64) void self_weight_kernel(
    const T* __restrict__ q, const int32_t* __restrict__ src_rows, const int32_t* __restrict__ q_pos,
    const int32_t* __restrict__ slot_map, const T* __restrict__ k_pool, int n_blocks, int hq, int hkv,
    InvFreq inv_freq, const float* __restrict__ lse, float* __restrict__ row_self) {
  const int j = blockIdx.x, lane = threadIdx.x;
  const int jq = src_rows != nullptr ? src_rows[j] : j;       // row of q the list row reads
  const int slot = slot_map[j];
  const bool ok = slot >= 0 && slot / kBlock < n_blocks;
  const bool own = lane < D / 2;
  float c = 1.f, sn = 0.f;
  if (ok && own) rot_cos_sin(q_pos[j], inv_freq.f[lane], &c, &sn);
  const int group = hq / hkv;
  float acc = 0.f;
  if (ok) {
    for (int kvh = 0; kvh < hkv; ++kvh) {
      float kx = 0.f, ky = 0.f;
      if (own) {
        const T* kp = k_pool + ((static_cast<size_t>(slot / kBlock) * hkv + kvh) * kBlock + slot % kBlock) * D;
        kx = to_float(kp[lane]);
        ky = to_float(kp[lane + D / 2]);
      }
      for (int g = 0; g < group; ++g) {
        const int h = kvh * group + g;
        float part = 0.f;
        if (own) {
          const T* qp = q + (static_cast<size_t>(jq) * hq + h) * D;
          const float x = to_float(qp[lane]), y = to_float(qp[lane + D / 2]);
          part = (x * c - y * sn) * kx + (y * c + x * sn) * ky;
        }
        const float logit = wave_sum(part) * rsqrtf(static_cast<float>(D));
        acc += __expf(logit - lse[static_cast<size_t>(j) * hq + h]);
      }
    }
  }
  if (lane == 0) row_self[j] = acc;
}

__global__ __launch_bounds__(256) void self_sum_kernel(
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q, const cc_segment* __restrict__ segs,
    int n_requests, int hq, const float* __restrict__ row_self, float* __restrict__ self_mass) {
  const int s = blockIdx.x;
  const cc_segment sg = segs[s];
  float acc = 0.f;
  if (sg.req >= 0 && sg.req < n_requests) {
    const int j0 = cu_q[sg.req], n = cu_q[sg.req + 1] - j0;
    for (int u = threadIdx.x; u < n; u += 256) {
      const int pos = q_pos[j0 + u];
      if (pos >= sg.logical_start && pos < sg.logical_start + sg.n_tokens) acc += row_self[j0 + u];
    }
  }
  const float tot = block_sum_256(acc);
  if (threadIdx.x == 0) self_mass[s] = tot / static_cast<float>(hq);
}

// ---- question rows of the batch, numbered request after request ("snap rows") ------------------------
// m_req[r] = question rows of request r (at most max_rows)
__global__ __launch_bounds__(256) void snap_count_kernel(
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

// snap_base[r] = snap rows before request r; snap_base[n_requests] = their total
__global__ __launch_bounds__(256) void snap_scan_kernel(int n_requests, const int32_t* __restrict__ m_req,
                                                         int32_t* __restrict__ snap_base) {
  __shared__ int carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int r0 = 0; r0 < n_requests; r0 += 256) {
    const int r = r0 + threadIdx.x;
    const int m = r < n_requests ? m_req[r] : 0;
    int total;
    const int incl = block_scan_256(m, &total);
    const int carry = carry_s;
    if (r < n_requests) snap_base[r] = carry + incl - m;
    __syncthreads();
    if (threadIdx.x == 0) carry_s = carry + total;
    __syncthreads();
  }
  if (threadIdx.x == 0) snap_base[n_requests] = carry_s;
}

// snap_index[j] = snap row of list row j (-1: not a question row); snap_rows / snap_req: the way back
__global__ __launch_bounds__(256) void snap_fill_kernel(
    const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off,
    const int32_t* __restrict__ snap_base, int32_t* __restrict__ snap_index,
    int32_t* __restrict__ snap_rows, int32_t* __restrict__ snap_req) {
  const int r = blockIdx.x;
  const int base = snap_base[r], m = snap_base[r + 1] - base;
  const int qs = question_start(segs, req_seg_off, r);
  int done = 0;
  for (int j0 = cu_q[r]; j0 < cu_q[r + 1]; j0 += 256) {      // (uniform trip count)
    const int j = j0 + threadIdx.x;
    const bool in = j < cu_q[r + 1];
    const int take = (in && q_pos[j] >= qs) ? 1 : 0;
    int total;
    const int ord = done + block_scan_256(take, &total) - take;
    if (in) snap_index[j] = (take && ord < m) ? base + ord : -1;
    if (take && ord < m) {
      snap_rows[base + ord] = j;
      snap_req[base + ord] = r;
    }
    done += total;
  }
}

// Cumulative log-sum-exp per segment for the snap rows the wide attention kernel did not finish
// (its redo flags; every snap row when redo is NULL): one wavefront per snap row walks, head after
// head, the request's keys in prompt order with a running maximum, lane i owning rotation pair
// (i, i + d/2).  (Slow, and meant to be: it only ever runs for rows whose logits overflowed.)
template <typename T, int D>
__global__ __launch_bounds__(64) void cum_scalar_kernel(
    const T* __restrict__ q, const int32_t* __restrict__ src_rows, const int32_t* __restrict__ q_pos,
    const int32_t* __restrict__ cu_q,
    const int32_t* __restrict__ snap_base, int n_requests, const int32_t* __restrict__ snap_rows,
    const int32_t* __restrict__ snap_req, const int32_t* __restrict__ redo,
    const T* __restrict__ k_pool, int n_blocks, const int32_t* __restrict__ block_tab,
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int hq, int hkv,
    InvFreq inv_freq, float* __restrict__ cum, int s_max) {
  const int u = blockIdx.x, lane = threadIdx.x;
  if (u >= snap_base[n_requests]) return;
  // (no maps: every list row is a snap row, snap_base is cu_q itself)
  const int j = snap_rows != nullptr ? snap_rows[u] : u;
  int r = 0;
  if (snap_req != nullptr) r = snap_req[u];
  else
    while (r + 1 < n_requests && cu_q[r + 1] <= j) ++r;
  if (redo != nullptr && redo[redo_index(cu_q[r] + ((j - cu_q[r]) / 64) * 64)] == 0) return;
  const int p = q_pos[j];
  const bool own = lane < D / 2;
  for (int h = 0; h < hq; ++h) {
  const int kvh = h / (hq / hkv);
  float qx = 0.f, qy = 0.f;
  if (own) {
    const T* qp = q + (static_cast<size_t>(src_rows != nullptr ? src_rows[j] : j) * hq + h) * D;
    float x = to_float(qp[lane]), y = to_float(qp[lane + D / 2]), c, sn;
    rot_cos_sin(p, inv_freq.f[lane], &c, &sn);
    qx = x * c - y * sn;
    qy = y * c + x * sn;
  }
  const float scale = rsqrtf(static_cast<float>(D));
  float m = -INFINITY, z = 0.f;
  for (int s = req_seg_off[r]; s < req_seg_off[r + 1]; ++s) {
    const cc_segment ks = segs[s];
    const int n_vis = min(ks.n_tokens, p - ks.logical_start + 1);
    for (int tk = 0; tk < n_vis; ++tk) {
      const int blk = block_tab[ks.tab_off + tk / kBlock];
      if (blk < 0 || blk >= n_blocks) continue;
      const T* kp = k_pool + ((static_cast<size_t>(blk) * hkv + kvh) * kBlock + tk % kBlock) * D;
      const float part = own ? qx * to_float(kp[lane]) + qy * to_float(kp[lane + D / 2]) : 0.f;
      const float logit = wave_sum(part) * scale;
      if (logit > m) {
        z *= expf(m - logit);
        m = logit;
      }
      z += expf(logit - m);
    }
    const int sl = s - req_seg_off[r];
    if (lane == 0 && sl < s_max) cum[(static_cast<size_t>(u) * hq + h) * s_max + sl] = m + logf(z);
  }
  }
}

// seg_mass[s] from the cumulative log-sum-exps: weight on segment s = exp(cum_s - lse) - exp(cum_{s-1} - lse);
// the request's last segment takes what is left (its own cum entry is never read: rows of a tile
// end at different keys there).
__global__ __launch_bounds__(256) void seg_mass_from_cum_kernel(
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int n_requests,
    const int32_t* __restrict__ snap_base, const int32_t* __restrict__ snap_rows, int hq,
    const float* __restrict__ cum, int s_max, const float* __restrict__ lse, float* __restrict__ seg_mass) {
  const int s = blockIdx.x;
  const int r = segs[s].req;
  float acc = 0.f;
  if (r >= 0 && r < n_requests) {
    const int sl = s - req_seg_off[r], n_r = req_seg_off[r + 1] - req_seg_off[r];
    const int base = snap_base[r], m = snap_base[r + 1] - base;
    if (sl < s_max) {
      for (int i = threadIdx.x; i < m * hq; i += 256) {
        const int u = base + i / hq, h = i % hq;
        const float total = lse[static_cast<size_t>(snap_rows[u]) * hq + h];
        const float* c = cum + (static_cast<size_t>(u) * hq + h) * s_max;
        const float upto = sl + 1 < n_r ? __expf(c[sl] - total) : 1.f;
        const float before = sl > 0 ? __expf(c[sl - 1] - total) : 0.f;
        acc += upto - before;
      }
    }
  }
  const float tot = block_sum_256(acc);
  if (threadIdx.x == 0) seg_mass[s] = tot / static_cast<float>(hq);
}

// pair_mass from the cumulative log-sum-exps of EVERY row (snap row = list row): workgroup t sums,
// over the rows of segment t (they sit at [sel_off, sel_off + n_select) of the list, as cc_select
// lays them out) and all heads, the weight on each segment s <= t of the same request:
// exp(cum_s - lse) - exp(cum_{s-1} - lse) for s < t, and what is left for s = t.
__global__ __launch_bounds__(256) void pair_mass_from_cum_kernel(
    const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int n_requests, int n_q_tot,
    int hq, const float* __restrict__ cum, int s_max, const float* __restrict__ lse,
    float* __restrict__ pair_mass, int n_pairs) {
  const int t = blockIdx.x, sl = blockIdx.y;               // (row segment, key segment's index in the request)
  const cc_segment sg = segs[t];
  const int r = sg.req;
  if (r < 0 || r >= n_requests) return;
  const int tl = t - req_seg_off[r];
  if (sl > tl) return;
  int pair_base = 0;
  for (int r2 = 0; r2 < r; ++r2) {
    const int n2 = req_seg_off[r2 + 1] - req_seg_off[r2];
    pair_base += n2 * (n2 + 1) / 2;
  }
  const int row0 = max(sg.sel_off, 0), n_rows = max(min(sg.n_select, n_q_tot - row0), 0);
  float acc = 0.f;
  if (tl < s_max) {
    for (int i = threadIdx.x; i < n_rows * hq; i += 256) {
      const int u = row0 + i / hq, h = i % hq;
      const float total = lse[static_cast<size_t>(u) * hq + h];
      const float* c = cum + (static_cast<size_t>(u) * hq + h) * s_max;
      const float upto = sl < tl ? __expf(c[sl] - total) : 1.f;
      const float before = sl > 0 ? __expf(c[sl - 1] - total) : 0.f;
      acc += upto - before;
    }
  }
  const float tot = block_sum_256(acc);
  const int pi = pair_base + tl * (tl + 1) / 2 + sl;
  if (threadIdx.x == 0 && pi < n_pairs) pair_mass[pi] = tot / static_cast<float>(hq);
}

// seg_mass[s] = the entry of the pair matrix whose rows are the request's question segment
__global__ __launch_bounds__(256) void seg_mass_from_pairs_kernel(
    const cc_segment* __restrict__ segs, int n_segs, const int32_t* __restrict__ req_seg_off, int n_requests,
    const float* __restrict__ pair_mass, int n_pairs, float* __restrict__ seg_mass) {
  const int s = blockIdx.x * 256 + threadIdx.x;
  if (s >= n_segs) return;
  const int r = segs[s].req;
  float v = 0.f;
  if (r >= 0 && r < n_requests) {
    int pair_base = 0;
    for (int r2 = 0; r2 < r; ++r2) {
      const int n2 = req_seg_off[r2 + 1] - req_seg_off[r2];
      pair_base += n2 * (n2 + 1) / 2;
    }
    int tq = -1;                                           // the request's question segment (the last one of that kind)
    for (int t = req_seg_off[r]; t < req_seg_off[r + 1]; ++t)
      if (segs[t].kind == CC_SEG_QUESTION) tq = t - req_seg_off[r];
    const int sl = s - req_seg_off[r];
    if (tq >= sl) {
      const int pi = pair_base + tq * (tq + 1) / 2 + sl;
      if (pi < n_pairs) v = pair_mass[pi];
    }
  }
  seg_mass[s] = v;
}

__global__ __launch_bounds__(256) void fill_kernel(float* __restrict__ p, size_t n, float v) {
  const size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}

// entry row j (of cu_v[n_segs] in all): q row src_rows[q_map[j]], position q_pos[q_map[j]]
__global__ __launch_bounds__(256) void fold_maps_kernel(const int32_t* __restrict__ cu_v, int n_segs,
                                                         const int32_t* __restrict__ q_map,
                                                         const int32_t* __restrict__ src_rows,
                                                         const int32_t* __restrict__ q_pos,
                                                         int32_t* __restrict__ q_map_src, int32_t* __restrict__ pos_src) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= cu_v[n_segs]) return;
  const int row = q_map[j];
  q_map_src[j] = src_rows[row];
  pos_src[j] = q_pos[row];
}

size_t up256(size_t v) { return (v + 255) / 256 * 256; }

// the workspace, cut up
struct ListBuffers {
  void* plan_ws;
  int32_t *m_seg, *cu_v, *seg_iota, *q_map, *row_seg, *q_map_src, *pos_src;
  float *lse_seg, *row_self;
};

}  // namespace

void launch_fill_zero(float* p, int n, hipStream_t stream) {
  if (n > 0) hipLaunchKernelGGL(fill_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p, static_cast<size_t>(n), 0.f);
}

// workspace: tile plan | m_seg[n_segs+1] | cu_v[n_segs+1] | seg_iota[n_segs+1] | q_map[cap] |
//            row_seg[cap] | q_map_src[cap] | pos_src[cap] | lse_seg[cap][Hq] | row_self[n_q_tot] (sized for Hq floats per row) (the last only for the pair matrix)
size_t segment_mass_bytes(const cc_ctx* ctx, int n_segs, int max_tiles, int max_rows, int n_q_tot_self) {
  const size_t cap = static_cast<size_t>(n_segs) * max_rows;
  return up256(mfma_plan_bytes(n_segs, max_tiles, static_cast<int>(cap))) +
         3 * up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t)) + 4 * up256(cap * sizeof(int32_t)) +
         up256(cap * ctx->cfg.n_q_heads * sizeof(float)) +
         up256(static_cast<size_t>(n_q_tot_self) * ctx->cfg.n_q_heads * sizeof(float));
}

static ListBuffers cut_workspace(const cc_ctx* ctx, void* workspace, int n_segs, int max_tiles, int max_rows) {
  const size_t cap = static_cast<size_t>(n_segs) * max_rows;
  ListBuffers b;
  char* w = static_cast<char*>(workspace);
  b.plan_ws = w;
  w += up256(mfma_plan_bytes(n_segs, max_tiles, static_cast<int>(cap)));
  b.m_seg = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t));
  b.cu_v = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t));
  b.seg_iota = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_segs + 1) * sizeof(int32_t));
  b.q_map = reinterpret_cast<int32_t*>(w);
  w += up256(cap * sizeof(int32_t));
  b.row_seg = reinterpret_cast<int32_t*>(w);
  w += up256(cap * sizeof(int32_t));
  b.q_map_src = reinterpret_cast<int32_t*>(w);
  w += up256(cap * sizeof(int32_t));
  b.pos_src = reinterpret_cast<int32_t*>(w);
  w += up256(cap * sizeof(int32_t));
  b.lse_seg = reinterpret_cast<float*>(w);
  w += up256(cap * ctx->cfg.n_q_heads * sizeof(float));
  b.row_self = reinterpret_cast<float*>(w);
  return b;
}

// builds the list of one-segment requests and runs the attention kernels over it (log-sum-exp only)
static void run_segment_list(const cc_ctx* ctx, const ListBuffers& b, const void* q, const int32_t* src_rows,
                             const int32_t* q_pos, const int32_t* cu_q, int max_rows, bool question_only, const void* k_pool,
                             const void* v_pool, int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                             int n_segs, const int32_t* req_seg_off, int n_requests, int max_tiles,
                             hipStream_t stream) {
  const int hq = ctx->cfg.n_q_heads;
  const int cap = n_segs * max_rows;
  hipLaunchKernelGGL(entry_count_kernel, dim3(n_segs), dim3(256), 0, stream, q_pos, cu_q, segs, req_seg_off,
                     n_requests, max_rows, question_only, b.m_seg);
  hipLaunchKernelGGL(list_scan_kernel, dim3(1), dim3(256), 0, stream, n_segs, b.m_seg, b.cu_v, b.seg_iota);
  hipLaunchKernelGGL(row_map_kernel, dim3(n_segs), dim3(256), 0, stream, q_pos, cu_q, segs, req_seg_off,
                     n_requests, b.cu_v, hq, question_only, b.q_map, question_only ? nullptr : b.row_seg,
                     b.lse_seg);
  // The kernels take one row map: entry row j reads q and q_pos at row q_map[j].  When the list rows
  // themselves read q through src_rows, the two maps are folded into one and the positions are
  // laid out by entry row, so that the kernels index them directly.
  const int32_t* map = b.q_map;
  const int32_t* pos = q_pos;
  int map_pos = 1;
  if (src_rows != nullptr) {
    hipLaunchKernelGGL(fold_maps_kernel, dim3((cap + 255) / 256), dim3(256), 0, stream, b.cu_v, n_segs, b.q_map,
                       src_rows, q_pos, b.q_map_src, b.pos_src);
    map = b.q_map_src; pos = b.pos_src; map_pos = 0;
  }
  if (ctx->impl != CC_IMPL_SCALAR && attn_mfma_supported(ctx))
    launch_attn_mfma(ctx, q, pos, b.cu_v, cap, max_rows, k_pool, v_pool, n_blocks, block_tab, segs, n_segs,
                     b.seg_iota, n_segs, nullptr, b.lse_seg, b.plan_ws, max_tiles, map, map_pos, stream);
  else
    launch_attn_scalar(ctx, q, pos, b.cu_v, cap, max_rows, k_pool, v_pool, n_blocks, block_tab, segs,
                       b.seg_iota, n_segs, nullptr, b.lse_seg, map, map_pos, stream);
}

void launch_question_mass(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* cu_q,
                          int max_question_rows, const void* k_pool, const void* v_pool, int n_blocks,
                          const int32_t* block_tab, const cc_segment* segs, int n_segs,
                          const int32_t* req_seg_off, int n_requests, const float* lse, float* seg_mass,
                          void* workspace, int max_tiles, hipStream_t stream) {
  const ListBuffers b = cut_workspace(ctx, workspace, n_segs, max_tiles, max_question_rows);
  run_segment_list(ctx, b, q, src_rows, q_pos, cu_q, max_question_rows, true, k_pool, v_pool, n_blocks, block_tab, segs,
                   n_segs, req_seg_off, n_requests, max_tiles, stream);
  hipLaunchKernelGGL(seg_mass_kernel, dim3(n_segs), dim3(256), 0, stream, b.cu_v, b.q_map, ctx->cfg.n_q_heads,
                     b.lse_seg, lse, seg_mass);
}

void launch_chunk_attention(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                            const int32_t* cu_q, int n_q_tot, int max_q_per_req, const void* k_pool,
                            const void* v_pool, int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                            int n_segs, const int32_t* req_seg_off, int n_requests, const float* lse,
                            float* pair_mass, int n_pairs, float* self_mass, void* workspace, int max_tiles,
                            hipStream_t stream) {
  const ListBuffers b = cut_workspace(ctx, workspace, n_segs, max_tiles, max_q_per_req);
  const int hq = ctx->cfg.n_q_heads, hkv = ctx->cfg.n_kv_heads;
  run_segment_list(ctx, b, q, src_rows, q_pos, cu_q, max_q_per_req, false, k_pool, v_pool, n_blocks, block_tab, segs,
                   n_segs, req_seg_off, n_requests, max_tiles, stream);
  hipLaunchKernelGGL(pair_mass_kernel, dim3(n_segs), dim3(256), 0, stream, segs, req_seg_off, n_requests,
                     b.cu_v, b.q_map, b.row_seg, hq, b.lse_seg, lse, pair_mass, n_pairs);
  if (self_mass != nullptr) {
    const bool bf = ctx->cfg.dtype == CC_BF16;
    const int d = ctx->cfg.head_dim;
#define CC_LAUNCH(T, D)                                                                              \
  hipLaunchKernelGGL((self_weight_kernel<T, D>), dim3(n_q_tot), dim3(64), 0, stream,                 \
                     static_cast<const T*>(q), src_rows, q_pos, slot_map, static_cast<const T*>(k_pool), n_blocks, \
                     hq, hkv, ctx->inv_freq, lse, b.row_self)
    if (bf && d == 128) CC_LAUNCH(bf16_t, 128);
    else if (bf && d == 64) CC_LAUNCH(bf16_t, 64);
    else if (!bf && d == 128) CC_LAUNCH(float, 128);
    else CC_LAUNCH(float, 64);
#undef CC_LAUNCH
    hipLaunchKernelGGL(self_sum_kernel, dim3(n_segs), dim3(256), 0, stream, q_pos, cu_q, segs, n_requests, hq,
                       b.row_self, self_mass);
  }
}

// workspace of the prefill that also returns the question's masses:
//   tile plan of the attention | m_req[n_requests+1] | snap_base[n_requests+1] | snap_index[n_q_tot] |
//   snap_rows[cap] | snap_req[cap] | cum[cap][Hq][s_max] | workspace of launch_question_mass
// with cap = n_requests * max_question_rows.
size_t prefill_mass_bytes(const cc_ctx* ctx, int n_ctx_tokens, int n_segs, int n_requests, int max_tiles,
                          int max_question_rows, int s_max) {
  const size_t cap = static_cast<size_t>(n_requests) * max_question_rows;
  return up256(mfma_plan_bytes(n_segs, max_tiles, n_ctx_tokens)) +
         2 * up256(static_cast<size_t>(n_requests + 1) * sizeof(int32_t)) +
         up256(static_cast<size_t>(n_ctx_tokens) * sizeof(int32_t)) + 2 * up256(cap * sizeof(int32_t)) +
         up256(cap * ctx->cfg.n_q_heads * s_max * sizeof(float)) +
         segment_mass_bytes(ctx, n_segs, max_tiles, max_question_rows, 0);
}

void launch_prefill_mass(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* cu_q,
                         int n_q_tot, int max_q_per_req, int max_question_rows, int s_max, const void* k_pool,
                         const void* v_pool, int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                         int n_segs, const int32_t* req_seg_off, int n_requests, int n_ctx_tokens, void* out,
                         float* lse, float* seg_mass, void* workspace, int max_tiles, hipStream_t stream,
                         const ValueSource& vs) {
  const int hq = ctx->cfg.n_q_heads, hkv = ctx->cfg.n_kv_heads;
  const size_t cap = static_cast<size_t>(n_requests) * max_question_rows;
  char* w = static_cast<char*>(workspace);
  void* plan_ws = w;
  w += up256(mfma_plan_bytes(n_segs, max_tiles, n_ctx_tokens));
  int32_t* m_req = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_requests + 1) * sizeof(int32_t));
  int32_t* snap_base = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_requests + 1) * sizeof(int32_t));
  int32_t* snap_index = reinterpret_cast<int32_t*>(w);
  w += up256(static_cast<size_t>(n_ctx_tokens) * sizeof(int32_t));
  int32_t* snap_rows = reinterpret_cast<int32_t*>(w);
  w += up256(cap * sizeof(int32_t));
  int32_t* snap_req = reinterpret_cast<int32_t*>(w);
  w += up256(cap * sizeof(int32_t));
  float* cum = reinterpret_cast<float*>(w);
  w += up256(cap * hq * s_max * sizeof(float));
  void* fallback_ws = w;

  const bool mfma = ctx->impl != CC_IMPL_SCALAR && attn_mfma_supported(ctx);
  AttnByProduct by{snap_index, cum, s_max, false, nullptr};
  if (mfma) {
    hipLaunchKernelGGL(snap_count_kernel, dim3(n_requests), dim3(256), 0, stream, q_pos, cu_q, segs, req_seg_off,
                       max_question_rows, m_req);
    hipLaunchKernelGGL(snap_scan_kernel, dim3(1), dim3(256), 0, stream, n_requests, m_req, snap_base);
    hipLaunchKernelGGL(snap_fill_kernel, dim3(n_requests), dim3(256), 0, stream, q_pos, cu_q, segs, req_seg_off,
                       snap_base, snap_index, snap_rows, snap_req);
    // (a segment without tokens, or before the first tile, keeps "no key yet")
    const size_t n_cum = cap * hq * s_max;
    hipLaunchKernelGGL(fill_kernel, dim3(static_cast<unsigned>((n_cum + 255) / 256)), dim3(256), 0, stream, cum, n_cum,
                       -INFINITY);
    launch_attn_mfma(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks, block_tab, segs,
                     n_segs, req_seg_off, n_requests, out, lse, plan_ws, max_tiles, src_rows, 0, stream, &by, vs);
  } else {
    launch_attn_scalar(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks, block_tab, segs,
                       req_seg_off, n_requests, out, lse, src_rows, 0, stream, vs);
  }
  if (by.wide) {
    // rows the wide kernel flagged (normally none: every wavefront reads one flag and leaves)
    const bool bf = ctx->cfg.dtype == CC_BF16;
    const int d = ctx->cfg.head_dim;
#define CC_LAUNCH(T, D)                                                                                  \
  hipLaunchKernelGGL((cum_scalar_kernel<T, D>), dim3(static_cast<unsigned>(cap)), dim3(64), 0, stream, \
                     static_cast<const T*>(q), src_rows, q_pos, cu_q, snap_base, n_requests, snap_rows, snap_req,   \
                     by.redo, static_cast<const T*>(k_pool), n_blocks, block_tab, segs, req_seg_off, hq,  \
                     hkv, ctx->inv_freq, cum, s_max)
    if (bf && d == 128) CC_LAUNCH(bf16_t, 128);
    else if (bf && d == 64) CC_LAUNCH(bf16_t, 64);
    else if (!bf && d == 128) CC_LAUNCH(float, 128);
    else CC_LAUNCH(float, 64);
#undef CC_LAUNCH
    hipLaunchKernelGGL(seg_mass_from_cum_kernel, dim3(n_segs), dim3(256), 0, stream, segs, req_seg_off, n_requests,
                       snap_base, snap_rows, hq, cum, s_max, lse, seg_mass);
  } else {
    // the kernels that ran carry no by-product: the pass of its own
    launch_question_mass(ctx, q, src_rows, q_pos, cu_q, max_question_rows, k_pool, v_pool, n_blocks, block_tab, segs,
                         n_segs, req_seg_off, n_requests, lse, seg_mass, fallback_ws, max_tiles, stream);
  }
}

// workspace of the prefill that also returns the whole segment-to-segment matrix:
//   tile plan of the attention | cum[n_q_tot][Hq][s_max] | row_self[n_q_tot] (sized for Hq floats per row) | workspace of launch_chunk_attention
size_t prefill_pairs_bytes(const cc_ctx* ctx, int n_ctx_tokens, int n_segs, int max_tiles, int n_q_tot,
                           int max_q_per_req, int s_max) {
  const size_t hq = ctx->cfg.n_q_heads;
  return up256(mfma_plan_bytes(n_segs, max_tiles, n_ctx_tokens)) +
         up256(static_cast<size_t>(n_q_tot) * hq * s_max * sizeof(float)) +
         up256(static_cast<size_t>(n_q_tot) * hq * sizeof(float)) +
         segment_mass_bytes(ctx, n_segs, max_tiles, max_q_per_req, n_q_tot);
}

void launch_prefill_pairs(const cc_ctx* ctx, const void* q, const int32_t* src_rows, const int32_t* q_pos, const int32_t* slot_map,
                          const int32_t* cu_q, int n_q_tot, int max_q_per_req, int s_max, const void* k_pool,
                          const void* v_pool, int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                          int n_segs, const int32_t* req_seg_off, int n_requests, int n_ctx_tokens, void* out,
                          float* lse, float* seg_mass, float* pair_mass, int n_pairs, float* self_mass,
                          void* workspace, int max_tiles, hipStream_t stream, const ValueSource& vs) {
  const int hq = ctx->cfg.n_q_heads, hkv = ctx->cfg.n_kv_heads;
  char* w = static_cast<char*>(workspace);
  void* plan_ws = w;
  w += up256(mfma_plan_bytes(n_segs, max_tiles, n_ctx_tokens));
  float* cum = reinterpret_cast<float*>(w);
  const size_t n_cum = static_cast<size_t>(n_q_tot) * hq * s_max;
  w += up256(n_cum * sizeof(float));
  float* row_self = reinterpret_cast<float*>(w);
  w += up256(static_cast<size_t>(n_q_tot) * hq * sizeof(float));
  void* fallback_ws = w;

  const bool mfma = ctx->impl != CC_IMPL_SCALAR && attn_mfma_supported(ctx);
  AttnByProduct by{nullptr, cum, s_max, false, nullptr};          // no index: every row is a snap row
  if (mfma) {
    hipLaunchKernelGGL(fill_kernel, dim3(static_cast<unsigned>((n_cum + 255) / 256)), dim3(256), 0, stream, cum, n_cum,
                       -INFINITY);
    launch_attn_mfma(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks, block_tab, segs,
                     n_segs, req_seg_off, n_requests, out, lse, plan_ws, max_tiles, src_rows, 0, stream, &by, vs);
  } else {
    launch_attn_scalar(ctx, q, q_pos, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks, block_tab, segs,
                       req_seg_off, n_requests, out, lse, src_rows, 0, stream, vs);
  }
  const bool bf = ctx->cfg.dtype == CC_BF16;
  const int d = ctx->cfg.head_dim;
  if (by.wide) {
#define CC_LAUNCH(T, D)                                                                                       \
  hipLaunchKernelGGL((cum_scalar_kernel<T, D>), dim3(static_cast<unsigned>(n_q_tot)), dim3(64), 0, stream,     \
                     static_cast<const T*>(q), src_rows, q_pos, cu_q, cu_q, n_requests, static_cast<const int32_t*>(nullptr), \
                     static_cast<const int32_t*>(nullptr), by.redo, static_cast<const T*>(k_pool), n_blocks,   \
                     block_tab, segs, req_seg_off, hq, hkv, ctx->inv_freq, cum, s_max)
    if (bf && d == 128) CC_LAUNCH(bf16_t, 128);
    else if (bf && d == 64) CC_LAUNCH(bf16_t, 64);
    else if (!bf && d == 128) CC_LAUNCH(float, 128);
    else CC_LAUNCH(float, 64);
#undef CC_LAUNCH
    hipLaunchKernelGGL(pair_mass_from_cum_kernel, dim3(n_segs, s_max), dim3(256), 0, stream, segs, req_seg_off, n_requests,
                       n_q_tot, hq, cum, s_max, lse, pair_mass, n_pairs);
    if (self_mass != nullptr) {
#define CC_LAUNCH(T, D)                                                                              \
  hipLaunchKernelGGL((self_weight_kernel<T, D>), dim3(n_q_tot), dim3(64), 0, stream,                 \
                     static_cast<const T*>(q), src_rows, q_pos, slot_map, static_cast<const T*>(k_pool), n_blocks, \
                     hq, hkv, ctx->inv_freq, lse, row_self)
      if (bf && d == 128) CC_LAUNCH(bf16_t, 128);
      else if (bf && d == 64) CC_LAUNCH(bf16_t, 64);
      else if (!bf && d == 128) CC_LAUNCH(float, 128);
      else CC_LAUNCH(float, 64);
#undef CC_LAUNCH
      hipLaunchKernelGGL(self_sum_kernel, dim3(n_segs), dim3(256), 0, stream, q_pos, cu_q, segs, n_requests, hq,
                         row_self, self_mass);
    }
  } else {
    launch_chunk_attention(ctx, q, src_rows, q_pos, slot_map, cu_q, n_q_tot, max_q_per_req, k_pool, v_pool, n_blocks,
                           block_tab, segs, n_segs, req_seg_off, n_requests, lse, pair_mass, n_pairs, self_mass,
                           fallback_ws, max_tiles, stream);
  }
  if (seg_mass != nullptr)
    hipLaunchKernelGGL(seg_mass_from_pairs_kernel, dim3((n_segs + 255) / 256), dim3(256), 0, stream, segs, n_segs,
                       req_seg_off, n_requests, pair_mass, n_pairs, seg_mass);
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

// ---- reuse scores (host) ------------------------------------------------------------------------------
int cc_chunk_ab(const double* inter, const int32_t* prefix_len, int32_t n_prefix, double intra,
                int32_t chunk_len, double* a, double* b) {
  if (a == nullptr || b == nullptr || chunk_len <= 0 || n_prefix < 0) return CC_ERR_INVALID_ARG;
  if (n_prefix > 0 && (inter == nullptr || prefix_len == nullptr)) return CC_ERR_INVALID_ARG;
  double acc = 0.0;
  for (int j = 0; j < n_prefix; ++j) {
    if (prefix_len[j] <= 0 || !std::isfinite(inter[j])) return CC_ERR_INVALID_ARG;
    acc += inter[j] / (static_cast<double>(chunk_len) * prefix_len[j]);
  }
  if (!std::isfinite(intra)) return CC_ERR_INVALID_ARG;
  *a = acc;
  *b = intra / (static_cast<double>(chunk_len) * chunk_len);
  return CC_OK;
}

int cc_chunk_cci(const double* a, const double* b, int32_t n_layers, double* cci) {
  if (a == nullptr || b == nullptr || cci == nullptr || n_layers <= 0) return CC_ERR_INVALID_ARG;
  double sa = 0.0, sb = 0.0;
  for (int l = 0; l < n_layers; ++l) {
    if (!std::isfinite(a[l]) || !std::isfinite(b[l]) || a[l] < 0.0 || b[l] < 0.0) return CC_ERR_INVALID_ARG;
    sa += a[l];
    sb += b[l];
  }
  const double abar = sa / n_layers, bbar = sb / n_layers;
  // no outside influence at all: ratio 0 whatever b is; outside influence but none from inside: infinite ratio
  const double ratio = abar == 0.0 ? 0.0 : (bbar == 0.0 ? INFINITY : abar / bbar);
  *cci = 1.0 / (1.0 + std::exp(-ratio));
  return CC_OK;
}

int cc_chunk_reuse(const int64_t* old_prefix, const double* old_inter, int32_t n_old,
                   const int64_t* new_prefix, int32_t n_new, double cci, double alpha,
                   int32_t chunk_len, cc_reuse* out) {
  if (out == nullptr || n_old < 0 || n_new < 0 || chunk_len < 0) return CC_ERR_INVALID_ARG;
  if ((n_old > 0 && (old_prefix == nullptr || old_inter == nullptr)) || (n_new > 0 && new_prefix == nullptr))
    return CC_ERR_INVALID_ARG;
  if (!std::isfinite(cci) || !std::isfinite(alpha) || alpha < 0.0) return CC_ERR_INVALID_ARG;
  // position of every old prefix chunk in the new prefix (-1: not there)
  std::vector<int> where(n_old, -1);
  double kept = 0.0, all = 0.0;
  for (int i = 0; i < n_old; ++i) {
    if (!std::isfinite(old_inter[i]) || old_inter[i] < 0.0) return CC_ERR_INVALID_ARG;
    for (int j = 0; j < n_new; ++j)
      if (new_prefix[j] == old_prefix[i]) { where[i] = j; break; }
    all += old_inter[i];
    if (where[i] >= 0) kept += old_inter[i];
  }
  // a cache that depended on no prefix chunk has lost none of its context
  out->beta = all > 0.0 ? kept / all : 1.0;
  // discordant pairs among the common chunks: old order i < j, new order reversed
  long long m = 0, discordant = 0;
  for (int i = 0; i < n_old; ++i) {
    if (where[i] < 0) continue;
    ++m;
    for (int j = i + 1; j < n_old; ++j)
      if (where[j] >= 0 && where[j] < where[i]) ++discordant;
  }
  out->gamma = m >= 2 ? static_cast<double>(discordant) / (static_cast<double>(m) * (m - 1) / 2.0) : 0.0;
  out->beta_adj = out->beta * (1.0 - out->gamma);
  out->cfo = std::min(1.0, std::max(0.0, alpha * cci * (1.0 - out->beta_adj)));
  const double n = std::ceil(out->cfo * chunk_len - 1e-9);
  out->n_recompute = static_cast<int32_t>(std::min<double>(chunk_len, std::max(0.0, n)));
  return CC_OK;
}

}  // extern "C"
