// cc_sparse_prefill, plain kernels: row gather, rotate-and-scatter of the recomputed K/V into the
// paged cache ("fix", Sec. 3.4.3), and the scalar reference-grade attention (per-token form of
// Eq. (1)); Sec. 4 "Selective Token Recomputation".
#include "device_util.h"

namespace cc {

// dst[i] = src[row_idx[i]], 16 bytes per lane.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4* __restrict__ src,
                                                          int n_src_rows,
                                                          const int32_t* __restrict__ row_idx,
                                                          int n_rows, int vec_per_row,
                                                          uint4* __restrict__ dst) {
  const int rows_per_block = max(1, 256 / vec_per_row);
  const int v_stride = (vec_per_row >= 256) ? 256 : vec_per_row;
  const int local_row = (vec_per_row >= 256) ? 0 : threadIdx.x / vec_per_row;
  const int v0 = (vec_per_row >= 256) ? threadIdx.x : threadIdx.x % vec_per_row;
  const int row = blockIdx.x * rows_per_block + local_row;
  if (row >= n_rows || local_row >= rows_per_block) return;
  const int s = row_idx[row];
  if (s < 0 || s >= n_src_rows) return;
  const uint4* sp = src + static_cast<size_t>(s) * vec_per_row;
  uint4* dp = dst + static_cast<size_t>(row) * vec_per_row;
  for (int v = v0; v < vec_per_row; v += v_stride) dp[v] = sp[v];
}

void launch_gather_rows(const void* src, int n_src_rows, const int32_t* row_idx, int n_rows,
                        size_t row_bytes, void* dst, hipStream_t stream) {
  const int vec_per_row = static_cast<int>(row_bytes / 16);
  const int rows_per_block = vec_per_row >= 256 ? 1 : 256 / vec_per_row;
  dim3 grid((n_rows + rows_per_block - 1) / rows_per_block);
  hipLaunchKernelGGL(gather_rows_kernel, grid, dim3(256), 0, stream,
                     static_cast<const uint4*>(src), n_src_rows, row_idx, n_rows, vec_per_row,
                     static_cast<uint4*>(dst));
}

// Rotate-and-scatter of the recomputed K/V rows into their cache slots.  Rows of the compact query
// list that fall into the same 16-token block are adjacent (the order cc_select emits) and form a
// run.  A workgroup looks at 16 consecutive rows and handles every run that STARTS among them (a
// run may reach into the next workgroup's rows; it is still handled where it starts).
//   K rows are token-major and written directly, in 16-byte pieces.
//   The V block is dimension-major -- a token is one element in each of the block's d rows of 16
//   slots -- and isolated 2-byte stores cost a full memory write each, so every (head, dim) row
//   of the block is read, patched with the run's tokens in registers, and written back whole.
//   This needs all rows of a block to sit in ONE run.
// Per run the source row, position and slot of every token are looked up once and kept in LDS; a
// thread then issues all the loads of its items before it uses the first (the items of a run are
// independent), so that the kernel is bound by bytes and not by a chain of load latencies.
constexpr int kScatterRows = 16;     // candidate rows per workgroup (4 or 8 measured the same, 1 or 2 slower)

template <typename T, int D>
__global__ __launch_bounds__(256) void rope_scatter_kernel(
    const T* __restrict__ k_new, const T* __restrict__ v_new, const int32_t* __restrict__ q_pos,
    const int32_t* __restrict__ slot_map, int n_q_tot, int hkv, InvFreq inv_freq,
    T* __restrict__ k_pool, T* __restrict__ v_pool, int n_blocks, const int32_t* __restrict__ src_rows,
    const T* __restrict__ v_shared, int n_shared_blocks, int32_t* __restrict__ v_map) {
  // slots of rows base-1 .. base+kScatterRows+14: the row before the first candidate (is it the same
  // block?) and the 15 rows a run starting at the last candidate can still cover; -1 = no row /
  // invalid slot
  __shared__ int sl[kScatterRows + kBlock];
  __shared__ int run_row[kBlock], run_pos[kBlock], run_slot[kBlock];   // by token of the run
  __shared__ int row_of_slot[kBlock];                                  // by slot of the block (-1: not in the run)
  const int tid = threadIdx.x, base = blockIdx.x * kScatterRows;
  if (tid < kScatterRows + kBlock) {
    const int j = base - 1 + tid;
    int v = -1;
    if (j >= 0 && j < n_q_tot) {
      v = slot_map[j];
      if (v < 0 || v >= n_blocks * kBlock) v = -1;
    }
    sl[tid] = v;
  }
  __syncthreads();
  for (int c = 0; c < kScatterRows; ++c) {                 // candidate row base + c (workgroup-uniform loop)
    const int slot0 = sl[c + 1];
    if (slot0 < 0) continue;
    const int blk = slot0 / kBlock;
    if (sl[c] >= 0 && sl[c] / kBlock == blk) continue;     // not the first row of its run
    int n_run = 1;
    while (n_run < kBlock && sl[c + 1 + n_run] >= 0 && sl[c + 1 + n_run] / kBlock == blk) ++n_run;
    const int j0 = base + c;
    __syncthreads();                                       // (the previous run's readers are done)
    if (tid < kBlock) {
      row_of_slot[tid] = -1;
      if (tid < n_run) {
        run_row[tid] = src_rows != nullptr ? src_rows[j0 + tid] : j0 + tid;   // (row of k_new, v_new this list row reads)
        run_pos[tid] = q_pos[j0 + tid];
        run_slot[tid] = sl[c + 1 + tid] % kBlock;
      }
    }
    __syncthreads();
    if (tid < n_run) row_of_slot[run_slot[tid]] = run_row[tid];
    __syncthreads();

    // K: one (token, KV head, 16-byte piece of the head's first half) per thread and item, together
    // with the matching piece of the second half: two 16-byte loads, kPer rotations, two 16-byte stores
    constexpr int kPer = 16 / sizeof(T), kPieces = D / 2 / kPer, kItems = 4;
    const int n_items = n_run * hkv * kPieces;
    for (int i0 = tid; i0 < n_items; i0 += 256 * kItems) {
      uint4 xv[kItems], yv[kItems];
#pragma unroll
      for (int u = 0; u < kItems; ++u) {
        const int idx = i0 + 256 * u;
        if (idx < n_items) {
          const int p = idx % kPieces, h = (idx / kPieces) % hkv, t = idx / (kPieces * hkv);
          const T* kp = k_new + (static_cast<size_t>(run_row[t]) * hkv + h) * D + kPer * p;
          xv[u] = *reinterpret_cast<const uint4*>(kp);
          yv[u] = *reinterpret_cast<const uint4*>(kp + D / 2);
        }
      }
#pragma unroll
      for (int u = 0; u < kItems; ++u) {
        const int idx = i0 + 256 * u;
        if (idx < n_items) {
          const int p = idx % kPieces, h = (idx / kPieces) % hkv, t = idx / (kPieces * hkv);
          const int pos = run_pos[t];
          T* ko = k_pool + ((static_cast<size_t>(blk) * hkv + h) * kBlock + run_slot[t]) * D + kPer * p;
          T x[kPer], y[kPer], ox[kPer], oy[kPer];
          *reinterpret_cast<uint4*>(x) = xv[u];
          *reinterpret_cast<uint4*>(y) = yv[u];
#pragma unroll
          for (int e = 0; e < kPer; ++e) {
            float cs, sn;
            if (sizeof(T) == 2) rot_cos_sin_fast(pos, inv_freq.f[kPer * p + e], &cs, &sn);   // (the result is rounded to bf16)
            else rot_cos_sin(pos, inv_freq.f[kPer * p + e], &cs, &sn);
            const float xf = to_float(x[e]), yf = to_float(y[e]);
            ox[e] = from_float<T>(xf * cs - yf * sn);
            oy[e] = from_float<T>(yf * cs + xf * sn);
          }
          *reinterpret_cast<uint4*>(ko) = *reinterpret_cast<uint4*>(ox);
          *reinterpret_cast<uint4*>(ko + D / 2) = *reinterpret_cast<uint4*>(oy);
        }
      }
    }

    // V: one (head, dim) row of 16 slots per thread and step.  The rows that are patched come
    // from the block that holds the page's values now: the request's own block, or - the first
    // time a token of the page is recomputed - the stored block the value map still points at
    // (copy-on-write; the map entry is cleared once the whole block has been written).
    constexpr int kVec = kBlock * sizeof(T) / 16;          // 16-byte vectors per row
    const size_t block_elems = static_cast<size_t>(hkv) * D * kBlock;
    const T* v_from = value_block<T>(v_pool, v_shared, n_shared_blocks, v_map, blk, block_elems);
    const bool pending = v_from != v_pool + static_cast<size_t>(blk) * block_elems;
    int src_of[kBlock];                                    // (workgroup-uniform: scalar registers)
#pragma unroll
    for (int k = 0; k < kBlock; ++k) src_of[k] = __builtin_amdgcn_readfirstlane(row_of_slot[k]);
    for (int idx = tid; idx < hkv * D; idx += 256) {
      const int h = idx / D, dcol = idx % D;
      uint4* rowp = reinterpret_cast<uint4*>(v_pool + ((static_cast<size_t>(blk) * hkv + h) * D + dcol) * kBlock);
      const uint4* fromp = reinterpret_cast<const uint4*>(v_from + (static_cast<size_t>(h) * D + dcol) * kBlock);
      T e[kBlock];
      if (n_run < kBlock) {
#pragma unroll
        for (int v = 0; v < kVec; ++v) reinterpret_cast<uint4*>(e)[v] = fromp[v];
      }
      const T* vcol = v_new + static_cast<size_t>(h) * D + dcol;
#pragma unroll
      for (int k = 0; k < kBlock; ++k)
        if (src_of[k] >= 0) e[k] = vcol[static_cast<size_t>(src_of[k]) * hkv * D];
#pragma unroll
      for (int v = 0; v < kVec; ++v) rowp[v] = reinterpret_cast<uint4*>(e)[v];
    }
    if (pending) {                       // (workgroup-uniform)
      __syncthreads();                   // every thread has looked the block up
      if (tid == 0) v_map[blk] = -1;
    }
  }
}

// Check of the order the scatter relies on: the rows of a 16-token block must form ONE run of
// adjacent list rows.  mark[block] (-1 on entry) takes the first row of the first run that names
// the block; every further run that names it counts as a violation.
__global__ __launch_bounds__(256) void fill_int_kernel(int32_t* __restrict__ p, int n, int32_t v) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ __launch_bounds__(256) void list_order_kernel(const int32_t* __restrict__ slot_map, int n_rows,
                                                          int n_blocks, int32_t* __restrict__ mark,
                                                          int32_t* __restrict__ n_violations) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j >= n_rows) return;
  const int slot = slot_map[j];
  if (slot < 0 || slot >= n_blocks * kBlock) return;            // (such rows are skipped by the scatter too)
  const int blk = slot / kBlock;
  if (j > 0) {
    const int prev = slot_map[j - 1];
    if (prev >= 0 && prev < n_blocks * kBlock && prev / kBlock == blk) return;   // not the first row of its run
  }
  if (atomicCAS(&mark[blk], -1, j) != -1) atomicAdd(n_violations, 1);
}

void launch_list_order_check(const int32_t* slot_map, int n_rows, int n_blocks, int32_t* mark,
                             int32_t* n_violations, hipStream_t stream) {
  hipLaunchKernelGGL(fill_int_kernel, dim3((n_blocks + 255) / 256), dim3(256), 0, stream, mark, n_blocks, -1);
  hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(256), 0, stream, n_violations, 1, 0);
  if (n_rows > 0)
    hipLaunchKernelGGL(list_order_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, stream, slot_map, n_rows,
                       n_blocks, mark, n_violations);
}

void launch_rope_scatter(const cc_ctx* ctx, const void* k_new, const void* v_new,
                         const int32_t* q_pos, const int32_t* slot_map, int n_q_tot, void* k_pool,
                         void* v_pool, int n_blocks, const int32_t* src_rows, hipStream_t stream,
                         const ValueSource& vs) {
  if (n_q_tot <= 0) return;
  const bool bf = ctx->cfg.dtype == CC_BF16;
  const int d = ctx->cfg.head_dim, hkv = ctx->cfg.n_kv_heads;
#define CC_LAUNCH(T, D)                                                                          \
  hipLaunchKernelGGL((rope_scatter_kernel<T, D>), dim3((n_q_tot + kScatterRows - 1) / kScatterRows), dim3(256), 0, stream,           \
                     static_cast<const T*>(k_new), static_cast<const T*>(v_new), q_pos, slot_map, \
                     n_q_tot, hkv, ctx->inv_freq, static_cast<T*>(k_pool), static_cast<T*>(v_pool), n_blocks, src_rows, \
                     static_cast<const T*>(vs.v_shared), vs.n_shared_blocks, vs.v_map)
  if (bf && d == 128) CC_LAUNCH(bf16_t, 128);
  else if (bf && d == 64) CC_LAUNCH(bf16_t, 64);
  else if (!bf && d == 128) CC_LAUNCH(float, 128);
  else CC_LAUNCH(float, 64);
#undef CC_LAUNCH
}

// Scalar attention: one wavefront per (query row, query head).  Lane i owns rotation pair
// (i, i + d/2) of q and the same two output dimensions.
template <typename T, int D>
__global__ __launch_bounds__(64) void attn_scalar_kernel(
    const T* __restrict__ q, const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    int n_requests, const T* __restrict__ k_pool, const T* __restrict__ v_pool, int n_blocks,
    const int32_t* __restrict__ block_tab, const cc_segment* __restrict__ segs,
    const int32_t* __restrict__ req_seg_off, int hq, int hkv, InvFreq inv_freq,
    T* __restrict__ out, float* __restrict__ lse, const int32_t* __restrict__ q_map, int map_pos,
    const T* __restrict__ v_shared, int n_shared_blocks, const int32_t* __restrict__ v_map) {
  const int j = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
  int r = 0;
  while (r + 1 < n_requests && cu_q[r + 1] <= j) ++r;
  if (j >= cu_q[n_requests]) return;                 // (the list may be shorter than its capacity)
  // with a row map, list row j takes its query from row q_map[j] of q (and, if map_pos, its
  // position from q_pos[q_map[j]])
  const int src = q_map != nullptr ? q_map[j] : j;
  const int p = q_pos[map_pos ? src : j];
  const int kvh = h / (hq / hkv);
  const bool own = lane < D / 2;
  float qx = 0.f, qy = 0.f;
  if (own) {
    const T* qp = q + (static_cast<size_t>(src) * hq + h) * D;
    float x = to_float(qp[lane]), y = to_float(qp[lane + D / 2]), c, s;
    rot_cos_sin(p, inv_freq.f[lane], &c, &s);
    qx = x * c - y * s;
    qy = y * c + x * s;
  }
  const float scale = rsqrtf(static_cast<float>(D));
  float m = -INFINITY, z = 0.f, ox = 0.f, oy = 0.f;
  for (int s = req_seg_off[r]; s < req_seg_off[r + 1]; ++s) {
    const cc_segment ks = segs[s];
    const int n_vis = min(ks.n_tokens, p - ks.logical_start + 1);
    for (int tk = 0; tk < n_vis; ++tk) {
      const int blk = block_tab[ks.tab_off + tk / kBlock];
      if (blk < 0 || blk >= n_blocks) continue;
      const size_t bh = static_cast<size_t>(blk) * hkv + kvh;
      const T* kp = k_pool + (bh * kBlock + tk % kBlock) * D;
      float part = own ? qx * to_float(kp[lane]) + qy * to_float(kp[lane + D / 2]) : 0.f;
      const float logit = wave_sum(part) * scale;
      if (logit > m) {
        const float a = expf(m - logit);
        z *= a; ox *= a; oy *= a;
        m = logit;
      }
      const float e = expf(logit - m);
      z += e;
      if (own) {
        const T* vp = value_block<T>(v_pool, v_shared, n_shared_blocks, v_map, blk, static_cast<size_t>(hkv) * D * kBlock) +
                      static_cast<size_t>(kvh) * D * kBlock + tk % kBlock;
        ox += e * to_float(vp[static_cast<size_t>(lane) * kBlock]);
        oy += e * to_float(vp[static_cast<size_t>(lane + D / 2) * kBlock]);
      }
    }
  }
  if (own && out != nullptr) {
    T* op = out + (static_cast<size_t>(j) * hq + h) * D;
    op[lane] = from_float<T>(ox / z);
    op[lane + D / 2] = from_float<T>(oy / z);
  }
  if (lse != nullptr && lane == 0) lse[static_cast<size_t>(j) * hq + h] = m + logf(z);
}

void launch_attn_scalar(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                        int n_q_tot, int max_q_per_req, const void* k_pool, const void* v_pool,
                        int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                        const int32_t* req_seg_off, int n_requests, void* out, float* lse,
                        const int32_t* q_map, int map_pos, hipStream_t stream, const ValueSource& vs) {
  (void)max_q_per_req;
  if (n_q_tot <= 0) return;
  const bool bf = ctx->cfg.dtype == CC_BF16;
  const int d = ctx->cfg.head_dim, hq = ctx->cfg.n_q_heads, hkv = ctx->cfg.n_kv_heads;
#define CC_LAUNCH(T, D)                                                                         \
  hipLaunchKernelGGL((attn_scalar_kernel<T, D>), dim3(n_q_tot, hq), dim3(64), 0, stream,        \
                     static_cast<const T*>(q), q_pos, cu_q, n_requests,                         \
                     static_cast<const T*>(k_pool), static_cast<const T*>(v_pool), n_blocks,    \
                     block_tab, segs, req_seg_off, hq, hkv, ctx->inv_freq, static_cast<T*>(out), lse, q_map, map_pos, \
                     static_cast<const T*>(vs.v_shared), vs.n_shared_blocks, vs.v_map)
  if (bf && d == 128) CC_LAUNCH(bf16_t, 128);
  else if (bf && d == 64) CC_LAUNCH(bf16_t, 64);
  else if (!bf && d == 128) CC_LAUNCH(float, 128);
  else CC_LAUNCH(float, 64);
#undef CC_LAUNCH
}

}  // namespace cc
