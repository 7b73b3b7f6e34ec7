// cc_select, plain kernels: per-token prior-chunk attention mass (scalar reference-grade path)
// and the per-chunk top-N (Eq. (2), Eq. (10), Sec. 3.2.1).
#include "device_util.h"

namespace cc {

// ---------------------------------------------------------------------------------------------
// Scalar score kernel: one wavefront per (chunk token, query head).  Lane i owns rotation pair
// (i, i + d/2) of the query; keys of the request are visited in logical order, each logit is a
// wavefront reduction.  Used for fp32 and as the fallback for shapes the MFMA kernel lacks.
// ---------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(64) void score_scalar_kernel(
    const T* __restrict__ q, const T* __restrict__ k_pool, int n_blocks,
    const int32_t* __restrict__ block_tab, const cc_segment* __restrict__ segs,
    const int32_t* __restrict__ req_seg_off, int hq, int hkv, InvFreq inv_freq,
    float* __restrict__ mass) {
  const cc_segment sg = segs[blockIdx.y];
  const int t = blockIdx.x, h = blockIdx.z, lane = threadIdx.x;
  if (sg.kind != CC_SEG_CHUNK || t >= sg.n_tokens) return;
  const size_t row = static_cast<size_t>(sg.tok_off) + t;
  if (sg.logical_start == 0) {              // first chunk: no prior chunk to attend to
    if (lane == 0) mass[row * hq + h] = 0.f;
    return;
  }
  const int p = sg.logical_start + t;
  const int kvh = h / (hq / hkv);
  const bool own = lane < D / 2;
  float qx = 0.f, qy = 0.f;
  if (own) {
    const T* qp = q + (row * hq + h) * D;
    float x = to_float(qp[lane]), y = to_float(qp[lane + D / 2]), c, s;
    rot_cos_sin(p, inv_freq.f[lane], &c, &s);
    qx = x * c - y * s;
    qy = y * c + x * s;
  }
  const float scale = rsqrtf(static_cast<float>(D));
  float m = -INFINITY, z_prior = 0.f, z_all = 0.f;
  const int s_begin = req_seg_off[sg.req], s_self = blockIdx.y;
  for (int s = s_begin; s <= s_self; ++s) {
    const cc_segment ks = segs[s];
    const int n_vis = min(ks.n_tokens, p - ks.logical_start + 1);
    float z_seg = 0.f;
    for (int tk = 0; tk < n_vis; ++tk) {
      const int blk = block_tab[ks.tab_off + tk / kBlock];
      if (blk < 0 || blk >= n_blocks) continue;
      const T* kp = k_pool + ((static_cast<size_t>(blk) * hkv + kvh) * kBlock + tk % kBlock) * D;
      float part = own ? qx * to_float(kp[lane]) + qy * to_float(kp[lane + D / 2]) : 0.f;
      const float logit = wave_sum(part) * scale;
      if (logit > m) {                       // wave-uniform
        const float a = expf(m - logit);
        z_all *= a; z_seg *= a; z_prior *= a;
        m = logit;
      }
      const float e = expf(logit - m);
      z_all += e; z_seg += e;
    }
    if (s < s_self) z_prior += z_seg;
  }
  if (lane == 0) mass[row * hq + h] = z_prior / z_all;
}

template <typename T, int D>
static void launch_score_t(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks,
                           const int32_t* block_tab, const cc_segment* segs, int n_segs,
                           const int32_t* req_seg_off, int max_seg_tokens, float* mass,
                           hipStream_t stream) {
  dim3 grid(max_seg_tokens, n_segs, ctx->cfg.n_q_heads);
  hipLaunchKernelGGL((score_scalar_kernel<T, D>), grid, dim3(64), 0, stream,
                     static_cast<const T*>(q), static_cast<const T*>(k_pool), n_blocks, block_tab,
                     segs, req_seg_off, ctx->cfg.n_q_heads, ctx->cfg.n_kv_heads, ctx->inv_freq, mass);
}

void launch_score_scalar(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks,
                         const int32_t* block_tab, const cc_segment* segs, int n_segs,
                         const int32_t* req_seg_off, int max_seg_tokens, float* mass,
                         hipStream_t stream) {
  const bool bf = ctx->cfg.dtype == CC_BF16;
  const int d = ctx->cfg.head_dim;
#define CC_ARGS ctx, q, k_pool, n_blocks, block_tab, segs, n_segs, req_seg_off, max_seg_tokens, mass, stream
  if (bf && d == 128) launch_score_t<bf16_t, 128>(CC_ARGS);
  else if (bf && d == 64) launch_score_t<bf16_t, 64>(CC_ARGS);
  else if (!bf && d == 128) launch_score_t<float, 128>(CC_ARGS);
  else launch_score_t<float, 64>(CC_ARGS);
#undef CC_ARGS
}

// ---------------------------------------------------------------------------------------------
// Top-N per chunk.  One workgroup per segment.  score = mean over heads of the mass; the N-th
// largest score is found by building its bit pattern from the top bit down (32 counting rounds
// with wavefront ballots), then tokens above it, and the lowest-index tokens equal to it, are
// written in ascending index order through a workgroup-wide prefix count.  Equal scores go to
// the lower index, so the result is unique.
// ---------------------------------------------------------------------------------------------
constexpr int kTopnThreads = 256;
constexpr int kTopnLds = 4096;              // chunk lengths up to this are ranked out of LDS

__device__ __forceinline__ uint32_t ordered_key(float v) {   // monotone float -> uint
  uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int block_sum_i(int v, int* red) {  // sum over 256 threads, all get it
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(kTopnThreads) void topn_kernel(
    const float* __restrict__ mass, int hq, bool given, const int32_t* __restrict__ block_tab,
    const cc_segment* __restrict__ segs, int32_t* __restrict__ sel_idx, int32_t* __restrict__ q_row,
    int32_t* __restrict__ q_pos, int32_t* __restrict__ slot_map, float* __restrict__ scores,
    uint32_t* __restrict__ key_buf) {
  __shared__ uint32_t lds_keys[kTopnLds];
  __shared__ int red[4];
  __shared__ int wave_off[2][4];
  const cc_segment sg = segs[blockIdx.x];
  const int n = sg.n_tokens, tid = threadIdx.x;
  auto emit = [&](int j, int idx) {
    const int o = sg.sel_off + j;
    sel_idx[o] = idx;
    if (q_row) q_row[o] = sg.tok_off + idx;
    if (q_pos) q_pos[o] = sg.logical_start + idx;
    if (slot_map) slot_map[o] = block_tab[sg.tab_off + idx / kBlock] * kBlock + idx % kBlock;
  };
  if (sg.kind != CC_SEG_CHUNK) {            // question: every token is a query
    for (int i = tid; i < n; i += kTopnThreads) emit(i, i);
    return;
  }
  const int n_sel = min(max(sg.n_select, 0), n);
  uint32_t* keys = (n <= kTopnLds) ? lds_keys : key_buf + sg.tok_off;
  const float inv_h = 1.f / static_cast<float>(hq);
  for (int i = tid; i < n; i += kTopnThreads) {
    float sc = 0.f;
    if (given) {                            // scores supplied by the caller, one per token
      sc = mass[static_cast<size_t>(sg.tok_off) + i];
    } else if (sg.logical_start > 0) {
      // (summed head by head in index order whatever the load width, so the result does not
      //  depend on it)
      const float* mp = mass + (static_cast<size_t>(sg.tok_off) + i) * hq;
      if ((hq & 3) == 0) {
        const float4* mp4 = reinterpret_cast<const float4*>(mp);
#pragma unroll 8
        for (int h4 = 0; h4 < hq / 4; ++h4) {
          const float4 v = mp4[h4];
          sc += v.x; sc += v.y; sc += v.z; sc += v.w;
        }
      } else {
        for (int h = 0; h < hq; ++h) sc += mp[h];
      }
      sc *= inv_h;
    }
    if (scores) scores[sg.tok_off + i] = sc;
    keys[i] = ordered_key(sc);
  }
  __syncthreads();
  if (n_sel == 0) return;
  // N-th largest key, most significant bit first
  // (a wavefront counts with ballots; the four wavefront counts meet in LDS, in two alternating
  //  sets of cells so that one barrier per round is enough)
  __shared__ int round_cnt[2][4];
  uint32_t thr = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = thr | (1u << bit);
    int cnt = 0;
    for (int i0 = 0; i0 < n; i0 += kTopnThreads) {
      const int i = i0 + tid;
      cnt += __popcll(__ballot(i < n && keys[i] >= cand));
    }
    int* cell = round_cnt[bit & 1];
    if ((tid & 63) == 0) cell[tid >> 6] = cnt;
    __syncthreads();
    if (cell[0] + cell[1] + cell[2] + cell[3] >= n_sel) thr = cand;
  }
  int cnt = 0;
  for (int i = tid; i < n; i += kTopnThreads) cnt += keys[i] > thr;
  const int n_gt = block_sum_i(cnt, red);
  const int n_eq_take = n_sel - n_gt;       // how many of the ties (lowest indices) are kept
  // ordered compaction, 256 tokens per round
  int base_sel = 0, base_eq = 0;
  const int lane = tid & 63, w = tid >> 6;
  for (int i0 = 0; i0 < n; i0 += kTopnThreads) {
    const int i = i0 + tid;
    const uint32_t k = i < n ? keys[i] : 0u;
    const bool gt = i < n && k > thr, eq = i < n && k == thr;
    const unsigned long long b_eq = __ballot(eq);
    const unsigned long long below = (1ull << lane) - 1ull;
    __syncthreads();
    if (lane == 0) wave_off[0][w] = __popcll(b_eq);
    __syncthreads();
    int eq_rank = base_eq + __popcll(b_eq & below);
    for (int ww = 0; ww < w; ++ww) eq_rank += wave_off[0][ww];
    const int eq_round = wave_off[0][0] + wave_off[0][1] + wave_off[0][2] + wave_off[0][3];
    const bool take = gt || (eq && eq_rank < n_eq_take);
    const unsigned long long b_tk = __ballot(take);
    if (lane == 0) wave_off[1][w] = __popcll(b_tk);
    __syncthreads();
    int pos = base_sel + __popcll(b_tk & below);
    for (int ww = 0; ww < w; ++ww) pos += wave_off[1][ww];
    if (take) emit(pos, i);
    base_sel += wave_off[1][0] + wave_off[1][1] + wave_off[1][2] + wave_off[1][3];
    base_eq += eq_round;
  }
}

void launch_topn(const cc_ctx* ctx, const float* mass, const int32_t* block_tab,
                 const cc_segment* segs, int n_segs, int32_t* sel_idx, int32_t* q_row,
                 int32_t* q_pos, int32_t* slot_map, float* scores, uint32_t* key_buf,
                 bool given, hipStream_t stream) {
  hipLaunchKernelGGL(topn_kernel, dim3(n_segs), dim3(kTopnThreads), 0, stream, mass,
                     ctx->cfg.n_q_heads, given, block_tab, segs, sel_idx, q_row, q_pos, slot_map, scores,
                     key_buf);
}

}  // namespace cc
