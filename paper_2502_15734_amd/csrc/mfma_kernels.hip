// MFMA (bf16, head_dim 128) kernels of cc_select's score stage and cc_sparse_prefill's attention.
//
// Both stages are "few queries against all earlier keys" (Sec. 4 "Selective Token Recomputation";
// per-token form of Eq. (1)).  One workgroup owns 32 query tokens of one request and one KV head;
// wavefront w owns query head kvh*G + w, so all G heads of the group share every K/V tile that
// is staged in LDS (grouped-query packing).  Key tiles are 64 keys (4 blocks of 16 tokens) and
// never straddle a segment, so block padding only shows up in a segment's last tile.
//
// Orientation: S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16.  In the 32x32 result
// a lane holds ONE query column (lane % 32) and 16 rows, so the softmax of a query (running max,
// exponentials, sum, rescale of O) is lane-local; the two lane halves, which hold different keys
// of the same query, exchange one value per tile.  P^T feeds the second product straight from the
// accumulator registers: within a 32-key block the MFMA row m of S^T is assigned the key
// swap_bits_2_3(m), which makes the 8 values a lane-half contributes to one 16-key step the keys
// 8*half .. 8*half+7 of one 16-token block -- exactly one 16-byte row piece of the dimension-major
// V block.
//
// LDS image of a tile (16-byte pieces; every MFMA operand read is one conflict-free 1 KiB run):
//   K piece (block b of 32 keys, k-step kk, half hh, row m):  (b*8+kk)*64 + hh*32 + (m ^ ((2kk+hh)&7))
//   V piece (page pg, 32-dim group db, half hh, dim n):       1024 + (pg*4+db)*64 + hh*32 + (n ^ 4hh)
// The XOR terms spread the *writes* of a coalesced global read over the LDS banks.
#include "device_util.h"

namespace cc {

namespace {

constexpr int kD = 128;
constexpr int kTile = 64;                      // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int swap23(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }

// Walks the key tiles of one request in prompt order, up to logical position p_max.
struct TileIter {
  const cc_segment* segs;
  int s, s_end, p_max;
  int kt, n_kt, seg_start, seg_ntok, seg_tab;
  bool valid;
  __device__ __forceinline__ void init(const cc_segment* sg, int s_begin, int s_end_, int p_max_) {
    segs = sg; s = s_begin - 1; s_end = s_end_; p_max = p_max_;
    kt = 0; n_kt = 0; seg_start = 0; seg_ntok = 0; seg_tab = 0; valid = true;
    advance();
  }
  __device__ __forceinline__ void advance() {
    ++kt;
    while (kt >= n_kt) {
      ++s;
      if (s >= s_end) { valid = false; return; }
      const cc_segment g = segs[s];
      if (g.logical_start > p_max) { valid = false; return; }
      seg_start = g.logical_start; seg_ntok = g.n_tokens; seg_tab = g.tab_off;
      const int n_keys = min(g.n_tokens, p_max - g.logical_start + 1);
      n_kt = (n_keys + kTile - 1) / kTile;
      kt = 0;
    }
  }
  __device__ __forceinline__ int kpos0() const { return seg_start + kTile * kt; }
  __device__ __forceinline__ int nvalid() const { return min(kTile, seg_ntok - kTile * kt); }
  __device__ __forceinline__ int tab0() const { return seg_tab + (kTile / kBlock) * kt; }
};

// Staging of one key tile (and, if WITH_V, the value tile) of KV head `kvh`: every thread owns
// PER 16-byte pieces, piece c = tid + NT*i of the tile in pool order (K pages 0..3, then V pages
// 0..3), so a wavefront instruction reads one contiguous KiB.  With NT a multiple of 256 a thread
// keeps the same place inside every page, and its LDS destination is one base per pool plus a
// constant per piece.  load() leaves the pieces in registers (issued one tile ahead of their
// use), store() writes them to LDS.  Slots past the segment's end are staged as zeros so that
// stale or non-finite padding can never reach a product.
template <int NT, bool WITH_V>
struct Stager {
  static_assert(NT % 256 == 0 || NT == 64 || NT == 128, "unsupported workgroup size");
  static constexpr int kPieces = WITH_V ? 2048 : 1024;
  static constexpr int PER = kPieces / NT;
  static constexpr int kBatch = PER < 8 ? PER : 8;      // pieces held in registers at a time
  static constexpr bool kPrefetch = PER <= 8;           // whole tile fits in registers
  uint4 reg[kBatch];
  const bf16_t* k_head;  // pools offset to this KV head
  const bf16_t* v_head;
  size_t blk_stride;     // elements per block (all heads)
  int n_blocks;
  int tid;

  __device__ __forceinline__ int piece(int i) const { return tid + NT * i; }
  __device__ __forceinline__ int page_of(int i) const { return (piece(i) & 1023) >> 8; }
  __device__ __forceinline__ bool is_v(int i) const { return WITH_V && piece(i) >= 1024; }
  __device__ __forceinline__ int src_of(int i) const { return (piece(i) & 255) * 8; }
  __device__ __forceinline__ int dst_of(int i) const {
    const int cc_ = piece(i) & 255, pg = page_of(i);
    if (!is_v(i)) {
      const int slot = cc_ >> 4, ch = cc_ & 15;
      // key a = 16*pg + slot of the tile -> block a/32, MFMA row swap23(a%32)
      return ((pg >> 1) * 8 + (ch >> 1)) * 64 + (ch & 1) * 32 + (((pg & 1) * 16 + swap23(slot)) ^ (ch & 7));
    }
    const int dcol = cc_ >> 1, hh = cc_ & 1;
    return 1024 + (pg * 4 + (dcol >> 5)) * 64 + hh * 32 + ((dcol & 31) ^ (4 * hh));
  }

  __device__ __forceinline__ void init(const bf16_t* k_pool, const bf16_t* v_pool, int n_blocks_,
                                       int hkv, int kvh, int tid_) {
    k_head = k_pool + static_cast<size_t>(kvh) * (kBlock * kD);
    v_head = WITH_V ? v_pool + static_cast<size_t>(kvh) * (kBlock * kD) : nullptr;
    blk_stride = static_cast<size_t>(hkv) * (kBlock * kD);
    n_blocks = n_blocks_;
    tid = tid_;
  }

  // pieces [i0, i0 + kBatch) of the tile -> reg
  __device__ __forceinline__ void load(const int32_t* __restrict__ block_tab, int tab0, int nvalid, int i0 = 0) {
    if (nvalid == kTile) {                         // whole tile present (wave-uniform)
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int i = i0 + j;
        const int blk = block_tab[tab0 + page_of(i)];
        const bool ok = blk >= 0 && blk < n_blocks;
        const bf16_t* base = (is_v(i) ? v_head : k_head) + static_cast<size_t>(ok ? blk : 0) * blk_stride;
        reg[j] = ok ? *reinterpret_cast<const uint4*>(base + src_of(i)) : make_uint4(0u, 0u, 0u, 0u);
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int i = i0 + j;
      const int pg = page_of(i), src = src_of(i);
      const int nv = min(max(nvalid - kBlock * pg, 0), kBlock);
      int blk = -1;
      if (nv > 0) blk = block_tab[tab0 + pg];
      const bool ok = blk >= 0 && blk < n_blocks;
      uint4 val = make_uint4(0u, 0u, 0u, 0u);
      if (ok) {
        if (!is_v(i)) {
          if ((src >> 7) < nv)                     // src/8 = piece in page, /16 = token slot
            val = *reinterpret_cast<const uint4*>(k_head + static_cast<size_t>(blk) * blk_stride + src);
        } else {
          val = *reinterpret_cast<const uint4*>(v_head + static_cast<size_t>(blk) * blk_stride + src);
          if (nv < kBlock) {                       // zero the padding slots of a partly filled block
            const int hh = (src >> 3) & 1;
            unsigned short e[8];
            *reinterpret_cast<uint4*>(e) = val;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) if (8 * hh + jj >= nv) e[jj] = 0;
            val = *reinterpret_cast<uint4*>(e);
          }
        }
      }
      reg[j] = val;
    }
  }

  __device__ __forceinline__ void store(uint4* lds, int i0 = 0) const {
#pragma unroll
    for (int j = 0; j < kBatch; ++j) lds[dst_of(i0 + j)] = reg[j];
  }

  // small workgroups: the tile does not fit in registers, copy it batch by batch
  __device__ __forceinline__ void copy(uint4* lds, const int32_t* __restrict__ block_tab, int tab0, int nvalid) {
#pragma unroll 1
    for (int i0 = 0; i0 < PER; i0 += kBatch) {
      load(block_tab, tab0, nvalid, i0);
      store(lds, i0);
    }
  }
};

__device__ __forceinline__ float max16(const f32x16& v) {
  float a = fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3]));
  float b = fmaxf(fmaxf(v[4], v[5]), fmaxf(v[6], v[7]));
  float c = fmaxf(fmaxf(v[8], v[9]), fmaxf(v[10], v[11]));
  float d = fmaxf(fmaxf(v[12], v[13]), fmaxf(v[14], v[15]));
  return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

// SCORE = true : queries are 32 consecutive tokens of a chunk segment; result is the share of the
//                softmax mass that falls on keys of earlier segments (Eq. (2), Eq. (10)).
// SCORE = false: queries are 32 rows of the compact query list; result is the attention output
//                and log-sum-exp (Eq. (1)).
template <int G, bool SCORE>
__global__ __launch_bounds__(64 * G, 2) void sparse_qk_kernel(
    const bf16_t* __restrict__ q, const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool, int n_blocks,
    const int32_t* __restrict__ block_tab, const cc_segment* __restrict__ segs,
    const int32_t* __restrict__ req_seg_off, int hq, int hkv, int n_tiles_x, InvFreq inv_freq,
    bf16_t* __restrict__ out, float* __restrict__ lse, float* __restrict__ mass) {
  constexpr int NT = 64 * G;
  constexpr int kImage = SCORE ? 1024 : 2048;      // 16-byte pieces per tile image
  __shared__ uint4 lds_all[2 * kImage];            // double-buffered
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, hh = lane >> 5;
  const int kvh = blockIdx.x % hkv;
  const int tile = n_tiles_x - 1 - blockIdx.x / hkv;       // late (long) tiles are dispatched first
  const int h = kvh * G + wave;

  // ---- which queries ------------------------------------------------------------------------
  int row, p, s_begin, s_end, s_self = -1;
  bool row_valid;
  if constexpr (SCORE) {
    const cc_segment sg = segs[blockIdx.y];
    const int t0 = tile * 32;
    if (sg.kind != CC_SEG_CHUNK || t0 >= sg.n_tokens || sg.logical_start == 0) return;
    const int t = min(t0 + n, sg.n_tokens - 1);
    row_valid = t0 + n < sg.n_tokens;
    row = sg.tok_off + t;
    p = sg.logical_start + t;
    s_begin = req_seg_off[sg.req];
    s_self = blockIdx.y;
    s_end = s_self + 1;
  } else {
    const int r = blockIdx.y;
    const int q0 = cu_q[r] + tile * 32, q_end = cu_q[r + 1];
    if (q0 >= q_end) return;
    row = min(q0 + n, q_end - 1);
    row_valid = q0 + n < q_end;
    p = q_pos[row];
    s_begin = req_seg_off[r];
    s_end = req_seg_off[r + 1];
  }
  const int p_max = wave_max_i(p), p_min = wave_min_i(p);

  // ---- load the query rows and rotate them to their positions ---------------------------------
  // lane (n, hh) keeps, for k-step kk, dims 16kk + 8hh .. +7; dims < 64 pair with dims + 64.
  bf16x8 qreg[8];
  {
    const bf16_t* qp = q + (static_cast<size_t>(row) * hq + h) * kD + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      qreg[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + 16 * kk));
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float c, s;
        rot_cos_sin_fast(p, inv_freq.f[16 * kk + 8 * hh + j], &c, &s);
        const float x = static_cast<float>(qreg[kk][j]), y = static_cast<float>(qreg[kk + 4][j]);
        qreg[kk][j] = static_cast<bf16_t>(x * c - y * s);
        qreg[kk + 4][j] = static_cast<bf16_t>(y * c + x * s);
      }
    }
  }

  const float c2 = 0.08838834764831845f * kLog2e;           // log2(e) / sqrt(128)
  float m_run = -INFINITY, l_run = 0.f, l_prior = 0.f;
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

  Stager<NT, !SCORE> stg;
  stg.init(k_pool, v_pool, n_blocks, hkv, kvh, tid);
  TileIter it;
  it.init(segs, s_begin, s_end, p_max);
  constexpr bool kPrefetch = Stager<NT, !SCORE>::kPrefetch;
  if (it.valid) stg.copy(lds_all, block_tab, it.tab0(), it.nvalid());
  __syncthreads();
  int buf = 0;
  while (it.valid) {
    if constexpr (SCORE) {
      // entering the query's own segment: everything summed so far is prior-chunk mass
      if (it.s == s_self && it.kt == 0) { l_prior = l_run; l_run = 0.f; }
    }
    const int kpos0 = it.kpos0(), nvalid = it.nvalid();
    const uint4* lds = lds_all + buf * kImage;
    it.advance();
    if (kPrefetch && it.valid) stg.load(block_tab, it.tab0(), it.nvalid());   // next tile: loads in flight

    // ---- S^T = K Q^T : 2 blocks of 32 keys x 32 queries ------------------------------------
    f32x16 sacc[2];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) sacc[b][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
      for (int b = 0; b < 2; ++b) {
        const bf16x8 a = __builtin_bit_cast(
            bf16x8, lds[(b * 8 + kk) * 64 + hh * 32 + (n ^ ((2 * kk + hh) & 7))]);
        sacc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[kk], sacc[b], 0, 0, 0);
      }
    }
    // accumulator register i of block b holds key 32b + 16(i/8) + 8hh + i%8 of the tile
    if (nvalid < kTile || kpos0 + kTile - 1 > p_min) {     // wave-uniform: padding or causal edge
      const int lim = min(nvalid - 1, p - kpos0) - 8 * hh;
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          sacc[b][i] = (32 * b + 16 * (i / 8) + (i % 8) <= lim) ? sacc[b][i] : -INFINITY;
    }
    // ---- online softmax, one query per lane --------------------------------------------------
    float tmax = fmaxf(max16(sacc[0]), max16(sacc[1]));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(m_run, tmax);
    if (__any(m_new > m_run)) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c2);
      l_run *= alpha;
      if constexpr (SCORE) l_prior *= alpha;
      else {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
      }
      m_run = m_new;
    }
    const float mc = m_run * c2;
    float lsum = 0.f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        sacc[b][i] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[b][i], c2, -mc));
        lsum += sacc[b][i];
      }
    l_run += lsum;

    if constexpr (!SCORE) {
      // ---- O^T += V^T P^T : P^T comes straight from the accumulator registers ----------------
#pragma unroll
      for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          bf16x8 pb;
#pragma unroll
          for (int j = 0; j < 8; ++j) pb[j] = static_cast<bf16_t>(sacc[b][8 * u + j]);
          const int pg = 2 * b + u;
#pragma unroll
          for (int db = 0; db < 4; ++db) {
            const bf16x8 a = __builtin_bit_cast(
                bf16x8, lds[1024 + (pg * 4 + db) * 64 + hh * 32 + (n ^ (4 * hh))]);
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, o[db], 0, 0, 0);
          }
        }
      }
    }
    if (it.valid) {
      if (kPrefetch) stg.store(lds_all + (buf ^ 1) * kImage);
      else stg.copy(lds_all + (buf ^ 1) * kImage, block_tab, it.tab0(), it.nvalid());
    }
    __syncthreads();
    buf ^= 1;
  }

  // ---- epilogue ---------------------------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if constexpr (SCORE) {
    const float lp = l_prior + __shfl_xor(l_prior, 32, 64);
    if (row_valid && hh == 0) mass[static_cast<size_t>(row) * hq + h] = lp / (lp + l_tot);
  } else {
    const float inv = 1.f / l_tot;
    if (row_valid) {
      bf16_t* op = out + (static_cast<size_t>(row) * hq + h) * kD;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16_t v4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v4[e] = static_cast<bf16_t>(o[db][4 * g4 + e] * inv);
          // accumulator register i holds output dim 32db + 8(i/4) + 4hh + i%4
          *reinterpret_cast<uint2*>(op + 32 * db + 8 * g4 + 4 * hh) = *reinterpret_cast<uint2*>(v4);
        }
      if (lse != nullptr && hh == 0)
        lse[static_cast<size_t>(row) * hq + h] = kLn2 * (m_run * c2 + __builtin_amdgcn_logf(l_tot));
    }
  }
}

template <int G>
void launch_attn_g(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                   int max_q_per_req, const void* k_pool, const void* v_pool, int n_blocks,
                   const int32_t* block_tab, const cc_segment* segs, const int32_t* req_seg_off,
                   int n_requests, void* out, float* lse, hipStream_t stream) {
  const int hkv = ctx->cfg.n_kv_heads, n_tiles = (max_q_per_req + 31) / 32;
  dim3 grid(hkv * n_tiles, n_requests);
  hipLaunchKernelGGL((sparse_qk_kernel<G, false>), grid, dim3(64 * G), 0, stream,
                     static_cast<const bf16_t*>(q), q_pos, cu_q, static_cast<const bf16_t*>(k_pool),
                     static_cast<const bf16_t*>(v_pool), n_blocks, block_tab, segs, req_seg_off,
                     ctx->cfg.n_q_heads, hkv, n_tiles, ctx->inv_freq, static_cast<bf16_t*>(out), lse,
                     static_cast<float*>(nullptr));
}

template <int G>
void launch_score_g(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks,
                    const int32_t* block_tab, const cc_segment* segs, int n_segs,
                    const int32_t* req_seg_off, int max_seg_tokens, float* mass, hipStream_t stream) {
  const int hkv = ctx->cfg.n_kv_heads, n_tiles = (max_seg_tokens + 31) / 32;
  dim3 grid(hkv * n_tiles, n_segs);
  hipLaunchKernelGGL((sparse_qk_kernel<G, true>), grid, dim3(64 * G), 0, stream,
                     static_cast<const bf16_t*>(q), static_cast<const int32_t*>(nullptr),
                     static_cast<const int32_t*>(nullptr), static_cast<const bf16_t*>(k_pool),
                     static_cast<const bf16_t*>(nullptr), n_blocks, block_tab, segs, req_seg_off,
                     ctx->cfg.n_q_heads, hkv, n_tiles, ctx->inv_freq, static_cast<bf16_t*>(nullptr),
                     static_cast<float*>(nullptr), mass);
}

bool group_supported(const cc_ctx* ctx) {
  if (ctx->cfg.dtype != CC_BF16 || ctx->cfg.head_dim != kD) return false;
  const int g = ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads;
  return g == 1 || g == 2 || g == 4 || g == 8;
}

}  // namespace

bool attn_mfma_supported(const cc_ctx* ctx) { return group_supported(ctx); }
bool score_mfma_supported(const cc_ctx* ctx) { return group_supported(ctx); }

void launch_attn_mfma(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                      int n_q_tot, int max_q_per_req, const void* k_pool, const void* v_pool,
                      int n_blocks, const int32_t* block_tab, const cc_segment* segs,
                      const int32_t* req_seg_off, int n_requests, void* out, float* lse,
                      hipStream_t stream) {
  (void)n_q_tot;
#define CC_ARGS ctx, q, q_pos, cu_q, max_q_per_req, k_pool, v_pool, n_blocks, block_tab, segs, req_seg_off, n_requests, out, lse, stream
  switch (ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads) {
    case 1: launch_attn_g<1>(CC_ARGS); break;
    case 2: launch_attn_g<2>(CC_ARGS); break;
    case 4: launch_attn_g<4>(CC_ARGS); break;
    default: launch_attn_g<8>(CC_ARGS); break;
  }
#undef CC_ARGS
}

void launch_score_mfma(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks,
                       const int32_t* block_tab, const cc_segment* segs, int n_segs,
                       const int32_t* req_seg_off, int max_seg_tokens, float* mass,
                       hipStream_t stream) {
#define CC_ARGS ctx, q, k_pool, n_blocks, block_tab, segs, n_segs, req_seg_off, max_seg_tokens, mass, stream
  switch (ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads) {
    case 1: launch_score_g<1>(CC_ARGS); break;
    case 2: launch_score_g<2>(CC_ARGS); break;
    case 4: launch_score_g<4>(CC_ARGS); break;
    default: launch_score_g<8>(CC_ARGS); break;
  }
#undef CC_ARGS
}

}  // namespace cc
