// cc_select's score stage for head groups that are a multiple of 4 (bf16, head_dim 128): share of a
// chunk token's softmax mass that falls on keys of earlier chunks (Eq. (2), block matrix below
// Eq. (3), Eq. (10)).
//
// One workgroup = 4 wavefronts = 4 query heads of one KV head x 128 consecutive tokens of a chunk;
// a wavefront owns one head and all 128 tokens (four 32-row MFMA column blocks), so every K operand
// it reads from LDS feeds four MFMAs and one staged K tile serves 512 (token, head) columns.  The
// four rotated query blocks sit in accumulation registers (128), one S block in vector registers
// (64): 256 registers in all, so two workgroups share a compute unit.  A wavefront alternates
// between the 32 MFMAs of a 32-key block and the block's 64 exponentials; the two wavefronts of a
// SIMD fall out of phase, so the matrix pipe works for one while the vector ALU works for the
// other.  The two phases cost about the same (one exp2 and one add per 2 d flops).
//
// Orientation, key permutation and masking are those of mfma_tile.h: S^T = K Q^T with
// v_mfma_f32_32x32x16_bf16, a lane holds one token column, the sums stay lane-local.  The query is
// pre-multiplied by log2(e)/sqrt(d), so p = exp2(S): no reference is subtracted.  That is exact as
// long as the sums stay in range; a workgroup whose sums leave the safe range (logits beyond about
// +-60) flags its tokens and the kernel that carries a movable reference redoes them (see the
// launcher).
//
// Staging: four K-tile images in LDS (16 KiB each), filled by loads that write LDS directly
// (global_load_lds, lane L of an instruction fills piece base + L):
//   K piece (block b of 32 keys, k-step kk, half hh, MFMA row m):  (b*8+kk)*64 + hh*32 + m
// In iteration t the wavefronts read image t and start the loads of image t+3; before the
// iteration's barrier each wavefront waits until its loads of image t+2 have landed.  Padding
// slots of K never reach a sum: their S entries are masked by selection.
#include <type_traits>

#include "mfma_tile.h"

namespace cc {

using namespace tile;

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kQB = 4;            // 32-token column blocks per wavefront
constexpr int kTQ = 32 * kQB;     // tokens per workgroup
constexpr int kImageK = 1024;     // 16-byte pieces per K tile image
constexpr int kBufs = 4;
constexpr int kDepth = 4;         // operand reads in flight ahead of the MFMAs (each feeds four of them)
// p = exp2(S) with no reference: sums outside this range leave too little headroom (above) or may
// have lost small terms to underflow (below)
constexpr float kSafeSum = 1.0e30f;
constexpr float kTinySum = 1.0e-18f;

// 64 lanes x 16 bytes from global memory straight into LDS: lane L's 16 bytes land at
// lds_addr + 16 L (lds_addr wave-uniform).  Written as an instruction the compiler does not model:
// it would otherwise drain every outstanding load before the next LDS read, because it cannot see
// that the image being filled is not the image being read.  Completion is counted by vmcnt.
__device__ __forceinline__ void load_to_lds(const void* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(src), "s"(lds_addr) : "memory", "m0");
}

// MFMA forms with fixed register classes (see attn_mfma2.hip): S accumulates in vector registers,
// the rotated query is the B operand out of accumulation registers.  The results are opaque to the
// compiler's hazard handling, so the vector ALU reads them only behind mfma_result_wait().
__device__ __forceinline__ void mfma_s_first(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_s_acc(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_result_wait() {
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}
// l += exp2(a0) + exp2(a1).  Written out so that it stays where it is placed, under one MFMA (the
// compiler otherwise lumps all exponentials of a block together right after its last MFMA); each
// exponential is two instructions ahead of the add that reads it, which covers the wait state a
// transcendental result needs.
__device__ __forceinline__ void exp2_sum2(float& l, float a0, float a1) {
  float t0, t1;
  asm volatile("v_exp_f32 %1, %3\n\tv_exp_f32 %2, %4\n\tv_add_f32 %0, %0, %1\n\tv_add_f32 %0, %0, %2"
               : "+v"(l), "=&v"(t0), "=&v"(t1) : "v"(a0), "v"(a1));
}
// one 16-byte LDS piece straight into accumulation registers
__device__ __forceinline__ u32x4 lds_to_acc(const uint4* p) {
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)p));   // LDS byte offset
  u32x4 r;
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=a"(r) : "v"(addr) : "memory");
  return r;
}

// RAGGED = false: the workgroups whose four column blocks all hold tokens of the chunk (straight-line
//                  loop body; a chunk's last workgroup leaves at once if it holds fewer).
// RAGGED = true : one workgroup per (segment, head group) for exactly those last workgroups: the
//                  column blocks past the chunk's end cost no MFMA and no exponential (uniform
//                  branches around them, which the straight-line form does not have to carry).
template <bool RAGGED>
__global__ __launch_bounds__(256, 2) void score_v2_kernel(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_pool, int n_blocks,
    const TileDesc* __restrict__ tiles, int max_tiles,
    const WorkItem* __restrict__ items, int hq, int hkv, int n_sub, int n_tiles_x,
    InvFreq inv_freq, float* __restrict__ mass, int32_t* __restrict__ redo) {
  __shared__ uint4 lds_all[kBufs * kImageK];
  const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
  const int n = lane & 31, hh = lane >> 5;
  const int per_tile = hkv * n_sub;
  const int rem = blockIdx.x % per_tile;
  const int kvh = rem % hkv, hsub = rem / hkv;
  const int h = kvh * (4 * n_sub) + hsub * 4 + wave;

  // ---- which tokens ---------------------------------------------------------------------------
  // (one load; the fields go to scalar registers, token indices are recomputed from them where
  // needed, which keeps the vector registers for the queries and the S blocks)
  const uint4* ip = reinterpret_cast<const uint4*>(items + blockIdx.y);      // heaviest segments first
  const uint4 i0 = ip[0], i1 = ip[1];
  const int sg_kind = uniform(i0.y), sg_start = uniform(i0.z), sg_ntok = uniform(i0.w);
  const int sg_tok_off = uniform(i1.x), j_begin = uniform(i1.y), j_own = uniform(i1.z);
  // (RAGGED: the grid has one x-row per head group, and the tile is the chunk's last)
  const int tile = RAGGED ? max(sg_ntok - 1, 0) / kTQ : n_tiles_x - 1 - blockIdx.x / per_tile;    // late (long) tiles are dispatched first
  const int t0 = tile * kTQ;
  if (sg_kind != CC_SEG_CHUNK || t0 >= sg_ntok || sg_start == 0) return;
  // column blocks that hold tokens of the chunk
  const int n_cols = uniform((min(t0 + kTQ, sg_ntok) - t0 + 31) >> 5);
  if (RAGGED ? n_cols == kQB : n_cols < kQB) return;
  // token of column block qb in this lane (clamped into the chunk)
  auto token = [&](int qb) __attribute__((always_inline)) { return min(t0 + 32 * qb + n, sg_ntok - 1); };
  const int p_min = sg_start + t0;
  const int p_max = sg_start + min(t0 + kTQ, sg_ntok) - 1;

  // ---- key tiles: everything before the chunk, then the chunk's own tiles up to the last token --
  const int n_t = uniform(min(j_own + (p_max - sg_start) / kTile + 1, max_tiles) - j_begin);
  const int t_own = uniform(j_own - j_begin);                         // first tile of the token's own chunk
  if (n_t <= 0) return;

  // ---- load the query rows, rotate them to their positions, fold the softmax scale -------------
  // lane (n, hh) keeps, for k-step kk, dims 16kk + 8hh .. +7; dims < 64 pair with dims + 64.
  const float c2 = 0.08838834764831845f * kLog2e;            // log2(e) / sqrt(128)
  __shared__ uint4 q_bounce[256];     // one piece per lane: the way into the accumulation registers
  u32x4 qreg[kQB][8];
  // (called after the first tile loads are on their way, so that the trigonometry hides their latency)
  // The four column blocks of a lane sit 32 positions apart, so only the first block's angles take
  // the double-precision path; each further block turns them by the fixed angle 32 f (a single-
  // precision product is exact enough for that small angle).  Columns past the chunk's end get a
  // query row and a position that do not belong together; nothing of theirs is written.
  auto load_queries = [&]() __attribute__((always_inline)) {
    const bf16_t* qp[kQB];
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb)
      qp[qb] = q + (static_cast<size_t>(sg_tok_off + token(qb)) * hq + h) * kD + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 xv[kQB], yv[kQB];
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        xv[qb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp[qb] + 16 * kk));
        yv[qb] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp[qb] + 16 * kk + 64));
      }
      float cs[8], sn[8], ct[8], st[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const double f = inv_freq.f[16 * kk + 8 * hh + j];
        rot_cos_sin_fast(sg_start + t0 + n, f, &cs[j], &sn[j]);
        cs[j] *= c2; sn[j] *= c2;
        const float turn = static_cast<float>(f) * (32.f * 0.15915494309189535f);    // revolutions
        ct[j] = __builtin_amdgcn_cosf(turn);
        st[j] = __builtin_amdgcn_sinf(turn);
      }
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float x = static_cast<float>(xv[qb][j]), y = static_cast<float>(yv[qb][j]);
          xv[qb][j] = static_cast<bf16_t>(x * cs[j] - y * sn[j]);
          yv[qb][j] = static_cast<bf16_t>(y * cs[j] + x * sn[j]);
          const float c = cs[j], s_ = sn[j];
          cs[j] = c * ct[j] - s_ * st[j];
          sn[j] = s_ * ct[j] + c * st[j];
        }
        q_bounce[tid] = __builtin_bit_cast(uint4, xv[qb]);
        qreg[qb][kk] = lds_to_acc(&q_bounce[tid]);
        q_bounce[tid] = __builtin_bit_cast(uint4, yv[qb]);
        qreg[qb][kk + 4] = lds_to_acc(&q_bounce[tid]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  const int lane16 = lane * 16;
  const char* lds_bytes = reinterpret_cast<const char*>(lds_all);
  float l_run[kQB], l_prior[kQB];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) { l_run[qb] = 0.f; l_prior[qb] = 0.f; }

  // ---- descriptors and staging --------------------------------------------------------------------
  // The descriptors of 64 consecutive tiles sit in vector registers, one tile per lane, and are
  // handed out with v_readlane: no memory access per tile.
  int win_base = 0;
  TileDesc win = fetch_desc(tiles, j_begin + min(lane, n_t - 1), max_tiles);
  auto desc_of = [&](int t) __attribute__((always_inline)) {           // t in [win_base, win_base + 64)
    const int l = t - win_base;
    TileDesc d;
    d.kpos0 = __builtin_amdgcn_readlane(win.kpos0, l);
    d.nvalid = __builtin_amdgcn_readlane(win.nvalid, l);
#pragma unroll
    for (int i = 0; i < 4; ++i) d.blk[i] = __builtin_amdgcn_readlane(win.blk[i], l);
    d.seg = 0; d.pad = 0;
    return d;
  };
  auto image_off = [&](int t) __attribute__((always_inline)) { return (t & (kBufs - 1)) * (kImageK * 16); };   // bytes
  // Loads of one K tile, straight into image `img_off`.  Wavefront w brings operand groups
  // 4w..4w+3: lane (hh, m) of group (b, kk) reads slot swap23(m % 16) of page 2b + m / 16, 16 bytes
  // at dim 16kk + 8hh.
  const size_t blk_bytes = static_cast<size_t>(hkv) * (kBlock * kD) * sizeof(bf16_t);
  const char* k_head = reinterpret_cast<const char*>(k_pool) + static_cast<size_t>(kvh) * (kBlock * kD * sizeof(bf16_t));
  const int k_lane_off = swap23(n & 15) * (kD * 2) + hh * 16 + (wave & 1) * 128;
  const bool k_second_page = (n >> 4) != 0;
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t lds_base = uniform(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)lds_all)));   // LDS byte address
  auto dma_tile = [&](const TileDesc& d, int img_off) __attribute__((always_inline)) {
    const bool upper = wave >= 2;                                        // K block this wavefront feeds
    const size_t o0 = static_cast<size_t>(max(upper ? d.blk[2] : d.blk[0], 0)) * blk_bytes;
    const size_t o1 = static_cast<size_t>(max(upper ? d.blk[3] : d.blk[1], 0)) * blk_bytes;
    const char* src = k_head + (k_second_page ? o1 : o0) + k_lane_off;
    const uint32_t dst = lds_base + img_off + (4 * wave) * 1024;
#pragma unroll
    for (int j = 0; j < 4; ++j) load_to_lds(src + 32 * j, dst + 1024 * j);
  };
  // wait until at most `newer` of this wavefront's vector-memory operations are outstanding
  auto wait_loads = [&](auto newer) __attribute__((always_inline)) {
    constexpr int kN = decltype(newer)::value;
    __builtin_amdgcn_s_waitcnt((kN & 15) | ((kN >> 4) << 14) | (7 << 4) | (15 << 8));
    asm volatile("" ::: "memory");
  };
  auto barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // ---- one 32-key block: S, masking, exponentials, sums ---------------------------------------------
  u32x4 ring[kDepth];
  f32x16 sacc[kQB];
  auto piece = [&](int img_off, int step) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4*>(lds_bytes + img_off + step * 1024 + lane16);
  };
  // tile block blk of image img_off; the ring holds the block's first kDepth pieces on entry and
  // the next block's (nimg_off, nblk) on exit
  auto block = [&](int img_off, int blk, int nimg_off, int nblk, const TileDesc& d) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        if (!RAGGED || qb < n_cols) {
          if (kk == 0) mfma_s_first(sacc[qb], ring[kk % kDepth], qreg[qb][kk]);
          else mfma_s_acc(sacc[qb], ring[kk % kDepth], qreg[qb][kk]);
        }
      }
      const int s = kk + kDepth;
      ring[kk % kDepth] = s < 8 ? piece(img_off, blk * 8 + s) : piece(nimg_off, nblk * 8 + (s - 8));
      __builtin_amdgcn_sched_barrier(0);
    }
    mfma_result_wait();          // (idle issue slots: the SIMD's other wavefront runs meanwhile)
    // padding / causal edge: entries the token must not see become -inf
    // (accumulator register i holds key 32 blk + 16(i/8) + 8hh + i%8 of the tile)
    if (d.nvalid < kTile || d.kpos0 + kTile - 1 > p_min) {
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) {
        if (RAGGED && qb >= n_cols) continue;
        int lim = min(d.nvalid - 1, sg_start + token(qb) - d.kpos0) - 8 * hh - 32 * blk;
        asm volatile("" : "+v"(lim));
#pragma unroll
        for (int i = 0; i < 16; ++i)
          sacc[qb][i] = (16 * (i / 8) + (i % 8) <= lim) ? sacc[qb][i] : -INFINITY;
      }
    }
    // (an overflow shows in the sums: inf stays inf)
#pragma unroll
    for (int qb = 0; qb < kQB; ++qb) {
      if (RAGGED && qb >= n_cols) continue;
#pragma unroll
      for (int j = 0; j < 8; ++j) exp2_sum2(l_run[qb], sacc[qb][2 * j], sacc[qb][2 * j + 1]);
    }
  };

  // ---- prologue: images 0, 1, 2 ---------------------------------------------------------------------
  TileDesc d0 = desc_of(0), d1 = desc_of(min(1, n_t - 1)), d2 = desc_of(min(2, n_t - 1)), d3 = d2;
  dma_tile(d0, image_off(0));
  dma_tile(d1, image_off(1));
  dma_tile(d2, image_off(2));
  load_queries();
  wait_loads(std::integral_constant<int, 0>{});
  __syncthreads();
#pragma unroll
  for (int s = 0; s < kDepth; ++s) ring[s] = piece(image_off(0), s);

  // ---- the tile loop --------------------------------------------------------------------------------
  for (int t = 0; t < n_t; ++t) {
    const int img = image_off(t);
    const int nimg = t + 1 < n_t ? image_off(t + 1) : img;
    if (t + 3 - win_base >= 64) {                        // next 64 descriptors (rare)
      win_base += 64;
      win = fetch_desc(tiles, j_begin + min(win_base + lane, n_t - 1), max_tiles);
      __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));      // vmcnt(0) here, so the hot path never waits for it
    }
    // entering the token's own chunk: everything summed so far is prior-chunk mass
    if (t == t_own) {
#pragma unroll
      for (int qb = 0; qb < kQB; ++qb) { l_prior[qb] = l_run[qb]; l_run[qb] = 0.f; }
    }
    // loads of image t+3 (past the last tile they repeat the last tile into an image nobody reads)
    d3 = desc_of(min(t + 3, n_t - 1));
    dma_tile(d3, image_off(t + 3));
    block(img, 0, img, 1, d0);
    block(img, 1, nimg, 0, d0);
    // image t+2 (loads started one iteration ago) must be whole before anyone reads it
    wait_loads(std::integral_constant<int, 4>{});
    barrier();
    d0 = d1; d1 = d2; d2 = d3;
  }

  // ---- epilogue ---------------------------------------------------------------------------------
  bool bad = false;
  float lp[kQB], lt[kQB];
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb) {
    lt[qb] = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
    lp[qb] = l_prior[qb] + __shfl_xor(l_prior[qb], 32, 64);
    const float tot = lp[qb] + lt[qb];
    bad = bad || (qb < n_cols && !(tot > kTinySum && tot < kSafeSum));
  }
  // tokens whose sums left the safe range are redone by the kernel that carries a reference
  if (__any(bad)) {
    const int r0 = sg_tok_off + t0, r1 = sg_tok_off + min(t0 + kTQ, sg_ntok) - 1;
    if (lane <= (r1 >> 6) - (r0 >> 6)) redo[(r0 >> 6) + lane] = 1;
    return;
  }
#pragma unroll
  for (int qb = 0; qb < kQB; ++qb)
    if (t0 + 32 * qb + n < sg_ntok && hh == 0)
      mass[static_cast<size_t>(sg_tok_off + token(qb)) * hq + h] = lp[qb] / (lp[qb] + lt[qb]);
}

}  // namespace

bool score_v2_supported(const cc_ctx* ctx) {
  if (ctx->cfg.dtype != CC_BF16 || ctx->cfg.head_dim != kD) return false;
  return (ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads) % 4 == 0;
}

void launch_score_v2(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks, const Plan& pl,
                     const cc_segment* segs, int n_segs, const int32_t* req_seg_off, int max_seg_tokens,
                     float* mass, int32_t* redo, hipStream_t stream) {
  const int hkv = ctx->cfg.n_kv_heads, n_sub = ctx->cfg.n_q_heads / hkv / 4;
  const int n_tiles = (max_seg_tokens + kTQ - 1) / kTQ;
  dim3 grid(hkv * n_sub * n_tiles, n_segs);
  // The chunks' last, partly empty workgroups run as a launch of their own behind the others, so that
  // the straight-line body of the full workgroups does not have to carry the branches that skip empty
  // column blocks (inside one kernel those branches, or a second copy of the loop, cost the full
  // workgroups 4-5 %).  (Run beside the first launch on a second stream instead, the second launch
  // gains another 1 % of the call on the 8B batch: not worth a stream of the library's own.)
  hipLaunchKernelGGL(score_v2_kernel<false>, grid, dim3(256), 0, stream, static_cast<const bf16_t*>(q),
                     static_cast<const bf16_t*>(k_pool), n_blocks, pl.tiles, pl.max_tiles,
                     pl.items, ctx->cfg.n_q_heads, hkv, n_sub, n_tiles, ctx->inv_freq,
                     mass, redo);
  hipLaunchKernelGGL(score_v2_kernel<true>, dim3(hkv * n_sub, n_segs), dim3(256), 0, stream,
                     static_cast<const bf16_t*>(q), static_cast<const bf16_t*>(k_pool), n_blocks, pl.tiles,
                     pl.max_tiles, pl.items, ctx->cfg.n_q_heads, hkv, n_sub, n_tiles, ctx->inv_freq, mass, redo);
}

}  // namespace cc
