// MFMA (bf16, head_dim 128) kernels of cc_select's score stage and cc_sparse_prefill's attention.
//
// Both stages are "few queries against all earlier keys" (Sec. 4 "Selective Token Recomputation";
// per-token form of Eq. (1)).  One workgroup owns 32*QB query tokens of one request and one KV
// head; wavefront w owns query head kvh*G + w, so all G heads of the group share every K/V tile
// that is staged in LDS (grouped-query packing).  Key tiles are 64 keys (4 blocks of 16 tokens)
// and never straddle a segment, so block padding only shows up in a segment's last tile.
//
// Orientation: S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16.  In the 32x32 result
// a lane holds ONE query column (lane % 32) and 16 rows, so the softmax of a query (reference
// max, exponentials, sum, rescale of O) is lane-local; the two lane halves, which hold different
// keys of the same query, only talk when the reference max moves.  P^T feeds the second product
// straight from the accumulator registers: within a 32-key block the MFMA row m of S^T is
// assigned the key swap_bits_2_3(m), which makes the 8 values a lane-half contributes to one
// 16-key step the keys 8*half .. 8*half+7 of one 16-token block -- exactly one 16-byte row piece
// of the dimension-major V block.
//
// Softmax bookkeeping: the query is pre-multiplied by log2(e)/sqrt(d) before it is rounded to
// bf16, so S is in log2 units and p = exp2(S - m_ref).  The reference m_ref is fixed by the first
// block of the request -- 0 if that block's maximum is within +-2^24 of it (then the subtraction
// is skipped altogether), else that maximum -- and afterwards moves only when a block's sum of
// exponentials exceeds kBig (entries far above the reference); that block is then redone with the
// reference raised and the sums and O rescaled.  Until then p is merely "large": fp32 and bf16
// share the exponent range, so nothing is lost.
//
// LDS image of a tile (16-byte pieces; every MFMA operand read is one conflict-free 1 KiB run):
//   K piece (block b of 32 keys, k-step kk, half hh, row m):  (b*8+kk)*64 + hh*32 + (m ^ ((2kk+hh)&7))
//   V piece (page pg, 32-dim group db, half hh, dim n):       1024 + (pg*4+db)*64 + hh*32 + (n ^ 4hh)
// The XOR terms spread the *writes* of a coalesced global read over the LDS banks.
#include <type_traits>

#include "mfma_tile.h"

namespace cc {

using namespace tile;

namespace {

// Small workgroups (64 or 128 threads; head groups of 1 or 2): the tile does not fit in registers,
// so it is copied piece by piece without prefetch.  Correct, not fast.
template <int NT, bool WITH_V>
__device__ __forceinline__ void stage_direct(uint4* lds, const bf16_t* __restrict__ k_pool,
                                             const bf16_t* __restrict__ v_pool, int n_blocks,
                                             const TileDesc& d, int hkv, int kvh, int tid,
                                             const bf16_t* __restrict__ v_shared, int n_shared_blocks,
                                             const int32_t* __restrict__ v_map) {
  const int nvalid = d.nvalid;
  constexpr int kPieces = WITH_V ? 2048 : 1024;
#pragma unroll 4
  for (int i = 0; i < kPieces / NT; ++i) {
    const int c = tid + NT * i;
    const bool is_v = WITH_V && c >= 1024;
    const int pg = (c & 1023) >> 8, cc_ = c & 255;
    const int nv = min(max(nvalid - kBlock * pg, 0), kBlock);
    const int blk = d.blk[pg];
    const bool ok = nv > 0 && blk >= 0 && blk < n_blocks;
    const size_t off = (static_cast<size_t>(ok ? blk : 0) * hkv + kvh) * (kBlock * kD) + cc_ * 8;
    uint4 val = make_uint4(0u, 0u, 0u, 0u);
    if (ok) {
      if (!is_v) {
        if ((cc_ >> 4) < nv) val = *reinterpret_cast<const uint4*>(k_pool + off);
      } else {
        const bf16_t* vb = value_block<bf16_t>(v_pool, v_shared, n_shared_blocks, v_map, blk,
                                               static_cast<size_t>(hkv) * (kBlock * kD));
        val = *reinterpret_cast<const uint4*>(vb + static_cast<size_t>(kvh) * (kBlock * kD) + cc_ * 8);
        if (nv < kBlock) val = zero_pad_slots(val, cc_ & 1, nv);
      }
    }
    lds[is_v ? v_piece_dst(pg, cc_) : k_piece_dst(pg, cc_)] = val;
  }
}

// SCORE = true : queries are 32*QB consecutive tokens of a chunk segment; result is the share of
//                the softmax mass that falls on keys of earlier segments (Eq. (2), Eq. (10)).
// SCORE = false: queries are 32*QB rows of the compact query list; result is the attention
//                output and log-sum-exp (Eq. (1)).
// REDO = true : second pass behind the wide kernels.  One workgroup per segment (score) or request
//                (attention) looks up, in parallel, which of its row tiles the wide kernel flagged
//                and walks those, one KV head after the other; without flags - the normal case -
//                it is gone after one round of loads, so the pass costs a few hundred short
//                workgroups instead of one per (tile, KV head).
template <int G, bool SCORE, int QB, bool REDO>
__global__ __launch_bounds__(64 * G, 2) void sparse_qk_kernel(
    const bf16_t* __restrict__ q, const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool, int n_blocks,
    const TileDesc* __restrict__ tiles, const int32_t* __restrict__ seg_tile_off, int max_tiles,
    const int32_t* __restrict__ order, const cc_segment* __restrict__ segs, const int32_t* __restrict__ req_seg_off, int hq, int hkv,
    int n_tiles_x, InvFreq inv_freq, bf16_t* __restrict__ out, float* __restrict__ lse,
    float* __restrict__ mass, const int32_t* __restrict__ redo, const int32_t* __restrict__ q_map,
    int map_pos, const bf16_t* __restrict__ v_shared, int n_shared_blocks, const int32_t* __restrict__ v_map) {
  constexpr int NT = 64 * G;
  constexpr int TQ = 32 * QB;                       // query tokens per workgroup
  constexpr bool kPrefetch = NT >= 256;
  constexpr int kImage = SCORE ? 1024 : 2048;       // 16-byte pieces per tile image
  // operand reads in flight ahead of the MFMAs (16 bytes per lane each)
  constexpr int kDepth = (QB == 2 || NT <= 256) ? 4 : 8;
  static_assert(16 % kDepth == 0, "ring slots must line up from one tile to the next");
  // attention: double-buffered.  score: three images, because the previous tile's image must stay
  // readable (repair path of its deferred block) while the next tile is being stored.
  constexpr int kBufs = SCORE ? 3 : 2;
  __shared__ uint4 lds_all[kBufs * kImage];
  const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
  const int n = lane & 31, hh = lane >> 5;
  // ---- which row tiles ----------------------------------------------------------------------
  const int y_item = order[blockIdx.y];     // segment (score; heaviest first) or request (attention; longest context first)
  cc_segment sg_own = {};
  int q_first = 0, q_end = 0;
  if constexpr (SCORE) sg_own = segs[y_item];
  else { q_first = cu_q[y_item]; q_end = cu_q[y_item + 1]; }
  // is row tile t of this item flagged for the second pass?
  auto flagged = [&](int t) {
    if constexpr (SCORE) {
      const int t0 = t * TQ;
      if (sg_own.kind != CC_SEG_CHUNK || t0 >= sg_own.n_tokens || sg_own.logical_start == 0) return false;
      return (redo[(sg_own.tok_off + t0) >> 6] | redo[(sg_own.tok_off + t0 + TQ - 1) >> 6]) != 0;
    } else {
      if (q_first + t * TQ >= q_end) return false;
      return redo[redo_index(q_first + (t * TQ / 64) * 64)] != 0;
    }
  };
  __shared__ int todo[REDO ? NT : 1];
  __shared__ int n_todo;
  const int n_rounds = REDO ? (n_tiles_x + NT - 1) / NT : 1;
  for (int round = 0; round < n_rounds; ++round) {
  int n_work = 1;
  if constexpr (REDO) {
    __syncthreads();                                  // (the previous round's list has been walked)
    if (tid == 0) n_todo = 0;
    __syncthreads();
    const int t = round * NT + tid;
    if (t < n_tiles_x && flagged(t)) todo[atomicAdd(&n_todo, 1)] = t;
    __syncthreads();
    n_work = n_todo * hkv;
  }
  for (int work = 0; work < n_work; ++work) {
  if constexpr (REDO) __syncthreads();                // (LDS images of the previous tile are free)
  const int kvh = REDO ? work % hkv : blockIdx.x % hkv;
  const int tile = REDO ? todo[work / hkv] : n_tiles_x - 1 - blockIdx.x / hkv;       // late (long) tiles are dispatched first
  const int h = kvh * G + wave;

  // ---- which queries ------------------------------------------------------------------------
  // (attention with a row map: list row j takes its query from row q_map[j] of q - and, if
  // map_pos, its position from q_pos[q_map[j]]; results are always indexed by the list row)
  int row[QB], src_row[QB], p[QB], s_begin, s_end, s_self = -1;
  bool row_valid[QB];
  if constexpr (SCORE) {
    const int seg_id = y_item;
    const cc_segment sg = sg_own;
    const int t0 = tile * TQ;
    if (sg.kind != CC_SEG_CHUNK || t0 >= sg.n_tokens || sg.logical_start == 0) continue;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int t = min(t0 + 32 * qb + n, sg.n_tokens - 1);
      row_valid[qb] = t0 + 32 * qb + n < sg.n_tokens;
      row[qb] = sg.tok_off + t;
      src_row[qb] = row[qb];
      p[qb] = sg.logical_start + t;
    }
    s_begin = req_seg_off[sg.req];
    s_self = seg_id;
    s_end = s_self + 1;
  } else {
    const int r = y_item;
    const int q0 = q_first + tile * TQ;
    if (q0 >= q_end) continue;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      row[qb] = min(q0 + 32 * qb + n, q_end - 1);
      row_valid[qb] = q0 + 32 * qb + n < q_end;
      src_row[qb] = q_map != nullptr ? q_map[row[qb]] : row[qb];
      p[qb] = q_pos[map_pos ? src_row[qb] : row[qb]];
    }
    s_begin = req_seg_off[r];
    s_end = req_seg_off[r + 1];
  }
  int pmx = p[0], pmn = p[0];
#pragma unroll
  for (int qb = 1; qb < QB; ++qb) { pmx = max(pmx, p[qb]); pmn = min(pmn, p[qb]); }
  const int p_max = uniform(wave_max_i(pmx)), p_min = uniform(wave_min_i(pmn));

  // ---- load the query rows, rotate them to their positions, fold the softmax scale -------------
  // lane (n, hh) keeps, for k-step kk, dims 16kk + 8hh .. +7; dims < 64 pair with dims + 64.
  const float c2 = 0.08838834764831845f * kLog2e;           // log2(e) / sqrt(128)
  bf16x8 qreg[QB][8];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const bf16_t* qp = q + (static_cast<size_t>(src_row[qb]) * hq + h) * kD + 8 * hh;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 xv = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + 16 * kk));
      bf16x8 yv = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qp + 16 * kk + 64));
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float c, s;
        rot_cos_sin_fast(p[qb], inv_freq.f[16 * kk + 8 * hh + j], &c, &s);
        c *= c2; s *= c2;
        const float x = static_cast<float>(xv[j]), y = static_cast<float>(yv[j]);
        xv[j] = static_cast<bf16_t>(x * c - y * s);
        yv[j] = static_cast<bf16_t>(y * c + x * s);
      }
      qreg[qb][kk] = xv;
      qreg[qb][kk + 4] = yv;
      __builtin_amdgcn_sched_barrier(0);     // keep the prologue's register footprint small
    }
  }

  // lane-dependent part of the operand addresses (pieces), constant over the whole loop
  int kx[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) kx[j] = hh * 32 + (n ^ ((2 * j + hh) & 7));
  const int vx = 1024 + hh * 32 + (n ^ (4 * hh));

  float m_ref[QB], l_run[QB], l_prior[QB];
  f32x16 o[QB][SCORE ? 1 : 4];
  f32x16 sacc[QB][2];                 // S (then p) of the two 32-key blocks in flight
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_ref[qb] = 0.f; l_run[qb] = 0.f; l_prior[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < (SCORE ? 1 : 4); ++db) o[qb][db] = splat16(0.f);
  }

  // ---- building blocks of the tile pipeline -----------------------------------------------------
  // S block b of the tile image `img`: 8 k-steps, operand reads kDepth steps ahead of the MFMAs;
  // `side(kk)` is VALU work of ANOTHER block that is slotted in after every k-step so that it runs
  // while the matrix pipe is busy.  raw = true ignores the reference (used by the repair path).
  // The MFMA operands of a tile form one stream of kSteps 16-byte pieces per lane (K pieces of S
  // block 0, S block 1, then the V pieces of the four pages); `ring` keeps kDepth of them in flight
  // ahead of the MFMA that consumes them, across the stages of the tile, so that LDS latency is
  // paid once per tile and not once per stage.
  constexpr int kSteps = SCORE ? 16 : 32;
  uint4 ring[kDepth];
  // step t of the current image; steps >= kSteps are the first K pieces of the next image `nimg`
  // (nullptr: there is no next tile, or it may not be read yet)
  auto issue = [&](const uint4* img, const uint4* nimg, int t) {   // t: compile-time step index
    if (t < kSteps) {
      ring[t % kDepth] = t < 16 ? img[t * 64 + kx[t & 3]] : img[(t - 16) * 64 + vx];
    } else if (nimg != nullptr) {
      const int t2 = t - kSteps;
      ring[t % kDepth] = nimg[t2 * 64 + kx[t2 & 3]];
    }
  };
  auto prime = [&](const uint4* img) {
#pragma unroll
    for (int t = 0; t < kDepth; ++t) issue(img, nullptr, t);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto qk_block = [&](const uint4* img, const uint4* nimg, int b, auto&& side) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int t = b * 8 + kk;
      const bf16x8 a = __builtin_bit_cast(bf16x8, ring[t % kDepth]);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        sacc[qb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            a, qreg[qb][kk], kk == 0 ? splat16(0.f) : sacc[qb][b], 0, 0, 0);
      issue(img, nimg, t + kDepth);
      side(kk);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // repair path only: raw S of block b straight from the image (does not touch the ring)
  auto qk_block_raw = [&](const uint4* img, int b) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, img[(b * 8 + kk) * 64 + kx[kk & 3]]);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb)
        sacc[qb][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
            a, qreg[qb][kk], kk == 0 ? splat16(0.f) : sacc[qb][b], 0, 0, 0);
    }
  };
  // exponentials of elements 2kk, 2kk+1 of block b (all query blocks); sums go to lsum[]
  float lsum[QB];
  // While every query's reference is still exactly 0 (zero_ref: the first block's maximum was
  // small, which is the normal case for attention logits) the subtraction is skipped; the
  // accumulators always hold raw S, so switching between the two forms needs no fix-up.
  bool zero_ref = true;
  auto exp_pair = [&](auto zero, int b, int kk) {
    constexpr bool kZero = decltype(zero)::value;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int i = 2 * kk + e;
        const float v = __builtin_amdgcn_exp2f(kZero ? sacc[qb][b][i] : sacc[qb][b][i] - m_ref[qb]);
        sacc[qb][b][i] = v;
        lsum[qb] += v;
      }
  };
  using ZeroT = std::integral_constant<bool, true>;
  using SubT = std::integral_constant<bool, false>;
  auto no_side = [&](int) {};
  // padding / causal edge: entries of block b that the query must not see become -inf
  // (accumulator register i of block b holds key 32b + 16(i/8) + 8hh + i%8 of the tile)
  auto mask_block = [&](int b, int kpos0, int nvalid) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      int lim = min(nvalid - 1, p[qb] - kpos0) - 8 * hh - 32 * b;
      asm volatile("" : "+v"(lim));                        // keep the compares inside the branch
#pragma unroll
      for (int i = 0; i < 16; ++i)
        sacc[qb][b][i] = (16 * (i / 8) + (i % 8) <= lim) ? sacc[qb][b][i] : -INFINITY;
      asm volatile("" : "+v"(sacc[qb][b]));
    }
  };
  // move the reference of every query up to the maximum of block b (raw S); rescale what has been
  // summed so far.  init: first block of the request -- the reference stays 0 if every query's
  // maximum is within +-kZeroBand, else it becomes that maximum.
  auto raise_ref = [&](int b, bool init) {
    float t[QB];
    bool small = true;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      t[qb] = max16(sacc[qb][b]);
      t[qb] = fmaxf(t[qb], __shfl_xor(t[qb], 32, 64));
      small = small && fabsf(t[qb]) <= kZeroBand;
    }
    if (init && __all(small)) return;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float d = init ? t[qb] : fmaxf(t[qb] - m_ref[qb], 0.f);
      const float alpha = init ? 1.f : __builtin_amdgcn_exp2f(-d);
      l_run[qb] *= alpha;
      if constexpr (SCORE) l_prior[qb] *= alpha;
      else {
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[qb][db][i] *= alpha;
      }
      m_ref[qb] += d;
    }
    zero_ref = false;
  };
  // close block b after its exponentials: normally just add the sums.  If a sum is huge or not
  // finite, entries ran far above the reference: recompute the block's S from the LDS image,
  // raise the reference (rescaling sums and O), and redo the exponentials.  Rare.
  auto close_block = [&](const uint4* img, int b, int kpos0, int nvalid, bool edge) {
    bool bad = false;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) bad = bad || !(lsum[qb] < kBig);
    if (__any(bad)) {
      asm volatile("" ::: "memory");
      qk_block_raw(img, b);
      if (edge) mask_block(b, kpos0, nvalid);
      raise_ref(b, false);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        lsum[qb] = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float v = __builtin_amdgcn_exp2f(sacc[qb][b][i] - m_ref[qb]);
          sacc[qb][b][i] = v;
          lsum[qb] += v;
        }
      }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { l_run[qb] += lsum[qb]; lsum[qb] = 0.f; }
  };
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) lsum[qb] = 0.f;

  // ---- the tile loop ------------------------------------------------------------------------------
  // Tiles of the request are listed by the plan kernels; tile j is usable if j < j_end and its
  // first key is visible to some query of the workgroup.  Three things run ahead of the math of
  // tile t: the descriptor of tile t+3 (a broadcast vector load), the global loads of tile t+2
  // (into registers, issued right after the barrier), and the LDS image of tile t+1 (stored in the
  // middle of tile t).  The workgroup barrier sits before the last stage of a tile, whose operands
  // are already in registers, so that the first operand reads of the next image are in flight
  // while that stage's MFMAs run.
  const int j_begin = seg_tile_off[s_begin];
  const int j_end = min(seg_tile_off[s_end], max_tiles);
  const int j_own = SCORE ? seg_tile_off[s_self] : -1;
  auto usable = [&](const TileDesc& d, int j) { return j < j_end && uniform(d.kpos0) <= p_max; };

  Stager<kPrefetch ? NT : 256, !SCORE> stg;
  if constexpr (kPrefetch) stg.init(k_pool, v_pool, n_blocks, hkv, kvh, tid, v_shared, n_shared_blocks, v_map);
  auto stage_load = [&](const TileDesc& d) {            // global -> registers
    if constexpr (kPrefetch) stg.load(d);
  };
  auto stage_store = [&](const TileDesc& d, int b_) {   // registers (or global) -> LDS image b_
    if constexpr (kPrefetch) stg.store(lds_all + b_ * kImage);
    else stage_direct<NT, !SCORE>(lds_all + b_ * kImage, k_pool, v_pool, n_blocks, d, hkv, kvh, tid, v_shared,
                                  n_shared_blocks, v_map);
  };

  int j = j_begin;
  TileDesc d0 = to_scalar(fetch_desc(tiles, j, max_tiles));
  TileDesc d1 = to_scalar(fetch_desc(tiles, j + 1, max_tiles));
  TileDesc d2 = to_scalar(fetch_desc(tiles, j + 2, max_tiles));
  bool v0 = usable(d0, j), v1 = v0 && usable(d1, j + 1), v2 = v1 && usable(d2, j + 2);
  int buf = 0;
  if (v0) { stage_load(d0); stage_store(d0, 0); }
  if (v1) stage_load(d1);
  __syncthreads();
  if (v0) prime(lds_all);
  bool first = true;
  // SCORE: block 1 of the previous tile waits in sacc[*][1] for its exponentials, which are
  // slotted under the next tile's first S block
  bool pending = false;
  int prev_kpos0 = 0, prev_nvalid = 0;
  bool prev_edge = false;
  while (v0) {
    const bool enter_own = SCORE && j == j_own;
    const int kpos0 = uniform(d0.kpos0), nvalid = uniform(d0.nvalid);
    const bool edge = nvalid < kTile || kpos0 + kTile - 1 > p_min;   // padding or causal edge
    const int next_buf = (buf + 1) % kBufs;
    const uint4* img = lds_all + buf * kImage;
    const uint4* next_img = lds_all + next_buf * kImage;
    const uint4* prev_img = lds_all + ((buf + kBufs - 1) % kBufs) * kImage;
    TileDesc d3 = fetch_desc(tiles, j + 3, max_tiles);             // three tiles ahead
    TileDesc d3s;                                                  // ... made wave-uniform mid-tile

    // ---- stage 0: S block 0 ----------------------------------------------------------------------
    if constexpr (SCORE) {
      if (pending) {
        if (zero_ref) qk_block(img, nullptr, 0, [&](int kk) { exp_pair(ZeroT{}, 1, kk); });
        else qk_block(img, nullptr, 0, [&](int kk) { exp_pair(SubT{}, 1, kk); });
        close_block(prev_img, 1, prev_kpos0, prev_nvalid, prev_edge);
      } else {
        qk_block(img, nullptr, 0, no_side);
      }
      // entering the query's own segment: everything summed so far is prior-chunk mass
      if (enter_own) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) { l_prior[qb] = l_run[qb]; l_run[qb] = 0.f; }
      }
    } else {
      qk_block(img, nullptr, 0, no_side);
    }
    if (edge) mask_block(0, kpos0, nvalid);
    if (first) {                       // key 0 of the request is in this block and visible to all
      raise_ref(0, true);
      first = false;
    }
    if constexpr (SCORE) {
      // all operand reads of this image are issued; publish the next image and meet
      if (v1) stage_store(d1, next_buf);
      __syncthreads();
      d3s = to_scalar(d3);             // its load is the only one in flight here: waiting is free
      if (v2) stage_load(d2);
      // ---- stage 1: S block 1, exponentials of block 0 underneath; first reads of the next image
      if (zero_ref) qk_block(img, v1 ? next_img : nullptr, 1, [&](int kk) { exp_pair(ZeroT{}, 0, kk); });
      else qk_block(img, v1 ? next_img : nullptr, 1, [&](int kk) { exp_pair(SubT{}, 0, kk); });
      if (edge) mask_block(1, kpos0, nvalid);
      close_block(img, 0, kpos0, nvalid, edge);
      pending = true; prev_kpos0 = kpos0; prev_nvalid = nvalid; prev_edge = edge;
    } else {
      // ---- stage 1: S block 1, exponentials of block 0 underneath -----------------------------------
      // (the attention kernel is bound by LDS operand reads, not by the VALU: one form is enough)
      qk_block(img, nullptr, 1, [&](int kk) { exp_pair(SubT{}, 0, kk); });
      if (edge) mask_block(1, kpos0, nvalid);
      close_block(img, 0, kpos0, nvalid, edge);
      if (v1) stage_store(d1, next_buf);
      // ---- stages 2, 3: O^T += V^T P^T, P^T straight from the accumulator registers ------------------
      // block b covers pages 2b, 2b+1 of the tile; step st = (u, db): page 2b+u, 32-dim group db
      auto pv_block = [&](const uint4* nimg, int b, auto&& side) {
        bf16x8 pb[QB];
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          const int u = st >> 2, db = st & 3, t = 16 + b * 8 + st;
          if (db == 0) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
              for (int jj = 0; jj < 8; ++jj) pb[qb][jj] = static_cast<bf16_t>(sacc[qb][b][8 * u + jj]);
          }
          const bf16x8 a = __builtin_bit_cast(bf16x8, ring[t % kDepth]);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb], o[qb][db], 0, 0, 0);
          issue(img, nimg, t + kDepth);
          side(st);
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      pv_block(nullptr, 0, [&](int st) { exp_pair(SubT{}, 1, st); });
      close_block(img, 1, kpos0, nvalid, edge);
      // every read of this image has been issued; meet, then finish the tile out of registers
      // while the first operand reads of the next image are in flight
      __syncthreads();
      d3s = to_scalar(d3);             // its load is the only one in flight here: waiting is free
      if (v2) stage_load(d2);
      pv_block(v1 ? next_img : nullptr, 1, no_side);
    }
    ++j;
    d0 = d1; d1 = d2; d2 = d3s;
    v0 = v1; v1 = v2; v2 = v2 && usable(d2, j + 2);
    buf = next_buf;
  }
  if constexpr (SCORE) {
    if (pending) {                     // exponentials of the very last block
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) exp_pair(SubT{}, 1, kk);
      close_block(lds_all + ((buf + kBufs - 1) % kBufs) * kImage, 1, prev_kpos0, prev_nvalid, prev_edge);
    }
  }

  // ---- epilogue ---------------------------------------------------------------------------------
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
    if constexpr (SCORE) {
      const float lp = l_prior[qb] + __shfl_xor(l_prior[qb], 32, 64);
      if (row_valid[qb] && hh == 0) mass[static_cast<size_t>(row[qb]) * hq + h] = lp / (lp + l_tot);
    } else {
      const float inv = 1.f / l_tot;
      if (row_valid[qb]) {
        if (out != nullptr) {                // (a caller that only wants the log-sum-exp passes none)
          bf16_t* op = out + (static_cast<size_t>(row[qb]) * hq + h) * kD;
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
              bf16_t v4[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) v4[e] = static_cast<bf16_t>(o[qb][db][4 * g4 + e] * inv);
              // accumulator register i holds output dim 32db + 8(i/4) + 4hh + i%4
              *reinterpret_cast<uint2*>(op + 32 * db + 8 * g4 + 4 * hh) = *reinterpret_cast<uint2*>(v4);
            }
        }
        if (lse != nullptr && hh == 0)
          lse[static_cast<size_t>(row[qb]) * hq + h] = kLn2 * (m_ref[qb] + __builtin_amdgcn_logf(l_tot));
      }
    }
  }
  }   // work items of the round
  }   // rounds
}

// ---- plan: the key tiles of every segment, in prompt order ---------------------------------------
// seg_tile_off[s] = number of tiles before segment s (exclusive scan of ceil(n_tokens/64)); run by
// one whole workgroup of 256 threads, into global memory or into LDS.
__device__ __forceinline__ void plan_scan(const cc_segment* __restrict__ segs, int n_segs,
                                          int32_t* seg_tile_off) {
  __shared__ int wsum[4];
  __shared__ int carry_s;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  for (int s0 = 0; s0 < n_segs; s0 += 256) {
    const int s = s0 + tid;
    const int nt = s < n_segs ? (max(segs[s].n_tokens, 0) + kTile - 1) / kTile : 0;
    int incl = nt;                                   // inclusive scan inside the wavefront
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int up = __shfl_up(incl, o, 64);
      if (lane >= o) incl += up;
    }
    if (lane == 63) wsum[w] = incl;
    __syncthreads();
    int base = carry_s;
    for (int ww = 0; ww < w; ++ww) base += wsum[ww];
    if (s < n_segs) seg_tile_off[s] = base + incl - nt;
    __syncthreads();
    if (tid == 255) carry_s = base + incl;
    __syncthreads();
  }
  if (tid == 0) seg_tile_off[n_segs] = carry_s;
  __syncthreads();
}

__global__ __launch_bounds__(256) void plan_scan_kernel(const cc_segment* __restrict__ segs, int n_segs,
                                                         int32_t* __restrict__ seg_tile_off) {
  plan_scan(segs, n_segs, seg_tile_off);
}

// descriptor of tile j (and the redo flags cleared, spread over the n_fill workgroups that do this)
__device__ __forceinline__ void plan_fill(const cc_segment* __restrict__ segs, int n_segs,
                                          const int32_t* seg_tile_off, const int32_t* __restrict__ block_tab,
                                          int n_blocks, int max_tiles, TileDesc* __restrict__ tiles,
                                          int32_t* __restrict__ redo, int n_redo, int j, int n_fill) {
  for (int i = j; i < n_redo; i += n_fill * 256) redo[i] = 0;
  if (j >= min(seg_tile_off[n_segs], max_tiles)) return;
  int lo = 0, hi = n_segs - 1;                       // last segment with seg_tile_off[s] <= j
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (seg_tile_off[mid] <= j) lo = mid; else hi = mid - 1;
  }
  const cc_segment sg = segs[lo];
  const int kt = j - seg_tile_off[lo];
  TileDesc d;
  d.kpos0 = sg.logical_start + kTile * kt;
  d.nvalid = min(kTile, sg.n_tokens - kTile * kt);
  for (int i = 0; i < 4; ++i) {
    int b = -1;
    if (kBlock * i < d.nvalid) b = block_tab[sg.tab_off + (kTile / kBlock) * kt + i];
    d.blk[i] = (b >= 0 && b < n_blocks) ? b : -1;
  }
  d.seg = lo;
  d.pad = 0;
  tiles[j] = d;
}

__global__ __launch_bounds__(256) void plan_fill_kernel(const cc_segment* __restrict__ segs, int n_segs,
                                                         const int32_t* __restrict__ seg_tile_off,
                                                         const int32_t* __restrict__ block_tab, int n_blocks,
                                                         int max_tiles, TileDesc* __restrict__ tiles,
                                                         int32_t* __restrict__ redo, int n_redo) {
  plan_fill(segs, n_segs, seg_tile_off, block_tab, n_blocks, max_tiles, tiles, redo, n_redo,
            blockIdx.x * 256 + threadIdx.x, gridDim.x);
}

// Dispatch order of the grid's y index: items sorted by decreasing key-side work, so that the last
// workgroups to start are the short ones.  BY_REQUEST: item = request, key = end of its context;
// otherwise item = segment, key = end of the segment (0 for segments that are not scored).
// order[rank] = item; ties keep index order, so the result is always a permutation.  More than
// kMaxOrdered items: identity.
constexpr int kMaxOrdered = 4096;

//
// Beside order[] one 32-byte work item per rank is written, so that a workgroup of the
// wide kernels finds everything it needs to start with ONE load instead of a chain of dependent
// ones (order -> segment -> request -> tile offsets).  Called by whole workgroups; `block` is the
// workgroup's index among those that do this.
template <bool BY_REQUEST>
__device__ __forceinline__ void plan_order(const cc_segment* __restrict__ segs,
                                           const int32_t* __restrict__ req_seg_off,
                                           const int32_t* seg_tile_off, int n_items,
                                           int32_t* __restrict__ order, WorkItem* __restrict__ items, int block) {
  __shared__ int key[kMaxOrdered];
  const int i = block * 256 + threadIdx.x;
  auto emit = [&](int rank, int item) {
    order[rank] = item;
    WorkItem w;
    if constexpr (BY_REQUEST) {
      w.id = item; w.kind = 0; w.start = 0; w.n_tokens = 0; w.tok_off = 0;
      w.j_begin = seg_tile_off[req_seg_off[item]];
      w.j_own = seg_tile_off[req_seg_off[item + 1]];           // end of the request's tiles
    } else {
      const cc_segment sg = segs[item];
      w.id = item; w.kind = sg.kind; w.start = sg.logical_start; w.n_tokens = sg.n_tokens; w.tok_off = sg.tok_off;
      w.j_begin = seg_tile_off[req_seg_off[sg.req]];
      w.j_own = seg_tile_off[item];
    }
    w.pad = 0;
    items[rank] = w;
  };
  if (n_items > kMaxOrdered) {
    if (i < n_items) emit(i, i);
    return;
  }
  for (int j = threadIdx.x; j < n_items; j += 256) {
    int kv = 0;
    if constexpr (BY_REQUEST) {
      const int s_last = req_seg_off[j + 1] - 1;
      if (s_last >= req_seg_off[j]) kv = segs[s_last].logical_start + segs[s_last].n_tokens;
    } else {
      const cc_segment sg = segs[j];
      if (sg.kind == CC_SEG_CHUNK && sg.logical_start > 0) kv = sg.logical_start + sg.n_tokens;
    }
    key[j] = kv;
  }
  __syncthreads();
  if (i >= n_items) return;
  const int mine = key[i];
  int rank = 0;
  for (int j = 0; j < n_items; ++j) {
    const int other = key[j];
    rank += (other > mine || (other == mine && j < i)) ? 1 : 0;
  }
  emit(rank, i);
}

template <bool BY_REQUEST>
__global__ __launch_bounds__(256) void plan_order_kernel(const cc_segment* __restrict__ segs,
                                                          const int32_t* __restrict__ req_seg_off,
                                                          const int32_t* __restrict__ seg_tile_off,
                                                          int n_items, int32_t* __restrict__ order,
                                                          WorkItem* __restrict__ items) {
  plan_order<BY_REQUEST>(segs, req_seg_off, seg_tile_off, n_items, order, items, blockIdx.x);
}

// The whole plan in ONE launch, for batches of up to kPlanFused segments: every workgroup repeats
// the (tiny) scan into LDS, then the first n_fill workgroups write descriptors and the others the
// dispatch order.  Two launches and two waits between dependent kernels fewer per call, which is
// what a single request's step (a dozen kernels of a few microseconds) is made of.
constexpr int kPlanFused = 1024;

template <bool BY_REQUEST>
__global__ __launch_bounds__(256) void plan_fused_kernel(const cc_segment* __restrict__ segs, int n_segs,
                                                          const int32_t* __restrict__ req_seg_off, int n_items,
                                                          const int32_t* __restrict__ block_tab, int n_blocks,
                                                          int max_tiles, int32_t* __restrict__ seg_tile_off,
                                                          int32_t* __restrict__ order, WorkItem* __restrict__ items,
                                                          TileDesc* __restrict__ tiles, int32_t* __restrict__ redo,
                                                          int n_redo, int n_fill) {
  __shared__ int32_t s_off[kPlanFused + 1];
  plan_scan(segs, n_segs, s_off);
  if (blockIdx.x == 0)
    for (int s = threadIdx.x; s <= n_segs; s += 256) seg_tile_off[s] = s_off[s];
  if (static_cast<int>(blockIdx.x) < n_fill)
    plan_fill(segs, n_segs, s_off, block_tab, n_blocks, max_tiles, tiles, redo, n_redo,
              blockIdx.x * 256 + threadIdx.x, n_fill);
  else
    plan_order<BY_REQUEST>(segs, req_seg_off, s_off, n_items, order, items, blockIdx.x - n_fill);
}

constexpr int kAttnQB = 1;     // 32 query tokens per workgroup in the attention kernel
constexpr int kScoreQB = 2;    // 64 in the score kernel (no O accumulator, so registers allow it)

template <int G>
void launch_attn_g(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                   int max_q_per_req, const void* k_pool, const void* v_pool, int n_blocks,
                   const Plan& pl, const cc_segment* segs, const int32_t* req_seg_off,
                   int n_requests, void* out, float* lse, const int32_t* redo, const int32_t* q_map,
                   int map_pos, hipStream_t stream, const ValueSource& vs) {
  const int hkv = ctx->cfg.n_kv_heads, n_tiles = (max_q_per_req + 32 * kAttnQB - 1) / (32 * kAttnQB);
#define CC_KARGS static_cast<const bf16_t*>(q), q_pos, cu_q, static_cast<const bf16_t*>(k_pool),                 \
                 static_cast<const bf16_t*>(v_pool), n_blocks, pl.tiles, pl.seg_tile_off, pl.max_tiles,         \
                 pl.order, segs, req_seg_off, ctx->cfg.n_q_heads, hkv, n_tiles, ctx->inv_freq,                  \
                 static_cast<bf16_t*>(out), lse, static_cast<float*>(nullptr), redo, q_map, map_pos,            \
                 static_cast<const bf16_t*>(vs.v_shared), vs.n_shared_blocks, static_cast<const int32_t*>(vs.v_map)
  if (redo != nullptr)
    hipLaunchKernelGGL((sparse_qk_kernel<G, false, kAttnQB, true>), dim3(1, n_requests), dim3(64 * G), 0, stream, CC_KARGS);
  else
    hipLaunchKernelGGL((sparse_qk_kernel<G, false, kAttnQB, false>), dim3(hkv * n_tiles, n_requests), dim3(64 * G), 0,
                       stream, CC_KARGS);
#undef CC_KARGS
}

template <int G>
void launch_score_g(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks, const Plan& pl,
                    const cc_segment* segs, int n_segs, const int32_t* req_seg_off, int max_seg_tokens,
                    float* mass, const int32_t* redo, hipStream_t stream) {
  const int hkv = ctx->cfg.n_kv_heads, n_tiles = (max_seg_tokens + 32 * kScoreQB - 1) / (32 * kScoreQB);
#define CC_KARGS static_cast<const bf16_t*>(q), static_cast<const int32_t*>(nullptr),                             \
                 static_cast<const int32_t*>(nullptr), static_cast<const bf16_t*>(k_pool),                      \
                 static_cast<const bf16_t*>(nullptr), n_blocks, pl.tiles, pl.seg_tile_off, pl.max_tiles,        \
                 pl.order, segs, req_seg_off, ctx->cfg.n_q_heads, hkv, n_tiles, ctx->inv_freq,                  \
                 static_cast<bf16_t*>(nullptr), static_cast<float*>(nullptr), mass, redo,                       \
                 static_cast<const int32_t*>(nullptr), 0, static_cast<const bf16_t*>(nullptr), 0,               \
                 static_cast<const int32_t*>(nullptr)
  if (redo != nullptr)
    hipLaunchKernelGGL((sparse_qk_kernel<G, true, kScoreQB, true>), dim3(1, n_segs), dim3(64 * G), 0, stream, CC_KARGS);
  else
    hipLaunchKernelGGL((sparse_qk_kernel<G, true, kScoreQB, false>), dim3(hkv * n_tiles, n_segs), dim3(64 * G), 0, stream,
                       CC_KARGS);
#undef CC_KARGS
}

bool group_supported(const cc_ctx* ctx) {
  if (ctx->cfg.dtype != CC_BF16 || ctx->cfg.head_dim != kD) return false;
  const int g = ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads;
  return g == 1 || g == 2 || g == 4 || g == 8;
}

}  // namespace

// workspace: seg_tile_off[n_segs + 1] | order[n_segs] (requests never outnumber segments) |
//            items[n_segs] | tiles | redo flags
static size_t plan_ints_bytes(int n_segs) {
  return (static_cast<size_t>(2 * n_segs + 1) * sizeof(int32_t) + 255) / 256 * 256;
}
size_t plan_head_bytes(int n_segs) {
  return plan_ints_bytes(n_segs) + (static_cast<size_t>(n_segs) * sizeof(WorkItem) + 255) / 256 * 256;
}

static size_t plan_bytes_impl(int n_segs, int max_tiles) {
  return plan_head_bytes(n_segs) + static_cast<size_t>(max_tiles) * sizeof(TileDesc);
}

Plan run_plan(void* ws, const cc_segment* segs, int n_segs, const int32_t* req_seg_off, int n_requests,
              const int32_t* block_tab, int n_blocks, int max_tiles, int n_redo, hipStream_t stream) {
  Plan pl;
  pl.seg_tile_off = static_cast<int32_t*>(ws);
  pl.order = pl.seg_tile_off + n_segs + 1;
  pl.items = reinterpret_cast<WorkItem*>(static_cast<char*>(ws) + plan_ints_bytes(n_segs));
  pl.tiles = reinterpret_cast<TileDesc*>(static_cast<char*>(ws) + plan_head_bytes(n_segs));
  pl.max_tiles = max_tiles;
  pl.redo = n_redo > 0 ? reinterpret_cast<int32_t*>(pl.tiles + max_tiles) : nullptr;
  if (n_segs <= kPlanFused) {
    const int n_fill = (max_tiles + 255) / 256;
    if (n_requests > 0)
      hipLaunchKernelGGL(plan_fused_kernel<true>, dim3(n_fill + (n_requests + 255) / 256), dim3(256), 0, stream, segs,
                         n_segs, req_seg_off, n_requests, block_tab, n_blocks, max_tiles, pl.seg_tile_off, pl.order,
                         pl.items, pl.tiles, pl.redo, n_redo, n_fill);
    else
      hipLaunchKernelGGL(plan_fused_kernel<false>, dim3(n_fill + (n_segs + 255) / 256), dim3(256), 0, stream, segs,
                         n_segs, req_seg_off, n_segs, block_tab, n_blocks, max_tiles, pl.seg_tile_off, pl.order,
                         pl.items, pl.tiles, pl.redo, n_redo, n_fill);
    return pl;
  }
  hipLaunchKernelGGL(plan_scan_kernel, dim3(1), dim3(256), 0, stream, segs, n_segs, pl.seg_tile_off);
  if (n_requests > 0)                                  // attention: the grid's y index walks requests
    hipLaunchKernelGGL(plan_order_kernel<true>, dim3((n_requests + 255) / 256), dim3(256), 0, stream, segs,
                       req_seg_off, pl.seg_tile_off, n_requests, pl.order, pl.items);
  else                                                 // score: it walks segments
    hipLaunchKernelGGL(plan_order_kernel<false>, dim3((n_segs + 255) / 256), dim3(256), 0, stream, segs,
                       req_seg_off, pl.seg_tile_off, n_segs, pl.order, pl.items);
  hipLaunchKernelGGL(plan_fill_kernel, dim3((max_tiles + 255) / 256), dim3(256), 0, stream, segs, n_segs,
                     pl.seg_tile_off, block_tab, n_blocks, max_tiles, pl.tiles, pl.redo, n_redo);
  return pl;
}

// Fewest workgroups for which the wide SCORE kernel is chosen (three per compute unit of an MI355X:
// below that the narrow kernel's twice as many, half as long workgroups fill the machine better;
// measured on batches of 1-8 requests, 32 and 64 query heads: 10-25 % for the narrow kernel at
// 200-600 workgroups, equal at ~800, 5-15 % for the wide one above).  The wide ATTENTION kernel is
// faster at every size measured, down to 64 workgroups (7-25 %), so it has no such limit.
constexpr int kMinWideGrid = 768;

bool attn_mfma_supported(const cc_ctx* ctx) { return group_supported(ctx); }
bool score_mfma_supported(const cc_ctx* ctx) { return group_supported(ctx); }

size_t mfma_plan_bytes(int n_segs, int max_tiles, int n_q_max) {
  return plan_bytes_impl(n_segs, max_tiles) + redo_entries(n_q_max) * sizeof(int32_t);
}

void launch_attn_mfma(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                      int n_q_tot, int max_q_per_req, const void* k_pool, const void* v_pool,
                      int n_blocks, const int32_t* block_tab, const cc_segment* segs, int n_segs,
                      const int32_t* req_seg_off, int n_requests, void* out, float* lse,
                      void* plan_ws, int max_tiles, const int32_t* q_map, int map_pos, hipStream_t stream,
                      const AttnByProduct* by, const ValueSource& vs) {
  // Wide kernel first where the head group allows it; the narrow kernel then redoes the 64-row
  // tiles the wide one flagged (normally none: its workgroups read one flag and exit).
  const bool wide = ctx->impl != CC_IMPL_MFMA_NARROW && attn_v2_supported(ctx);
  const int n_redo = wide ? static_cast<int>(redo_entries(n_q_tot)) : 0;
  const Plan pl = run_plan(plan_ws, segs, n_segs, req_seg_off, n_requests, block_tab, n_blocks, max_tiles, n_redo, stream);
  if (wide)
    launch_attn_v2(ctx, q, q_pos, cu_q, max_q_per_req, k_pool, v_pool, n_blocks, pl, req_seg_off, n_requests,
                   out, lse, pl.redo, q_map, map_pos, by != nullptr ? by->snap_index : nullptr,
                   by != nullptr ? by->cum : nullptr, by != nullptr ? by->s_max : 0, stream, vs);
  if (by != nullptr) {
    by->wide = wide;
    by->redo = pl.redo;
  }
  const int32_t* redo = pl.redo;
#define CC_ARGS ctx, q, q_pos, cu_q, max_q_per_req, k_pool, v_pool, n_blocks, pl, segs, req_seg_off, n_requests, out, lse, redo, q_map, map_pos, stream, vs
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
                       void* plan_ws, int max_tiles, int n_tok, hipStream_t stream) {
  // Wide kernel first where the head group allows it; the narrow kernel then redoes the granules
  // the wide one flagged (normally none: its workgroups read two flags and exit).
  const int wide_wgs = ctx->cfg.n_q_heads / 4 * ((max_seg_tokens + 127) / 128) * n_segs;
  const bool wide = ctx->impl != CC_IMPL_MFMA_NARROW && score_v2_supported(ctx) &&
                    (wide_wgs >= kMinWideGrid || ctx->impl == CC_IMPL_MFMA_WIDE);
  const int n_redo = wide ? static_cast<int>(score_redo_entries(n_tok)) : 0;
  const Plan pl = run_plan(plan_ws, segs, n_segs, req_seg_off, 0, block_tab, n_blocks, max_tiles, n_redo, stream);
  if (wide)
    launch_score_v2(ctx, q, k_pool, n_blocks, pl, segs, n_segs, req_seg_off, max_seg_tokens, mass, pl.redo, stream);
  const int32_t* redo = pl.redo;
#define CC_ARGS ctx, q, k_pool, n_blocks, pl, segs, n_segs, req_seg_off, max_seg_tokens, mass, redo, stream
  switch (ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads) {
    case 1: launch_score_g<1>(CC_ARGS); break;
    case 2: launch_score_g<2>(CC_ARGS); break;
    case 4: launch_score_g<4>(CC_ARGS); break;
    default: launch_score_g<8>(CC_ARGS); break;
  }
#undef CC_ARGS
}

}  // namespace cc
