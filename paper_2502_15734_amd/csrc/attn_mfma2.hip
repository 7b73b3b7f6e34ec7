// cc_sparse_prefill's attention for head groups that are a multiple of 4 (bf16, head_dim 128):
// per-token form of Eq. (1); Sec. 4 "Selective Token Recomputation".
//
// One workgroup = 4 wavefronts = 4 query heads of one KV head x 64 query rows of the compact list;
// a wavefront owns one head and all 64 rows (two 32-row MFMA column blocks), so every K / V operand
// it reads from LDS feeds two MFMAs.  One wavefront per SIMD (up to 512 registers): the running
// output (128 registers), the rotated queries (64) and two 32-key score blocks (64) stay in
// registers for the whole key loop.
//
// Orientation, LDS image and key permutation are those of mfma_tile.h: S^T = K Q^T, O^T = V^T P^T
// with v_mfma_f32_32x32x16_bf16, a lane holds one query column, P^T goes from the accumulators to
// the second product without leaving the lane.
//
// Schedule.  Keys advance in 32-key blocks b = 0, 1, 2, ... (two per 64-key tile).  The matrix pipe
// sees   S(b+1), PV(b), S(b+2), PV(b+1), ...   16 MFMAs each, and under every MFMA one exponential
// of a block whose S is already complete is computed: the first half of exp(b) under PV(b-1), the
// second half under S(b+1).  So the vector ALU work per MFMA is constant (one exp2, one add, half a
// pack) and never waits for a matrix result that was issued less than 16 MFMAs ago.
//
// Softmax reference: as in the other MFMA kernels the reference m_ref is fixed by the first block
// (0 if that block's maximum is within +-2^24, and then p = exp2(S) with no subtraction) and moves
// only if a block's sum of exponentials explodes; that block is then redone from its LDS image
// with the reference raised and everything summed so far rescaled.
//
// Staging: four tile images in LDS, filled by loads that write LDS directly (global_load_lds, 16
// bytes per lane: lane L of an instruction fills piece base + L, so the image layout is chosen by
// the global address each lane is given).  Image of a tile (16-byte pieces):
//   K piece (block b of 32 keys, k-step kk, half hh, MFMA row m):  (b*8+kk)*64 + hh*32 + m
//   V piece (page pg, 32-dim group db, half hh, dim n):            1024 + (pg*4+db)*64 + hh*32 + n
// so every MFMA operand read is the contiguous KiB  step*64 + lane.  In iteration t the wavefronts
// read image t and (for S of the next tile's first block) image t+1 and start the loads of image
// t+3; before the iteration's barrier each wavefront waits until its loads of image t+2 have
// landed.  One s_barrier per tile.  LDS reads of a wavefront return in order, so when it reaches
// the barrier its reads of image t have returned.  Block padding: K padding never reaches a
// product (its S entries are masked by selection); V padding would, as 0 x garbage, so the
// wavefront that loaded a V page blanks the page's padding slots in LDS before the barrier, in a
// branch only a segment's last tile takes.
#include <type_traits>

#include "mfma_tile.h"

namespace cc {

using namespace tile;

namespace {

typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kImage = 2048;    // 16-byte pieces per tile image (K: 1024, V: 1024)
constexpr int kBufs = 4;
#ifndef CC_RING_DEPTH
#define CC_RING_DEPTH 4
#endif
constexpr int kDepth = CC_RING_DEPTH;       // operand reads in flight ahead of the MFMAs
// p = exp2(S - reference) may be large (fp32 and bf16 share the exponent range); a block sum
// beyond this leaves no headroom for the row sum and O
constexpr float kSafeSum = 1.0e30f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}


// MFMA forms with fixed register classes (the compiler's own choice shuffles accumulators between
// the two register files once a wavefront uses more than 256 registers): S accumulates in vector
// registers, where the vector ALU reads it; O accumulates in accumulation registers; the rotated
// query sits in accumulation registers as the B operand.  The matrix results are opaque to the
// compiler's hazard handling, so every vector-ALU read of them is either at least two MFMAs
// behind its producer (steady state) or behind mfma_result_wait().
__device__ __forceinline__ void mfma_s_first(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_s_acc(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_o_acc(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}
__device__ __forceinline__ void zero_acc(f32x16& d) {
#pragma unroll
  for (int i = 0; i < 16; ++i) asm volatile("v_accvgpr_write_b32 %0, 0" : "=a"(d[i]));
}
// 32 idle issue slots: longer than the 8 passes of the MFMA plus its write-back
__device__ __forceinline__ void mfma_result_wait() {
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
}
// 64 lanes x 16 bytes from global memory straight into LDS: lane L's 16 bytes land at
// lds_addr + 16 L (lds_addr wave-uniform).  Written as an instruction the compiler does not model:
// it would otherwise drain every outstanding load before the next LDS read, because it cannot see
// that the image being filled is not the image being read.  Completion is counted by vmcnt.
__device__ __forceinline__ void load_to_lds(const void* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(src), "s"(lds_addr) : "memory", "m0");
}
// v = exp2(a - m); l += pending (the previous element's exponential).  Written out so that it stays
// where it is placed, under one MFMA (the compiler otherwise lumps the exponentials of a block
// together or sinks them to their use), and so that the transcendental result is not read by
// the instruction right behind it.
__device__ __forceinline__ float exp2_sub_sum(float& l, float pending, float a, float m) {
  float t, v;
  asm volatile("v_sub_f32 %1, %4, %5\n\tv_exp_f32 %2, %1\n\tv_add_f32 %0, %0, %3"
               : "+v"(l), "=&v"(t), "=&v"(v) : "v"(pending), "v"(a), "v"(m));
  return v;
}
// one 16-byte LDS piece straight into accumulation registers
__device__ __forceinline__ u32x4 lds_to_acc(const uint4* p) {
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)p));   // LDS byte offset
  u32x4 r;
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=a"(r) : "v"(addr) : "memory");
  return r;
}

template <int QB>
__global__ __launch_bounds__(256, 1) void attn_v2_kernel(
    const bf16_t* __restrict__ q, const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool, int n_blocks,
    const TileDesc* __restrict__ tiles, const int32_t* __restrict__ seg_tile_off, int max_tiles,
    const int32_t* __restrict__ order, const int32_t* __restrict__ req_seg_off, int hq, int hkv,
    int n_sub, int n_tiles_x, InvFreq inv_freq, bf16_t* __restrict__ out, float* __restrict__ lse,
    int32_t* __restrict__ redo, const int32_t* __restrict__ q_map, int map_pos,
    const int32_t* __restrict__ snap_index, float* __restrict__ cum, int s_max) {
  constexpr int TQ = 32 * QB;
  __shared__ uint4 lds_all[kBufs * kImage];
  const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
  const int n = lane & 31, hh = lane >> 5;
  const int per_tile = hkv * n_sub;
  const int tile = n_tiles_x - 1 - blockIdx.x / per_tile;    // late (long) tiles are dispatched first
  const int rem = blockIdx.x % per_tile;
  const int kvh = rem % hkv, hsub = rem / hkv;
  const int h = kvh * (4 * n_sub) + hsub * 4 + wave;

  // ---- which queries ------------------------------------------------------------------------
  const int r = order[blockIdx.y];                           // longest contexts are dispatched first
  const int q0 = cu_q[r] + tile * TQ, q_end = cu_q[r + 1];
  if (q0 >= q_end) return;
  // (with a row map, list row j takes its query from row q_map[j] of q - and, if map_pos, its
  // position from q_pos[q_map[j]]; results are always indexed by the list row)
  int row[QB], src_row[QB], p[QB];
  bool row_valid[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    row[qb] = min(q0 + 32 * qb + n, q_end - 1);
    row_valid[qb] = q0 + 32 * qb + n < q_end;
    src_row[qb] = q_map != nullptr ? q_map[row[qb]] : row[qb];
    p[qb] = q_pos[map_pos ? src_row[qb] : row[qb]];
  }
  int pmx = p[0], pmn = p[0];
#pragma unroll
  for (int qb = 1; qb < QB; ++qb) { pmx = max(pmx, p[qb]); pmn = min(pmn, p[qb]); }
  const int p_max = uniform(wave_max_i(pmx)), p_min = uniform(wave_min_i(pmn));

  // ---- tiles of the request whose first key some query of the workgroup sees ------------------
  // (tiles are listed in prompt order, so these form a prefix)
  const int j_begin = seg_tile_off[req_seg_off[r]];
  const int j_end = min(seg_tile_off[req_seg_off[r + 1]], max_tiles);
  int n_t = 0;
  for (int j0 = j_begin; j0 < j_end; j0 += 256) {
    const int j = j0 + tid;
    n_t += __syncthreads_count(j < j_end && tiles[min(j, j_end - 1)].kpos0 <= p_max);
  }
  n_t = uniform(n_t);
  if (n_t == 0) return;                                      // cannot happen for a valid prompt

  // ---- load the query rows, rotate them to their positions, fold the softmax scale -------------
  // lane (n, hh) keeps, for k-step kk, dims 16kk + 8hh .. +7; dims < 64 pair with dims + 64.
  const float c2 = 0.08838834764831845f * kLog2e;            // log2(e) / sqrt(128)
  __shared__ uint4 q_bounce[256];     // one piece per lane: the way into the accumulation registers
  u32x4 qreg[QB][8];
  // (called after the first tile loads are on their way, so that the trigonometry hides their latency)
  auto load_queries = [&]() __attribute__((always_inline)) {
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
        q_bounce[tid] = __builtin_bit_cast(uint4, xv);
        qreg[qb][kk] = lds_to_acc(&q_bounce[tid]);
        q_bounce[tid] = __builtin_bit_cast(uint4, yv);
        qreg[qb][kk + 4] = lds_to_acc(&q_bounce[tid]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  // byte offset of this lane's piece inside every 64-piece operand group
  const int lane16 = lane * 16;
  const char* lds_bytes = reinterpret_cast<const char*>(lds_all);
  float m_ref[QB], l_run[QB], lsum[QB], ev[QB], vprev[QB];
  f32x16 o[QB][4];                    // running output, accumulation registers for the whole loop
  f32x16 sacc[QB][2];                 // S of the two 32-key blocks in flight (vector registers)
  uint32_t pk[QB][2][2][4];           // P^T of [block parity][16-key half], packed bf16 pairs
  bool overflow = false;              // some block's sum of exponentials left the safe range
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_ref[qb] = 0.f; l_run[qb] = 0.f; lsum[qb] = 0.f; ev[qb] = 0.f; vprev[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db) zero_acc(o[qb][db]);
  }

  // ---- operand ring ---------------------------------------------------------------------------
  // Steps of one iteration (tile t, image img; nimg = image of tile t+1):
  //    0.. 7  K pieces of block 1 of img        (S of the tile's second block)
  //    8..15  V pieces of pages 0, 1 of img     (PV of the first block)
  //   16..23  K pieces of block 0 of nimg       (S of the next tile's first block)
  //   24..31  V pieces of pages 2, 3 of img     (PV of the second block)
  //   32..35  = steps 0..3 of the next iteration
  // Without a next tile steps 16..23 are the V pieces of pages 2, 3 and nothing follows.
  u32x4 ring[kDepth];
  // operand group `step` of an image: 0..15 = K (block*8 + k-step), 16..31 = V (page*4 + dim group)
  auto piece = [&](int img_off, int step) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4*>(lds_bytes + img_off + step * 1024 + lane16);
  };
  auto issue = [&](int img, int nimg, bool has_next, int s) __attribute__((always_inline)) {   // s: compile-time
    if (s < 8) ring[s % kDepth] = piece(img, 8 + s);
    else if (s < 16) ring[s % kDepth] = piece(img, 16 + (s - 8));
    else if (s < 24) ring[s % kDepth] = has_next ? piece(nimg, s - 16) : piece(img, 16 + (s - 8));
    else if (s < 32) ring[s % kDepth] = piece(img, 16 + (s - 16));
    else ring[s % kDepth] = piece(nimg, 8 + (s - 32));      // harmless when there is no next tile
  };

  // one exponential: element i (0..15) of block parity bp; pairs are packed as they complete.  The
  // add into the row sum runs one element behind (vprev), so that no instruction reads a
  // transcendental result right after it was issued.
  auto exp_one = [&](int qb, int bp, int i) __attribute__((always_inline)) {
    const float v = exp2_sub_sum(lsum[qb], vprev[qb], sacc[qb][bp][i], m_ref[qb]);
    vprev[qb] = v;
    if ((i & 1) == 0) ev[qb] = v;
    else {
      pk[qb][bp][i >> 3][(i & 7) >> 1] = pack_bf16(ev[qb], v);
      asm volatile("" :: "v"(pk[qb][bp][i >> 3][(i & 7) >> 1]));     // keep the pack here, not at its use
    }
  };
  // S block into parity bp from the ring; side(kk, qb) runs after each MFMA
  auto s_slot = [&](int img, int nimg, bool has_next, int s0, int bp, auto&& side) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (kk == 0) mfma_s_first(sacc[qb][bp], ring[(s0 + kk) % kDepth], qreg[qb][kk]);
        else mfma_s_acc(sacc[qb][bp], ring[(s0 + kk) % kDepth], qreg[qb][kk]);
        if (qb == QB - 1) issue(img, nimg, has_next, s0 + kk + kDepth);
        side(kk, qb);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // PV of block parity bp: step st = (u, db): 16-key half u (page), 32-dim group db
  auto pv_slot = [&](int img, int nimg, bool has_next, int s0, int bp, auto&& side) __attribute__((always_inline)) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const int u = st >> 2, db = st & 3;
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const u32x4 pw = {pk[qb][bp][u][0], pk[qb][bp][u][1], pk[qb][bp][u][2], pk[qb][bp][u][3]};
        mfma_o_acc(o[qb][db], ring[(s0 + st) % kDepth], pw);
        if (qb == QB - 1) issue(img, nimg, has_next, s0 + st + kDepth);
        side(st, qb);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  auto no_side = [&](int, int) __attribute__((always_inline)) {};

  // padding / causal edge: entries of block parity bp (tile block blk) the query must not see
  // become -inf (register i of block blk holds key 32 blk + 16(i/8) + 8hh + i%8 of the tile)
  auto mask_block = [&](int bp, int blk, int kpos0, int nvalid) __attribute__((always_inline)) {
    mfma_result_wait();
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      int lim = min(nvalid - 1, p[qb] - kpos0) - 8 * hh - 32 * blk;
      asm volatile("" : "+v"(lim));
#pragma unroll
      for (int i = 0; i < 16; ++i)
        sacc[qb][bp][i] = (16 * (i / 8) + (i % 8) <= lim) ? sacc[qb][bp][i] : -INFINITY;
      asm volatile("" : "+v"(sacc[qb][bp]));
    }
  };
  // close the block whose exponentials are in lsum.  A sum that is huge or not finite means
  // entries ran far above the reference: the workgroup's rows are then redone by the kernel that
  // can move its reference (see the launcher).
  auto close_block = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      lsum[qb] += vprev[qb];
      vprev[qb] = 0.f;
      overflow = overflow || !(lsum[qb] < kSafeSum);
      l_run[qb] += lsum[qb];
      lsum[qb] = 0.f;
    }
  };

  // ---- descriptors and staging --------------------------------------------------------------------
  // What the loop needs of 64 consecutive tiles sits in vector registers, one tile per lane, and is
  // handed out with v_readlane: no memory access per tile.  The pages this wavefront brings in (its
  // V page and the two pages of its K groups) are picked once per window, so that a tile's
  // descriptor is a handful of scalars and never an indexed array.
  struct HotDesc {
    int kpos0;     // logical position of the tile's first key
    int nvalid;    // keys of the tile that exist
    int seg;       // segment of the tile
    int own;       // physical block of V page `wave` (-1: none)
    int ka, kb;    // physical blocks of the two pages of the K block this wavefront feeds
    int edge;      // the tile has padding slots or missing pages
  };
  int win_base = 0;
  int w_kpos0, w_nvalid, w_seg, w_own, w_ka, w_kb, w_edge;
  auto fill_window = [&](int base) __attribute__((always_inline)) {
    const TileDesc v = fetch_desc(tiles, j_begin + min(base + lane, n_t - 1), max_tiles);
    const int b0 = v.blk[0], b1 = v.blk[1], b2 = v.blk[2], b3 = v.blk[3];
    w_kpos0 = v.kpos0; w_nvalid = v.nvalid; w_seg = v.seg;
    w_own = wave == 0 ? b0 : wave == 1 ? b1 : wave == 2 ? b2 : b3;
    w_ka = wave >= 2 ? b2 : b0;
    w_kb = wave >= 2 ? b3 : b1;
    w_edge = (v.nvalid < kTile || (b0 | b1 | b2 | b3) < 0) ? 1 : 0;
  };
  fill_window(0);
  auto desc_of = [&](int t) __attribute__((always_inline)) {           // t in [win_base, win_base + 64)
    const int l = t - win_base;
    HotDesc d;
    d.kpos0 = __builtin_amdgcn_readlane(w_kpos0, l);
    d.nvalid = __builtin_amdgcn_readlane(w_nvalid, l);
    d.seg = __builtin_amdgcn_readlane(w_seg, l);
    d.own = __builtin_amdgcn_readlane(w_own, l);
    d.ka = __builtin_amdgcn_readlane(w_ka, l);
    d.kb = __builtin_amdgcn_readlane(w_kb, l);
    d.edge = __builtin_amdgcn_readlane(w_edge, l);
    return d;
  };
  auto image_off = [&](int t) __attribute__((always_inline)) { return (t & (kBufs - 1)) * (kImage * 16); };   // bytes
  // Loads of one tile, straight into image `img_off`.  Wavefront w brings K operand groups
  // 4w..4w+3 (half a 32-key block over all 16 slots of two pages) and V page w.
  const size_t blk_bytes = static_cast<size_t>(hkv) * (kBlock * kD) * sizeof(bf16_t);
  const char* k_head = reinterpret_cast<const char*>(k_pool) + static_cast<size_t>(kvh) * (kBlock * kD * sizeof(bf16_t));
  const char* v_head = reinterpret_cast<const char*>(v_pool) + static_cast<size_t>(kvh) * (kBlock * kD * sizeof(bf16_t));
  // K: lane (hh, m) of group (b, kk) reads slot swap23(m % 16) of page 2b + m / 16, 16 bytes at dim 16kk + 8hh
  const int k_lane_off = swap23(n & 15) * (kD * 2) + hh * 16;
  const bool k_second_page = (n >> 4) != 0;
  // V: lane (hh, n) of group (pg, db) reads slots 8hh.. of dim row 32db + n
  const int v_lane_off = n * 32 + hh * 16;
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t lds_base = uniform(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)lds_all)));   // LDS byte address
  const char* k_src = nullptr;                                           // of the tile being loaded
  const char* v_src = nullptr;
  uint32_t k_dst = 0;
  auto dma_begin = [&](const HotDesc& d, int img_off) __attribute__((always_inline)) {
    const size_t o0 = static_cast<size_t>(max(d.ka, 0)) * blk_bytes;
    const size_t o1 = static_cast<size_t>(max(d.kb, 0)) * blk_bytes;
    k_src = k_head + (k_second_page ? o1 : o0) + k_lane_off + (wave & 1) * 128;
    v_src = v_head + static_cast<size_t>(max(d.own, 0)) * blk_bytes + v_lane_off;
    k_dst = lds_base + img_off + (4 * wave) * 1024;
  };
  auto dma_part = [&](int j) __attribute__((always_inline)) {           // j = 0..3: one K group, one V group
    load_to_lds(k_src + 32 * j, k_dst + 1024 * j);
    load_to_lds(v_src + 1024 * j, k_dst + 16 * 1024 + 1024 * j);
  };
  auto dma_tile = [&](const HotDesc& d, int img_off) __attribute__((always_inline)) {
    dma_begin(d, img_off);
#pragma unroll
    for (int j = 0; j < 4; ++j) dma_part(j);
  };
  // blank the padding slots of the V page this wavefront loaded (rare; after its loads have landed)
  auto blank_padding = [&](const HotDesc& d, int img_off) __attribute__((always_inline)) {
    if (d.edge) {
      const int nv = d.own < 0 ? 0 : min(max(d.nvalid - kBlock * wave, 0), kBlock);
      if (nv < kBlock) {
        uint4* vp = reinterpret_cast<uint4*>(const_cast<char*>(lds_bytes) + img_off + (16 + 4 * wave) * 1024 + lane16);
#pragma unroll
        for (int j = 0; j < 4; ++j) vp[j * 64] = zero_pad_slots(vp[j * 64], hh, nv);
        // (a rare branch leaves nothing pending, so that the code behind the join waits for no more
        // than the straight path does)
        __builtin_amdgcn_s_waitcnt((15) | (3 << 14) | (7 << 4) | (0 << 8));      // lgkmcnt(0)
      }
    }
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

  // prologue: images 0, 1, 2; S of block 0 and the first half of its exponentials
  HotDesc d0 = desc_of(0), d1 = desc_of(min(1, n_t - 1)), d2 = desc_of(min(2, n_t - 1)), d3 = d2;
  dma_tile(d0, image_off(0));
  dma_tile(d1, image_off(1));
  dma_tile(d2, image_off(2));
  load_queries();
  wait_loads(std::integral_constant<int, 0>{});
  blank_padding(d0, image_off(0));
  blank_padding(d1, image_off(1));
  blank_padding(d2, image_off(2));
  __syncthreads();
  {
    const int img = image_off(0);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const u32x4 a = piece(img, kk);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (kk == 0) mfma_s_first(sacc[qb][0], a, qreg[qb][kk]);
        else mfma_s_acc(sacc[qb][0], a, qreg[qb][kk]);
      }
    }
    if (d0.nvalid < kTile || d0.kpos0 + kTile - 1 > p_min) mask_block(0, 0, d0.kpos0, d0.nvalid);
    else mfma_result_wait();
    // first block of the request: its key 0 is visible to every query, so the maximum is finite;
    // it is the reference for the whole row
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float t = max16(sacc[qb][0]);
      m_ref[qb] = fmaxf(t, __shfl_xor(t, 32, 64));
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) exp_one(qb, 0, i);
#pragma unroll
    for (int s = 0; s < kDepth; ++s) issue(img, img, false, s);     // steps 0..3 of iteration 0
    __builtin_amdgcn_sched_barrier(0);
  }

  // ---- the tile loop --------------------------------------------------------------------------------
  // on entry: parity 0 holds S of the tile's first block (masked) with the first half of its
  // exponentials done.  The last tile is peeled off, so the loop body is straight-line code apart
  // from the masking branches.
  // By-product for rows that ask for it (snap_index >= 0: the question rows; or every row): when the tile that
  // has just been closed is the last one of its segment, the log-sum-exp over all keys up to here
  // goes to cum[snap row][head][segment's index in its request].  The reference never moves in this
  // kernel, so these running sums subtract exactly.  (Rare: once per segment of the request.)
  const int seg_first = cum != nullptr ? req_seg_off[order[blockIdx.y]] : 0;
  // (segments without tokens have no tile: the value also stands for those between this tile's
  // segment and the next tile's)
  auto snapshot = [&](int seg, int seg_next) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
      const int sr = snap_index != nullptr ? snap_index[row[qb]] : row[qb];     // (no index: every row is a snap row)
      if (row_valid[qb] && hh == 0 && sr >= 0) {
        const float v = kLn2 * (m_ref[qb] + __builtin_amdgcn_logf(tot));
        for (int sl = max(seg - seg_first, 0); sl < min(seg_next - seg_first, s_max); ++sl)
          cum[(static_cast<size_t>(sr) * hq + h) * s_max + sl] = v;
      }
    }
    __builtin_amdgcn_s_waitcnt((15) | (3 << 14) | (7 << 4) | (0 << 8));          // lgkmcnt(0): see blank_padding
  };
  auto tile_front = [&](auto next_tag, int t) __attribute__((always_inline)) {
    constexpr bool kNext = decltype(next_tag)::value;
    const int img = image_off(t);
    const int nimg = kNext ? image_off(t + 1) : img;
    // slot 1: S of the tile's second block; second half of the first block's exponentials.
    // Underneath: the loads of image t+3 (past the last tile they repeat the last tile into an
    // image nobody reads).
    s_slot(img, nimg, kNext, 0, 1, [&](int kk, int qb) __attribute__((always_inline)) {
      exp_one(qb, 0, 8 + kk);
      if (kNext && qb == QB - 1) {                       // two loads under each of four k-steps
        if (kk == 0) { d3 = desc_of(min(t + 3, n_t - 1)); dma_begin(d3, image_off(t + 3)); }
        if (kk >= 1 && kk <= 4) dma_part(kk - 1);
      }
    });
    close_block();
    if (d0.nvalid < kTile || d0.kpos0 + kTile - 1 > p_min) mask_block(1, 1, d0.kpos0, d0.nvalid);
    // slot 2: PV of the first block; first half of the second block's exponentials
    pv_slot(img, nimg, kNext, 8, 0, [&](int st, int qb) __attribute__((always_inline)) { exp_one(qb, 1, st); });
  };
  using NextT = std::integral_constant<bool, true>;
  using LastT = std::integral_constant<bool, false>;
  int t = 0;
  for (; t + 1 < n_t; ++t) {
    const int img = image_off(t), nimg = image_off(t + 1);
    if (t + 3 - win_base >= 64) {                        // next 64 descriptors (rare)
      win_base += 64;
      fill_window(win_base);
      __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));      // vmcnt(0) here, so the hot path never waits for it
    }
    tile_front(NextT{}, t);
    // slot 3: S of the next tile's first block; second half of the second block's exponentials
    s_slot(img, nimg, true, 16, 0, [&](int kk, int qb) __attribute__((always_inline)) { exp_one(qb, 1, 8 + kk); });
    close_block();
    if (cum != nullptr && d0.seg != d1.seg) snapshot(d0.seg, d1.seg);          // tile t was the last of its segment
    if (d1.nvalid < kTile || d1.kpos0 + kTile - 1 > p_min) mask_block(0, 0, d1.kpos0, d1.nvalid);
    // slot 4: PV of the second block; first half of the next block's exponentials
    pv_slot(img, nimg, true, 24, 1, [&](int st, int qb) __attribute__((always_inline)) { exp_one(qb, 0, st); });
    // image t+2 (loads started one iteration ago) must be whole before anyone reads it
    wait_loads(std::integral_constant<int, 8>{});
    blank_padding(d2, image_off(t + 2));
    barrier();
    d0 = d1; d1 = d2; d2 = d3;
  }
  {
    tile_front(LastT{}, t);
#pragma unroll
    for (int i = 8; i < 16; ++i)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) exp_one(qb, 1, i);
    close_block();
    pv_slot(image_off(t), image_off(t), false, 16, 1, no_side);
  }
  mfma_result_wait();

  // ---- epilogue ---------------------------------------------------------------------------------
  float l_tot[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    l_tot[qb] = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
    overflow = overflow || !(l_tot[qb] > 0.f && l_tot[qb] < kSafeSum);
  }
  // rows whose sums left the safe range are redone by the kernel that can move its reference
  if (__any(overflow)) {
    if (lane == 0) redo[redo_index(q0)] = 1;
    return;
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float inv = 1.f / l_tot[qb];
    if (row_valid[qb]) {
      if (out != nullptr) {                  // (a caller that only wants the log-sum-exp passes none)
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
        lse[static_cast<size_t>(row[qb]) * hq + h] = kLn2 * (m_ref[qb] + __builtin_amdgcn_logf(l_tot[qb]));
    }
  }
}

}  // namespace

bool attn_v2_supported(const cc_ctx* ctx) {
  if (ctx->cfg.dtype != CC_BF16 || ctx->cfg.head_dim != kD) return false;
  return (ctx->cfg.n_q_heads / ctx->cfg.n_kv_heads) % 4 == 0;
}

void launch_attn_v2(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                    int max_q_per_req, const void* k_pool, const void* v_pool, int n_blocks,
                    const Plan& pl, const int32_t* req_seg_off, int n_requests, void* out, float* lse,
                    int32_t* redo, const int32_t* q_map, int map_pos, const int32_t* snap_index, float* cum,
                    int s_max, hipStream_t stream) {
  constexpr int QB = 2;
  const int hkv = ctx->cfg.n_kv_heads, n_sub = ctx->cfg.n_q_heads / hkv / 4;
  const int n_tiles = (max_q_per_req + 32 * QB - 1) / (32 * QB);
  dim3 grid(hkv * n_sub * n_tiles, n_requests);
  hipLaunchKernelGGL((attn_v2_kernel<QB>), grid, dim3(256), 0, stream, static_cast<const bf16_t*>(q), q_pos,
                     cu_q, static_cast<const bf16_t*>(k_pool), static_cast<const bf16_t*>(v_pool), n_blocks,
                     pl.tiles, pl.seg_tile_off, pl.max_tiles, pl.order, req_seg_off, ctx->cfg.n_q_heads, hkv,
                     n_sub, n_tiles, ctx->inv_freq, static_cast<bf16_t*>(out), lse, redo, q_map, map_pos, snap_index, cum, s_max);
}

}  // namespace cc
