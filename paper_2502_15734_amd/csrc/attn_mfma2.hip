// cc_sparse_prefill's attention for head groups that are a multiple of 4 (bf16, head_dim 128):
// per-token form of Eq. (1); Sec. 4 "Selective Token Recomputation".
//
// One workgroup = 4 wavefronts = 4 query heads of one KV head x 64 query rows of the compact list;
// a wavefront owns one head and all 64 rows (two 32-row MFMA column blocks), so every K / V operand
// it reads from LDS feeds two MFMAs.  One wavefront per SIMD (up to 512 registers): the running
// output (128 registers) and the rotated queries (64) sit in accumulation registers, two 32-key
// score blocks (64), the packed probabilities (32) and the operand ring (32) in vector registers.
//
// Orientation and key permutation are those of mfma_tile.h: S^T = K Q^T, O^T = V^T P^T with
// v_mfma_f32_32x32x16_bf16, a lane holds one query column, P^T goes from the accumulators to
// the second product without leaving the lane.
//
// A SIMD with a single wavefront issues at most one instruction of any kind every four clocks, and
// a 32x32x16 MFMA occupies the matrix pipe for 32: the loop can keep the pipe full only if it
// spends at most seven other instructions per MFMA.  Everything below serves that count.
//
// Schedule.  Keys advance in 32-key blocks b = 0, 1, 2, ... (two per 64-key tile).  The matrix pipe
// sees   S(b+1), PV(b), S(b+2), PV(b+1), ...   16 MFMAs each, and under every MFMA one exponential
// of a block whose S is already complete: the first half of exp(b) under PV(b-1), the second half
// under S(b+1).  Per element that is one v_exp_f32 and one add into the row sum: the reference is
// already subtracted (it enters through the C operand of the block's first MFMA).  The row sum
// takes the unrounded exponentials (summing the bf16 roundings instead - one v_dot2c_f32_bf16 per
// pair - was measured too: it biases the log-sum-exp by up to 1.4e-3 when the weights are nearly
// uniform, and saves nothing that shows).  The pack of a pair to bf16 and its two adds run one step
// late, in front of the next exponential, so that no instruction reads a transcendental result
// right behind its issue.
//
// Softmax reference: m_ref = maximum of the row's first 32-key block, for the whole row (fp32 and
// bf16 share the exponent range, so p = exp2(S - m_ref) may grow to 1e30 without loss).  Rows whose
// sum leaves the safe range are flagged and redone by the kernel that can move its reference
// (see the launcher).
//
// Staging: four tile images in LDS, filled by loads that write LDS directly (global_load_lds, 16
// bytes per lane: lane L of an instruction fills piece base + L, so the image layout is chosen by
// the global address each lane is given).  Wavefront w brings page w (16 tokens) of the tile, K and
// V, each with four instructions whose addresses are one scalar base + one per-lane constant + an
// immediate: no vector arithmetic per tile.  Image of a tile (16-byte pieces):
//   K piece (MFMA row m of 32-key block b, k-step kk, half hh):
//       ((b*2 + kk/4)*4 + m/8)*64 + ((kk%4)*2 + (hh ^ (m/8)%2))*8 + m%8
//     (an instruction = 8 token slots x 128 bytes: whole cache lines; with 64-byte runs per slot the
//     K loads cost three times what the V loads cost for the same bytes)
//   V piece (page pg, 32-dim group db, half hh, dim n):  1024 + (pg*4+db)*64 + hh*32 + n
// An MFMA operand read takes contiguous runs of 128 bytes that alternate between the two halves
// of the 256-byte bank sweep (K) or one contiguous KiB (V): no bank conflicts.  In iteration t the wavefronts read image t and (for S of
// the next tile's first block) image t+1 and start the loads of image t+3; before the iteration's
// barrier each wavefront waits until its loads of image t+2 have landed.  One s_barrier per tile.
// Block padding: K padding never reaches a product (its S entries are masked by selection); V
// padding would, as 0 x garbage, so the wavefront that loaded a V page blanks the page's padding
// slots in LDS before the barrier, in a branch only a segment's last tile takes.
#include <type_traits>

#include "mfma_tile.h"

namespace cc {

using namespace tile;

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kImage = 2048;    // 16-byte pieces per tile image (K: 1024, V: 1024)
constexpr int kBufs = 4;
#ifndef CC_RING_DEPTH
#define CC_RING_DEPTH 8
#endif
constexpr int kDepth = CC_RING_DEPTH;       // operand reads in flight ahead of the MFMAs (even)
static_assert(kDepth % 2 == 0 && kDepth >= 4 && kDepth <= 8, "operand reads are issued in pairs");
// p = exp2(S - reference) may be large (fp32 and bf16 share the exponent range); a row sum
// beyond this leaves no headroom for O
constexpr float kSafeSum = 1.0e30f;

// MFMA forms with fixed register classes (the compiler's own choice shuffles accumulators between
// the two register files once a wavefront uses more than 256 registers): S accumulates in vector
// registers, where the vector ALU reads it; O accumulates in accumulation registers; the rotated
// query sits in accumulation registers as the B operand.  The matrix results are opaque to the
// compiler's hazard handling, so every vector-ALU read of them is either at least two MFMAs
// behind its producer (steady state) or behind mfma_result_wait().
__device__ __forceinline__ void mfma_s_zero(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(d) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_s_first(f32x16& d, const u32x4& a, const u32x4& b, const f32x16& c) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "a"(b), "v"(c));
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
// Loads of 64 lanes x 16 bytes from global memory straight into LDS: lane L's 16 bytes land at
// M0 + immediate + 16 L, read from base + voff(L) + immediate (the immediate counts on both sides).
// Written as instructions the compiler does not model: it would otherwise drain every outstanding
// load before the next LDS read, because it cannot see that the image being filled is not the
// image being read.  Completion is counted by vmcnt.
template <int IMM>
__device__ __forceinline__ void dma_one(uint32_t voff, const char* base, uint32_t m0v) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:%3"
               :: "v"(voff), "s"(base), "s"(m0v), "n"(IMM) : "memory", "m0");
}
template <int IMM0, int IMM1>
__device__ __forceinline__ void dma_two(uint32_t voff, const char* base, uint32_t m0v) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:%3\n\t"
               "global_load_lds_dwordx4 %0, %1 offset:%4"
               :: "v"(voff), "s"(base), "s"(m0v), "n"(IMM0), "n"(IMM1) : "memory", "m0");
}
// The exponentials.  exp_only: t = exp2(s).  exp_behind_pack: first the pair that is still pending
// (e = its even element, v = its odd one) is packed to bf16 and both are added to the row sum, then
// e = exp2(s).  Written out so that each stays where it is placed, under one MFMA (the compiler
// otherwise lumps the exponentials of a block together or sinks them to their use).
__device__ __forceinline__ void exp_only(float& t, float s) {
  asm volatile("v_exp_f32 %0, %1" : "=v"(t) : "v"(s));
}
__device__ __forceinline__ void exp_behind_pack(uint32_t& pk, float& l, float& e, float v, float s) {
  asm volatile("v_cvt_pk_bf16_f32 %0, %2, %3\n\tv_add_f32 %1, %1, %2\n\tv_add_f32 %1, %1, %3\n\tv_exp_f32 %2, %4"
               : "=&v"(pk), "+v"(l), "+v"(e) : "v"(v), "v"(s));
}
// one 16-byte LDS piece straight into accumulation registers
__device__ __forceinline__ u32x4 lds_to_acc(const uint4* p) {
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t addr = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)p));   // LDS byte offset
  u32x4 r;
  asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=a"(r) : "v"(addr) : "memory");
  return r;
}
// s_waitcnt with only the LDS counter set (vector-memory and export counters left alone)
template <int N>
__device__ __forceinline__ void wait_lds() {
  __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (7 << 4) | (N << 8));
}

// QB = 2: 4 wavefronts, each one head x 64 rows (one wavefront per SIMD, up to 512 registers);
// QB = 1: 8 wavefronts, each one head x 32 rows (two per SIMD, up to 256 registers each): the workgroup
// covers the same 4 heads x 64 rows, and while one wavefront of a SIMD waits (for LDS, for its
// exponentials - a transcendental does not run beside a matrix instruction of its own wavefront)
// the other one keeps the matrix pipe busy.
template <int QB>
__global__ __launch_bounds__(512 / QB, 1) void attn_v2_kernel(
    const bf16_t* __restrict__ q, const int32_t* __restrict__ q_pos, const int32_t* __restrict__ cu_q,
    const bf16_t* __restrict__ k_pool, const bf16_t* __restrict__ v_pool, int n_blocks,
    const TileDesc* __restrict__ tiles, const int32_t* __restrict__ seg_tile_off, int max_tiles,
    const int32_t* __restrict__ order, const int32_t* __restrict__ req_seg_off, int hq, int hkv,
    int n_sub, int n_tiles_x, InvFreq inv_freq, bf16_t* __restrict__ out, float* __restrict__ lse,
    int32_t* __restrict__ redo, const int32_t* __restrict__ q_map, int map_pos,
    const int32_t* __restrict__ snap_index, float* __restrict__ cum, int s_max,
    const bf16_t* __restrict__ v_shared, int n_shared_blocks, const int32_t* __restrict__ v_map) {
  constexpr int TQ = 64;                    // query rows per workgroup
  constexpr int NT = 512 / QB;              // threads
  __shared__ uint4 lds_all[kBufs * kImage];
  const int tid = threadIdx.x, lane = tid & 63, wave = uniform(tid >> 6);
  const int n = lane & 31, hh = lane >> 5;
  const int whead = wave & 3, wrows = (wave >> 2) * 32;     // this wavefront's head of the four, its first row of the 64
  const int per_tile = hkv * n_sub;
  const int tile = n_tiles_x - 1 - blockIdx.x / per_tile;    // late (long) tiles are dispatched first
  const int rem = blockIdx.x % per_tile;
  const int kvh = rem % hkv, hsub = rem / hkv;
  const int h = kvh * (4 * n_sub) + hsub * 4 + whead;

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
    row[qb] = min(q0 + wrows + 32 * qb + n, q_end - 1);
    row_valid[qb] = q0 + wrows + 32 * qb + n < q_end;
    src_row[qb] = q_map != nullptr ? q_map[row[qb]] : row[qb];
    p[qb] = q_pos[map_pos ? src_row[qb] : row[qb]];
  }
  // first and last position over all 64 rows of the workgroup (every wavefront walks the same tiles)
  int pmx, pmn;
  {
    const int ra = min(q0 + n, q_end - 1), rb = min(q0 + 32 + n, q_end - 1);
    const int pa = q_pos[map_pos ? (q_map != nullptr ? q_map[ra] : ra) : ra];
    const int pb = q_pos[map_pos ? (q_map != nullptr ? q_map[rb] : rb) : rb];
    pmx = max(pa, pb); pmn = min(pa, pb);
  }
  const int p_max = uniform(wave_max_i(pmx)), p_min = uniform(wave_min_i(pmn));

  // ---- tiles of the request whose first key some query of the workgroup sees ------------------
  // (tiles are listed in prompt order, so these form a prefix)
  const int j_begin = seg_tile_off[req_seg_off[r]];
  const int j_end = min(seg_tile_off[req_seg_off[r + 1]], max_tiles);
  int n_t = 0;
  for (int j0 = j_begin; j0 < j_end; j0 += NT) {
    const int j = j0 + tid;
    n_t += __syncthreads_count(j < j_end && tiles[min(j, j_end - 1)].kpos0 <= p_max);
  }
  n_t = uniform(n_t);
  if (n_t == 0) return;                                      // cannot happen for a valid prompt

  // ---- load the query rows, rotate them to their positions, fold the softmax scale -------------
  // lane (n, hh) keeps, for k-step kk, dims 16kk + 8hh .. +7; dims < 64 pair with dims + 64.
  const float c2 = 0.08838834764831845f * kLog2e;            // log2(e) / sqrt(128)
  __shared__ uint4 q_bounce[NT];      // one piece per lane: the way into the accumulation registers
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

  const char* lds_bytes = reinterpret_cast<const char*>(lds_all);
  // byte offsets of this lane's operand pieces inside an image (see the layout above)
  const int k_rd = (n >> 3) * 1024 + (hh ^ ((n >> 3) & 1)) * 128 + (n & 7) * 16;
  const int v_rd = 16384 + lane * 16;
  float m_ref[QB], lsum[QB], ev[QB], vodd[QB];
  f32x16 cinit[QB];                   // -m_ref in all 16 registers: the C operand that opens an S block
  f32x16 o[QB][4];                    // running output, accumulation registers for the whole loop
  f32x16 sacc[QB][2];                 // S of the two 32-key blocks in flight (vector registers)
  uint32_t pk[QB][2][2][4];           // P^T of [block parity][16-key half], packed bf16 pairs
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_ref[qb] = 0.f; lsum[qb] = 0.f; ev[qb] = 0.f; vodd[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db) zero_acc(o[qb][db]);
  }

  // ---- operand ring ---------------------------------------------------------------------------
  // Steps of one iteration (tile t, image img; nimg = image of tile t+1):
  //    0.. 7  K pieces of block 1 of img        (S of the tile's second block)
  //    8..15  V pieces of pages 0, 1 of img     (PV of the first block)
  //   16..23  K pieces of block 0 of nimg       (S of the next tile's first block)
  //   24..31  V pieces of pages 2, 3 of img     (PV of the second block)
  //   32..39  = steps 0..7 of the next iteration
  // (behind the last tile the "next image" holds stale keys: that S block is masked as a whole)
  // Reads are issued two at a time behind every odd step (into the slots of the two pieces just
  // used), and one wait in front of every even step covers that step and the next.
  u32x4 ring[kDepth];
  auto k_piece = [&](int img_off, int b, int kk) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4*>(lds_bytes + img_off + k_rd + b * 8192 + (kk >> 2) * 4096 + (kk & 3) * 256);
  };
  auto v_piece = [&](int img_off, int j) __attribute__((always_inline)) {      // j = page * 4 + dim group
    return *reinterpret_cast<const u32x4*>(lds_bytes + img_off + v_rd + j * 1024);
  };
  auto issue = [&](int img, int nimg, int s) __attribute__((always_inline)) {   // s: compile-time
    if (s < 8) ring[s % kDepth] = k_piece(img, 1, s);
    else if (s < 16) ring[s % kDepth] = v_piece(img, s - 8);
    else if (s < 24) ring[s % kDepth] = k_piece(nimg, 0, s - 16);
    else if (s < 32) ring[s % kDepth] = v_piece(img, s - 16);
    else ring[s % kDepth] = k_piece(nimg, 1, s - 32);
  };

  // one exponential: element i (0..15) of block parity bp.  An even element first packs the pair
  // in front of it (element 0: the last pair of the block before, which has the other parity).
  auto exp_step = [&](int qb, int bp, int i) __attribute__((always_inline)) {
    const float s = sacc[qb][bp][i];
    if (i & 1) exp_only(vodd[qb], s);
    else if (i == 0) exp_behind_pack(pk[qb][bp ^ 1][1][3], lsum[qb], ev[qb], vodd[qb], s);
    else exp_behind_pack(pk[qb][bp][(i - 2) >> 3][((i - 2) & 7) >> 1], lsum[qb], ev[qb], vodd[qb], s);
  };
  // S block into parity bp from the ring; side(kk, qb) runs after each MFMA
  auto s_slot = [&](int img, int nimg, int s0, int bp, auto&& side) __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      if ((kk & 1) == 0) wait_lds<kDepth - 2>();
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (kk == 0) mfma_s_first(sacc[qb][bp], ring[(s0 + kk) % kDepth], qreg[qb][kk], cinit[qb]);
        else mfma_s_acc(sacc[qb][bp], ring[(s0 + kk) % kDepth], qreg[qb][kk]);
        if (qb == QB - 1 && (kk & 1)) {
          issue(img, nimg, s0 + kk - 1 + kDepth);
          issue(img, nimg, s0 + kk + kDepth);
        }
        side(kk, qb);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // PV of block parity bp: step st = (u, db): 16-key half u (page), 32-dim group db
  auto pv_slot = [&](int img, int nimg, int s0, int bp, auto&& side) __attribute__((always_inline)) {
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      const int u = st >> 2, db = st & 3;
      if ((st & 1) == 0) wait_lds<kDepth - 2>();
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const u32x4 pw = {pk[qb][bp][u][0], pk[qb][bp][u][1], pk[qb][bp][u][2], pk[qb][bp][u][3]};
        mfma_o_acc(o[qb][db], ring[(s0 + st) % kDepth], pw);
        if (qb == QB - 1 && (st & 1)) {
          issue(img, nimg, s0 + st - 1 + kDepth);
          issue(img, nimg, s0 + st + kDepth);
        }
        side(st, qb);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

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

  // ---- descriptors and staging --------------------------------------------------------------------
  // What the loop needs of 64 consecutive tiles sits in vector registers, one tile per lane, and is
  // handed out with v_readlane: no memory access per tile.  The straight path reads two values per
  // tile (the flags of tile t+2, the page of tile t+3 this wavefront brings in); positions, key
  // counts and segments are read only inside the branches that need them.
  //   flag 1: the tile needs masking for some row (padding, or its last key lies behind p_min)
  //   flag 2: the tile has padding slots or missing pages
  //   flag 4: the next tile belongs to another segment
  int win_base = 0;
  // w_own: block of the page this wavefront brings in (-1: none); w_vown: where that page's values
  // are - the same block of v_pool, or (<= -2) block -2 - w_vown of v_shared while the value map
  // still points there (copy-on-write pending)
  int w_kpos0, w_nvalid, w_seg, w_seg_next, w_own, w_vown, w_flags;
  auto fill_window = [&](int base) __attribute__((always_inline)) {
    const int jl = min(base + lane, n_t - 1);
    const TileDesc v = fetch_desc(tiles, j_begin + jl, max_tiles);
    const int b0 = v.blk[0], b1 = v.blk[1], b2 = v.blk[2], b3 = v.blk[3];
    w_kpos0 = v.kpos0; w_nvalid = v.nvalid; w_seg = v.seg;
    int jn = min(max(j_begin + min(jl + 1, n_t - 1), 0), max_tiles - 1);
    asm volatile("" : "+v"(jn));                   // (a vector load, like the descriptor itself: see fetch_desc)
    w_seg_next = tiles[jn].seg;
    w_own = whead == 0 ? b0 : whead == 1 ? b1 : whead == 2 ? b2 : b3;
    w_vown = w_own;
    if (v_map != nullptr && w_own >= 0) {
      const int m = v_map[w_own];
      if (m >= 0 && m < n_shared_blocks) w_vown = -2 - m;
    }
    const bool edge = v.nvalid < kTile || (b0 | b1 | b2 | b3) < 0;
    w_flags = ((edge || v.kpos0 + kTile - 1 > p_min) ? 1 : 0) | (edge ? 2 : 0) | (w_seg_next != v.seg ? 4 : 0);
  };
  fill_window(0);
  auto lane_of = [&](int t) __attribute__((always_inline)) { return min(t, n_t - 1) - win_base; };
  auto image_off = [&](int t) __attribute__((always_inline)) { return (t & (kBufs - 1)) * (kImage * 16); };   // bytes
  // Loads of one tile, straight into image `img_off`: wavefront w brings page w % 4 - K and V if
  // there are four wavefronts, else K (w < 4) or V.
  //   K: instruction (rg, kq) brings rows 8 rg .. 8 rg + 7 of the page (row r sits in token slot
  //      swap23(r)), 128 bytes each at dim 64 kq: lane L reads row 8 rg + L % 8, piece (L / 8) ^ rg
  //   V: lane (hh, n) reads slots 8hh.. of dim row 32 j + n
  const size_t blk_bytes = static_cast<size_t>(hkv) * (kBlock * kD) * sizeof(bf16_t);
  const char* k_head = reinterpret_cast<const char*>(k_pool) + static_cast<size_t>(kvh) * (kBlock * kD * sizeof(bf16_t));
  const char* v_head = reinterpret_cast<const char*>(v_pool) + static_cast<size_t>(kvh) * (kBlock * kD * sizeof(bf16_t));
  const char* v_head_shared = v_shared == nullptr ? v_head
      : reinterpret_cast<const char*>(v_shared) + static_cast<size_t>(kvh) * (kBlock * kD * sizeof(bf16_t));
  const uint32_t k_voff0 = swap23(lane & 7) * (kD * 2) + (lane >> 3) * 16;
  const uint32_t k_voff1 = swap23(8 + (lane & 7)) * (kD * 2) + ((lane >> 3) ^ 1) * 16;
  const uint32_t v_voff = n * 32 + hh * 16;
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t lds_base = uniform(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)lds_all)));   // LDS byte address
  const int page = whead;
  const bool brings_k = QB == 2 || wave < 4, brings_v = QB == 2 || wave >= 4;
  const uint32_t k_img = lds_base + ((page >> 1) * 8 + (page & 1) * 2) * 1024;   // this wavefront's first K group in image 0
  const uint32_t v_img = lds_base + (16 + 4 * page) * 1024;                   // ... and its V page
  const char* k_src = nullptr;                                                // page of the tile being loaded (scalar)
  const char* v_src = nullptr;
  uint32_t k_dst = 0, v_dst = 0;
  auto dma_begin = [&](int l, int img_off) __attribute__((always_inline)) {          // l: the tile's lane in the window
    const int own = __builtin_amdgcn_readlane(w_own, l), vown = __builtin_amdgcn_readlane(w_vown, l);
    k_src = k_head + static_cast<size_t>(max(own, 0)) * blk_bytes;
    v_src = vown <= -2 ? v_head_shared + static_cast<size_t>(-2 - vown) * blk_bytes
                       : v_head + static_cast<size_t>(max(vown, 0)) * blk_bytes;
    k_dst = k_img + img_off;
    v_dst = v_img + img_off;
  };
  // (the two halves of a row are 4 KiB apart in the image and 128 bytes apart in memory; the two
  // row groups of a page are neighbours in the image)
  auto dma_k = [&](int j) __attribute__((always_inline)) {
    if (!brings_k) return;
    if (j == 0) dma_one<0>(k_voff0, k_src, k_dst);
    else if (j == 1) dma_one<128>(k_voff0, k_src, k_dst + (4096 - 128));
    else if (j == 2) dma_one<0>(k_voff1, k_src, k_dst + 1024);
    else dma_one<128>(k_voff1, k_src, k_dst + 1024 + (4096 - 128));
  };
  auto dma_v = [&](int half) __attribute__((always_inline)) {
    if (!brings_v) return;
    if (half == 0) dma_two<0, 1024>(v_voff, v_src, v_dst);
    else dma_two<2048, 3072>(v_voff, v_src, v_dst);
  };
  auto dma_tile = [&](int t, int img_off) __attribute__((always_inline)) {
    dma_begin(lane_of(t), img_off);
#pragma unroll
    for (int j = 0; j < 4; ++j) dma_k(j);
    dma_v(0);
    dma_v(1);
  };
  // blank the padding slots of the V page this wavefront loaded (rare; after its loads have landed)
  auto blank_padding = [&](int t, int img_off) __attribute__((always_inline)) {
    const int l = lane_of(t);
    const int nvalid = __builtin_amdgcn_readlane(w_nvalid, l), own = __builtin_amdgcn_readlane(w_own, l);
    const int nv = own < 0 ? 0 : min(max(nvalid - kBlock * page, 0), kBlock);
    if (brings_v && nv < kBlock) {
      uint4* vp = reinterpret_cast<uint4*>(const_cast<char*>(lds_bytes) + img_off + (16 + 4 * page) * 1024 + lane * 16);
#pragma unroll
      for (int j = 0; j < 4; ++j) vp[j * 64] = zero_pad_slots(vp[j * 64], hh, nv);
      // (a rare branch leaves nothing pending, so that the code behind the join waits for no more
      // than the straight path does)
      wait_lds<0>();
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
  dma_tile(0, image_off(0));
  dma_tile(1, image_off(1));
  dma_tile(2, image_off(2));
  load_queries();
  wait_loads(std::integral_constant<int, 0>{});
  {
    const int f012 = __builtin_amdgcn_readlane(w_flags, lane_of(0)) | __builtin_amdgcn_readlane(w_flags, lane_of(1)) |
                     __builtin_amdgcn_readlane(w_flags, lane_of(2));
    if (f012 & 2) {
      blank_padding(0, image_off(0));
      blank_padding(1, image_off(1));
      blank_padding(2, image_off(2));
    }
  }
  __syncthreads();
  int f_cur = __builtin_amdgcn_readlane(w_flags, lane_of(0));      // flags of tile t, t+1 (carried from tile to tile)
  int f_next = __builtin_amdgcn_readlane(w_flags, lane_of(1));
  {
    const int img = image_off(0);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const u32x4 a = k_piece(img, 0, kk);
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        if (kk == 0) mfma_s_zero(sacc[qb][0], a, qreg[qb][kk]);
        else mfma_s_acc(sacc[qb][0], a, qreg[qb][kk]);
      }
    }
    if (f_cur & 1) mask_block(0, 0, __builtin_amdgcn_readlane(w_kpos0, 0), __builtin_amdgcn_readlane(w_nvalid, 0));
    else mfma_result_wait();
    // first block of the request: its key 0 is visible to every query, so the maximum is finite;
    // it is the reference for the whole row
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float t = max16(sacc[qb][0]);
      m_ref[qb] = fmaxf(t, __shfl_xor(t, 32, 64));
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        sacc[qb][0][i] -= m_ref[qb];
        cinit[qb][i] = -m_ref[qb];
      }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) exp_only(ev[qb], sacc[qb][0][0]);
#pragma unroll
    for (int i = 1; i < 8; ++i)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) exp_step(qb, 0, i);
#pragma unroll
    for (int s = 0; s < kDepth; ++s) issue(img, img, s);     // steps 0..kDepth-1 of iteration 0
    __builtin_amdgcn_sched_barrier(0);
  }

  // ---- the tile loop --------------------------------------------------------------------------------
  // on entry: parity 0 holds S of the tile's first block (masked) with the first half of its
  // exponentials done.  Every tile runs through the same straight-line body (the masking branches
  // apart): behind the last tile the "next tile" is a phantom whose S block is masked as a whole, so
  // that its exponentials are zeros.  (A peeled copy of the body for the last tile would save those
  // 16 MFMAs per workgroup; but the register allocator then settles the accumulators differently in
  // the two copies and moves them around between MFMAs it cannot see into, without the wait states
  // such moves need in front of a matrix instruction.)
  // By-product for rows that ask for it (snap_index >= 0: the question rows; or every row): when the tile that
  // has just been closed is the last one of its segment, the log-sum-exp over all keys up to here
  // goes to cum[snap row][head][segment's index in its request].  The reference never moves in this
  // kernel, so these running sums subtract exactly.  (Rare: once per segment of the request.)
  const int seg_first = cum != nullptr ? req_seg_off[order[blockIdx.y]] : 0;
  // (segments without tokens have no tile: the value also stands for those between this tile's
  // segment and the next tile's; the row sum is taken with the pair that is still to be packed)
  auto snapshot = [&](int t) __attribute__((always_inline)) {
    const int l = lane_of(t);
    const int seg = __builtin_amdgcn_readlane(w_seg, l), seg_next = __builtin_amdgcn_readlane(w_seg_next, l);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float mine = lsum[qb] + (ev[qb] + vodd[qb]);
      const float tot = mine + __shfl_xor(mine, 32, 64);
      const int sr = snap_index != nullptr ? snap_index[row[qb]] : row[qb];     // (no index: every row is a snap row)
      if (row_valid[qb] && hh == 0 && sr >= 0) {
        const float v = kLn2 * (m_ref[qb] + __builtin_amdgcn_logf(tot));
        for (int sl = max(seg - seg_first, 0); sl < min(seg_next - seg_first, s_max); ++sl)
          cum[(static_cast<size_t>(sr) * hq + h) * s_max + sl] = v;
      }
    }
    wait_lds<0>();                                 // (see blank_padding)
  };
  int f_far = 0;                                   // flags of tile t+2
  for (int t = 0; t < n_t; ++t) {
    const int img = image_off(t), nimg = image_off(t + 1);
    if (min(t + 3, n_t - 1) - win_base >= 64) {          // next 64 descriptors, starting at tile t (rare)
      win_base = t;
      fill_window(t);
      __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));      // vmcnt(0) here, so the hot path never waits for it
    }
    // slot 1: S of the tile's second block; second half of the first block's exponentials.
    // Underneath: the loads of image t+3 (past the last tile they repeat the last tile into an
    // image nobody reads), one instruction group per k-step.
    s_slot(img, nimg, 0, 1, [&](int kk, int qb) __attribute__((always_inline)) {
      exp_step(qb, 0, 8 + kk);
      if (qb == QB - 1) {
        if (kk == 0) {
          f_far = __builtin_amdgcn_readlane(w_flags, lane_of(t + 2));
          dma_begin(lane_of(t + 3), image_off(t + 3));
        }
        if (kk >= 1 && kk <= 4) dma_k(kk - 1);
        if (kk == 5) dma_v(0);
        if (kk == 6) dma_v(1);
      }
    });
    if (f_cur & 1) {
      const int l = lane_of(t);
      mask_block(1, 1, __builtin_amdgcn_readlane(w_kpos0, l), __builtin_amdgcn_readlane(w_nvalid, l));
    }
    // slot 2: PV of the first block; first half of the second block's exponentials
    pv_slot(img, nimg, 8, 0, [&](int st, int qb) __attribute__((always_inline)) { exp_step(qb, 1, st); });
    // slot 3: S of the next tile's first block; second half of the second block's exponentials
    s_slot(img, nimg, 16, 0, [&](int kk, int qb) __attribute__((always_inline)) { exp_step(qb, 1, 8 + kk); });
    if (cum != nullptr && (f_cur & 4)) snapshot(t);          // tile t was the last of its segment
    const bool phantom = t + 1 >= n_t;                       // no next tile: none of its keys exists
    if ((f_next & 1) || phantom) {
      const int l = lane_of(t + 1);
      mask_block(0, 0, __builtin_amdgcn_readlane(w_kpos0, l), phantom ? 0 : __builtin_amdgcn_readlane(w_nvalid, l));
    }
    // slot 4: PV of the second block; first half of the next block's exponentials
    pv_slot(img, nimg, 24, 1, [&](int st, int qb) __attribute__((always_inline)) { exp_step(qb, 0, st); });
    // image t+2 (loads started one iteration ago) must be whole before anyone reads it
    wait_loads(std::integral_constant<int, 4 * QB>{});
    if (f_far & 2) blank_padding(t + 2, image_off(t + 2));
    barrier();
    f_cur = f_next; f_next = f_far;
  }
  mfma_result_wait();

  // ---- epilogue ---------------------------------------------------------------------------------
  float l_tot[QB];
  bool overflow = false;              // some row's sum left the safe range (the sums only grow)
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    l_tot[qb] = lsum[qb] + __shfl_xor(lsum[qb], 32, 64);
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
                    int s_max, hipStream_t stream, const ValueSource& vs) {
  const int hkv = ctx->cfg.n_kv_heads, n_sub = ctx->cfg.n_q_heads / hkv / 4;
  const int n_tiles = (max_q_per_req + 63) / 64;
  dim3 grid(hkv * n_sub * n_tiles, n_requests);
  // Eight wavefronts of 32 rows (two per SIMD) rather than four of 64: the same speed on long prompts
  // and a few percent faster on short ones (measured on the 8B continuous batch: 2.14 vs 2.20 ms).
  constexpr int QB = 1;
  hipLaunchKernelGGL((attn_v2_kernel<QB>), grid, dim3(512 / QB), 0, stream, static_cast<const bf16_t*>(q), q_pos,
                     cu_q, static_cast<const bf16_t*>(k_pool), static_cast<const bf16_t*>(v_pool), n_blocks,
                     pl.tiles, pl.seg_tile_off, pl.max_tiles, pl.order, req_seg_off, ctx->cfg.n_q_heads, hkv,
                     n_sub, n_tiles, ctx->inv_freq, static_cast<bf16_t*>(out), lse, redo, q_map, map_pos, snap_index, cum, s_max,
                     static_cast<const bf16_t*>(vs.v_shared), vs.n_shared_blocks, static_cast<const int32_t*>(vs.v_map));
}

}  // namespace cc
