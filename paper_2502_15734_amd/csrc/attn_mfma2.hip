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
// Staging: three tile images in LDS.  In iteration t the wavefronts read image t and (for S of the
// next tile's first block) image t+1, write image t+2 from registers and start the global loads
// of tile t+3.  One s_barrier per tile.  LDS operations of a wavefront complete in order, so when
// a wavefront reaches the barrier its stores to image t+2 have landed and its reads of image t
// have returned; no counter has to be drained at the barrier.
#include <type_traits>

#include "mfma_tile.h"

namespace cc {

using namespace tile;

namespace {

typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kImage = 2048;    // 16-byte pieces per tile image (K: 1024, V: 1024)
constexpr int kBufs = 3;
constexpr int kDepth = 4;       // operand reads in flight ahead of the MFMAs
// p = exp2(S - reference) may be large (fp32 and bf16 share the exponent range); a block sum
// beyond this leaves no headroom for the row sum and O
constexpr float kSafeSum = 1.0e30f;

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}


// Staging of one 64-key tile (K and V of one KV head) for 256 threads: a thread owns the same
// 16-byte piece of each of the tile's four pages in both pools (thread t -> piece t, so a wavefront
// instruction reads one contiguous KiB).  The loads are unconditional -- a page the tile does not
// have is read from block 0 -- so the hot loop has no branch in them; padding slots and missing
// pages are blanked in the registers when the image is stored, in a branch only a segment's last
// tile takes.  (K padding never reaches a product: its S entries are masked by selection.  V
// padding would, as 0 x garbage, so it must be exactly zero.)
struct TileStager {
  uint4 reg[8];                  // K pages 0..3, V pages 0..3
  const bf16_t* k_src;           // pool + head offset + this thread's piece
  const bf16_t* v_src;
  size_t blk_stride;             // elements per block (all heads)
  int piece;

  __device__ __forceinline__ void init(const bf16_t* k_pool, const bf16_t* v_pool, int hkv, int kvh, int tid) {
    piece = tid;
    k_src = k_pool + static_cast<size_t>(kvh) * (kBlock * kD) + tid * 8;
    v_src = v_pool + static_cast<size_t>(kvh) * (kBlock * kD) + tid * 8;
    blk_stride = static_cast<size_t>(hkv) * (kBlock * kD);
  }
  __device__ __forceinline__ void load(const TileDesc& d) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const size_t off = static_cast<size_t>(max(d.blk[j], 0)) * blk_stride;
      reg[j] = *reinterpret_cast<const uint4*>(k_src + off);
      reg[4 + j] = *reinterpret_cast<const uint4*>(v_src + off);
    }
  }
  __device__ __forceinline__ void store(uint4* lds, const TileDesc& d) {
    if (d.nvalid < kTile || (d.blk[0] | d.blk[1] | d.blk[2] | d.blk[3]) < 0) {     // wave-uniform, rare
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int nv = d.blk[j] < 0 ? 0 : min(max(d.nvalid - kBlock * j, 0), kBlock);
        if ((piece >> 4) >= nv) reg[j] = make_uint4(0u, 0u, 0u, 0u);
        if (nv < kBlock) reg[4 + j] = zero_pad_slots(reg[4 + j], piece & 1, nv);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      lds[k_piece_dst(j, piece)] = reg[j];
      lds[v_piece_dst(j, piece)] = reg[4 + j];
    }
  }
};

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
    int32_t* __restrict__ redo) {
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
  int row[QB], p[QB];
  bool row_valid[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    row[qb] = min(q0 + 32 * qb + n, q_end - 1);
    row_valid[qb] = q0 + 32 * qb + n < q_end;
    p[qb] = q_pos[row[qb]];
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
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const bf16_t* qp = q + (static_cast<size_t>(row[qb]) * hq + h) * kD + 8 * hh;
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

  // lane-dependent part of the operand addresses (pieces), constant over the whole loop
  int kx[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) kx[j] = hh * 32 + (n ^ ((2 * j + hh) & 7));
  const int vx = 1024 + hh * 32 + (n ^ (4 * hh));

  float m_ref[QB], l_run[QB], lsum[QB], ev[QB];
  f32x16 o[QB][4];                    // running output, accumulation registers for the whole loop
  f32x16 sacc[QB][2];                 // S of the two 32-key blocks in flight (vector registers)
  uint32_t pk[QB][2][2][4];           // P^T of [block parity][16-key half], packed bf16 pairs
  bool overflow = false;              // some block's sum of exponentials left the safe range
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_ref[qb] = 0.f; l_run[qb] = 0.f; lsum[qb] = 0.f; ev[qb] = 0.f;
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
  auto k_piece = [&](const uint4* im, int blk, int kk) __attribute__((always_inline)) { return *reinterpret_cast<const u32x4*>(&im[(blk * 8 + kk) * 64 + kx[kk & 3]]); };
  auto v_piece = [&](const uint4* im, int idx) __attribute__((always_inline)) { return *reinterpret_cast<const u32x4*>(&im[idx * 64 + vx]); };
  auto issue = [&](const uint4* img, const uint4* nimg, bool has_next, int s) __attribute__((always_inline)) {   // s: compile-time
    if (s < 8) ring[s % kDepth] = k_piece(img, 1, s);
    else if (s < 16) ring[s % kDepth] = v_piece(img, s - 8);
    else if (s < 24) {
      const uint4* a = &nimg[(s - 16) * 64 + kx[s & 3]];
      const uint4* b = &img[(s - 8) * 64 + vx];
      ring[s % kDepth] = *reinterpret_cast<const u32x4*>(has_next ? a : b);
    } else if (s < 32) ring[s % kDepth] = v_piece(img, s - 16);
    else ring[s % kDepth] = k_piece(nimg, 1, s - 32);       // harmless when there is no next tile
  };

  // one exponential: element i (0..15) of block parity bp; pairs are packed as they complete
  auto exp_one = [&](int qb, int bp, int i) __attribute__((always_inline)) {
    const float v = __builtin_amdgcn_exp2f(sacc[qb][bp][i] - m_ref[qb]);
    lsum[qb] += v;
    if ((i & 1) == 0) ev[qb] = v;
    else pk[qb][bp][i >> 3][(i & 7) >> 1] = pack_bf16(ev[qb], v);
    // fake uses: keep the work under the MFMA it was placed under (otherwise it is sunk to its use)
    if ((i & 1) == 0) asm volatile("" :: "v"(lsum[qb]), "v"(ev[qb]));
    else asm volatile("" :: "v"(lsum[qb]), "v"(pk[qb][bp][i >> 3][(i & 7) >> 1]));
  };
  // S block into parity bp from the ring; side(kk, qb) runs after each MFMA
  auto s_slot = [&](const uint4* img, const uint4* nimg, bool has_next, int s0, int bp, auto&& side) __attribute__((always_inline)) {
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
  auto pv_slot = [&](const uint4* img, const uint4* nimg, bool has_next, int s0, int bp, auto&& side) __attribute__((always_inline)) {
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
      overflow = overflow || !(lsum[qb] < kSafeSum);
      l_run[qb] += lsum[qb];
      lsum[qb] = 0.f;
    }
  };

  // ---- descriptors and staging --------------------------------------------------------------------
  TileStager stg;
  stg.init(k_pool, v_pool, hkv, kvh, tid);
  auto image = [&](int t) __attribute__((always_inline)) { return lds_all + (t % kBufs) * kImage; };   // t >= 0
  auto desc_at = [&](int t) __attribute__((always_inline)) { return fetch_desc(tiles, j_begin + min(t, n_t - 1), max_tiles); };
  auto barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // prologue: images 0 and 1, loads of tile 2, S of block 0 and the first half of its exponentials
  TileDesc d0 = to_scalar(desc_at(0)), d1 = to_scalar(desc_at(1)), d2 = to_scalar(desc_at(2));
  TileDesc d3 = to_scalar(desc_at(3));
  stg.load(d0); stg.store(image(0), d0);
  if (n_t > 1) { stg.load(d1); stg.store(image(1), d1); }
  stg.load(d2);
  TileDesc d4v = desc_at(4), d4 = d3;
  __syncthreads();
  {
    const uint4* img = image(0);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const u32x4 a = k_piece(img, 0, kk);
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
  auto tile_front = [&](auto next_tag, int t) __attribute__((always_inline)) {
    constexpr bool kNext = decltype(next_tag)::value;
    const uint4* img = image(t);
    const uint4* nimg = kNext ? image(t + 1) : img;
    // slot 1: S of the tile's second block; second half of the first block's exponentials.
    // Underneath: image t+2 out of the staging registers, loads of tile t+3, descriptor of tile
    // t+5 (past the last tile these repeat the last tile into an image nobody reads).
    uint4* wimg = image(t + 2);
    s_slot(img, nimg, kNext, 0, 1, [&](int kk, int qb) __attribute__((always_inline)) {
      exp_one(qb, 0, 8 + kk);
      if (qb == QB - 1) {
        if (kk == 1) stg.store(wimg, d2);
        if (kk == 3) { d4 = to_scalar(d4v); stg.load(d3); }
        if (kk == 5) d4v = desc_at(t + 5);
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
    const uint4* img = image(t);
    const uint4* nimg = image(t + 1);
    tile_front(NextT{}, t);
    // slot 3: S of the next tile's first block; second half of the second block's exponentials
    s_slot(img, nimg, true, 16, 0, [&](int kk, int qb) __attribute__((always_inline)) { exp_one(qb, 1, 8 + kk); });
    close_block();
    if (d1.nvalid < kTile || d1.kpos0 + kTile - 1 > p_min) mask_block(0, 0, d1.kpos0, d1.nvalid);
    // slot 4: PV of the second block; first half of the next block's exponentials
    pv_slot(img, nimg, true, 24, 1, [&](int st, int qb) __attribute__((always_inline)) { exp_one(qb, 0, st); });
    barrier();
    d0 = d1; d1 = d2; d2 = d3; d3 = d4;
  }
  {
    tile_front(LastT{}, t);
#pragma unroll
    for (int i = 8; i < 16; ++i)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) exp_one(qb, 1, i);
    close_block();
    pv_slot(image(t), image(t), false, 16, 1, no_side);
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
                    int32_t* redo, hipStream_t stream) {
  constexpr int QB = 2;
  const int hkv = ctx->cfg.n_kv_heads, n_sub = ctx->cfg.n_q_heads / hkv / 4;
  const int n_tiles = (max_q_per_req + 32 * QB - 1) / (32 * QB);
  dim3 grid(hkv * n_sub * n_tiles, n_requests);
  hipLaunchKernelGGL((attn_v2_kernel<QB>), grid, dim3(256), 0, stream, static_cast<const bf16_t*>(q), q_pos,
                     cu_q, static_cast<const bf16_t*>(k_pool), static_cast<const bf16_t*>(v_pool), n_blocks,
                     pl.tiles, pl.seg_tile_off, pl.max_tiles, pl.order, req_seg_off, ctx->cfg.n_q_heads, hkv,
                     n_sub, n_tiles, ctx->inv_freq, static_cast<bf16_t*>(out), lse, redo);
}

}  // namespace cc
