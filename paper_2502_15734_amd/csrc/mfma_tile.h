// Shared pieces of the MFMA (bf16, head_dim 128) kernels: the 64-key tile descriptor written by the
// plan kernels, the LDS image layout of a staged K/V tile, and the register-prefetch stager.
//
// LDS image of a tile (16-byte pieces; every MFMA operand read is one conflict-free 1 KiB run):
//   K piece (block b of 32 keys, k-step kk, half hh, row m):  (b*8+kk)*64 + hh*32 + (m ^ ((2kk+hh)&7))
//   V piece (page pg, 32-dim group db, half hh, dim n):       1024 + (pg*4+db)*64 + hh*32 + (n ^ 4hh)
// The XOR terms spread the *writes* of a coalesced global read over the LDS banks.  Within a
// 32-key block the MFMA row m holds the key swap_bits_2_3(m), so that the 8 accumulator values a
// lane-half feeds to one 16-key step of the second product are slots 8*half..8*half+7 of one
// 16-token block -- one 16-byte piece of the dimension-major V block.
#pragma once

#include "device_util.h"

namespace cc {
namespace tile {

constexpr int kD = 128;
constexpr int kTile = 64;                      // keys per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kBig = 1.0e12f;                // a tile sum above this moves the reference maximum
constexpr float kZeroBand = 24.f;              // first-block maxima within this keep the reference at 0

__device__ __forceinline__ int swap23(int m) { return (m & ~12) | ((m & 4) << 1) | ((m & 8) >> 1); }
__device__ __forceinline__ int uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }

// One key tile as the plan kernels lay it out (32 bytes, read with two 16-byte loads).
struct TileDesc {
  int32_t kpos0;     // logical position of the tile's first key
  int32_t nvalid;    // keys of the tile that exist (1..64); the rest is block padding
  int32_t blk[4];    // physical block of each of the four 16-token pages (-1: none)
  int32_t seg;       // segment the tile belongs to
  int32_t pad;
};
static_assert(sizeof(TileDesc) == 32, "descriptor is read as two 16-byte vectors");

// a descriptor that came in through a (broadcast) vector load, moved to scalar registers
__device__ __forceinline__ TileDesc to_scalar(const TileDesc& v) {
  TileDesc d;
  d.kpos0 = __builtin_amdgcn_readfirstlane(v.kpos0);
  d.nvalid = __builtin_amdgcn_readfirstlane(v.nvalid);
#pragma unroll
  for (int i = 0; i < 4; ++i) d.blk[i] = __builtin_amdgcn_readfirstlane(v.blk[i]);
  d.seg = 0;
  d.pad = 0;
  return d;
}

// The index is laundered through a vector register on purpose: a scalar (SMEM) load here would
// share the LDS operand reads' completion counter, return out of order, and force a full drain
// of the operand ring every tile; a broadcast vector load is counted with the global loads.
__device__ __forceinline__ TileDesc fetch_desc(const TileDesc* __restrict__ tiles, int j, int max_tiles) {
  int jj = min(max(j, 0), max_tiles - 1);
  asm volatile("" : "+v"(jj));
  const uint4* src = reinterpret_cast<const uint4*>(tiles + jj);
  union { uint4 v[2]; TileDesc d; } u;
  u.v[0] = src[0];
  u.v[1] = src[1];
  return u.d;
}

// LDS piece index of piece `cc_` (0..255, pool order) of page `pg` of the K / V tile image.
__device__ __forceinline__ int k_piece_dst(int pg, int cc_) {
  const int slot = cc_ >> 4, ch = cc_ & 15;
  // key a = 16*pg + slot of the tile -> block a/32, MFMA row swap23(a%32)
  return ((pg >> 1) * 8 + (ch >> 1)) * 64 + (ch & 1) * 32 + (((pg & 1) * 16 + swap23(slot)) ^ (ch & 7));
}
__device__ __forceinline__ int v_piece_dst(int pg, int cc_) {
  const int dcol = cc_ >> 1, hh = cc_ & 1;
  return 1024 + (pg * 4 + (dcol >> 5)) * 64 + hh * 32 + ((dcol & 31) ^ (4 * hh));
}
// V piece with the slots >= nv (padding of a partly filled block) zeroed.
__device__ __forceinline__ uint4 zero_pad_slots(uint4 val, int hh, int nv) {
  unsigned short e[8];
  *reinterpret_cast<uint4*>(e) = val;
#pragma unroll
  for (int j = 0; j < 8; ++j) if (8 * hh + j >= nv) e[j] = 0;
  return *reinterpret_cast<uint4*>(e);
}

// Staging of one key tile (and, if WITH_V, the value tile) of KV head `kvh` for workgroups of 256
// or 512 threads.  A thread owns the same 16-byte piece of every page it stages (thread t ->
// piece t % 256, so a wavefront instruction reads one contiguous KiB of a page); with 512 threads
// the lower half of the workgroup takes pages {0,1} and the upper half pages {2,3}.  Block ids
// come from the tile descriptor (already in registers), so all data loads are issued back to back
// with no memory access in between, one tile ahead of their use (load), and are written to the
// LDS image later (store).
// Slots past the segment's end are staged as zeros so that stale or non-finite padding can never
// reach a product.
template <int NT, bool WITH_V>
struct Stager {
  static_assert(NT == 256 || NT == 512, "register-prefetch staging needs 256 or 512 threads");
  static constexpr int kPagesPerThread = 1024 / NT;          // 4 or 2 pages of each pool
  static constexpr int PER = kPagesPerThread * (WITH_V ? 2 : 1);
  uint4 reg[PER];
  const bf16_t* k_src;   // pool + head offset + this thread's piece
  const bf16_t* v_src;
  const bf16_t* v_src_shared;   // the same piece of a block of the shared value pool
  const int32_t* v_map;         // see value_block()
  size_t blk_stride;     // elements per block (all heads)
  int n_blocks, n_shared_blocks, in_page, pg0;

  __device__ __forceinline__ void init(const bf16_t* k_pool, const bf16_t* v_pool, int n_blocks_,
                                       int hkv, int kvh, int tid, const bf16_t* v_shared = nullptr,
                                       int n_shared_blocks_ = 0, const int32_t* v_map_ = nullptr) {
    v_map = v_map_;
    n_shared_blocks = n_shared_blocks_;
    v_src_shared = (WITH_V && v_shared != nullptr)
                       ? v_shared + static_cast<size_t>(kvh) * (kBlock * kD) + (tid & 255) * 8 : nullptr;
    in_page = tid & 255;
    pg0 = NT == 512 ? uniform(tid >> 8) * 2 : 0;             // first page this thread stages
    k_src = k_pool + static_cast<size_t>(kvh) * (kBlock * kD) + in_page * 8;
    v_src = WITH_V ? v_pool + static_cast<size_t>(kvh) * (kBlock * kD) + in_page * 8 : nullptr;
    blk_stride = static_cast<size_t>(hkv) * (kBlock * kD);
    n_blocks = n_blocks_;
  }

  // this thread's piece of the values that belong to key block blk (a valid block id)
  __device__ __forceinline__ const bf16_t* value_piece(int blk) const {
    if (v_map != nullptr) {
      const int m = uniform(v_map[blk]);
      if (m >= 0 && m < n_shared_blocks) return v_src_shared + static_cast<size_t>(m) * blk_stride;
    }
    return v_src + static_cast<size_t>(blk) * blk_stride;
  }

  __device__ __forceinline__ void load(const TileDesc& d) {
    const int nvalid = uniform(d.nvalid);
    int blk[kPagesPerThread];
    bool all_ok = nvalid == kTile;
#pragma unroll
    for (int j = 0; j < kPagesPerThread; ++j) {
      blk[j] = uniform(NT == 512 ? (pg0 ? d.blk[2 + j] : d.blk[j]) : d.blk[j]);
      all_ok = all_ok && blk[j] >= 0 && blk[j] < n_blocks;
    }
    if (all_ok) {                                            // whole tile present (wave-uniform)
#pragma unroll
      for (int j = 0; j < kPagesPerThread; ++j) {
        reg[j] = *reinterpret_cast<const uint4*>(k_src + static_cast<size_t>(blk[j]) * blk_stride);
        if constexpr (WITH_V)
          reg[kPagesPerThread + j] = *reinterpret_cast<const uint4*>(value_piece(blk[j]));
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < kPagesPerThread; ++j) {
      const int pg = pg0 + j;
      const int nv = min(max(nvalid - kBlock * pg, 0), kBlock);
      const bool ok = nv > 0 && blk[j] >= 0 && blk[j] < n_blocks;
      uint4 kv = make_uint4(0u, 0u, 0u, 0u), vv = make_uint4(0u, 0u, 0u, 0u);
      if (ok) {
        if ((in_page >> 4) < nv)                             // token slot of this K piece
          kv = *reinterpret_cast<const uint4*>(k_src + static_cast<size_t>(blk[j]) * blk_stride);
        if constexpr (WITH_V) {
          vv = *reinterpret_cast<const uint4*>(value_piece(blk[j]));
          if (nv < kBlock) vv = zero_pad_slots(vv, in_page & 1, nv);
        }
      }
      reg[j] = kv;
      if constexpr (WITH_V) reg[kPagesPerThread + j] = vv;
    }
  }

  __device__ __forceinline__ void store(uint4* lds) const {
#pragma unroll
    for (int j = 0; j < kPagesPerThread; ++j) {
      lds[k_piece_dst(pg0 + j, in_page)] = reg[j];
      if constexpr (WITH_V) lds[v_piece_dst(pg0 + j, in_page)] = reg[kPagesPerThread + j];
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

__device__ __forceinline__ f32x16 splat16(float v) {
  f32x16 r;
#pragma unroll
  for (int i = 0; i < 16; ++i) r[i] = v;
  return r;
}


}  // namespace tile

// ---- tile plan (built by plan kernels on the stream, kept in the caller's workspace) ----------
// What the workgroups of grid row y need to start: the segment (score) or request (attention) of
// dispatch rank y and where its key tiles begin.
struct WorkItem {
  int32_t id;         // segment / request index
  int32_t kind;       // segment kind (score)
  int32_t start;      // segment's logical start (score)
  int32_t n_tokens;   // segment length (score)
  int32_t tok_off;    // segment's first row in per-token tensors (score)
  int32_t j_begin;    // first key tile of the request
  int32_t j_own;      // first tile of the segment itself (score); end of the request's tiles (attention)
  int32_t pad;
};
static_assert(sizeof(WorkItem) == 32, "read as two 16-byte vectors");
struct Plan { int32_t* seg_tile_off; int32_t* order; WorkItem* items; tile::TileDesc* tiles; int max_tiles; int32_t* redo; };
size_t plan_head_bytes(int n_segs);
// n_requests > 0: dispatch order over requests (attention); 0: over segments (score).
// n_redo > 0: the plan also holds n_redo redo flags (after the tiles), cleared by the plan kernels.
Plan run_plan(void* ws, const cc_segment* segs, int n_segs, const int32_t* req_seg_off, int n_requests,
              const int32_t* block_tab, int n_blocks, int max_tiles, int n_redo, hipStream_t stream);

// The wide attention kernel (64 query rows per wavefront) keeps one softmax reference per row; rows
// whose sums leave the safe range are flagged in redo[] and redone by the narrow kernel, which can
// move its reference.  q0 is the first row of the 64-row tile (the request's first row + 64 k);
// two tiles of different requests may share an entry, which only costs a spurious redo.
__host__ __device__ inline int redo_index(int q0) { return q0 >> 5; }
inline size_t redo_entries(int n_q_tot) { return static_cast<size_t>(n_q_tot) / 32 + 2; }

void launch_attn_v2(const cc_ctx* ctx, const void* q, const int32_t* q_pos, const int32_t* cu_q,
                    int max_q_per_req, const void* k_pool, const void* v_pool, int n_blocks,
                    const Plan& pl, const int32_t* req_seg_off, int n_requests, void* out, float* lse,
                    int32_t* redo, const int32_t* q_map, int map_pos, const int32_t* snap_index, float* cum,
                    int s_max, hipStream_t stream, const ValueSource& vs);

// The wide score kernel (128 tokens per wavefront, no softmax reference) flags 64-row granules of
// the per-token tensors whose sums left the safe range; the narrow kernel redoes them.
inline size_t score_redo_entries(int n_tok) { return static_cast<size_t>(n_tok) / 64 + 2; }
void launch_score_v2(const cc_ctx* ctx, const void* q, const void* k_pool, int n_blocks, const Plan& pl,
                     const cc_segment* segs, int n_segs, const int32_t* req_seg_off, int max_seg_tokens,
                     float* mass, int32_t* redo, hipStream_t stream);

}  // namespace cc
