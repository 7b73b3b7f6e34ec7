// cc_rope_shift: re-position cached keys (Sec. 3.4.3; Sec. 4 "RPE Management").
//
// HBM-bound streaming kernel.  One workgroup moves one 16-token block of one chunk instance for
// all KV heads: in both pools a block is one contiguous run of Hkv*16*d elements, so every
// wavefront reads and writes whole contiguous kilobytes with 16-byte accesses per lane.  A lane
// owns the same group of rotation pairs AND the same token slot for the whole block (its rows are
// 32 apart: two heads further, same slot), so it evaluates its cos/sin once - also in the mode
// where the store holds keys without any rotation and every token is turned by its own absolute
// position (ABSOLUTE: angle (delta_pos + t) f instead of delta_pos f).  Every lane issues the
// loads of several rows before it turns and stores the first of them (eight 16-byte requests per
// lane in flight); one block per workgroup measured better than two or four.
#include "device_util.h"

namespace cc {

template <typename T> struct Vec16;   // 16 bytes of T
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16_t> { static constexpr int N = 8; };

typedef unsigned int vec16 __attribute__((ext_vector_type(4)));
// Loads are ordinary: a chunk that several requests of the batch use is read once from HBM and
// then from the cache (measured: non-temporal loads cost 25 % on such a batch and gain 3 % on one
// without sharing).  Stores are non-temporal: the request's pages are written once here and read
// by later kernels only after much other traffic (measured: 2-27 % faster).
__device__ __forceinline__ vec16 load16(const void* p) { return *static_cast<const vec16*>(p); }
__device__ __forceinline__ void store16(void* p, vec16 v) {
  __builtin_nontemporal_store(v, static_cast<vec16*>(p));
}

template <typename T, int D, bool ABSOLUTE>
__global__ __launch_bounds__(256) void rope_shift_kernel(
    const T* __restrict__ k_src, const T* __restrict__ v_src, int n_src_blocks,
    T* __restrict__ k_dst, T* __restrict__ v_dst, int n_dst_blocks,
    const int32_t* __restrict__ src_tab, const int32_t* __restrict__ dst_tab,
    const cc_shift_desc* __restrict__ descs, int hkv, InvFreq inv_freq, int32_t* __restrict__ v_map) {
  constexpr int N = Vec16<T>::N;          // elements per 16-byte vector
  constexpr int UPR = (D / 2) / N;        // vector pairs per (head, token) row
  static_assert(256 % UPR == 0, "a lane must keep its pair group across iterations");
  static_assert((256 / UPR) % kBlock == 0, "a lane must keep its token slot across iterations");
  const cc_shift_desc dsc = descs[blockIdx.y];
  const int page = blockIdx.x;
  const int n_pages = (dsc.n_tokens + kBlock - 1) / kBlock;
  if (page >= n_pages) return;
  const int sb = src_tab[dsc.src_tab_off + page];
  const int db = dst_tab[dsc.dst_tab_off + page];
  if (sb < 0 || sb >= n_src_blocks || db < 0 || db >= n_dst_blocks) return;
  const int n_valid = min(kBlock, dsc.n_tokens - page * kBlock);
  const size_t page_elems = static_cast<size_t>(hkv) * kBlock * D;
  const T* ks = k_src + sb * page_elems;
  T* kd = k_dst + db * page_elems;

  const int tid = threadIdx.x;
  const int c = tid % UPR;                // pair group: pairs c*N .. c*N+N-1
  // token of this lane's rows within the instance (fixed: rows advance by a multiple of 16)
  const int turn = ABSOLUTE ? dsc.delta_pos + page * kBlock + (tid / UPR) % kBlock : dsc.delta_pos;
  // values carry no position: plain block copy.  Its first loads go out before the trigonometry.
  constexpr int UV = 8;                   // 16-byte loads of a lane in flight
  // (with a value map the values stay where they are: the map records which stored block holds
  //  the values of the page whose keys now sit in block db)
  const bool has_v = v_map == nullptr && v_src != nullptr && v_dst != nullptr;
  if (v_map != nullptr && threadIdx.x == 0) v_map[db] = sb;
  const vec16* vs = reinterpret_cast<const vec16*>(v_src + sb * page_elems);
  const int n_vec = static_cast<int>(page_elems / N);
  vec16 tv[UV];
  if (has_v) {
#pragma unroll
    for (int u = 0; u < UV; ++u)
      if (tid + u * 256 < n_vec) tv[u] = load16(vs + tid + u * 256);
  }
  // ... and so do the loads of the first group of key rows
  constexpr int RPI = 256 / UPR;          // rows the workgroup covers per pass
  constexpr int U = 4;                    // passes whose loads are issued together
  const int rows = hkv * kBlock;          // (head, slot) rows of the block
  // (padding slots are neither read nor written; a lane's slot is the same in every pass)
  const bool lane_valid = ((tid / UPR) % kBlock) < n_valid;
  vec16 xv[U], yv[U];
  auto load_rows = [&](int row0) __attribute__((always_inline)) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int row = row0 + u * RPI;
      if (row < rows) {
        const T* px = ks + row * D + c * N;
        xv[u] = load16(px);
        yv[u] = load16(px + D / 2);
      }
    }
  };
  if (lane_valid) load_rows(tid / UPR);
  float cs[N], sn[N];
  double freq[N];                         // (read together: one wait, not one per frequency)
#pragma unroll
  for (int j = 0; j < N; ++j) freq[j] = inv_freq.f[c * N + j];
#pragma unroll
  for (int j = 0; j < N; ++j) {
    if (sizeof(T) == 2) rot_cos_sin_fast(turn, freq[j], &cs[j], &sn[j]);   // (the result is rounded to bf16)
    else rot_cos_sin(turn, freq[j], &cs[j], &sn[j]);
  }

  // Every lane issues all the loads of a group of rows before it turns and stores the first of them,
  // so that several 16-byte requests per lane are in flight.
  if (lane_valid) {
    for (int row0 = tid / UPR; row0 < rows; row0 += U * RPI) {
      if (row0 != tid / UPR) load_rows(row0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int row = row0 + u * RPI;
        if (row < rows) {
          T x[N], y[N], ox[N], oy[N];
          *reinterpret_cast<vec16*>(x) = xv[u];
          *reinterpret_cast<vec16*>(y) = yv[u];
#pragma unroll
          for (int j = 0; j < N; ++j) {
            float xf = to_float(x[j]), yf = to_float(y[j]);
            ox[j] = from_float<T>(xf * cs[j] - yf * sn[j]);
            oy[j] = from_float<T>(yf * cs[j] + xf * sn[j]);
          }
          T* po = kd + row * D + c * N;
          store16(po, *reinterpret_cast<const vec16*>(ox));
          store16(po + D / 2, *reinterpret_cast<const vec16*>(oy));
        }
      }
    }
  }

  if (has_v) {
    vec16* vd = reinterpret_cast<vec16*>(v_dst + db * page_elems);
    for (int i0 = tid; i0 < n_vec; i0 += UV * 256) {
      if (i0 != tid) {
#pragma unroll
        for (int u = 0; u < UV; ++u)
          if (i0 + u * 256 < n_vec) tv[u] = load16(vs + i0 + u * 256);
      }
#pragma unroll
      for (int u = 0; u < UV; ++u)
        if (i0 + u * 256 < n_vec) store16(vd + i0 + u * 256, tv[u]);
    }
  }
}

template <typename T, int D, bool ABSOLUTE>
static void launch_t(const cc_ctx* ctx, const void* k_src, const void* v_src, int n_src_blocks,
                     void* k_dst, void* v_dst, int n_dst_blocks, const int32_t* src_tab,
                     const int32_t* dst_tab, const cc_shift_desc* descs, int n_instances,
                     int max_tokens, int32_t* v_map, hipStream_t stream) {
  dim3 grid((max_tokens + kBlock - 1) / kBlock, n_instances);
  hipLaunchKernelGGL((rope_shift_kernel<T, D, ABSOLUTE>), grid, dim3(256), 0, stream,
                     static_cast<const T*>(k_src), static_cast<const T*>(v_src), n_src_blocks,
                     static_cast<T*>(k_dst), static_cast<T*>(v_dst), n_dst_blocks, src_tab, dst_tab,
                     descs, ctx->cfg.n_kv_heads, ctx->inv_freq, v_map);
}

void launch_rope_shift(const cc_ctx* ctx, const void* k_src, const void* v_src, int n_src_blocks,
                       void* k_dst, void* v_dst, int n_dst_blocks, const int32_t* src_tab,
                       const int32_t* dst_tab, const cc_shift_desc* descs, int n_instances,
                       int max_tokens, bool absolute, int32_t* v_map, hipStream_t stream) {
  const bool bf = ctx->cfg.dtype == CC_BF16;
  const int d = ctx->cfg.head_dim;
#define CC_ARGS ctx, k_src, v_src, n_src_blocks, k_dst, v_dst, n_dst_blocks, src_tab, dst_tab, descs, n_instances, max_tokens, v_map, stream
  if (absolute) {
    if (bf && d == 128) launch_t<bf16_t, 128, true>(CC_ARGS);
    else if (bf && d == 64) launch_t<bf16_t, 64, true>(CC_ARGS);
    else if (!bf && d == 128) launch_t<float, 128, true>(CC_ARGS);
    else launch_t<float, 64, true>(CC_ARGS);
  } else {
    if (bf && d == 128) launch_t<bf16_t, 128, false>(CC_ARGS);
    else if (bf && d == 64) launch_t<bf16_t, 64, false>(CC_ARGS);
    else if (!bf && d == 128) launch_t<float, 128, false>(CC_ARGS);
    else launch_t<float, 64, false>(CC_ARGS);
  }
#undef CC_ARGS
}

}  // namespace cc
