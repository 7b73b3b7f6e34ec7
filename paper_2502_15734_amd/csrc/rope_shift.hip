// cc_rope_shift: re-position cached keys (Sec. 3.4.3; Sec. 4 "RPE Management").
//
// HBM-bound streaming kernel.  One workgroup moves one 16-token block of one chunk instance for
// all KV heads: in both pools a block is one contiguous run of Hkv*16*d elements, so every
// wavefront reads and writes whole contiguous kilobytes with 16-byte accesses per lane.  A lane
// owns the same group of rotation pairs AND the same token slot for the whole block (its rows are
// 32 apart: two heads further, same slot), so it evaluates its cos/sin once - also in the mode
// where the store holds keys without any rotation and every token is turned by its own absolute
// position (ABSOLUTE: angle (delta_pos + t) f instead of delta_pos f).
#include "device_util.h"

namespace cc {

template <typename T> struct Vec16;   // 16 bytes of T
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16_t> { static constexpr int N = 8; };

template <typename T, int D, bool ABSOLUTE>
__global__ __launch_bounds__(256) void rope_shift_kernel(
    const T* __restrict__ k_src, const T* __restrict__ v_src, int n_src_blocks,
    T* __restrict__ k_dst, T* __restrict__ v_dst, int n_dst_blocks,
    const int32_t* __restrict__ src_tab, const int32_t* __restrict__ dst_tab,
    const cc_shift_desc* __restrict__ descs, int hkv, InvFreq inv_freq) {
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
  float cs[N], sn[N];
#pragma unroll
  for (int j = 0; j < N; ++j) rot_cos_sin(turn, inv_freq.f[c * N + j], &cs[j], &sn[j]);

  const int rows = hkv * kBlock;          // (head, slot) rows of the block
  for (int row = tid / UPR; row < rows; row += 256 / UPR) {
    if ((row % kBlock) >= n_valid) continue;        // padding slots: neither read nor written
    const T* px = ks + row * D + c * N;
    T* po = kd + row * D + c * N;
    T x[N], y[N];
    *reinterpret_cast<uint4*>(x) = *reinterpret_cast<const uint4*>(px);
    *reinterpret_cast<uint4*>(y) = *reinterpret_cast<const uint4*>(px + D / 2);
    T ox[N], oy[N];
#pragma unroll
    for (int j = 0; j < N; ++j) {
      float xf = to_float(x[j]), yf = to_float(y[j]);
      ox[j] = from_float<T>(xf * cs[j] - yf * sn[j]);
      oy[j] = from_float<T>(yf * cs[j] + xf * sn[j]);
    }
    *reinterpret_cast<uint4*>(po) = *reinterpret_cast<const uint4*>(ox);
    *reinterpret_cast<uint4*>(po + D / 2) = *reinterpret_cast<const uint4*>(oy);
  }

  if (v_src != nullptr && v_dst != nullptr) {       // values carry no position: plain block copy
    const uint4* vs = reinterpret_cast<const uint4*>(v_src + sb * page_elems);
    uint4* vd = reinterpret_cast<uint4*>(v_dst + db * page_elems);
    const int n_vec = static_cast<int>(page_elems / N);
    for (int i = tid; i < n_vec; i += 256) vd[i] = vs[i];
  }
}

template <typename T, int D, bool ABSOLUTE>
static void launch_t(const cc_ctx* ctx, const void* k_src, const void* v_src, int n_src_blocks,
                     void* k_dst, void* v_dst, int n_dst_blocks, const int32_t* src_tab,
                     const int32_t* dst_tab, const cc_shift_desc* descs, int n_instances,
                     int max_tokens, hipStream_t stream) {
  dim3 grid((max_tokens + kBlock - 1) / kBlock, n_instances);
  hipLaunchKernelGGL((rope_shift_kernel<T, D, ABSOLUTE>), grid, dim3(256), 0, stream,
                     static_cast<const T*>(k_src), static_cast<const T*>(v_src), n_src_blocks,
                     static_cast<T*>(k_dst), static_cast<T*>(v_dst), n_dst_blocks, src_tab, dst_tab,
                     descs, ctx->cfg.n_kv_heads, ctx->inv_freq);
}

void launch_rope_shift(const cc_ctx* ctx, const void* k_src, const void* v_src, int n_src_blocks,
                       void* k_dst, void* v_dst, int n_dst_blocks, const int32_t* src_tab,
                       const int32_t* dst_tab, const cc_shift_desc* descs, int n_instances,
                       int max_tokens, bool absolute, hipStream_t stream) {
  const bool bf = ctx->cfg.dtype == CC_BF16;
  const int d = ctx->cfg.head_dim;
#define CC_ARGS ctx, k_src, v_src, n_src_blocks, k_dst, v_dst, n_dst_blocks, src_tab, dst_tab, descs, n_instances, max_tokens, stream
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
