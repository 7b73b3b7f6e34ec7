// Device-side helpers shared by the gfx950 kernels: element conversion, rotary angles,
// wavefront (64-lane) reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "common.h"

namespace cc {

typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_float<bf16_t>(float v) { return static_cast<bf16_t>(v); }

// cos/sin of pos * inv_freq.  The product and its reduction to (-pi, pi] are done in fp64 so that
// positions up to ~10^5 with frequency 1 do not lose the angle in fp32; the sine/cosine of the
// reduced angle are then taken in fp32.  pos == 0 yields exactly (1, 0).
__device__ __forceinline__ void rot_cos_sin(int pos, double inv_freq, float* c, float* s) {
  const double kInvTwoPi = 0.15915494309189533576888;
  const double kTwoPi = 6.28318530717958647692529;
  double t = static_cast<double>(pos) * inv_freq * kInvTwoPi;
  t -= rint(t);
  float r = static_cast<float>(t * kTwoPi);
  sincosf(r, s, c);
}

// Same angle, hardware sine/cosine (their argument is in revolutions, which is what the fp64
// reduction produces); absolute error ~1e-6, used where the result is rounded to bf16 anyway.
__device__ __forceinline__ void rot_cos_sin_fast(int pos, double inv_freq, float* c, float* s) {
  const double kInvTwoPi = 0.15915494309189533576888;
  double t = static_cast<double>(pos) * inv_freq * kInvTwoPi;
  t -= rint(t);
  const float tf = static_cast<float>(t);
  *c = __builtin_amdgcn_cosf(tf);
  *s = __builtin_amdgcn_sinf(tf);
}

// Where the values of the page whose keys sit in block blk of the key pool are: block blk of v_own,
// or, while the value map still points at a stored block (copy-on-write pending), that block of
// v_shared.  Returns the first element of the block (all KV heads).
template <typename T>
__device__ __forceinline__ const T* value_block(const T* v_own, const T* v_shared, int n_shared_blocks,
                                                const int32_t* v_map, int blk, size_t block_elems) {
  if (v_map != nullptr) {
    const int m = v_map[blk];
    if (m >= 0 && m < n_shared_blocks) return v_shared + static_cast<size_t>(m) * block_elems;
  }
  return v_own + static_cast<size_t>(blk) * block_elems;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_max_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_min_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
  return v;
}

}  // namespace cc
