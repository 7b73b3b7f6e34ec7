// Cost of re-turning a workgroup's rotated query tile at a segment boundary (what folding the chunk's position offset
// into the query instead of into the keys would add): the tile lives in accumulation registers as bf16 pairs
// (score kernel: 4 column blocks x 8 pieces x 16 B per lane = 128 registers; attention kernel: 1 x 8 = 32), every
// boundary needs cos/sin of (delta x frequency) for the lane's 32 rotation pairs, then 2 FMAs per element on values
// unpacked to fp32 and packed back.  (From the rounded bf16 tile: the variant that keeps or re-reads the exact query
// would cost more.)
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __bf16 bf16_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
template <int QB>
__global__ __launch_bounds__(256, 2) void k(const uint32_t* __restrict__ rnd, const float* __restrict__ freq, int reps, float* __restrict__ sink) {
  u32x4 q[QB][8];
  const int tid = threadIdx.x, hh = (tid & 63) >> 5;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
#pragma unroll
      for (int j = 0; j < 4; ++j) q[qb][kk][j] = rnd[(tid * 13 + qb * 32 + kk * 4 + j) & 4095];
      asm volatile("" : "+a"(q[qb][kk]));
    }
  for (int r = 0; r < reps; ++r) {
    const float delta = static_cast<float>(rnd[r & 4095] & 1023);        // (uniform per boundary)
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      float cs[8], sn[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float t = delta * freq[16 * kk + 8 * hh + j];
        t -= rintf(t);
        cs[j] = __builtin_amdgcn_cosf(t); sn[j] = __builtin_amdgcn_sinf(t);
      }
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        bf16x8 xv = __builtin_bit_cast(bf16x8, q[qb][kk]), yv = __builtin_bit_cast(bf16x8, q[qb][kk + 4]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float x = static_cast<float>(xv[j]), y = static_cast<float>(yv[j]);
          xv[j] = static_cast<bf16_t>(x * cs[j] - y * sn[j]);
          yv[j] = static_cast<bf16_t>(y * cs[j] + x * sn[j]);
        }
        q[qb][kk] = __builtin_bit_cast(u32x4, xv); q[qb][kk + 4] = __builtin_bit_cast(u32x4, yv);
        asm volatile("" : "+a"(q[qb][kk]), "+a"(q[qb][kk + 4]));
      }
    }
  }
  uint32_t acc = 0;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) acc ^= q[qb][kk][0] ^ q[qb][kk][3];
  if (acc == 0x12345u) sink[tid] = 1.f;
}
template <int QB> void run(const char* name, const uint32_t* rnd, const float* freq, float* sink, int wgs) {
  const int reps = 2000;
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  hipLaunchKernelGGL((k<QB>), dim3(wgs), dim3(256), 0, 0, rnd, freq, reps, sink);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL((k<QB>), dim3(wgs), dim3(256), 0, 0, rnd, freq, reps, sink);
  (void)hipEventRecord(e1); (void)hipEventSynchronize(e1);
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  // wgs workgroups on 256 CUs, wgs/256 per CU, i.e. that many wavefronts per SIMD
  printf("%-40s %d workgroups: %.3f us per re-turn of a wavefront's tile (%.1f wavefronts per SIMD resident)\n", name, wgs, ms * 1e3 / reps, wgs / 256.0);
  fflush(stdout);
}
int main() {
  uint32_t h[4096]; uint32_t s = 99;
  for (int i = 0; i < 4096; ++i) { s = s * 1664525u + 1013904223u; h[i] = (0x3c003c00u + ((s >> 8) & 0x03ff03ffu)); }
  float f[64]; for (int i = 0; i < 64; ++i) f[i] = powf(5.0e5f, -i / 64.f) * 0.15915494f;
  uint32_t* rnd; float* fr; float* sink;
  (void)hipMalloc(&rnd, sizeof(h)); (void)hipMemcpy(rnd, h, sizeof(h), hipMemcpyHostToDevice);
  (void)hipMalloc(&fr, sizeof(f)); (void)hipMemcpy(fr, f, sizeof(f), hipMemcpyHostToDevice); (void)hipMalloc(&sink, 4096);
  run<4>("score tile (128 registers)", rnd, fr, sink, 256);
  run<4>("score tile (128 registers)", rnd, fr, sink, 512);
  run<1>("attention tile (32 registers)", rnd, fr, sink, 256);
  run<1>("attention tile (32 registers)", rnd, fr, sink, 512);
  return 0;
}
