// What runs beside a matrix instruction?  Streams of v_mfma_f32_32x32x16_bf16 on random operands with, per MFMA:
//   0 nothing, 1 one v_exp_f32, 2 one v_exp_f16, 3 seven plain VALU ops (fma chain), 4 one v_exp_f32 + 2 plain, 5 two v_exp_f32
// with one or two wavefronts per SIMD (256 / 512 threads; one workgroup per CU: 96 KiB of LDS).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
constexpr int ITER = 3000;

template <int MODE, int NT>
__global__ __launch_bounds__(NT, 1) void k(const uint32_t* __restrict__ rnd, float* __restrict__ sink) {
  __shared__ uint4 pad[6144];                    // 96 KiB: one workgroup per CU
  const int tid = threadIdx.x;
  if (rnd[0] == 0x7fffffffu) pad[tid] = make_uint4(1, 2, 3, 4);
  u32x4 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a[i][j] = rnd[(tid * 37 + i * 4 + j) & 4095];
      b[i][j] = rnd[(tid * 53 + i * 4 + j + 77) & 4095];
    }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  float x0 = __uint_as_float(0x3f000000u | (rnd[tid & 4095] & 0x7fffffu)), x1 = x0 * 0.5f, x2 = 0.f, x3 = 0.f;
  for (int it = 0; it < ITER; ++it) {
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[s & 3]) : "v"(a[s & 3]), "v"(b[(s >> 2) & 3]));
      if (MODE == 1) asm volatile("v_exp_f32 %0, %1" : "=v"(x2) : "v"(x0));
      if (MODE == 2) asm volatile("v_exp_f16 %0, %1" : "=v"(x2) : "v"(x0));
      if (MODE == 3) asm volatile("v_fma_f32 %0, %1, %1, %0\n\tv_fma_f32 %2, %1, %1, %2\n\tv_fma_f32 %0, %1, %1, %0\n\tv_fma_f32 %2, %1, %1, %2\n\t"
                                  "v_fma_f32 %0, %1, %1, %0\n\tv_fma_f32 %2, %1, %1, %2\n\tv_fma_f32 %0, %1, %1, %0" : "+v"(x2), "+v"(x1), "+v"(x3));
      if (MODE == 4) asm volatile("v_exp_f32 %0, %1\n\tv_fma_f32 %2, %1, %1, %2\n\tv_fma_f32 %3, %1, %1, %3" : "=v"(x2), "+v"(x0), "+v"(x1), "+v"(x3));
      if (MODE == 5) asm volatile("v_exp_f32 %0, %2\n\tv_exp_f32 %1, %2" : "=v"(x2), "=v"(x3) : "v"(x0));
      if (MODE == 6) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2\n\tv_cvt_pk_bf16_f32 %3, %1, %2" : "=v"(x2) : "v"(x0), "v"(x1), "v"(x3));
      if (MODE == 7) asm volatile("v_perm_b32 %0, %1, %2, %3\n\tv_perm_b32 %3, %1, %2, %3" : "=v"(x2) : "v"(x0), "v"(x1), "v"(x3));
      if (MODE == 8) asm volatile("v_add_f32 %0, %0, %1\n\tv_add_f32 %2, %2, %1" : "+v"(x2), "+v"(x1), "+v"(x3));
      if (MODE == 9) asm volatile("v_dot2c_f32_bf16 %0, %1, %2\n\tv_dot2c_f32_bf16 %3, %1, %2" : "+v"(x2) : "v"(x0), "v"(x1), "v"(x3));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float t = x1 + x2 + x3;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) t += acc[i][j];
  if (t == 1.2345f) sink[tid] = t;
}
template <int MODE, int NT> int run(const char* name, const uint32_t* rnd, float* sink) {
  hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  hipLaunchKernelGGL((k<MODE, NT>), dim3(1024), dim3(NT), 0, 0, rnd, sink);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  hipLaunchKernelGGL((k<MODE, NT>), dim3(1024), dim3(NT), 0, 0, rnd, sink);
  CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
  float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
  const double mfma = 1024.0 * (NT / 64) * ITER * 16;
  const double pf = mfma * 32768 / (ms * 1e-3) / 1e15;
  // per SIMD: MFMAs of all resident wavefronts
  const double per_simd = mfma / 1024.0;           // 1024 SIMDs
  printf("%-34s NT=%d %8.3f ms  %.3f PFLOP/s  %.1f ns per MFMA per SIMD\n", name, NT, ms, pf, ms * 1e6 / per_simd);
  fflush(stdout);
  return 0;
}
int main() {
  uint32_t h[4096]; uint32_t s = 12345;
  for (int i = 0; i < 4096; ++i) {                 // random bf16 pairs with moderate exponents
    s = s * 1664525u + 1013904223u; uint32_t lo = 0x3c00u + ((s >> 8) & 0x07ffu) | ((s >> 3) & 0x8000u);
    s = s * 1664525u + 1013904223u; uint32_t hi = 0x3c00u + ((s >> 8) & 0x07ffu) | ((s >> 3) & 0x8000u);
    h[i] = lo | (hi << 16);
  }
  uint32_t* rnd; float* sink;
  CHECK(hipMalloc(&rnd, sizeof(h))); CHECK(hipMemcpy(rnd, h, sizeof(h), hipMemcpyHostToDevice)); CHECK(hipMalloc(&sink, 4096));
  if (run<0, 256>("mfma only", rnd, sink)) return 1;
  if (run<1, 256>("mfma + v_exp_f32", rnd, sink)) return 1;
  if (run<2, 256>("mfma + v_exp_f16", rnd, sink)) return 1;
  if (run<3, 256>("mfma + 7 fma", rnd, sink)) return 1;
  if (run<4, 256>("mfma + v_exp_f32 + 2 fma", rnd, sink)) return 1;
  if (run<5, 256>("mfma + 2 v_exp_f32", rnd, sink)) return 1;
  if (run<6, 256>("mfma + 2 v_cvt_pk_bf16_f32", rnd, sink)) return 1;
  if (run<7, 256>("mfma + 2 v_perm_b32", rnd, sink)) return 1;
  if (run<8, 256>("mfma + 2 v_add_f32", rnd, sink)) return 1;
  if (run<9, 256>("mfma + 2 v_dot2c_f32_bf16", rnd, sink)) return 1;
  if (run<0, 512>("mfma only", rnd, sink)) return 1;
  if (run<6, 512>("mfma + 2 v_cvt_pk_bf16_f32", rnd, sink)) return 1;
  if (run<7, 512>("mfma + 2 v_perm_b32", rnd, sink)) return 1;
  if (run<8, 512>("mfma + 2 v_add_f32", rnd, sink)) return 1;
  if (run<9, 512>("mfma + 2 v_dot2c_f32_bf16", rnd, sink)) return 1;
  if (run<1, 512>("mfma + v_exp_f32", rnd, sink)) return 1;
  if (run<2, 512>("mfma + v_exp_f16", rnd, sink)) return 1;
  if (run<3, 512>("mfma + 7 fma", rnd, sink)) return 1;
  if (run<4, 512>("mfma + v_exp_f32 + 2 fma", rnd, sink)) return 1;
  if (run<5, 512>("mfma + 2 v_exp_f32", rnd, sink)) return 1;
  return 0;
}
