// LDS throughput probe: operand reads (ds_read_b128), direct-to-LDS loads of 16 and 4 bytes per lane, and both together.
// One workgroup of 256 threads per CU (LDS 128 KiB), 1024 workgroups, ITER iterations; every access is in bounds.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <vector>
#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("%s: %s\n", #x, hipGetErrorString(e)); return 1; } } while (0)
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
constexpr int ITER = 2000;

template <int MODE>   // 0: reads only; 1: x4 DMA only; 2: x1 DMA only; 3: reads + x4 DMA; 4: reads + x1 DMA
__global__ __launch_bounds__(256, 1) void k(const char* __restrict__ src, uint32_t* __restrict__ sink) {
  __shared__ uint4 buf[8192];                      // 128 KiB
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t lds = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)buf)));
  for (int i = tid; i < 8192; i += 256) buf[i] = make_uint4(i, 1, 2, 3);
  __syncthreads();
  const char* base = src + (blockIdx.x % 64) * 65536;           // 4 MiB of source, L2 resident
  u32x4 acc = {0, 0, 0, 0};
  const char* lb = reinterpret_cast<const char*>(buf);
  for (int it = 0; it < ITER; ++it) {
    // per iteration and wavefront: 32 reads of 1 KiB (like one key tile) and/or 8 KiB of direct loads
    if (MODE == 1 || MODE == 3) {
      const uint32_t dst = lds + ((it + 2) & 3) * 32768 + wave * 8192;
      const uint32_t voff = lane * 16;
      const char* b = base + wave * 8192 + (it & 7) * 8192 * 4 % 32768;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:0" :: "v"(voff), "s"(b + j * 1024), "s"(dst + j * 1024) : "memory", "m0");
    }
    if (MODE == 2 || MODE == 4) {
      const uint32_t dst = lds + ((it + 2) & 3) * 32768 + wave * 8192;
      const uint32_t voff = lane * 4;
      const char* b = base + wave * 8192 + (it & 7) * 8192 * 4 % 32768;
#pragma unroll
      for (int j = 0; j < 32; ++j)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1 offset:0" :: "v"(voff), "s"(b + j * 256), "s"(dst + j * 256) : "memory", "m0");
    }
    if (MODE == 0 || MODE >= 3) {
      const uint32_t ra = lds + (it & 3) * 32768 + lane * 16;
#pragma unroll
      for (int j = 0; j < 32; ++j) {
        u32x4 v;
        asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(ra), "n"(j * 1024));
        if (j == 31) acc += v;
      }
    }
    if (MODE == 1 || MODE == 3) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    if (MODE == 2 || MODE == 4) asm volatile("s_waitcnt vmcnt(32)" ::: "memory");
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  __syncthreads();
  if (acc[0] + acc[1] + acc[2] + acc[3] == 0x12345u) sink[tid] = acc[0];
}

template <int MODE> int run(const char* name, const char* src, uint32_t* sink, double bytes_rd, double bytes_dma) {
  hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
  hipLaunchKernelGGL(k<MODE>, dim3(1024), dim3(256), 0, 0, src, sink);
  CHECK(hipDeviceSynchronize());
  CHECK(hipEventRecord(e0));
  hipLaunchKernelGGL(k<MODE>, dim3(1024), dim3(256), 0, 0, src, sink);
  CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
  float ms; CHECK(hipEventElapsedTime(&ms, e0, e1));
  // 1024 workgroups over 256 CUs = 4 rounds; per workgroup ITER iterations
  const double per_cu_iter_us = ms * 1e3 / 4 / ITER;
  printf("%-22s %8.3f ms  per CU-iteration %.3f us  = %.0f clk @2.4GHz; reads %.0f B/clk, direct loads %.0f B/clk\n", name, ms, per_cu_iter_us,
         per_cu_iter_us * 2400, bytes_rd / (per_cu_iter_us * 2400), bytes_dma / (per_cu_iter_us * 2400));
  fflush(stdout);
  return 0;
}
int main() {
  char* src; uint32_t* sink;
  CHECK(hipMalloc(&src, 8 << 20)); CHECK(hipMemset(src, 1, 8 << 20)); CHECK(hipMalloc(&sink, 4096));
  const double rd = 4 * 32 * 1024.0, dma = 4 * 8192.0;
  if (run<0>("reads only", src, sink, rd, 0)) return 1;
  if (run<1>("x4 direct loads only", src, sink, 0, dma)) return 1;
  if (run<2>("x1 direct loads only", src, sink, 0, dma)) return 1;
  if (run<3>("reads + x4 direct", src, sink, rd, dma)) return 1;
  if (run<4>("reads + x1 direct", src, sink, rd, dma)) return 1;
  return 0;
}
