// plain copy / read / write bandwidth of the chip with 16-byte accesses (ceiling for cc_rope_shift)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
typedef unsigned int vec16 __attribute__((ext_vector_type(4)));
template <int U, bool NTS, bool NTL>
__global__ __launch_bounds__(256) void copy_k(const vec16* __restrict__ s, vec16* __restrict__ d, size_t n) {
  size_t base = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
  vec16 t[U];
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 256 < n) t[u] = NTL ? __builtin_nontemporal_load(s + base + u * 256) : s[base + u * 256];
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 256 < n) { if (NTS) __builtin_nontemporal_store(t[u], d + base + u * 256); else d[base + u * 256] = t[u]; }
}
// block index swizzled so that the 8 XCDs (workgroup i runs on XCD i % 8) do not each keep to one residue of the address
template <int U, bool NTS, bool NTL, int MODE>
__global__ __launch_bounds__(256) void copy_s(const vec16* __restrict__ s, vec16* __restrict__ d, size_t n) {
  unsigned b = blockIdx.x;
  if (MODE == 0) b = (b & ~7u) | ((b + (b >> 3)) & 7u);
  if (MODE == 1) { unsigned g = gridDim.x / 8; b = (b % 8) * g + b / 8; }       // XCD x takes a contiguous eighth
  size_t base = (size_t)b * (256 * U) + threadIdx.x;
  vec16 t[U];
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 256 < n) t[u] = NTL ? __builtin_nontemporal_load(s + base + u * 256) : s[base + u * 256];
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 256 < n) { if (NTS) __builtin_nontemporal_store(t[u], d + base + u * 256); else d[base + u * 256] = t[u]; }
}
// the K part of rope_shift without arithmetic: a workgroup moves one 32 KiB page of 128 rows x 256 B; lane (r, c) of pass u
// reads 16 bytes at row (r + 32u) * 256 + 16c and the 16 bytes 128 further on
template <bool NTS, int PAGE_KIB, bool NTL = false>
__global__ __launch_bounds__(256) void copy_xy(const vec16* __restrict__ s, vec16* __restrict__ d, size_t n) {
  constexpr int ROWS = PAGE_KIB * 4;                       // rows of 256 B per page
  const size_t page = (size_t)blockIdx.x * (PAGE_KIB * 64);   // in vec16
  if (page + PAGE_KIB * 64 > n) return;
  const int r = threadIdx.x >> 3, c = threadIdx.x & 7;
  for (int row0 = r; row0 < ROWS; row0 += 128) {
    vec16 x[4], y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) if (row0 + 32 * u < ROWS) {
      const vec16* px = s + page + (row0 + 32 * u) * 16 + c;
      x[u] = NTL ? __builtin_nontemporal_load(px) : *px; y[u] = NTL ? __builtin_nontemporal_load(px + 8) : px[8];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) if (row0 + 32 * u < ROWS) {
      vec16 a = x[u] + y[u], b = x[u] ^ y[u];
      if (NTS) { __builtin_nontemporal_store(a, d + page + (row0 + 32 * u) * 16 + c); __builtin_nontemporal_store(b, d + page + (row0 + 32 * u) * 16 + c + 8); }
      else { d[page + (row0 + 32 * u) * 16 + c] = a; d[page + (row0 + 32 * u) * 16 + c + 8] = b; }
    }
  }
}
// wave-contiguous: a wavefront's U loads cover U consecutive KiB
template <int U, bool NTS, bool NTL>
__global__ __launch_bounds__(256) void copy_w(const vec16* __restrict__ s, vec16* __restrict__ d, size_t n) {
  size_t base = (size_t)blockIdx.x * (256 * U) + (threadIdx.x >> 6) * (64 * U) + (threadIdx.x & 63);
  vec16 t[U];
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 64 < n) t[u] = NTL ? __builtin_nontemporal_load(s + base + u * 64) : s[base + u * 64];
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 64 < n) { if (NTS) __builtin_nontemporal_store(t[u], d + base + u * 64); else d[base + u * 64] = t[u]; }
}
template <int U>
__global__ __launch_bounds__(256) void read_k(const vec16* __restrict__ s, vec16* __restrict__ d, size_t n) {
  size_t base = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
  vec16 acc = {0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 256 < n) acc ^= s[base + u * 256];
  if (acc.x == 0x12345678u) d[0] = acc;
}
template <int U>
__global__ __launch_bounds__(256) void write_k(vec16* __restrict__ d, size_t n) {
  size_t base = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
  vec16 v = {1, 2, 3, (unsigned)threadIdx.x};
#pragma unroll
  for (int u = 0; u < U; ++u) if (base + u * 256 < n) __builtin_nontemporal_store(v, d + base + u * 256);
}
template <typename F> float timeit(F f, int reps) {
  hipEvent_t a, b; hipEventCreate(&a); hipEventCreate(&b);
  f(); f(); hipDeviceSynchronize();
  hipEventRecord(a); for (int i = 0; i < reps; ++i) f(); hipEventRecord(b); hipEventSynchronize(b);
  float ms; hipEventElapsedTime(&ms, a, b); return ms / reps;
}
// A short copy with cold caches: `mib` MiB moved once per measurement, a 1 GiB copy of other buffers before each one.
template <typename F> float cold(F f, vec16* fa, vec16* fb, size_t fn, int reps) {
  hipEvent_t a, b; (void)hipEventCreate(&a); (void)hipEventCreate(&b);
  float best = 1e9f, sum = 0.f;
  for (int i = 0; i < reps; ++i) {
    copy_k<4, false, false><<<(unsigned)((fn + 1023) / 1024), 256>>>(fa, fb, fn);
    (void)hipEventRecord(a); f(); (void)hipEventRecord(b); (void)hipEventSynchronize(b);
    float ms; (void)hipEventElapsedTime(&ms, a, b);
    if (i > 0) { sum += ms; best = ms < best ? ms : best; }
  }
  return sum / (reps - 1);
}

int main() {
  {
    const size_t fbytes = (size_t)1 << 30, fn = fbytes / 16;
    vec16 *fa, *fb; (void)hipMalloc(&fa, fbytes); (void)hipMalloc(&fb, fbytes); (void)hipMemset(fa, 1, fbytes);
    for (size_t mib : {160, 512}) {
      size_t bytes = mib << 20, n = bytes / 16;
      vec16 *s, *d; (void)hipMalloc(&s, bytes); (void)hipMalloc(&d, bytes); (void)hipMemset(s, 1, bytes); (void)hipMemset(d, 0, bytes);
      { unsigned g = (unsigned)(n / (32 * 64)); float ms = cold([&] { copy_xy<true, 32><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 32 KiB nt-store", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)(n / (16 * 64)); float ms = cold([&] { copy_xy<true, 16><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 16 KiB nt-store", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)(n / (8 * 64)); float ms = cold([&] { copy_xy<true, 8><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 8 KiB nt-store", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)(n / (8 * 64)); float ms = cold([&] { copy_xy<true, 8, true><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 8 KiB nt-both", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)(n / (32 * 64)); float ms = cold([&] { copy_xy<true, 32, true><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 32 KiB nt-both", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)((n + 255) / 256); float ms = cold([&] { copy_k<1, true, false><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "copy U1 nt-store", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)((n + 255) / 256); float ms = cold([&] { copy_k<1, false, false><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "copy U1", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)((n + 255) / 256); float ms = cold([&] { copy_k<1, true, true><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "copy U1 nt-both", ms, 2.0 * bytes / ms * 1e-9); }
      { unsigned g = (unsigned)((n + 1023) / 1024); float ms = cold([&] { copy_k<4, true, true><<<g, 256>>>(s, d, n); }, fa, fb, fn, 8);
        printf("cold %4zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "copy U4 nt-both", ms, 2.0 * bytes / ms * 1e-9); }
      fflush(stdout);
      (void)hipFree(s); (void)hipFree(d);
    }
    (void)hipFree(fa); (void)hipFree(fb);
  }
  for (size_t mib : {1024}) {
    size_t bytes = mib << 20, n = bytes / 16;
    vec16 *s, *d; hipMalloc(&s, bytes); hipMalloc(&d, bytes); hipMemset(s, 1, bytes); hipMemset(d, 0, bytes);
#define RUN(name, kern, U, moved) { unsigned g = (unsigned)((n + 256 * U - 1) / (256 * U)); \
      float ms = timeit([&] { kern; }, 20); printf("%5zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, name, ms, moved / ms * 1e-9); fflush(stdout); }
    RUN("copy U4",         (copy_k<4, false, false><<<g, 256>>>(s, d, n)), 4, 2.0 * bytes)
    RUN("copy U8",         (copy_k<8, false, false><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("copy U8 nt-store", (copy_k<8, true, false><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("copy U8 nt-both",  (copy_k<8, true, true><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("copy U16 nt-both", (copy_k<16, true, true><<<g, 256>>>(s, d, n)), 16, 2.0 * bytes)
    RUN("copy U2 nt-both",  (copy_k<2, true, true><<<g, 256>>>(s, d, n)), 2, 2.0 * bytes)
    RUN("copy U1",          (copy_k<1, false, false><<<g, 256>>>(s, d, n)), 1, 2.0 * bytes)
    RUN("copy U1 nt-store", (copy_k<1, true, false><<<g, 256>>>(s, d, n)), 1, 2.0 * bytes)
    RUN("copy U1 nt-both",  (copy_k<1, true, true><<<g, 256>>>(s, d, n)), 1, 2.0 * bytes)
    RUN("copy U2",          (copy_k<2, false, false><<<g, 256>>>(s, d, n)), 2, 2.0 * bytes)
    RUN("copy U2 nt-store", (copy_k<2, true, false><<<g, 256>>>(s, d, n)), 2, 2.0 * bytes)
    RUN("copy U4 nt-store", (copy_k<4, true, false><<<g, 256>>>(s, d, n)), 4, 2.0 * bytes)
    RUN("copy U4 nt-both",  (copy_k<4, true, true><<<g, 256>>>(s, d, n)), 4, 2.0 * bytes)
    RUN("wavecont U2 nt-store", (copy_w<2, true, false><<<g, 256>>>(s, d, n)), 2, 2.0 * bytes)
    RUN("wavecont U4 nt-store", (copy_w<4, true, false><<<g, 256>>>(s, d, n)), 4, 2.0 * bytes)
    RUN("wavecont U8 nt-store", (copy_w<8, true, false><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("wavecont U8 nt-both",  (copy_w<8, true, true><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("wavecont U16 nt-store", (copy_w<16, true, false><<<g, 256>>>(s, d, n)), 16, 2.0 * bytes)
    RUN("swz0 U8 nt-store", (copy_s<8, true, false, 0><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("swz0 U8 nt-both", (copy_s<8, true, true, 0><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("swz1 U8 nt-store", (copy_s<8, true, false, 1><<<g, 256>>>(s, d, n)), 8, 2.0 * bytes)
    RUN("swz0 U16 nt-store", (copy_s<16, true, false, 0><<<g, 256>>>(s, d, n)), 16, 2.0 * bytes)
    RUN("swz0 U4 nt-store", (copy_s<4, true, false, 0><<<g, 256>>>(s, d, n)), 4, 2.0 * bytes)
    RUN("swz0 U1 nt-store", (copy_s<1, true, false, 0><<<g, 256>>>(s, d, n)), 1, 2.0 * bytes)
    { unsigned g = (unsigned)(n / (32 * 64)); float ms = timeit([&] { copy_xy<true, 32><<<g, 256>>>(s, d, n); }, 20); printf("%5zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 32 KiB nt-store", ms, 2.0 * bytes / ms * 1e-9); }
    { unsigned g = (unsigned)(n / (32 * 64)); float ms = timeit([&] { copy_xy<false, 32><<<g, 256>>>(s, d, n); }, 20); printf("%5zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 32 KiB", ms, 2.0 * bytes / ms * 1e-9); }
    { unsigned g = (unsigned)(n / (16 * 64)); float ms = timeit([&] { copy_xy<true, 16><<<g, 256>>>(s, d, n); }, 20); printf("%5zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 16 KiB nt-store", ms, 2.0 * bytes / ms * 1e-9); }
    { unsigned g = (unsigned)(n / (8 * 64)); float ms = timeit([&] { copy_xy<true, 8><<<g, 256>>>(s, d, n); }, 20); printf("%5zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 8 KiB nt-store", ms, 2.0 * bytes / ms * 1e-9); }
    { unsigned g = (unsigned)(n / (64 * 64)); float ms = timeit([&] { copy_xy<true, 64><<<g, 256>>>(s, d, n); }, 20); printf("%5zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "xy pattern 64 KiB nt-store", ms, 2.0 * bytes / ms * 1e-9); }
    RUN("read U8",          (read_k<8><<<g, 256>>>(s, d, n)), 8, 1.0 * bytes)
    RUN("write U8 nt",      (write_k<8><<<g, 256>>>(d, n)), 8, 1.0 * bytes)
    hipMemcpyAsync(d, s, bytes, hipMemcpyDeviceToDevice, 0);
    { float ms = timeit([&] { hipMemcpyAsync(d, s, bytes, hipMemcpyDeviceToDevice, 0); }, 20); printf("%5zu MiB %-28s %.3f ms  %.2f TB/s\n", mib, "hipMemcpyAsync D2D", ms, 2.0 * bytes / ms * 1e-9); }
    hipFree(s); hipFree(d);
  }
  return 0;
}
