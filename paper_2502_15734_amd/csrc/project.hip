// cc_qkv_project: [q | k | v] = x W for the chosen tokens only (Sec. 3.4.3).
//
// bf16: MFMA GEMM, 128x128 output tile per workgroup (4 wavefronts, 64x64 each as 2x2 blocks of
// v_mfma_f32_32x32x16_bf16), K-step 32 staged through LDS.  fp32: plain LDS-tiled FMA kernel.
// The epilogue splits the fused output columns into the three tensors.
#include "device_util.h"

namespace cc {

template <typename T>
__device__ __forceinline__ void store_qkv(float v, int row, int col, int nq, int nk, T* q, T* k, T* vv) {
  if (col < nq) q[static_cast<size_t>(row) * nq + col] = from_float<T>(v);
  else if (col < nq + nk) k[static_cast<size_t>(row) * nk + (col - nq)] = from_float<T>(v);
  else vv[static_cast<size_t>(row) * nk + (col - nq - nk)] = from_float<T>(v);
}

// ---- plain kernel (any dtype): 64x64 tile, 256 threads, 4x4 outputs per thread ----------------
template <typename T>
__global__ __launch_bounds__(256) void qkv_project_plain_kernel(
    const T* __restrict__ x, const T* __restrict__ w, int n_rows, int hidden, int n_cols, int nq,
    int nk, T* __restrict__ q, T* __restrict__ k, T* __restrict__ v) {
  __shared__ float xs[16][64 + 1];
  __shared__ float ws[16][64 + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int row0 = blockIdx.y * 64, col0 = blockIdx.x * 64;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < hidden; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int r = i / 16, kk = i % 16;
      xs[kk][r] = (row0 + r < n_rows) ? to_float(x[static_cast<size_t>(row0 + r) * hidden + k0 + kk]) : 0.f;
      const int kk2 = i / 64, c = i % 64;
      ws[kk2][c] = (col0 + c < n_cols) ? to_float(w[static_cast<size_t>(k0 + kk2) * n_cols + col0 + c]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = xs[kk][ty * 4 + i]; b[i] = ws[kk][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int r = row0 + ty * 4 + i, c = col0 + tx * 4 + j;
      if (r < n_rows && c < n_cols) store_qkv<T>(acc[i][j], r, c, nq, nk, q, k, v);
    }
}

void launch_qkv_project(const cc_ctx* ctx, const void* x, const void* w, int n_rows, int hidden,
                        void* q, void* k, void* v, hipStream_t stream) {
  const int d = ctx->cfg.head_dim;
  const int nq = ctx->cfg.n_q_heads * d, nk = ctx->cfg.n_kv_heads * d, n_cols = nq + 2 * nk;
  dim3 grid((n_cols + 63) / 64, (n_rows + 63) / 64);
  if (ctx->cfg.dtype == CC_BF16)
    hipLaunchKernelGGL(qkv_project_plain_kernel<bf16_t>, grid, dim3(256), 0, stream,
                       static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w), n_rows, hidden,
                       n_cols, nq, nk, static_cast<bf16_t*>(q), static_cast<bf16_t*>(k),
                       static_cast<bf16_t*>(v));
  else
    hipLaunchKernelGGL(qkv_project_plain_kernel<float>, grid, dim3(256), 0, stream,
                       static_cast<const float*>(x), static_cast<const float*>(w), n_rows, hidden,
                       n_cols, nq, nk, static_cast<float*>(q), static_cast<float*>(k),
                       static_cast<float*>(v));
}

}  // namespace cc
