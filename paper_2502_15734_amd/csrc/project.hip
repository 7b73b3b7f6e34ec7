// cc_qkv_project: [q | k | v] = x W^T for the chosen tokens only (Sec. 3.4.3).
//
// x [n_rows][hidden], W [(Hq+2Hkv)d][hidden]: both operands have the contraction index contiguous.
// bf16: MFMA GEMM.  A workgroup of 8 wavefronts owns a 256 (features) x 256 (tokens) tile of the
// transposed product D^T = W x^T; wavefront (wn, wm) owns 64 features x 128 tokens = 2 x 4 blocks
// of v_mfma_f32_32x32x16_bf16, so 6 operand reads from LDS feed 8 MFMAs per 16-wide k-step.
// K-steps of 32 are double-buffered in LDS (2 x 32 KiB) with the next step's global loads held in
// registers.  In the transposed product a lane holds 4 consecutive features of ONE token, so the
// epilogue writes 8-byte pieces of an output row.  fp32 (and odd shapes): plain LDS-tiled kernel.
//
// The same GEMM kernels serve the other dense products of a decoder layer for the recomputed rows
// (Sec. 2.1, Sec. 3.4.3): y = x W^T (+ residual) and the feed-forward input
// silu(x W_gate^T) * (x W_up^T); only the epilogue and the rows of W a workgroup stages differ.
#include <type_traits>

#include "device_util.h"

namespace cc {

// what a GEMM kernel does with its accumulators
enum { kOutQkv = 0, kOutLinear = 1, kOutGated = 2 };
struct GemmOut {
  void *o0, *o1, *o2;          // qkv: q, k, v; linear / gated: y in o0
  const void* residual;        // linear: added to the product (may be y itself), or null
  int nq, nk;                  // qkv: widths of q and of k (= v)
  int width;                   // linear / gated: features of y
};

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
      ws[kk][r] = (col0 + r < n_cols) ? to_float(w[static_cast<size_t>(col0 + r) * hidden + k0 + kk]) : 0.f;
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

// ---- plain kernels of y = x W^T (+ residual) and of the gated feed-forward input ------------------
template <typename T, bool GATED>
__global__ __launch_bounds__(256) void linear_plain_kernel(
    const T* __restrict__ x, const T* __restrict__ w, const T* __restrict__ w2, const T* residual,
    int n_rows, int n_in, int n_out, T* y) {                      // (residual may be y itself)
  __shared__ float xs[16][64 + 1];
  __shared__ float ws[16][64 + 1];
  __shared__ float us[GATED ? 16 : 1][64 + 1];
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  const int row0 = blockIdx.y * 64, col0 = blockIdx.x * 64;
  float acc[4][4] = {}, acc2[4][4] = {};
  for (int k0 = 0; k0 < n_in; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int r = i / 16, kk = i % 16;
      const bool kin = k0 + kk < n_in;
      xs[kk][r] = (kin && row0 + r < n_rows) ? to_float(x[static_cast<size_t>(row0 + r) * n_in + k0 + kk]) : 0.f;
      ws[kk][r] = (kin && col0 + r < n_out) ? to_float(w[static_cast<size_t>(col0 + r) * n_in + k0 + kk]) : 0.f;
      if (GATED) us[kk][r] = (kin && col0 + r < n_out) ? to_float(w2[static_cast<size_t>(col0 + r) * n_in + k0 + kk]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4], c[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = xs[kk][ty * 4 + i];
        b[i] = ws[kk][tx * 4 + i];
        c[i] = GATED ? us[kk][tx * 4 + i] : 0.f;
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] += a[i] * b[j];
          if (GATED) acc2[i][j] += a[i] * c[j];
        }
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int r = row0 + ty * 4 + i, c = col0 + tx * 4 + j;
      if (r >= n_rows || c >= n_out) continue;
      const size_t at = static_cast<size_t>(r) * n_out + c;
      float v = acc[i][j];
      if (GATED) v = v / (1.f + expf(-v)) * acc2[i][j];
      else if (residual != nullptr) v += to_float(residual[at]);
      y[at] = from_float<T>(v);
    }
}

// ---- MFMA kernel (bf16) -----------------------------------------------------------------------
namespace {

constexpr int kTN = 256, kTM = 256;                   // workgroup tile: features x tokens

// ---- MFMA kernel, 128 x 128 outputs per wavefront -------------------------------------------------
// Workgroup = 4 wavefronts (2 x 2), one per SIMD, 256 features x 256 tokens; a wavefront owns
// 4 x 4 blocks of v_mfma_f32_32x32x16_bf16 (256 accumulation registers), so 8 operand reads from
// LDS feed 16 MFMAs per 16-wide k-step.
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

__device__ __forceinline__ void gemm_load_to_lds(const void* src, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(src), "s"(lds_addr) : "memory", "m0");
}
__device__ __forceinline__ void gemm_mfma(f32x16& d, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(d) : "v"(a), "v"(b));
}

// Epilogue of the 128 x 128-per-wavefront kernels.  D^T block (a, b): lane (nl, hh) holds token
// m0 + 128 wm + 32 b + nl, features n0 + 128 wn + 32 a + 8 (i/4) + 4 hh + i%4.
template <int MODE>
__device__ __forceinline__ void gemm_store_tile(f32x16 (&acc)[4][4], const GemmOut& out, int n_rows, int n0, int m0,
                                                int wn, int wm, int nl, int hh) {
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int row = m0 + wm * 128 + b * 32 + nl;
    if (row >= n_rows) continue;
    if (MODE == kOutGated) {
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        bf16_t* op = static_cast<bf16_t*>(out.o0) + static_cast<size_t>(row) * out.width + n0 / 2 + wn * 64 + a * 32 + 4 * hh;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16_t v4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float gate = acc[a][b][4 * g4 + e], up = acc[a + 2][b][4 * g4 + e];
            v4[e] = static_cast<bf16_t>(gate / (1.f + __expf(-gate)) * up);
          }
          *reinterpret_cast<uint2*>(op + 8 * g4) = *reinterpret_cast<uint2*>(v4);
        }
      }
      continue;
    }
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int col0 = n0 + wn * 128 + a * 32;        // a 32-feature block never straddles q | k | v
      bf16_t* base;
      int c_in, width;
      if (MODE == kOutLinear) { base = static_cast<bf16_t*>(out.o0); c_in = col0; width = out.width; }
      else if (col0 < out.nq) { base = static_cast<bf16_t*>(out.o0); c_in = col0; width = out.nq; }
      else if (col0 < out.nq + out.nk) { base = static_cast<bf16_t*>(out.o1); c_in = col0 - out.nq; width = out.nk; }
      else { base = static_cast<bf16_t*>(out.o2); c_in = col0 - out.nq - out.nk; width = out.nk; }
      const size_t at = static_cast<size_t>(row) * width + c_in + 4 * hh;
      bf16_t* op = base + at;
      const bf16_t* rp = MODE == kOutLinear && out.residual != nullptr ? static_cast<const bf16_t*>(out.residual) + at : nullptr;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        bf16_t v4[4];
        if (rp != nullptr) {
          bf16_t r4[4];
          *reinterpret_cast<uint2*>(r4) = *reinterpret_cast<const uint2*>(rp + 8 * g4);
#pragma unroll
          for (int e = 0; e < 4; ++e) v4[e] = static_cast<bf16_t>(acc[a][b][4 * g4 + e] + static_cast<float>(r4[e]));
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) v4[e] = static_cast<bf16_t>(acc[a][b][4 * g4 + e]);
        }
        *reinterpret_cast<uint2*>(op + 8 * g4) = *reinterpret_cast<uint2*>(v4);
      }
    }
  }
}

// Operands go straight from global memory into LDS (global_load_lds: lane L of an instruction fills
// piece base + L), whole cache lines per load.  A k-stage is 64 wide: 128 bytes = one cache line of
// every row of W and x.  A load instruction brings 8 rows x 128 bytes (8 consecutive lanes share a
// line; an image laid out in MFMA operand order instead - 32 rows x 32 bytes per instruction - was
// measured: it touches 32 lines for the same kilobyte, needs every line in two stages, and ran the
// gated product in 9.96 ms instead of 6.94), and the image in LDS is row-major, 128 bytes per row.  Operand reads walk down 32 rows at one 16-byte piece, so piece c of row r is kept at
// c ^ swz(r), swz(r) = ((r >> 1) & 7) ^ ((r & 1) << 2): any 8 or 16 consecutive rows then spread
// over all banks.  The permutation is applied on the global side (lane -> piece of the line),
// because the load fixes where a lane's bytes land in LDS.  Two images of 64 KiB; per stage the
// wavefronts meet once, at its end.
constexpr int kTK3 = 64;
constexpr int kStage3Bytes = (kTN + kTM) * kTK3 * 2;      // 64 KiB

__device__ __forceinline__ int gemm_swz(int r) { return ((r >> 1) & 7) ^ ((r & 1) << 2); }

//
// Which tile a workgroup takes: workgroups are handed to the 8 XCDs in turn, each XCD with an L2 of
// its own.  Workgroup L therefore takes entry (L % 8) * per_xcd + L / 8 of a tile order in which 32
// consecutive entries (what one XCD runs at a time) form a block of 4 feature tiles x 8 token tiles:
// the block's 32 workgroups ask their L2 for 12 different operand panels instead of up to 34
// (L2 hit rate 48 % -> 82 %, memory reads a third; 3 - 7 % faster for the plain products).  The
// gated product keeps the plain order (feature tile fastest): every blocked order tried was 5 - 10 %
// slower there although it, too, cut the reads that leave the L2s to a third - in the plain order
// all XCDs walk the same rows of token tiles together, so the activations stream from HBM once,
// and an XCD keeps to one fixed set of weight panels, which the memory-side cache can hold.
constexpr int kBlockN = 4, kBlockM = 8;

template <int MODE>
__global__ __launch_bounds__(256, 1) void gemm_mfma3_kernel(
    const bf16_t* __restrict__ x, const bf16_t* __restrict__ w, const bf16_t* __restrict__ w2, int n_rows,
    int hidden, int tiles_n, int tiles_m, GemmOut out) {
  __shared__ uint4 lds[2 * kStage3Bytes / 16];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nl = lane & 31, hh = lane >> 5;
  const int wn = wave & 1, wm = wave >> 1;
  int n0, m0;
  if (MODE == kOutGated) {                                 // (see above: plain order measured faster here)
    if (blockIdx.x >= tiles_n * tiles_m) return;
    n0 = (blockIdx.x % tiles_n) * kTN;
    m0 = (blockIdx.x / tiles_n) * kTM;
  } else {
    const int entry = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    if (entry >= tiles_n * tiles_m) return;                // (the grid is padded to a multiple of 8)
    const int strip = min(entry / (kBlockN * tiles_m), (tiles_n - 1) / kBlockN);   // strip of up to 4 feature tiles
    const int strip_w = min(kBlockN, tiles_n - strip * kBlockN);
    const int in_strip = entry - strip * kBlockN * tiles_m;
    const int blk = in_strip / (strip_w * kBlockM), in_blk = in_strip - blk * strip_w * kBlockM;
    n0 = (strip * kBlockN + in_blk % strip_w) * kTN;
    m0 = (blk * kBlockM + in_blk / strip_w) * kTM;
  }
  const int n_k = hidden / kTK3;

  // ---- staging: wavefront w brings image rows 128 w .. 128 w + 127 (rows 0..255: W, 256..511: x),
  // 8 rows per instruction: lane L -> row 8 j + L / 8, LDS piece L % 8 of that row
  const char* src[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int r = 128 * wave + 8 * j + (lane >> 3);            // image row
    const bf16_t* row;
    if (r >= kTN) row = x + static_cast<size_t>(min(m0 + r - kTN, n_rows - 1)) * hidden;
    else if (MODE != kOutGated) row = w + static_cast<size_t>(n0 + r) * hidden;
    else {
      // gated: of a wavefront's four 32-feature blocks, two are rows of W_gate and two the SAME
      // rows of W_up, so that a lane ends up holding both factors of an output
      const int blk = r >> 5;
      const int f = n0 / 2 + 64 * (blk >> 2) + 32 * (blk & 1) + (r & 31);
      row = ((blk & 2) ? w2 : w) + static_cast<size_t>(f) * hidden;
    }
    src[j] = reinterpret_cast<const char*>(row) + 16 * ((lane & 7) ^ gemm_swz(r));
  }
  typedef __attribute__((address_space(3))) const uint4 lds_piece;
  const uint32_t lds_base = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_piece*)lds)));
  // load j of stage t (past the last stage: a harmless repeat into the image nobody reads any more)
  auto dma_one = [&](int t, int j) __attribute__((always_inline)) {
    const uint32_t dst = lds_base + (t & 1) * kStage3Bytes + (128 * wave + 8 * j) * 128;
    gemm_load_to_lds(src[j] + static_cast<size_t>(min(t, n_k - 1)) * (kTK3 * sizeof(bf16_t)), dst);
  };
  auto wait_all_loads = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0 | (7 << 4) | (15 << 8));       // vmcnt(0)
    asm volatile("" ::: "memory");
  };
  auto barrier = [&]() __attribute__((always_inline)) {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  f32x16 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) asm volatile("v_accvgpr_write_b32 %0, 0" : "=a"(acc[a][b][i]));

  const char* lds_bytes = reinterpret_cast<const char*>(lds);
  const int swz = gemm_swz(nl);                                // (block bases are multiples of 32 rows)
  const int row_a = (128 * wn + nl) * 128, row_b = (kTN + 128 * wm + nl) * 128;
  auto read_a = [&](int t, int s, int a) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4*>(lds_bytes + (t & 1) * kStage3Bytes + row_a + a * 4096 + (((2 * s + hh) ^ swz) << 4));
  };
  auto read_b = [&](int t, int s, int b) __attribute__((always_inline)) {
    return *reinterpret_cast<const u32x4*>(lds_bytes + (t & 1) * kStage3Bytes + row_b + b * 4096 + (((2 * s + hh) ^ swz) << 4));
  };

#pragma unroll
  for (int j = 0; j < 16; ++j) dma_one(0, j);
  wait_all_loads();
  __syncthreads();
  u32x4 opa[2][4], opb[2][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { opa[0][i] = read_a(0, 0, i); opb[0][i] = read_b(0, 0, i); }

  for (int t = 0; t < n_k; ++t) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int cur = s & 1, nxt = cur ^ 1;
      if (s < 3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { opa[nxt][i] = read_a(t, s + 1, i); opb[nxt][i] = read_b(t, s + 1, i); }
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          gemm_mfma(acc[a][b], opa[cur][a], opb[cur][b]);
          // The 16 loads of the next image go out under the MFMAs of the first two k-steps.
          // Measured alternatives: all 16 under the first k-step +2 %, spread over all four +8 %;
          // a barrier before the last k-step (the next stage's first operands then come in under
          // MFMAs, but the loads have one k-step less to land) +4 %; that plus a second barrier
          // at the end of the stage +6 %.
          if (s < 2 && (b & 1)) dma_one(t + 1, 8 * s + 2 * a + (b >> 1));
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    // all loads of image t+1 have landed and everyone has left image t (the loads of the stage
    // after next may overwrite it); the next stage's first operands are read behind the barrier
    wait_all_loads();
    barrier();
#pragma unroll
    for (int i = 0; i < 4; ++i) { opa[0][i] = read_a(t + 1, 0, i); opb[0][i] = read_b(t + 1, 0, i); }
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  gemm_store_tile<MODE>(acc, out, n_rows, n0, m0, wn, wm, nl, hh);
}

// the 128 x 128-per-wavefront kernel (contraction length a multiple of 64)
template <int MODE>
void launch_gemm_wide(dim3 grid, hipStream_t stream, const void* x, const void* w, const void* w2, int n_rows, int n_in,
                      const GemmOut& out) {
  hipLaunchKernelGGL(gemm_mfma3_kernel<MODE>, dim3((grid.x * grid.y + 7) / 8 * 8), dim3(256), 0, stream,
                     static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w), static_cast<const bf16_t*>(w2),
                     n_rows, n_in, static_cast<int>(grid.x), static_cast<int>(grid.y), out);
}

// the MFMA GEMM takes outputs in tiles of 256 features and contraction lengths in stages of 64, at least two
inline bool gemm_wide_fits(int n_features, int n_in) { return n_features % kTN == 0 && n_in % kTK3 == 0 && n_in >= 2 * kTK3; }

}  // namespace

void launch_qkv_project(const cc_ctx* ctx, const void* x, const void* w, int n_rows, int hidden,
                        void* q, void* k, void* v, hipStream_t stream) {
  const int d = ctx->cfg.head_dim;
  const int nq = ctx->cfg.n_q_heads * d, nk = ctx->cfg.n_kv_heads * d, n_cols = nq + 2 * nk;
  if (ctx->cfg.dtype == CC_BF16 && ctx->impl != CC_IMPL_SCALAR && gemm_wide_fits(n_cols, hidden) &&
      nq % 32 == 0 && nk % 32 == 0) {
    dim3 grid(n_cols / kTN, (n_rows + kTM - 1) / kTM);
    launch_gemm_wide<kOutQkv>(grid, stream, x, w, nullptr, n_rows, hidden, GemmOut{q, k, v, nullptr, nq, nk, 0});
    return;
  }
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

// y [n_rows][n_out] = x [n_rows][n_in] W^T (+ residual [n_rows][n_out]); W [n_out][n_in]
void launch_linear(const cc_ctx* ctx, const void* x, const void* w, const void* residual, int n_rows, int n_in,
                   int n_out, void* y, hipStream_t stream) {
  const bool bf = ctx->cfg.dtype == CC_BF16;
  if (bf && ctx->impl != CC_IMPL_SCALAR && gemm_wide_fits(n_out, n_in)) {
    dim3 grid(n_out / kTN, (n_rows + kTM - 1) / kTM);
    launch_gemm_wide<kOutLinear>(grid, stream, x, w, nullptr, n_rows, n_in, GemmOut{y, nullptr, nullptr, residual, 0, 0, n_out});
    return;
  }
  dim3 grid((n_out + 63) / 64, (n_rows + 63) / 64);
  if (bf)
    hipLaunchKernelGGL((linear_plain_kernel<bf16_t, false>), grid, dim3(256), 0, stream, static_cast<const bf16_t*>(x),
                       static_cast<const bf16_t*>(w), static_cast<const bf16_t*>(nullptr),
                       static_cast<const bf16_t*>(residual), n_rows, n_in, n_out, static_cast<bf16_t*>(y));
  else
    hipLaunchKernelGGL((linear_plain_kernel<float, false>), grid, dim3(256), 0, stream, static_cast<const float*>(x),
                       static_cast<const float*>(w), static_cast<const float*>(nullptr),
                       static_cast<const float*>(residual), n_rows, n_in, n_out, static_cast<float*>(y));
}

// y [n_rows][n_ffn] = silu(x W_gate^T) * (x W_up^T); both W [n_ffn][n_in]
void launch_gated_linear(const cc_ctx* ctx, const void* x, const void* w_gate, const void* w_up, int n_rows,
                         int n_in, int n_ffn, void* y, hipStream_t stream) {
  const bool bf = ctx->cfg.dtype == CC_BF16;
  if (bf && ctx->impl != CC_IMPL_SCALAR && gemm_wide_fits(2 * n_ffn, n_in)) {
    dim3 grid(2 * n_ffn / kTN, (n_rows + kTM - 1) / kTM);
    launch_gemm_wide<kOutGated>(grid, stream, x, w_gate, w_up, n_rows, n_in, GemmOut{y, nullptr, nullptr, nullptr, 0, 0, n_ffn});
    return;
  }
  dim3 grid((n_ffn + 63) / 64, (n_rows + 63) / 64);
  if (bf)
    hipLaunchKernelGGL((linear_plain_kernel<bf16_t, true>), grid, dim3(256), 0, stream, static_cast<const bf16_t*>(x),
                       static_cast<const bf16_t*>(w_gate), static_cast<const bf16_t*>(w_up),
                       static_cast<const bf16_t*>(nullptr), n_rows, n_in, n_ffn, static_cast<bf16_t*>(y));
  else
    hipLaunchKernelGGL((linear_plain_kernel<float, true>), grid, dim3(256), 0, stream, static_cast<const float*>(x),
                       static_cast<const float*>(w_gate), static_cast<const float*>(w_up),
                       static_cast<const float*>(nullptr), n_rows, n_in, n_ffn, static_cast<float*>(y));
}

// ---- root-mean-square normalisation: y = x / sqrt(mean(x^2) + eps) * gain ---------------------------
// One wavefront per row (four rows per workgroup).  Rows of up to 64 x 16 pieces of 16 bytes stay
// in registers between the sum of squares and the scaling, so each row moves once in and once out
// of HBM; longer rows are read a second time.
// the elements of a 16-byte piece as floats, and back, without taking the piece's address (which
// would move a register array to scratch memory)
__device__ __forceinline__ void piece_to_floats(const uint4& p, float (&f)[8], bf16_t*) {
  const uint32_t u[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(u[i] << 16);
    f[2 * i + 1] = __uint_as_float(u[i] & 0xffff0000u);
  }
}
__device__ __forceinline__ void piece_to_floats(const uint4& p, float (&f)[4], float*) {
  f[0] = __uint_as_float(p.x); f[1] = __uint_as_float(p.y); f[2] = __uint_as_float(p.z); f[3] = __uint_as_float(p.w);
}

template <typename T>
__global__ __launch_bounds__(256) void rms_norm_kernel(const T* x, const T* __restrict__ gain, float eps,
                                                       int n_rows, int hidden, T* y) {          // (y may be x)
  const int row = blockIdx.x * 4 + threadIdx.x / 64, lane = threadIdx.x % 64;
  if (row >= n_rows) return;
  constexpr int kPer = 16 / sizeof(T);                 // elements per 16-byte piece
  constexpr int kKeep = 16;                            // pieces a lane keeps
  const T* xr = x + static_cast<size_t>(row) * hidden;
  T* yr = y + static_cast<size_t>(row) * hidden;
  const int n_pieces = hidden / kPer;                  // (the call checks that hidden is a multiple of kPer)
  const bool keep = n_pieces <= 64 * kKeep;
  uint4 held[kKeep];
  float ss = 0.f;
  if (keep) {
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
      const int p = lane + 64 * i;
      held[i] = p < n_pieces ? *reinterpret_cast<const uint4*>(xr + p * kPer) : uint4{0, 0, 0, 0};
    }
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
      float f[kPer];
      piece_to_floats(held[i], f, static_cast<T*>(nullptr));
#pragma unroll
      for (int e = 0; e < kPer; ++e) ss += f[e] * f[e];
    }
  } else {
    for (int p = lane; p < n_pieces; p += 64) {
      T v[kPer];
      *reinterpret_cast<uint4*>(v) = *reinterpret_cast<const uint4*>(xr + p * kPer);
#pragma unroll
      for (int e = 0; e < kPer; ++e) ss += to_float(v[e]) * to_float(v[e]);
    }
  }
  const float scale = rsqrtf(wave_sum(ss) / static_cast<float>(hidden) + eps);
  auto scaled = [&](const uint4& in, int p) __attribute__((always_inline)) {
    float f[kPer], g[kPer];
    T o[kPer];
    piece_to_floats(in, f, static_cast<T*>(nullptr));
    piece_to_floats(*reinterpret_cast<const uint4*>(gain + p * kPer), g, static_cast<T*>(nullptr));
#pragma unroll
    for (int e = 0; e < kPer; ++e) o[e] = from_float<T>(f[e] * scale * g[e]);
    *reinterpret_cast<uint4*>(yr + p * kPer) = *reinterpret_cast<uint4*>(o);
  };
  if (keep) {
#pragma unroll
    for (int i = 0; i < kKeep; ++i)
      if (lane + 64 * i < n_pieces) scaled(held[i], lane + 64 * i);
  } else {
    for (int p = lane; p < n_pieces; p += 64) scaled(*reinterpret_cast<const uint4*>(xr + p * kPer), p);
  }
}

void launch_rms_norm(const cc_ctx* ctx, const void* x, const void* gain, float eps, int n_rows, int hidden, void* y,
                     hipStream_t stream) {
  const dim3 grid((n_rows + 3) / 4);
  if (ctx->cfg.dtype == CC_BF16)
    hipLaunchKernelGGL(rms_norm_kernel<bf16_t>, grid, dim3(256), 0, stream, static_cast<const bf16_t*>(x),
                       static_cast<const bf16_t*>(gain), eps, n_rows, hidden, static_cast<bf16_t*>(y));
  else
    hipLaunchKernelGGL(rms_norm_kernel<float>, grid, dim3(256), 0, stream, static_cast<const float*>(x),
                       static_cast<const float*>(gain), eps, n_rows, hidden, static_cast<float*>(y));
}

}  // namespace cc
