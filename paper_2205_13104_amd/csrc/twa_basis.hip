// Kernels of the basis construction (arXiv 2205.13104, Sec. 3: U = span{w_i}; Sec. 4.1: the
// checkpoints are orthogonalised in their given order).  The sequential Schmidt process of the
// paper is replaced by CholeskyQR2, which yields the same factor W = P R (R upper triangular,
// positive diagonal) from two dense contractions per pass -- the only part of the library that
// is compute bound and therefore runs on the matrix cores:
//
//   gram_kernel        G = W^T W, fp32 inputs widened to fp64 (products exact), accumulated with
//                      v_mfma_f64_16x16x4_f64; LDS-staged D-tiles; only the upper-triangular
//                      16x16 blocks are computed; per-workgroup partial sums, reduced in a fixed
//                      order by gram_reduce_kernel.
//   apply_rinv_kernel  Q = W R^-1 (R^-1 upper triangular, fp32) with v_mfma_f32_16x16x4_f32;
//                      a workgroup owns a tile of rows for ALL n columns, so Q may overwrite W.
#include "twa_device.h"
#include "twa_host.h"

namespace twa {

using f64x4 = double __attribute__((ext_vector_type(4)));
using f32x4 = float __attribute__((ext_vector_type(4)));

constexpr int kTileRows = 64;                 // rows of W (along D) staged in LDS per step
constexpr int kGramStride = kTileRows + 2;    // floats; (2*col + row) mod 32 banks -> conflict free
constexpr int kApplyStride = kTileRows + 16;  // floats; 16-lane row groups land on disjoint banks
constexpr int kMaxBlocksPerWave = 9;          // 8*9/2 upper-triangular blocks over 4 waves

// Row of the 16x16 result held by register r of lane l (both MFMA shapes used here):
//   v_mfma_f32_16x16x4_f32 : row = 4*(l/16) + r
//   v_mfma_f64_16x16x4_f64 : row = 4*r + l/16
__device__ __forceinline__ int mfma_row_f32(int lane, int r) { return 4 * (lane >> 4) + r; }
__device__ __forceinline__ int mfma_row_f64(int lane, int r) { return 4 * r + (lane >> 4); }

// A tile = rows [i0, i0+kTileRows) of all NP (padded) columns; rows >= D and columns >= n are zero.
// It travels in two steps so that the loads of the NEXT tile are in flight while the matrix cores work
// on the current one: global memory -> registers (fetch_tile), registers -> LDS as tile[col*stride + row]
// (store_tile).  Without this the two workgroups of a compute unit fall into step -- both load, then both
// compute -- and the matrix cores idle half of the time (Gram 9.5 ms -> see the measurements).
constexpr int kTileQuads = TWA_MAX_N * (kTileRows / 4) / 256;    // float4 per thread for the widest matrix: 8

__device__ __forceinline__ void fetch_tile(const float* W, int64_t ldw, int64_t D, int n, int NP,
                                           int64_t i0, float4 (&pre)[kTileQuads]) {
  constexpr int V = kTileRows / 4;              // float4 per column
#pragma unroll
  for (int k = 0; k < kTileQuads; ++k) {
    const int idx = threadIdx.x + 256 * k;
    const int col = idx / V;
    const int r4 = idx - col * V;
    const int64_t row = i0 + 4 * r4;
    float4 x = {0.f, 0.f, 0.f, 0.f};
    if (idx < NP * V && col < n) {
      const float* p = W + (int64_t)col * ldw + row;
      if (row + 4 <= D) {
        x = *reinterpret_cast<const float4*>(p);
      } else {
        if (row + 0 < D) x.x = p[0];
        if (row + 1 < D) x.y = p[1];
        if (row + 2 < D) x.z = p[2];
        if (row + 3 < D) x.w = p[3];
      }
    }
    pre[k] = x;
  }
}

template <int STRIDE>
__device__ __forceinline__ void store_tile(int NP, const float4 (&pre)[kTileQuads], float* tile) {
  constexpr int V = kTileRows / 4;
#pragma unroll
  for (int k = 0; k < kTileQuads; ++k) {
    const int idx = threadIdx.x + 256 * k;
    if (idx < NP * V) {
      const int col = idx / V;
      const int r4 = idx - col * V;
      float* t = tile + col * STRIDE + 4 * r4;
      *reinterpret_cast<float2*>(t) = make_float2(pre[k].x, pre[k].y);
      *reinterpret_cast<float2*>(t + 2) = make_float2(pre[k].z, pre[k].w);
    }
  }
}

__global__ __launch_bounds__(256) void gram_kernel(const float* __restrict__ W, int64_t D, int n, int64_t ldw,
                                                   int NP, double* __restrict__ partial) {
  __shared__ float tile[TWA_MAX_N * kGramStride];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nb = NP / 16;
  const int T = nb * (nb + 1) / 2;

  // upper-triangular blocks t = wave, wave+4, ... of the enumeration (a, b >= a)
  int blk_a[kMaxBlocksPerWave], blk_b[kMaxBlocksPerWave];
#pragma unroll
  for (int q = 0; q < kMaxBlocksPerWave; ++q) {
    int t = wave + 4 * q, a = 0;
    if (t >= T) t = T - 1;                       // unused slot: any valid block, result discarded
    while (t >= nb - a) { t -= nb - a; ++a; }
    blk_a[q] = a;
    blk_b[q] = a + t;
  }
  f64x4 acc[kMaxBlocksPerWave];
#pragma unroll
  for (int q = 0; q < kMaxBlocksPerWave; ++q) acc[q] = {0.0, 0.0, 0.0, 0.0};

  const int64_t nchunks = (D + kTileRows - 1) / kTileRows;
  int64_t c0, c1;
  split_range(nchunks, (int)gridDim.x, (int)blockIdx.x, c0, c1);
  const int m = lane & 15, kq = lane >> 4;
  float4 pre[kTileQuads];
  if (c0 < c1) fetch_tile(W, ldw, D, n, NP, c0 * kTileRows, pre);
  for (int64_t c = c0; c < c1; ++c) {
    store_tile<kGramStride>(NP, pre, tile);
    __syncthreads();
    if (c + 1 < c1) fetch_tile(W, ldw, D, n, NP, (c + 1) * kTileRows, pre);     // in flight during the products
#pragma unroll 4
    for (int kk = 0; kk < kTileRows / 4; ++kk) {
#pragma unroll
      for (int q = 0; q < kMaxBlocksPerWave; ++q) {
        if (wave + 4 * q < T) {
          const double a = (double)tile[(16 * blk_a[q] + m) * kGramStride + 4 * kk + kq];
          const double b = (double)tile[(16 * blk_b[q] + m) * kGramStride + 4 * kk + kq];
          acc[q] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, acc[q], 0, 0, 0);
        }
      }
    }
    __syncthreads();
  }
  double* out = partial + (int64_t)blockIdx.x * NP * NP;
#pragma unroll
  for (int q = 0; q < kMaxBlocksPerWave; ++q) {
    if (wave + 4 * q < T) {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        out[(16 * blk_a[q] + mfma_row_f64(lane, r)) * NP + 16 * blk_b[q] + m] = acc[q][r];
    }
  }
}

// gram[i*NP + j] = sum over workgroups in workgroup order (upper-triangular blocks only).
// `accumulate`: the sum is added to what gram holds (rows that arrive in panels).
__global__ __launch_bounds__(256) void gram_reduce_kernel(const double* __restrict__ partial, int nparts, int NP,
                                                          double* __restrict__ gram, int accumulate) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= NP * NP) return;
  const int i = idx / NP, j = idx - i * NP;
  double a = 0.0;
  if ((j >> 4) >= (i >> 4))
    for (int b = 0; b < nparts; ++b) a += partial[(int64_t)b * NP * NP + idx];
  gram[idx] = accumulate ? gram[idx] + a : a;
}

// Q[:, j] = sum_{a <= j} W[:, a] * rinv[a][j];  rinv is NP x NP row major, zero outside the
// upper triangle and outside n x n.  As an MFMA: D[m = j][n' = i] = sum_a A[m][a] B[a][n'] with
// A = rinv^T (kept in registers for the wave's two column blocks) and B = the staged tile.
// (W and Q carry no no-alias promise: Q may be W.)
__global__ __launch_bounds__(256) void apply_rinv_kernel(const float* W, int64_t ldw, float* Q, int64_t ldq, int64_t D, int n,
                                                         int NP, const float* __restrict__ rinv) {
  __shared__ float tile[TWA_MAX_N * kApplyStride];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nb = NP / 16;
  const int m = lane & 15, kq = lane >> 4;
  constexpr int KK = TWA_MAX_N / 4;             // 32 k-steps at most
  constexpr int RG = kTileRows / 16;            // row groups per tile

  float afrag[2][KK];
#pragma unroll
  for (int jbi = 0; jbi < 2; ++jbi) {
    const int jb = wave + 4 * jbi;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int a = 4 * kk + kq, j = 16 * jb + m;
      afrag[jbi][kk] = (jb < nb && a < NP) ? rinv[a * NP + j] : 0.0f;
    }
  }

  const int64_t nchunks = (D + kTileRows - 1) / kTileRows;
  int64_t c0, c1;
  split_range(nchunks, (int)gridDim.x, (int)blockIdx.x, c0, c1);
  float4 pre[kTileQuads];
  if (c0 < c1) fetch_tile(W, ldw, D, n, NP, c0 * kTileRows, pre);
  for (int64_t c = c0; c < c1; ++c) {
    const int64_t i0 = c * kTileRows;
    store_tile<kApplyStride>(NP, pre, tile);
    __syncthreads();
    // the next tile's rows are other rows than this tile's, which are the only ones written below:
    // fetching them now is safe also when Q overwrites W
    if (c + 1 < c1) fetch_tile(W, ldw, D, n, NP, (c + 1) * kTileRows, pre);
    f32x4 acc[2][RG];
#pragma unroll
    for (int jbi = 0; jbi < 2; ++jbi)
#pragma unroll
      for (int rg = 0; rg < RG; ++rg) acc[jbi][rg] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (4 * kk < NP) {                                           // uniform
        float b[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) b[rg] = tile[(4 * kk + kq) * kApplyStride + 16 * rg + m];
#pragma unroll
        for (int jbi = 0; jbi < 2; ++jbi) {
          const int jb = wave + 4 * jbi;
          if (jb < nb && 4 * kk < 16 * (jb + 1)) {                 // uniform; rinv is upper triangular
#pragma unroll
            for (int rg = 0; rg < RG; ++rg)
              acc[jbi][rg] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag[jbi][kk], b[rg], acc[jbi][rg], 0, 0, 0);
          }
        }
      }
    }
    __syncthreads();      // every wave has read the tile; safe to overwrite W rows in place
#pragma unroll
    for (int jbi = 0; jbi < 2; ++jbi) {
      const int jb = wave + 4 * jbi;
      if (jb < nb) {
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) {
          const int64_t row = i0 + 16 * rg + m;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int col = 16 * jb + mfma_row_f32(lane, r);
            if (col < n && row < D) Q[(int64_t)col * ldq + row] = acc[jbi][rg][r];
          }
        }
      }
    }
  }
}

// Zero the padding [D, ld) of every vector.
__global__ __launch_bounds__(256) void zero_padding_kernel(float* __restrict__ Q, int64_t D, int64_t ld) {
  const int j = blockIdx.y;
  for (int64_t i = D + threadIdx.x; i < ld; i += blockDim.x) Q[(int64_t)j * ld + i] = 0.0f;
}

int launch_gram(const float* W, int64_t D, int n, int64_t ldw, double* partial, int grid, double* gram,
                bool accumulate, hipStream_t st) {
  const int NP = (n + 15) / 16 * 16;
  hipLaunchKernelGGL(gram_kernel, dim3(grid), dim3(256), 0, st, W, D, n, ldw, NP, partial);
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((NP * NP + 255) / 256), dim3(256), 0, st, partial, grid, NP, gram,
                     accumulate ? 1 : 0);
  return hip_check(hipGetLastError());
}

int launch_apply_rinv(const float* W, int64_t ldw, float* Q, int64_t ldq, int64_t D, int n, const float* rinv_dev,
                      int grid, bool zero_padding, hipStream_t st) {
  const int NP = (n + 15) / 16 * 16;
  hipLaunchKernelGGL(apply_rinv_kernel, dim3(grid), dim3(256), 0, st, W, ldw, Q, ldq, D, n, NP, rinv_dev);
  if (zero_padding && ldq > D) hipLaunchKernelGGL(zero_padding_kernel, dim3(1, n), dim3(256), 0, st, Q, D, ldq);
  return hip_check(hipGetLastError());
}

}  // namespace twa
