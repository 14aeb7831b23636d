// Kernels of the basis construction (arXiv 2205.13104, Sec. 3: U = span{w_i}; Sec. 4.1: the
// checkpoints are orthogonalised in their given order).  The sequential Schmidt process of the
// paper is replaced by CholeskyQR2, which yields the same factor W = P R (R upper triangular,
// positive diagonal) from two dense contractions per pass -- the only part of the library that
// is compute bound and therefore runs on the matrix cores:
//
//   gram_kernel        G = W^T W, fp32 inputs widened to fp64 (products exact), accumulated with
//                      v_mfma_f64_16x16x4_f64; LDS-staged D-tiles; only the upper-triangular
//                      16x16 blocks are computed; per-workgroup partial sums, reduced in a fixed
//                      order by gram_reduce_kernel.  For the second pass (input orthonormal to ~1e-4)
//                      the products of a tile run on v_mfma_f32_16x16x4_f32 and the tiles are summed in fp64.
//   apply_rinv_kernel  Q = W R^-1 (R^-1 upper triangular, fp32) with v_mfma_f32_16x16x4_f32;
//                      a workgroup owns a tile of rows for ALL n columns, so Q may overwrite W.
//
// Both kernels are compiled per number of 16-column blocks (1..8), and inside them every wave runs its own
// copy of the product loop in which block indices, operand registers and trip counts are constants: with
// run-time block indices the loop had a branch per block, the compiler could not move the LDS reads of a
// block ahead of the matrix instruction of the previous one, and every instruction waited out an LDS
// latency (Gram 7.7 -> 6.2 ms, apply 6.5 -> 4.9 ms at D = 25.6 M, n = 100).
#include <type_traits>
#include <utility>

#include "twa_device.h"
#include "twa_host.h"

namespace twa {

using f64x4 = double __attribute__((ext_vector_type(4)));
using f32x4 = float __attribute__((ext_vector_type(4)));

constexpr int kTileRows = 64;                 // rows of W (along D) staged in LDS per step
constexpr int kGramStride = kTileRows + 2;    // floats; (2*col + row) mod 32 banks -> conflict free
constexpr int kApplyStride = kTileRows + 16;  // floats; 16-lane row groups land on disjoint banks

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
        // streamed once per pass: non-temporal (1.5 % on the whole construction; non-temporal STORES of
        // the result cost 1.8 % instead -- the next pass reads it back)
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        x = make_float4(t[0], t[1], t[2], t[3]);
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

// The upper-triangular 16x16 blocks (a, b >= a) of an NB x NB block matrix, enumerated row by row; wave w
// owns blocks t = w, w + 4, ...  Everything here is a compile-time constant, so that the operands and the
// sums of a wave's blocks sit in registers with static indices and the compiler can order the LDS reads
// of a k-step ahead of its matrix instructions.
template <int NB> struct GramBlocks {
  static constexpr int T = NB * (NB + 1) / 2;
  static constexpr int NQ = (T + 3) / 4;                 // blocks per wave, at most
  static constexpr int row_of(int t) { int a = 0; while (t >= NB - a) { t -= NB - a; ++a; } return a; }
  static constexpr int col_of(int t) { int a = 0; while (t >= NB - a) { t -= NB - a; ++a; } return a + t; }
};

// T = double: fp32 inputs widened, v_mfma_f64_16x16x4_f64 (products and sums exact to fp64 rounding: what the
// first pass needs, whose Gram matrix has a condition number near 1/eps32).  T = float: v_mfma_f32_16x16x4_f32 at
// twice the rate, for a matrix that is orthonormal already to ~1e-4 (the second pass): the caller adds every
// tile's fp32 sums (16 k-steps) to fp64 sums, so rounding does not build up along D.
template <typename T> struct GramAcc;
template <> struct GramAcc<double> { using type = f64x4; };
template <> struct GramAcc<float> { using type = f32x4; };

template <int NB, int WV, int Q, typename T>
__device__ __forceinline__ void gram_block_step(const T (&x)[NB], typename GramAcc<T>::type (&acc)[GramBlocks<NB>::NQ]) {
  using B = GramBlocks<NB>;
  if constexpr (WV + 4 * Q < B::T) {
    constexpr int a = B::row_of(WV + 4 * Q), b = B::col_of(WV + 4 * Q);
    if constexpr (sizeof(T) == 8) acc[Q] = __builtin_amdgcn_mfma_f64_16x16x4f64(x[a], x[b], acc[Q], 0, 0, 0);
    else acc[Q] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[a], x[b], acc[Q], 0, 0, 0);
  }
}
template <int NB, int WV, typename T, int... Q>
__device__ __forceinline__ void gram_k_step(const T (&x)[NB], typename GramAcc<T>::type (&acc)[GramBlocks<NB>::NQ],
                                            std::integer_sequence<int, Q...>) {
  (gram_block_step<NB, WV, Q, T>(x, acc), ...);
}
// One staged tile: kTileRows / 4 k-steps.  Lane (m, kq) holds element [16c + m][4kk + kq] of column block c,
// which is its share of the block both as the left and as the right operand.
template <int NB, int WV, typename T>
__device__ __forceinline__ void gram_tile_products(const float* tile, int m, int kq,
                                                   typename GramAcc<T>::type (&acc)[GramBlocks<NB>::NQ]) {
  constexpr int kSteps = NB == 8 ? 8 : 16;      // unrolled k-steps: the widest matrix has no registers for 16 steps' operands
#pragma unroll kSteps
  for (int kk = 0; kk < kTileRows / 4; ++kk) {
    T x[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) x[c] = (T)tile[(16 * c + m) * kGramStride + 4 * kk + kq];
    gram_k_step<NB, WV, T>(x, acc, std::make_integer_sequence<int, GramBlocks<NB>::NQ>{});
  }
}
template <int NB, int WV, int Q, bool F64>
__device__ __forceinline__ void gram_block_out(const f64x4 (&acc)[GramBlocks<NB>::NQ], double* out, int NP, int lane) {
  using B = GramBlocks<NB>;
  if constexpr (WV + 4 * Q < B::T) {
    constexpr int a = B::row_of(WV + 4 * Q), b = B::col_of(WV + 4 * Q);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = F64 ? mfma_row_f64(lane, r) : mfma_row_f32(lane, r);   // the layout of the instruction used
      out[(16 * a + row) * NP + 16 * b + (lane & 15)] = acc[Q][r];
    }
  }
}
template <int NB, int WV, bool F64, int... Q>
__device__ __forceinline__ void gram_out(const f64x4 (&acc)[GramBlocks<NB>::NQ], double* out, int NP, int lane,
                                         std::integer_sequence<int, Q...>) {
  (gram_block_out<NB, WV, Q, F64>(acc, out, NP, lane), ...);
}

template <int NB, bool F64>
__global__ __launch_bounds__(256, 2) void gram_kernel(const float* __restrict__ W, int64_t D, int n, int64_t ldw,
                                                   double* __restrict__ partial) {
  using B = GramBlocks<NB>;
  using T = typename std::conditional<F64, double, float>::type;
  constexpr int NP = 16 * NB;
  __shared__ float tile[NP * kGramStride];
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  f64x4 acc[B::NQ];
#pragma unroll
  for (int q = 0; q < B::NQ; ++q) acc[q] = {0.0, 0.0, 0.0, 0.0};

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
    if constexpr (F64) {
      switch (wave) {                                                           // uniform per wave
        case 0: gram_tile_products<NB, 0, double>(tile, m, kq, acc); break;
        case 1: gram_tile_products<NB, 1, double>(tile, m, kq, acc); break;
        case 2: gram_tile_products<NB, 2, double>(tile, m, kq, acc); break;
        default: gram_tile_products<NB, 3, double>(tile, m, kq, acc); break;
      }
    } else {
      f32x4 part[B::NQ];                                                        // this tile's sums
#pragma unroll
      for (int q = 0; q < B::NQ; ++q) part[q] = {0.f, 0.f, 0.f, 0.f};
      switch (wave) {
        case 0: gram_tile_products<NB, 0, float>(tile, m, kq, part); break;
        case 1: gram_tile_products<NB, 1, float>(tile, m, kq, part); break;
        case 2: gram_tile_products<NB, 2, float>(tile, m, kq, part); break;
        default: gram_tile_products<NB, 3, float>(tile, m, kq, part); break;
      }
#pragma unroll
      for (int q = 0; q < B::NQ; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[q][r] += (double)part[q][r];
    }
    __syncthreads();
  }
  double* out = partial + (int64_t)blockIdx.x * NP * NP;
  constexpr auto slots = std::make_integer_sequence<int, B::NQ>{};
  switch (wave) {
    case 0: gram_out<NB, 0, F64>(acc, out, NP, lane, slots); break;
    case 1: gram_out<NB, 1, F64>(acc, out, NP, lane, slots); break;
    case 2: gram_out<NB, 2, F64>(acc, out, NP, lane, slots); break;
    default: gram_out<NB, 3, F64>(acc, out, NP, lane, slots); break;
  }
}

// gram[i*NP + j] = sum of the workgroups' partial sums (upper-triangular blocks only), in a fixed order:
// eight threads per element each add every eighth workgroup's term in rising order, then the eight
// subtotals are added in rising order -- one thread per element walked all the partial matrices alone
// and took 0.16 ms for 512 of them.
// `accumulate`: the sum is added to what gram holds (rows that arrive in panels).
constexpr int kReduceSplit = 8;
__global__ __launch_bounds__(256) void gram_reduce_kernel(const double* __restrict__ partial, int nparts, int NP,
                                                          double* __restrict__ gram, int accumulate) {
  constexpr int kElems = 256 / kReduceSplit;
  __shared__ double sub[kReduceSplit][kElems];
  const int e = threadIdx.x % kElems, part = threadIdx.x / kElems;
  const int idx = blockIdx.x * kElems + e;
  const bool live = idx < NP * NP && ((idx % NP) >> 4) >= ((idx / NP) >> 4);
  double a = 0.0;
  if (live)
    for (int b = part; b < nparts; b += kReduceSplit) a += partial[(int64_t)b * NP * NP + idx];
  sub[part][e] = a;
  __syncthreads();
  if (part == 0 && idx < NP * NP) {
    double t = 0.0;
#pragma unroll
    for (int q = 0; q < kReduceSplit; ++q) t += sub[q][e];
    gram[idx] = accumulate ? gram[idx] + t : t;
  }
}

// Q[:, j] = sum_{a <= j} W[:, a] * rinv[a][j];  rinv is NP x NP row major, zero outside the
// upper triangle and outside n x n.  As an MFMA: D[m = j][n' = i] = sum_a A[m][a] B[a][n'] with
// A = rinv^T (kept in registers for the wave's two column blocks) and B = the staged tile.
// (W and Q carry no no-alias promise: Q may be W.)
//
// Column block jb needs the k-steps of rows 0 .. 16 (jb + 1) only (rinv is upper triangular): its cost is
// jb + 1.  A wave takes at most two blocks, chosen at compile time so that the four waves carry the same
// load: the four widest blocks go to waves 0..3 in falling order, the remaining NB - 4 narrow ones in
// rising order to the LAST waves (NB = 7: {6}, {5,0}, {4,1}, {3,2}, seven units each).  -1 = no block.
template <int NB>
__host__ __device__ constexpr int apply_block_of(int wave, int which) {
  if (NB <= 4) return (which == 0 && wave < NB) ? wave : -1;
  if (which == 0) return NB - 1 - wave;
  return wave - (8 - NB) >= 0 ? wave - (8 - NB) : -1;
}

constexpr int kApplyRowGroups = kTileRows / 16;

// The products of one staged tile for wave WV: every index is a compile-time constant, so the LDS reads
// of later k-steps are issued while the matrix cores work on earlier ones.
template <int NB, int WV>
__device__ __forceinline__ void apply_tile_products(const float* tile, const float (&afrag)[2][4 * NB], int m, int kq,
                                                    f32x4 (&acc)[2][kApplyRowGroups]) {
  constexpr int RG = kApplyRowGroups;
  constexpr int jb0 = apply_block_of<NB>(WV, 0), jb1 = apply_block_of<NB>(WV, 1);
  constexpr int ksteps = 4 * ((jb0 > jb1 ? jb0 : jb1) + 1);
#pragma unroll
  for (int kk = 0; kk < ksteps; ++kk) {
    float b[RG];
#pragma unroll
    for (int rg = 0; rg < RG; ++rg) b[rg] = tile[(4 * kk + kq) * kApplyStride + 16 * rg + m];
    if (kk < 4 * (jb0 + 1)) {
#pragma unroll
      for (int rg = 0; rg < RG; ++rg)
        acc[0][rg] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag[0][kk], b[rg], acc[0][rg], 0, 0, 0);
    }
    if (kk < 4 * (jb1 + 1)) {
#pragma unroll
      for (int rg = 0; rg < RG; ++rg)
        acc[1][rg] = __builtin_amdgcn_mfma_f32_16x16x4f32(afrag[1][kk], b[rg], acc[1][rg], 0, 0, 0);
    }
  }
}

// What apply_rinv_kernel does with a finished tile of Q.  The sums of a tile leave the matrix instruction as
// 16-lane runs of 64 bytes per column; written to memory like that the kernel reached 4.0 TB/s (the plain copy
// of this device: 5.3).  They are therefore first written to LDS as out[col][row] (the staged input tile is
// dead by then and gives its place), and leave in the shape the destination wants:
//   EMIT_F32   Q as fp32 (this one leaves straight from the registers: see the kernel)
//   EMIT_BF16  the same rounded to bfloat16 (nearest even)
//   EMIT_I8 / EMIT_I4  the block-absmax integer codes of twa_quantize, bit for bit the recipe of that call (every
//              step one correctly rounded binary32 operation): Q in fp32 is then never written at all.  A
//              quantisation block of 128 rows spans two tiles: the first one waits in a second LDS buffer.
enum { EMIT_F32 = 0, EMIT_BF16 = 1, EMIT_I8 = 2, EMIT_I4 = 3 };
constexpr int kOutStride = kTileRows + 4;     // floats; 4 columns apart = 16 banks apart: the 16-lane runs of two
                                              // column quads of a matrix-instruction result land on disjoint banks

struct EmitTarget {
  float* q;             // EMIT_F32: Q, stride ldq                 (may be W itself)
  uint8_t* codes;       // other modes: values / codes of the whole matrix, vector stride `ld` elements
  uint8_t* scales;      // EMIT_I8 / EMIT_I4: span-interleaved scales of the whole matrix
  int64_t ld;           // elements between vectors in q / codes
  int64_t row0;         // first row of this panel in the whole matrix (a multiple of kScaleSpan for the integer modes)
  int64_t rows_out;     // rows to produce, >= the panel's rows: those behind the panel's end are padding (zeros)
  int block_shift;      // log2(quantisation block)
  float gscale, inv_gscale;
};

__device__ __forceinline__ uint32_t bf16_rne(float x) {
  const uint32_t u = as_u32(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  const uint32_t keep = u >> 16, rem = u & 0xffffu;
  return keep + ((rem > 0x8000u || (rem == 0x8000u && (keep & 1u))) ? 1u : 0u);
}

// `nt` tiles of kTileRows rows (tile 0 in buf0, tile 1 in buf1, laid out [col][row] with stride kOutStride) starting at panel
// row i0 leave for memory.  EL rows per thread: 4, or 8 for the 4-bit codes (one dword of codes either way).
template <int EMIT>
__device__ __forceinline__ void emit_rows(const EmitTarget& T, int n, int NP, int64_t i0, int nt, const float* buf0,
                                          const float* buf1) {
  constexpr int EL = EMIT == EMIT_I4 ? 8 : 4;
  constexpr int PER_TILE = kTileRows / EL;                       // threads per column and tile
  const int per_col = PER_TILE * nt;
  const int total = NP * per_col;
  for (int idx = threadIdx.x; idx < (total + 255) / 256 * 256; idx += 256) {
    const int col = idx / per_col;
    const int rr = idx - col * per_col;                          // run of EL rows inside the group of tiles
    const int t = rr / PER_TILE;
    const int r = rr - t * PER_TILE;
    const bool inside = idx < total && col < n;
    float x[EL];
#pragma unroll
    for (int e = 0; e < EL; e += 4) {
      const float4 v = inside ? *reinterpret_cast<const float4*>((t ? buf1 : buf0) + col * kOutStride + EL * r + e)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
      x[e] = v.x; x[e + 1] = v.y; x[e + 2] = v.z; x[e + 3] = v.w;
    }
    const int64_t row = i0 + (int64_t)t * kTileRows + EL * r;    // first of this thread's rows, inside the panel
    const int64_t grow = T.row0 + row;                           // ... and in the whole matrix
    const bool live = inside && row < T.rows_out;
    if constexpr (EMIT == EMIT_F32) {
      if (live) {
        float* dst = T.q + (int64_t)col * T.ld + row;
        if (row + 4 <= T.rows_out) {
          *reinterpret_cast<float4*>(dst) = make_float4(x[0], x[1], x[2], x[3]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) if (row + e < T.rows_out) dst[e] = x[e];
        }
      }
    } else if constexpr (EMIT == EMIT_BF16) {
      if (live) {                                                // rows_out is a multiple of 4 here (ld is)
        const uint2 v = {bf16_rne(x[0]) | (bf16_rne(x[1]) << 16), bf16_rne(x[2]) | (bf16_rne(x[3]) << 16)};
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(T.codes) + (int64_t)col * T.ld + grow) = v;
      }
    } else {
      // the recipe of twa_quantize; the block's absmax over the block / EL consecutive threads that hold it
      constexpr float QMAX = EMIT == EMIT_I8 ? 127.0f : 7.0f;
      const int lanes_per_block = (1 << T.block_shift) / EL;
      float amax = 0.0f;
#pragma unroll
      for (int e = 0; e < EL; ++e) amax = fmaxf(amax, fabsf(x[e]));
#pragma unroll
      for (int m = 1; m < 32; m <<= 1)
        if (m < lanes_per_block) amax = fmaxf(amax, __shfl_xor(amax, m, kWave));
      const float scale = amax / QMAX;
      float eff = scale;
      uint16_t hbits = 0;
      if constexpr (EMIT == EMIT_I4) {
        const _Float16 h = (_Float16)(scale * T.inv_gscale);
        hbits = __builtin_bit_cast(uint16_t, h);
        eff = (float)h * T.gscale;
      }
      const bool nonzero = eff != 0.0f;
      const float inv = nonzero ? 1.0f / eff : 0.0f;
      uint32_t word = 0;
#pragma unroll
      for (int e = 0; e < EL; ++e) {
        float c = __builtin_rintf(x[e] * inv);
        c = fminf(fmaxf(c, -QMAX), QMAX);
        const int q = nonzero ? (int)c : 0;
        if constexpr (EMIT == EMIT_I8) word |= ((uint32_t)q & 0xffu) << (8 * e);
        else word |= ((uint32_t)(q + 8) & 0xfu) << (4 * e);
      }
      if (live) {
        constexpr int BITS = EMIT == EMIT_I8 ? 8 : 4;
        *reinterpret_cast<uint32_t*>(T.codes + ((((int64_t)col * T.ld + grow) * BITS) >> 3)) = word;
        if ((rr & (lanes_per_block - 1)) == 0) {
          const int gshift = kScaleSpanShift - T.block_shift;
          const int64_t b = grow >> T.block_shift;
          const int64_t at = ((((b >> gshift) * n + col)) << gshift) + (b & (((int64_t)1 << gshift) - 1));
          if constexpr (EMIT == EMIT_I8) reinterpret_cast<float*>(T.scales)[at] = scale;
          else reinterpret_cast<uint16_t*>(T.scales)[at] = hbits;
        }
      }
    }
  }
}

// GROUP = tiles that are emitted together: 2 where a quantisation block of 128 rows spans two tiles, else 1.
template <int NB, int EMIT, int GROUP>
__global__ __launch_bounds__(256, 2) void apply_rinv_kernel(const float* W, int64_t ldw, int64_t D, int n,
                                                            const float* __restrict__ rinv, EmitTarget T) {
  constexpr int NP = 16 * NB;
  constexpr int KK = 4 * NB;                    // k-steps of the widest block
  constexpr int RG = kApplyRowGroups;           // row groups per tile
  static_assert(kOutStride <= kApplyStride, "a finished tile takes the place of the staged one");
  __shared__ float tile[NP * kApplyStride];
  __shared__ float first[GROUP == 2 ? NP * kOutStride : 1];      // the first tile of a pair waits here
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, kq = lane >> 4;
  const int jbs[2] = {apply_block_of<NB>(wave, 0), apply_block_of<NB>(wave, 1)};

  float afrag[2][KK];
#pragma unroll
  for (int jbi = 0; jbi < 2; ++jbi) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int a = 4 * kk + kq, j = 16 * jbs[jbi] + m;
      afrag[jbi][kk] = jbs[jbi] >= 0 ? rinv[a * NP + j] : 0.0f;
    }
  }

  // groups of GROUP tiles are dealt to the workgroups; rows behind the panel's end (up to rows_out) are zeros
  const int64_t ngroups = (T.rows_out + GROUP * kTileRows - 1) / (GROUP * kTileRows);
  int64_t g0, g1;
  split_range(ngroups, (int)gridDim.x, (int)blockIdx.x, g0, g1);
  const int64_t c0 = g0 * GROUP, c1 = g1 * GROUP;
  float4 pre[kTileQuads];
  if (c0 < c1) fetch_tile(W, ldw, D, n, NP, c0 * kTileRows, pre);
  for (int64_t c = c0; c < c1; ++c) {
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
    switch (wave) {                                                 // uniform per wave
      case 0: apply_tile_products<NB, 0>(tile, afrag, m, kq, acc); break;
      case 1: apply_tile_products<NB, 1>(tile, afrag, m, kq, acc); break;
      case 2: apply_tile_products<NB, 2>(tile, afrag, m, kq, acc); break;
      default: apply_tile_products<NB, 3>(tile, afrag, m, kq, acc); break;
    }
    __syncthreads();      // every wave has read the staged tile: the finished one may take its place
    if constexpr (EMIT == EMIT_F32) {
      // fp32 leaves straight from the registers, 64 bytes per column and 16-lane run: taking it through LDS for
      // runs of 256 bytes was measured and is 5 % SLOWER (two more barriers per tile; 5.4 against 5.1 ms)
      const int64_t i0 = c * kTileRows;
#pragma unroll
      for (int jbi = 0; jbi < 2; ++jbi) {
        const int jb = jbs[jbi];
        if (jb >= 0) {
#pragma unroll
          for (int rg = 0; rg < RG; ++rg) {
            const int64_t row = i0 + 16 * rg + m;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int col = 16 * jb + mfma_row_f32(lane, r);
              if (col < n && row < T.rows_out) T.q[(int64_t)col * T.ld + row] = acc[jbi][rg][r];
            }
          }
        }
      }
      continue;
    }
    const bool waits = GROUP == 2 && ((c - c0) & 1) == 0;          // first tile of a pair
    float* out = waits ? first : tile;
#pragma unroll
    for (int jbi = 0; jbi < 2; ++jbi) {
      const int jb = jbs[jbi];
      if (jb >= 0) {
#pragma unroll
        for (int rg = 0; rg < RG; ++rg)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            out[(16 * jb + mfma_row_f32(lane, r)) * kOutStride + 16 * rg + m] = acc[jbi][rg][r];
      }
    }
    if (waits) continue;                                           // (the next store_tile only touches `tile`)
    __syncthreads();
    emit_rows<EMIT>(T, n, NP, (c + 1 - GROUP) * kTileRows, GROUP, GROUP == 2 ? first : tile, tile);
    __syncthreads();      // the staged tile's place is free again
  }
}

// ---- the n x n algebra of a pass on the device (n <= 128): no host round trip, nothing synchronises --------
// G = R^T R (R upper triangular, positive diagonal), X = R^-1, in fp64 by ONE workgroup with the whole matrix in
// LDS (129 x 128 doubles = 132 KB: gfx950 gives a workgroup up to 160 KB).  The operations and their order are
// those of the host routines of the synchronous path (right-looking elimination visits the terms of every entry
// in the same order k = 0, 1, .. as the host's dot products; products and sums are rounded separately, as the host
// compiler does without fused multiply-add), so both paths give the same bits.
//   upper triangle of A: G, then R in place          lower triangle: X^T (X[i][j], i < j, at A[j][i])
//   xd: the diagonal of X
// A pivot d <= tol * max diag(G) stops the factorisation: *status (if still 0) becomes 1 + the index of that
// checkpoint, and rinv is filled with NaN so that everything computed from it says so.
constexpr int kFactorStride = TWA_MAX_N + 1;
__global__ __launch_bounds__(256) void gram_factor_kernel(const double* __restrict__ gram, int n, int NP,
                                                          float* __restrict__ rinv, double* __restrict__ Rout,
                                                          int* __restrict__ status, double tol) {
#pragma clang fp contract(off)            // products and sums rounded separately, as in the host routines
  __shared__ double A[TWA_MAX_N * kFactorStride];
  __shared__ double xd[TWA_MAX_N];
  const int tid = threadIdx.x;
  for (int idx = tid; idx < n * n; idx += 256) {
    const int r = idx / n, c = idx - r * n;
    if (r <= c) A[r * kFactorStride + c] = gram[r * NP + c];
  }
  __syncthreads();
  double dmax = 0.0;
  for (int i = 0; i < n; ++i) dmax = fmax(dmax, A[i * kFactorStride + i]);
  int bad = 0;
  for (int j = 0; j < n; ++j) {
    const double d = A[j * kFactorStride + j];                 // every thread reads the same value: uniform branch
    if (!(d > tol * dmax)) { bad = j + 1; break; }
    const double rjj = sqrt(d);
    for (int i = j + 1 + tid; i < n; i += 256) A[j * kFactorStride + i] = A[j * kFactorStride + i] / rjj;
    __syncthreads();
    if (tid == 0) A[j * kFactorStride + j] = rjj;
    const int b = tid & (TWA_MAX_N - 1);                       // column of the trailing matrix, two threads per column
    if (b > j && b < n) {
      const double rjb = A[j * kFactorStride + b];
      for (int a = j + 1 + (tid >> 7); a <= b; a += 2)
        A[a * kFactorStride + b] = A[a * kFactorStride + b] - A[j * kFactorStride + a] * rjb;
    }
    __syncthreads();
  }
  if (bad) {
    if (tid == 0 && *status == 0) *status = bad;
    const float nan = __builtin_nanf("");
    for (int idx = tid; idx < NP * NP; idx += 256) rinv[idx] = nan;
    if (Rout)
      for (int idx = tid; idx < n * n; idx += 256) Rout[idx] = __builtin_nan("");
    return;
  }
  // X = R^-1, row by row from the bottom; thread j owns column j and reads only what it wrote itself
  if (tid < n) xd[tid] = 1.0 / A[tid * kFactorStride + tid];
  __syncthreads();
  if (tid < n) {
    const int j = tid;
    for (int i = j - 1; i >= 0; --i) {
      double v = 0.0;
      for (int k = i + 1; k <= j; ++k) {
        const double xkj = k == j ? xd[j] : A[j * kFactorStride + k];
        v = v + A[i * kFactorStride + k] * xkj;
      }
      A[j * kFactorStride + i] = -v / A[i * kFactorStride + i];
    }
  }
  __syncthreads();
  for (int idx = tid; idx < NP * NP; idx += 256) {
    const int r = idx / NP, c = idx - r * NP;
    double x = 0.0;
    if (r < n && c < n && r <= c) x = r == c ? xd[r] : A[c * kFactorStride + r];
    rinv[idx] = (float)x;
  }
  if (Rout)
    for (int idx = tid; idx < n * n; idx += 256) {
      const int r = idx / n, c = idx - r * n;
      Rout[idx] = r <= c ? A[r * kFactorStride + c] : 0.0;
    }
}

// T = R * Rtot (both n x n upper triangular, row major): W = Q1 Rtot and Q1 = P R give W = P (R Rtot).  One
// thread per entry, the terms added in the order of the host routine.
__global__ __launch_bounds__(256) void compose_upper_kernel(const double* __restrict__ R, const double* __restrict__ Rtot,
                                                            double* __restrict__ T, int n) {
#pragma clang fp contract(off)
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= n * n) return;
  const int i = idx / n, j = idx - i * n;
  double v = 0.0;
  if (i <= j)
    for (int k = i; k <= j; ++k) v = v + R[i * n + k] * Rtot[k * n + j];
  T[idx] = v;
}
__global__ __launch_bounds__(256) void copy_doubles_kernel(const double* __restrict__ src, double* __restrict__ dst, int count) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx < count) dst[idx] = src[idx];
}
__global__ void zero_status_kernel(int* p) { *p = 0; }

int launch_zero_status(int* status, hipStream_t st) {
  hipLaunchKernelGGL(zero_status_kernel, dim3(1), dim3(1), 0, st, status);
  return hip_check(hipGetLastError());
}

// Factor the reduced Gram matrix on the device: rinv <- R^-1 (NP x NP floats), Rout <- R (n x n doubles) if wanted.
int launch_gram_factor(const double* gram, int n, float* rinv, double* Rout, int* status, hipStream_t st) {
  const int NP = (n + 15) / 16 * 16;
  hipLaunchKernelGGL(gram_factor_kernel, dim3(1), dim3(256), 0, st, gram, n, NP, rinv, Rout, status, 1e-12);
  return hip_check(hipGetLastError());
}

// Rtot <- R * Rtot through the scratch T (n x n doubles).
int launch_compose_upper(const double* R, double* Rtot, double* T, int n, hipStream_t st) {
  const int blocks = (n * n + 255) / 256;
  hipLaunchKernelGGL(compose_upper_kernel, dim3(blocks), dim3(256), 0, st, R, Rtot, T, n);
  hipLaunchKernelGGL(copy_doubles_kernel, dim3(blocks), dim3(256), 0, st, T, Rtot, n * n);
  return hip_check(hipGetLastError());
}

// Zero the padding [D, ld) of every vector.
__global__ __launch_bounds__(256) void zero_padding_kernel(float* __restrict__ Q, int64_t D, int64_t ld) {
  const int j = blockIdx.y;
  for (int64_t i = D + threadIdx.x; i < ld; i += blockDim.x) Q[(int64_t)j * ld + i] = 0.0f;
}

// `orthonormal_input`: W is orthonormal already to ~1e-4 (the second pass of CholeskyQR2): fp32 matrix instructions.
int launch_gram(const float* W, int64_t D, int n, int64_t ldw, double* partial, int grid, double* gram,
                bool accumulate, bool orthonormal_input, hipStream_t st) {
  const int NP = (n + 15) / 16 * 16;
  switch (NP / 16) {
#define TWA_GRAM(NB_)                                                                                          \
  case NB_:                                                                                                    \
    if (orthonormal_input)                                                                                     \
      hipLaunchKernelGGL((gram_kernel<NB_, false>), dim3(grid), dim3(256), 0, st, W, D, n, ldw, partial);      \
    else                                                                                                       \
      hipLaunchKernelGGL((gram_kernel<NB_, true>), dim3(grid), dim3(256), 0, st, W, D, n, ldw, partial);       \
    break
    TWA_GRAM(1); TWA_GRAM(2); TWA_GRAM(3); TWA_GRAM(4); TWA_GRAM(5); TWA_GRAM(6); TWA_GRAM(7); TWA_GRAM(8);
#undef TWA_GRAM
    default: return TWA_ERR_SHAPE;
  }
  constexpr int kElems = 256 / kReduceSplit;
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((NP * NP + kElems - 1) / kElems), dim3(256), 0, st, partial, grid, NP,
                     gram, accumulate ? 1 : 0);
  return hip_check(hipGetLastError());
}

template <int EMIT, int GROUP>
static int launch_apply_emit(const float* W, int64_t ldw, int64_t rows, int n, const float* rinv_dev, const EmitTarget& T,
                             int grid, hipStream_t st) {
  const int NP = (n + 15) / 16 * 16;
  switch (NP / 16) {
#define TWA_APPLY(NB_) case NB_: hipLaunchKernelGGL((apply_rinv_kernel<NB_, EMIT, GROUP>), dim3(grid), dim3(256), 0, st, W, ldw, rows, n, rinv_dev, T); break
    TWA_APPLY(1); TWA_APPLY(2); TWA_APPLY(3); TWA_APPLY(4); TWA_APPLY(5); TWA_APPLY(6); TWA_APPLY(7); TWA_APPLY(8);
#undef TWA_APPLY
    default: return TWA_ERR_SHAPE;
  }
  return hip_check(hipGetLastError());
}

int launch_apply_rinv(const float* W, int64_t ldw, float* Q, int64_t ldq, int64_t D, int n, const float* rinv_dev,
                      int grid, bool zero_padding, hipStream_t st) {
  const EmitTarget T{Q, nullptr, nullptr, ldq, 0, D, 0, 1.0f, 1.0f};
  int rc = launch_apply_emit<EMIT_F32, 1>(W, ldw, D, n, rinv_dev, T, grid, st);
  if (rc != TWA_OK) return rc;
  if (zero_padding && ldq > D) hipLaunchKernelGGL(zero_padding_kernel, dim3(1, n), dim3(256), 0, st, Q, D, ldq);
  return hip_check(hipGetLastError());
}

// Q = W R^-1 stored straight in the form `out` describes (rows [row0, row0 + rows) of the whole matrix; with
// `last` the padding behind them, up to out.ld, is produced too: zeros, code 0, scale 0).
int launch_apply_rinv_store(const float* W, int64_t ldw, int64_t rows, int n, const float* rinv_dev, const twa_pmat& out,
                            int64_t row0, bool last, int grid, hipStream_t st) {
  int shift = 0;
  while ((1 << shift) < out.block) ++shift;
  const int64_t rows_out = last ? out.ld - row0 : rows;
  const float gs = out.dtype == TWA_I4 ? out.gscale : 1.0f;
  const EmitTarget T{static_cast<float*>(out.data), static_cast<uint8_t*>(out.data), static_cast<uint8_t*>(out.scales),
                     out.ld, row0, rows_out, shift, gs, 1.0f / gs};
  switch (out.dtype) {
    case TWA_F32: {
      EmitTarget F = T;
      F.q = static_cast<float*>(out.data) + row0;              // (EMIT_F32 addresses rows inside the panel)
      return launch_apply_emit<EMIT_F32, 1>(W, ldw, rows, n, rinv_dev, F, grid, st);
    }
    case TWA_BF16: return launch_apply_emit<EMIT_BF16, 1>(W, ldw, rows, n, rinv_dev, T, grid, st);
    case TWA_I8:
      return out.block == 128 ? launch_apply_emit<EMIT_I8, 2>(W, ldw, rows, n, rinv_dev, T, grid, st)
                              : launch_apply_emit<EMIT_I8, 1>(W, ldw, rows, n, rinv_dev, T, grid, st);
    case TWA_I4:
      return out.block == 128 ? launch_apply_emit<EMIT_I4, 2>(W, ldw, rows, n, rinv_dev, T, grid, st)
                              : launch_apply_emit<EMIT_I4, 1>(W, ldw, rows, n, rinv_dev, T, grid, st);
    default: return TWA_ERR_DTYPE;
  }
}

}  // namespace twa
