// s = P^T g  (arXiv 2205.13104, Sec. 4.2: the gradient w.r.t. the averaging coefficients is the
// model gradient projected on the basis).  A tall-skinny reduction over D that is bound by the
// one pass over the stored P, so the kernel is a pure HBM stream:
//
//   * a persistent grid; workgroup b owns a contiguous, balanced range of D-tiles, so every
//     workgroup streams the same number of bytes (+-1 tile) and they all finish together;
//   * the 4 waves of a workgroup share the tile (same slice of g, kept in registers) and split
//     the n basis vectors between them, so a lane keeps <= 32 running sums in registers with
//     compile-time indices;
//   * every lane fetches 128 bits per load, a wave covers 1 KB contiguous of one basis vector;
//     int8 / int4 / bf16 are decoded in registers, the block scale is applied once per
//     (lane-vector, basis vector), never per element;
//   * all loads go through buffer descriptors: the ragged end of D and unused column slots
//     read zeros without memory traffic and without branches in the steady state;
//   * one cross-lane reduction per wave at the very end, per-workgroup partial sums in the
//     workspace, and a second tiny kernel adds them in a fixed order (fp64) -> deterministic.
#include "twa_device.h"
#include "twa_host.h"

namespace twa {

// KB = gradients handled together (1 or TWA_MAX_K slots), U = column slots per chunk,
// NCH = chunks, so a wave owns up to U*NCH basis vectors; VPL = 128-bit vectors per lane per
// basis vector and tile.
template <int DT, int KB, int U, int NCH, int VPL>
__global__ __launch_bounds__(256) void project_kernel(PView P, const float* __restrict__ g, int64_t ldg,
                                                      int kvalid, float* __restrict__ partial, int cpw) {
  using S = Store<DT>;
  constexpr int EPV = S::kEPV;
  constexpr int TILE = kWave * VPL * EPV;
  constexpr int SLOTS = U * NCH;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  const int64_t D = P.D;
  const int64_t ntiles = (D + TILE - 1) / TILE;
  int64_t t0, t1;
  split_range(ntiles, (int)gridDim.x, (int)blockIdx.x, t0, t1);

  const int c0 = wave * cpw;
  int ncol = P.n - c0;
  ncol = ncol < 0 ? 0 : (ncol > cpw ? cpw : ncol);

  // bytes of one stored vector, rounded up to whole dwords: the range check drops a dword that
  // is only partly inside, and the tail bytes are padding of the same vector (ld >= D, ld % 128 == 0)
  const uint32_t col_bytes = (uint32_t)((((D * S::kBitsPerElem + 7) >> 3) + 3) & ~(int64_t)3);
  const int64_t ld_bytes = (P.ld * S::kBitsPerElem) >> 3;
  const uint32_t nblk_valid = S::kScaled ? (uint32_t)((D + ((int64_t)1 << P.block_shift) - 1) >> P.block_shift) : 0u;
  const int64_t nblk_ld = S::kScaled ? (P.ld >> P.block_shift) : 0;
  const uint32_t g_bytes = (uint32_t)(D * 4);

  float acc[SLOTS][KB];
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl)
#pragma unroll
    for (int c = 0; c < KB; ++c) acc[sl][c] = 0.0f;

  for (int64_t t = t0; t < t1; ++t) {
    const int64_t e0 = t * TILE;
    const bool ragged = (e0 + TILE > D);   // uniform: only the last tile of all

    // ---- this lane's slice of the gradient(s) ------------------------------------------
    float gs[KB][VPL][EPV];
    float gcorr[KB][VPL];
#pragma unroll
    for (int c = 0; c < KB; ++c) {
      const rsrc_t rg = make_rsrc(g + (int64_t)c * ldg, c < kvalid ? g_bytes : 0u);
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        const uint32_t elem = (uint32_t)e0 + (uint32_t)(v * kWave + lane) * EPV;
#pragma unroll
        for (int q = 0; q < EPV / 4; ++q) {
          const u32x4 x = ld128(rg, (elem + 4u * q) * 4u);
#pragma unroll
          for (int r = 0; r < 4; ++r) gs[c][v][4 * q + r] = as_f32(x[r]);
        }
        if (ragged) {
#pragma unroll
          for (int e = 0; e < EPV; ++e)
            if ((int64_t)elem + e >= D) gs[c][v][e] = 0.0f;
        }
        if constexpr (DT == TWA_I4) {
          float sum = 0.0f;
#pragma unroll
          for (int e = 0; e < EPV; ++e) sum += gs[c][v][e];
          gcorr[c][v] = -8.0f * sum;                       // codes are stored as q+8
#pragma unroll
          for (int e = 1; e < EPV; e += 2) gs[c][v][e] *= 0.0625f;   // odd nibbles decode as 16*(q+8)
        } else {
          gcorr[c][v] = 0.0f;
        }
      }
    }

    // ---- stream this wave's basis vectors over the tile ----------------------------------
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      u32x4 raw[U][VPL];
      float sc[U][VPL];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int slot = ch * U + u;
        const bool valid = slot < ncol;
        const int col = valid ? c0 + slot : 0;
        const rsrc_t rc = make_rsrc(P.data + (int64_t)col * ld_bytes, valid ? col_bytes : 0u);
        rsrc_t rs = rc;
        if constexpr (S::kScaled)
          rs = make_rsrc(P.scales + (int64_t)col * nblk_ld * S::kScaleBytes,
                         valid ? nblk_valid * (uint32_t)S::kScaleBytes : 0u);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          const uint32_t elem = (uint32_t)e0 + (uint32_t)(v * kWave + lane) * EPV;
          raw[u][v] = ld128_stream(rc, (uint32_t)(((uint64_t)elem * S::kBitsPerElem) >> 3));
          if constexpr (S::kScaled)
            sc[u][v] = load_scale<DT>(rs, (elem >> P.block_shift) * (uint32_t)S::kScaleBytes, P.gscale);
          else
            sc[u][v] = 1.0f;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int slot = ch * U + u;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          float x[EPV];
          decode<DT>(raw[u][v], x);
#pragma unroll
          for (int c = 0; c < KB; ++c) {
            if constexpr (S::kScaled) {
              float d = gcorr[c][v];
#pragma unroll
              for (int e = 0; e < EPV; ++e) d = __builtin_fmaf(x[e], gs[c][v][e], d);
              acc[slot][c] = __builtin_fmaf(d, sc[u][v], acc[slot][c]);
            } else {
              float d = acc[slot][c];
#pragma unroll
              for (int e = 0; e < EPV; ++e) d = __builtin_fmaf(x[e], gs[c][v][e], d);
              acc[slot][c] = d;
            }
          }
        }
      }
    }
  }

  // ---- one reduction over the wave's lanes, then the per-workgroup partial sums -----------
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl) {
#pragma unroll
    for (int c = 0; c < KB; ++c) {
      const float tot = wave_sum(acc[sl][c]);
      if (lane == 0 && sl < ncol && c < kvalid)
        partial[((int64_t)blockIdx.x * kvalid + c) * P.n + c0 + sl] = tot;
    }
  }
}

// s[c*n + j] = sum over workgroups, in workgroup order, accumulated in fp64.
__global__ __launch_bounds__(64) void project_reduce_kernel(const float* __restrict__ partial, int nparts, int kn,
                                                            float* __restrict__ s) {
  const int idx = blockIdx.x;           // c*n + j
  const int lane = threadIdx.x;
  double a = 0.0;
  for (int b = lane; b < nparts; b += kWave) a += (double)partial[(int64_t)b * kn + idx];
  a = wave_sum(a);
  if (lane == 0) s[idx] = (float)a;
}

template <int DT, int KB, int VPL>
static int launch_project_dt(const PView& P, const float* g, int64_t ldg, int kvalid, float* partial, int grid,
                             hipStream_t st) {
  const int cpw = (P.n + 3) / 4;
  // chunks of 4 column slots; 25 columns per wave (n = 97..100) divide exactly into 5 chunks of 5
#define TWA_LAUNCH(U_, NCH_)                                                                         \
  hipLaunchKernelGGL((project_kernel<DT, KB, U_, NCH_, VPL>), dim3(grid), dim3(256), 0, st, P, g, ldg, \
                     kvalid, partial, cpw)
  if constexpr (KB > 1) {
    // the fused multi-gradient kernel is only used (and only built) for n <= 32
    if (cpw <= 4) TWA_LAUNCH(4, 1); else TWA_LAUNCH(4, 2);
  } else {
    if (cpw == 25) {
      TWA_LAUNCH(5, 5);
    } else {
      switch ((cpw + 3) / 4) {
        case 1: TWA_LAUNCH(4, 1); break;
        case 2: TWA_LAUNCH(4, 2); break;
        case 3: TWA_LAUNCH(4, 3); break;
        case 4: TWA_LAUNCH(4, 4); break;
        case 5: TWA_LAUNCH(4, 5); break;
        case 6: TWA_LAUNCH(4, 6); break;
        case 7: TWA_LAUNCH(4, 7); break;
        default: TWA_LAUNCH(4, 8); break;
      }
    }
  }
#undef TWA_LAUNCH
  return hip_check(hipGetLastError());
}

int project_tile_elems(int dtype) {
  switch (dtype) {
    case TWA_F32: return kWave * 4 * Store<TWA_F32>::kEPV;
    case TWA_BF16: return kWave * 2 * Store<TWA_BF16>::kEPV;
    case TWA_I8: return kWave * 2 * Store<TWA_I8>::kEPV;
    default: return kWave * 1 * Store<TWA_I4>::kEPV;
  }
}

// k == 1 path.  `partial` holds grid*n floats.
int launch_project(const PView& P, int dtype, const float* g, float* s, float* partial, int grid, hipStream_t st) {
  int rc;
  switch (dtype) {
    case TWA_F32: rc = launch_project_dt<TWA_F32, 1, 4>(P, g, 0, 1, partial, grid, st); break;
    case TWA_BF16: rc = launch_project_dt<TWA_BF16, 1, 2>(P, g, 0, 1, partial, grid, st); break;
    case TWA_I8: rc = launch_project_dt<TWA_I8, 1, 2>(P, g, 0, 1, partial, grid, st); break;
    case TWA_I4: rc = launch_project_dt<TWA_I4, 1, 1>(P, g, 0, 1, partial, grid, st); break;
    default: return TWA_ERR_DTYPE;
  }
  if (rc != TWA_OK) return rc;
  hipLaunchKernelGGL(project_reduce_kernel, dim3(P.n), dim3(kWave), 0, st, partial, grid, P.n, s);
  return hip_check(hipGetLastError());
}

// k > 1 gradients.  Up to 32 basis vectors (and not int4, whose 32-element vectors leave no
// registers for k gradient slices): one pass over P serves all k gradients -- each lane keeps k
// slices of G and k running sums per column slot.  Otherwise the gradients are projected one
// launch at a time.
template <int DT>
static int launch_project_batched_dt(const PView& P, const float* g, int64_t ldg, int k, float* s, float* partial,
                                     int grid, hipStream_t st) {
  if constexpr (DT != TWA_I4) {
    if (P.n <= 32) {
      int rc = launch_project_dt<DT, TWA_MAX_K, 1>(P, g, ldg, k, partial, grid, st);
      if (rc != TWA_OK) return rc;
      hipLaunchKernelGGL(project_reduce_kernel, dim3(P.n * k), dim3(kWave), 0, st, partial, grid, P.n * k, s);
      return hip_check(hipGetLastError());
    }
  }
  for (int c = 0; c < k; ++c) {
    int rc = launch_project(P, DT, g + (int64_t)c * ldg, s + (int64_t)c * P.n, partial, grid, st);
    if (rc != TWA_OK) return rc;
  }
  return TWA_OK;
}

int launch_project_batched(const PView& P, int dtype, const float* g, int64_t ldg, int k, float* s, float* partial,
                           int grid, hipStream_t st) {
  switch (dtype) {
    case TWA_F32: return launch_project_batched_dt<TWA_F32>(P, g, ldg, k, s, partial, grid, st);
    case TWA_BF16: return launch_project_batched_dt<TWA_BF16>(P, g, ldg, k, s, partial, grid, st);
    case TWA_I8: return launch_project_batched_dt<TWA_I8>(P, g, ldg, k, s, partial, grid, st);
    case TWA_I4: return launch_project_batched_dt<TWA_I4>(P, g, ldg, k, s, partial, grid, st);
    default: return TWA_ERR_DTYPE;
  }
}

}  // namespace twa
