// g~ = P s ;  w <- w - lr * g~   (arXiv 2205.13104, Sec. 4.2, weight-space form of the update rule
// with lambda = 0; Alg. 1, "update weights").  A broadcast-expand bound by the second pass over
// the stored P:
//
//   * a persistent grid of independent waves; wave v owns a contiguous balanced range of D-tiles;
//   * a lane owns VPL*EPV consecutive-by-vector outputs and keeps their sums in registers while
//     it walks over all n basis vectors, U of them per loop trip (U*VPL 128-bit loads in flight);
//   * s_j is wave-uniform (scalar loads); the block scale is folded into t = s_j * scale once per
//     (lane-vector, basis vector), then one convert + one FMA per stored element;
//   * w is read, updated and written in the epilogue of the tile (fused update), g~ optionally stored;
//   * buffer descriptors give the ragged end of D and the column remainder for free;
//   * optional descending tile order, so that the tail of P left in the memory-side cache by the
//     projection pass is consumed first.
#include "twa_device.h"
#include "twa_host.h"

namespace twa {

template <int DT, int U, int VPL>
__global__ __launch_bounds__(256) void expand_update_kernel(PView P, const float* __restrict__ s,
                                                            float* __restrict__ w, float lr,
                                                            float* __restrict__ g_tilde, int reverse) {
  using S = Store<DT>;
  constexpr int EPV = S::kEPV;
  constexpr int TILE = kWave * VPL * EPV;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nwaves = (int)gridDim.x * 4;
  const int gw = (int)blockIdx.x * 4 + wave;

  const int64_t D = P.D;
  const int n = P.n;
  const int64_t ntiles = (D + TILE - 1) / TILE;
  int64_t t0, t1;
  split_range(ntiles, nwaves, gw, t0, t1);

  // bytes of one stored vector, rounded up to whole dwords: the range check drops a dword that
  // is only partly inside, and the tail bytes are padding of the same vector (ld >= D, ld % 128 == 0)
  const uint32_t col_bytes = (uint32_t)((((D * S::kBitsPerElem + 7) >> 3) + 3) & ~(int64_t)3);
  const int64_t ld_bytes = (P.ld * S::kBitsPerElem) >> 3;
  const uint32_t nblk_valid = S::kScaled ? (uint32_t)((D + ((int64_t)1 << P.block_shift) - 1) >> P.block_shift) : 0u;
  const int64_t nblk_ld = S::kScaled ? (P.ld >> P.block_shift) : 0;
  const uint32_t w_bytes = (uint32_t)(D * 4);
  const rsrc_t rw = make_rsrc(w, w_bytes);
  const rsrc_t rgt = make_rsrc(g_tilde, g_tilde ? w_bytes : 0u);

  for (int64_t tt = t0; tt < t1; ++tt) {
    const int64_t t = reverse ? (t1 - 1 - (tt - t0)) : tt;
    const int64_t e0 = t * TILE;

    float acc[VPL][EPV];
    float tsum[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      tsum[v] = 0.0f;
#pragma unroll
      for (int e = 0; e < EPV; ++e) acc[v][e] = 0.0f;
    }

    for (int j0 = 0; j0 < n; j0 += U) {
      u32x4 raw[U][VPL];
      float tj[U][VPL];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = j0 + u;
        const bool valid = j < n;
        const int col = valid ? j : 0;
        const float sj = valid ? s[col] : 0.0f;
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
            tj[u][v] = sj * load_scale<DT>(rs, (elem >> P.block_shift) * (uint32_t)S::kScaleBytes, P.gscale);
          else
            tj[u][v] = sj;
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          float x[EPV];
          decode<DT>(raw[u][v], x);
          if constexpr (DT == TWA_I4) tsum[v] += tj[u][v];
#pragma unroll
          for (int e = 0; e < EPV; ++e) acc[v][e] = __builtin_fmaf(x[e], tj[u][v], acc[v][e]);
        }
      }
    }

    // ---- epilogue: g~ for this lane's elements, fused weight update --------------------------
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const uint32_t elem = (uint32_t)e0 + (uint32_t)(v * kWave + lane) * EPV;
      if constexpr (DT == TWA_I4) {
        // even nibbles decoded as q+8, odd nibbles as 16*(q+8)
#pragma unroll
        for (int e = 0; e < EPV; ++e)
          acc[v][e] = ((e & 1) ? acc[v][e] * 0.0625f : acc[v][e]) - 8.0f * tsum[v];
      }
#pragma unroll
      for (int q = 0; q < EPV / 4; ++q) {
        const uint32_t el = elem + 4u * q;
        const uint32_t off = el * 4u;
        const u32x4 wv = ld128(rw, off);
        u32x4 nw, gv;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float gt = acc[v][4 * q + r];
          gv[r] = as_u32(gt);
          nw[r] = as_u32(__builtin_fmaf(-lr, gt, as_f32(wv[r])));
        }
        if ((int64_t)el + 4 <= D) {
          st128(rw, off, nw);
          st128(rgt, off, gv);          // empty descriptor when g~ is not wanted: dropped
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if ((int64_t)el + r < D) {
              st32(rw, off + 4u * r, nw[r]);
              st32(rgt, off + 4u * r, gv[r]);
            }
        }
      }
    }
  }
}

int launch_expand_update(const PView& P, int dtype, const float* s, float* w, float lr, float* g_tilde, int grid,
                         bool reverse, hipStream_t st) {
  const int rev = reverse ? 1 : 0;
  switch (dtype) {
    case TWA_F32:
      hipLaunchKernelGGL((expand_update_kernel<TWA_F32, 8, 2>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, rev);
      break;
    case TWA_BF16:
      hipLaunchKernelGGL((expand_update_kernel<TWA_BF16, 8, 2>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, rev);
      break;
    case TWA_I8:
      hipLaunchKernelGGL((expand_update_kernel<TWA_I8, 4, 2>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, rev);
      break;
    case TWA_I4:
      hipLaunchKernelGGL((expand_update_kernel<TWA_I4, 4, 1>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, rev);
      break;
    default:
      return TWA_ERR_DTYPE;
  }
  return hip_check(hipGetLastError());
}

}  // namespace twa
