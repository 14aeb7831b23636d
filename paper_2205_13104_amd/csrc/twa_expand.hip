// g~ = P s ;  w <- w - lr * g~   (arXiv 2205.13104, Sec. 4.2, weight-space form of the update rule
// with lambda = 0; Alg. 1, "update weights").  A broadcast-expand bound by the second pass over
// the stored P:
//
//   * every workgroup owns the same number of consecutive D-tiles (the grid is sized so that the
//     division is exact up to the last workgroup); its 4 waves take neighbouring tiles, so the
//     workgroup reads and writes one contiguous window at a time;
//   * a lane owns VPL*EPV outputs and keeps their sums in registers while it walks over all n
//     basis vectors, U of them per loop trip (U*VPL 128-bit non-temporal loads in flight);
//   * s_j is wave-uniform (scalar loads); the block scale is folded into t = s_j * scale once per
//     (lane-vector, basis vector), then one convert + one FMA per stored element;
//   * the tile's slice of w is fetched at the START of the tile with fully coalesced loads, the
//     finished sums are transposed through a wave-private LDS buffer into the same coalesced
//     shape, and w (and optionally g~) is written with full-line stores (fused update);
//   * buffer descriptors give the ragged end of D and the column remainder for free.
#include "twa_device.h"
#include "twa_host.h"

namespace twa {

template <int DT> struct ExpandCfg;
template <> struct ExpandCfg<TWA_F32> { static constexpr int U = 8, VPL = 4; };
template <> struct ExpandCfg<TWA_BF16> { static constexpr int U = 8, VPL = 2; };
template <> struct ExpandCfg<TWA_I8> { static constexpr int U = 4, VPL = 2; };
template <> struct ExpandCfg<TWA_I4> { static constexpr int U = 4, VPL = 1; };

int expand_tile_elems(int dtype) {
  switch (dtype) {
    case TWA_F32: return kWave * ExpandCfg<TWA_F32>::VPL * Store<TWA_F32>::kEPV;
    case TWA_BF16: return kWave * ExpandCfg<TWA_BF16>::VPL * Store<TWA_BF16>::kEPV;
    case TWA_I8: return kWave * ExpandCfg<TWA_I8>::VPL * Store<TWA_I8>::kEPV;
    default: return kWave * ExpandCfg<TWA_I4>::VPL * Store<TWA_I4>::kEPV;
  }
}

template <int DT>
__global__ __launch_bounds__(256) void expand_update_kernel(PView P, const float* __restrict__ s,
                                                            float* __restrict__ w, float lr,
                                                            float* __restrict__ g_tilde, int tiles_per_wg) {
  using S = Store<DT>;
  constexpr int EPV = S::kEPV;
  constexpr int U = ExpandCfg<DT>::U;
  constexpr int VPL = ExpandCfg<DT>::VPL;
  constexpr int TILE = kWave * VPL * EPV;
  constexpr int VEC = kWave * EPV;               // elements one wave-vector covers
  constexpr int ROW = EPV + 4;                   // padded LDS row of one lane (bank-conflict free)
  static_assert(!S::kScaled || TILE == kScaleSpan, "integer formats: one tile = one scale span");
  __shared__ float tbuf[4][kWave * ROW];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  const int64_t D = P.D;
  const int n = P.n;
  const int64_t ntiles = (D + TILE - 1) / TILE;
  const int64_t wg_first = (int64_t)blockIdx.x * tiles_per_wg;
  int64_t wg_end = wg_first + tiles_per_wg;
  if (wg_end > ntiles) wg_end = ntiles;

  // bytes of one stored vector, rounded up to whole dwords: the range check drops a dword that
  // is only partly inside, and the tail bytes are padding of the same vector (ld >= D, ld % 128 == 0)
  const uint32_t col_bytes = (uint32_t)((((D * S::kBitsPerElem + 7) >> 3) + 3) & ~(int64_t)3);
  const int64_t ld_bytes = (P.ld * S::kBitsPerElem) >> 3;
  const int gshift = kScaleSpanShift - P.block_shift;            // log2(scales per span and vector)
  const uint32_t span_scale_bytes = S::kScaled ? ((uint32_t)n << gshift) * (uint32_t)S::kScaleBytes : 0u;
  const uint32_t w_bytes = (uint32_t)(D * 4);
  const rsrc_t rw = make_rsrc(w, w_bytes);
  const rsrc_t rgt = make_rsrc(g_tilde, g_tilde ? w_bytes : 0u);
  float* tb = tbuf[wave];

  for (int64_t t = wg_first + wave; t < wg_end; t += 4) {
    const int64_t e0 = t * TILE;

    // ---- this tile's slice of w, coalesced: lane l holds floats (q*64 + l)*4 .. +3 of each vector
    u32x4 wv[VPL][EPV / 4];
#pragma unroll
    for (int v = 0; v < VPL; ++v)
#pragma unroll
      for (int q = 0; q < EPV / 4; ++q)
        wv[v][q] = ld128(rw, ((uint32_t)e0 + (uint32_t)(v * VEC + (q * kWave + lane) * 4)) * 4u);

    float acc[VPL][EPV];
    float tsum[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      tsum[v] = 0.0f;
#pragma unroll
      for (int e = 0; e < EPV; ++e) acc[v][e] = 0.0f;
    }
    rsrc_t rs = rw;
    if constexpr (S::kScaled)
      rs = make_rsrc(P.scales + t * (int64_t)span_scale_bytes, span_scale_bytes);

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
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          const uint32_t loc = (uint32_t)(v * kWave + lane) * EPV;     // element inside the tile
          raw[u][v] = ld128_stream(rc, (uint32_t)((((uint64_t)e0 + loc) * S::kBitsPerElem) >> 3));
          if constexpr (S::kScaled) {
            // an unused column slot reads far outside the span's range and gets 0
            const uint32_t soff = valid ? (((uint32_t)col << gshift) + (loc >> P.block_shift)) * (uint32_t)S::kScaleBytes
                                        : 0x7fffff00u;
            tj[u][v] = sj * load_scale<DT>(rs, soff, P.gscale);
          } else {
            tj[u][v] = sj;
          }
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

    // ---- epilogue: transpose the sums into the coalesced shape, update w, store --------------
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      if constexpr (DT == TWA_I4) {
        // even nibbles were decoded as q+8, odd nibbles as 16*(q+8)
#pragma unroll
        for (int e = 0; e < EPV; ++e)
          acc[v][e] = ((e & 1) ? acc[v][e] * 0.0625f : acc[v][e]) - 8.0f * tsum[v];
      }
      if constexpr (EPV > 4) {
#pragma unroll
        for (int q = 0; q < EPV / 4; ++q)
          *reinterpret_cast<float4*>(tb + lane * ROW + 4 * q) =
              make_float4(acc[v][4 * q], acc[v][4 * q + 1], acc[v][4 * q + 2], acc[v][4 * q + 3]);
        wave_lds_sync();
      }
#pragma unroll
      for (int q = 0; q < EPV / 4; ++q) {
        const uint32_t m = (uint32_t)(q * kWave + lane) * 4u;       // element inside the wave-vector
        float4 gt;
        if constexpr (EPV > 4)
          gt = *reinterpret_cast<const float4*>(tb + (m / EPV) * ROW + (m % EPV));
        else
          gt = make_float4(acc[v][0], acc[v][1], acc[v][2], acc[v][3]);
        const uint32_t el = (uint32_t)e0 + (uint32_t)(v * VEC) + m;
        const uint32_t off = el * 4u;
        const u32x4 gv = {as_u32(gt.x), as_u32(gt.y), as_u32(gt.z), as_u32(gt.w)};
        u32x4 nw;
        nw[0] = as_u32(__builtin_fmaf(-lr, gt.x, as_f32(wv[v][q][0])));
        nw[1] = as_u32(__builtin_fmaf(-lr, gt.y, as_f32(wv[v][q][1])));
        nw[2] = as_u32(__builtin_fmaf(-lr, gt.z, as_f32(wv[v][q][2])));
        nw[3] = as_u32(__builtin_fmaf(-lr, gt.w, as_f32(wv[v][q][3])));
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
      if constexpr (EPV > 4) wave_lds_sync();
    }
  }
}

int launch_expand_update(const PView& P, int dtype, const float* s, float* w, float lr, float* g_tilde, int max_grid,
                         hipStream_t st) {
  const int tile = expand_tile_elems(dtype);
  const int64_t ntiles = (P.D + tile - 1) / tile;
  int64_t tiles_per_wg = (ntiles + max_grid - 1) / max_grid;
  tiles_per_wg = (tiles_per_wg + 3) / 4 * 4;                      // whole rounds of the 4 waves
  const int grid = (int)((ntiles + tiles_per_wg - 1) / tiles_per_wg);
  const int tpw = (int)tiles_per_wg;
  switch (dtype) {
    case TWA_F32:
      hipLaunchKernelGGL((expand_update_kernel<TWA_F32>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, tpw);
      break;
    case TWA_BF16:
      hipLaunchKernelGGL((expand_update_kernel<TWA_BF16>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, tpw);
      break;
    case TWA_I8:
      hipLaunchKernelGGL((expand_update_kernel<TWA_I8>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, tpw);
      break;
    case TWA_I4:
      hipLaunchKernelGGL((expand_update_kernel<TWA_I4>), dim3(grid), dim3(256), 0, st, P, s, w, lr, g_tilde, tpw);
      break;
    default:
      return TWA_ERR_DTYPE;
  }
  return hip_check(hipGetLastError());
}

}  // namespace twa
