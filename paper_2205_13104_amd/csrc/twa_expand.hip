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
//   * the finished sums are transposed through a wave-private LDS buffer into a fully coalesced
//     shape, w is read, updated with one FMA per element and written with full-line stores
//     (fused update); g~ is stored through a descriptor that is empty when it is not wanted;
//   * buffer descriptors give the ragged end of D and the column remainder for free.
//
// Writing w is the expensive part: on MI355X a thin stream of writes mixed into a saturating read
// stream costs several times its share of the bytes (102 MB of writes spread over the kernel
// cost as much as ~600 MB of reads), whereas the same bytes written in one burst when the reads
// are over cost about what their size suggests.  The kernel therefore keeps the finished sums
// of its LAST `HOLD` rounds of tiles in registers and writes them all at the very end; only
// earlier rounds (if the matrix is so long that a wave owns more tiles than it can hold) are
// written as they complete.  One more round is held in LDS.
#include "twa_device.h"
#include "twa_host.h"

namespace twa {

template <int DT, int U, int VPL, bool LAYERED>
struct Expander {
  using S = Store<DT>;
  static constexpr int EPV = S::kEPV;
  static constexpr int TILE = kWave * VPL * EPV;
  static constexpr int VEC = kWave * EPV;               // elements one wave-vector covers
  static constexpr int ROW = EPV + 4;                   // padded LDS row of one lane (conflict free)
  static constexpr int SPANS = TILE > kScaleSpan ? TILE / kScaleSpan : 1;
  static_assert(kScaleSpan % TILE == 0 || TILE % kScaleSpan == 0, "tiles and scale spans nest");
  static_assert(kLayerAlign % kScaleSpan == 0, "per-layer tiles keep the alignment of the scale spans");

  const PView& P;
  int lane;
  uint32_t col_bytes;
  int64_t ld_bytes;
  int gshift;
  uint32_t span_scale_bytes;
  rsrc_t rw, rgt;
  rsrc_t rw_in;                                         // where the old weights are read (normally = rw)
  bool out_of_place;                                    // ... and whether that is another buffer
  float lr;
  float* tb;                                            // this wave's LDS transpose buffer

  // sums of tile e0 over all basis vectors with the coefficients sv[0..n) (for I4 the bias / nibble
  // corrections are applied at the end)
  // Min-max formats (Sec. 4.6): mm_a scales every coefficient, and mm_b * sum_j s_j is added at the end
  // (mm_b = b_l + bias * a_l for codes stored relative to `bias`).
  __device__ __forceinline__ void accumulate(int64_t e0, float (&acc)[VPL][EPV], const float* __restrict__ sv,
                                             float mm_a = 1.0f, float mm_b = 0.0f) const {
    const int n = P.n;
    float ssum = 0.0f;
    float tsum[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      tsum[v] = 0.0f;
#pragma unroll
      for (int e = 0; e < EPV; ++e) acc[v][e] = 0.0f;
    }
    rsrc_t rs = rw;
    if constexpr (S::kScaled)      // (per-layer tiles start on the same grid as the scale spans)
      rs = make_rsrc(P.scales + (e0 >> kScaleSpanShift) * (int64_t)span_scale_bytes, SPANS * span_scale_bytes);
    const uint32_t in_span = (uint32_t)e0 & (uint32_t)(kScaleSpan - 1);   // tile offset inside its first span

    for (int j0 = 0; j0 < n; j0 += U) {
      u32x4 raw[U][VPL];
      float tj[U][VPL];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = j0 + u;
        const bool valid = j < n;
        const int col = valid ? j : 0;
        float sj = valid ? sv[col] : 0.0f;
        if constexpr (kMinMax<DT>) {
          ssum += sj;
          sj *= mm_a;
        }
        const rsrc_t rc = make_rsrc(P.data + (int64_t)col * ld_bytes, valid ? col_bytes : 0u);
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          const uint32_t loc = (uint32_t)(v * kWave + lane) * EPV;     // element inside the tile
          raw[u][v] = ld128_stream(rc, (uint32_t)((((uint64_t)e0 + loc) * S::kBitsPerElem) >> 3));
          if constexpr (S::kScaled) {
            // scale index inside the tile's run of spans: [span][vector][block in span];
            // an unused column slot reads far outside the range and gets 0
            const uint32_t pos = in_span + loc;
            const uint32_t soff =
                valid ? ((((pos >> kScaleSpanShift) * (uint32_t)n + (uint32_t)col) << gshift) +
                         ((pos & (uint32_t)(kScaleSpan - 1)) >> P.block_shift)) * (uint32_t)S::kScaleBytes
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
    if constexpr (DT == TWA_I4) {
      // even nibbles were decoded as q+8, odd nibbles as 16*(q+8)
#pragma unroll
      for (int v = 0; v < VPL; ++v)
#pragma unroll
        for (int e = 0; e < EPV; ++e)
          acc[v][e] = ((e & 1) ? acc[v][e] * 0.0625f : acc[v][e]) - 8.0f * tsum[v];
    }
    if constexpr (kMinMax<DT>) {
      const float add = mm_b * ssum;
#pragma unroll
      for (int v = 0; v < VPL; ++v)
#pragma unroll
        for (int e = 0; e < EPV; ++e)
          acc[v][e] = ((kNibbles<DT> && (e & 1)) ? acc[v][e] * 0.0625f : acc[v][e]) + add;   // odd nibbles: 16*code
    }
  }

  // coalesced position of this lane's q-th 128-bit piece of wave-vector v: floats (q*64 + lane)*4 ..
  __device__ __forceinline__ uint32_t piece(int64_t e0, int v, int q) const {
    return (uint32_t)e0 + (uint32_t)(v * VEC + (q * kWave + lane) * 4);
  }

  __device__ __forceinline__ void load_w(int64_t e0, u32x4 (&wv)[VPL][EPV / 4]) const {
#pragma unroll
    for (int v = 0; v < VPL; ++v)
#pragma unroll
      for (int q = 0; q < EPV / 4; ++q) wv[v][q] = ld128(rw_in, piece(e0, v, q) * 4u);
  }

  // lane's EPV sums of one wave-vector -> its padded row of an LDS buffer of kWave*ROW floats
  __device__ __forceinline__ void rows_to_lds(const float (&a)[EPV], float* buf) const {
#pragma unroll
    for (int q = 0; q < EPV / 4; ++q)
      *reinterpret_cast<float4*>(buf + lane * ROW + 4 * q) = make_float4(a[4 * q], a[4 * q + 1], a[4 * q + 2], a[4 * q + 3]);
  }

  // q-th coalesced 128-bit piece of wave-vector v: w <- w - lr * g~, store w (and g~); only the
  // elements [lo, hi) are written (the whole vector, or the tile's layer)
  __device__ __forceinline__ void finish_piece(int64_t e0, int v, int q, float4 gt, const u32x4& wq, uint32_t lo,
                                               uint32_t hi) const {
    const uint32_t el = piece(e0, v, q);
    const uint32_t off = el * 4u;
    const u32x4 gv = {as_u32(gt.x), as_u32(gt.y), as_u32(gt.z), as_u32(gt.w)};
    u32x4 nw;
    nw[0] = as_u32(__builtin_fmaf(-lr, gt.x, as_f32(wq[0])));
    nw[1] = as_u32(__builtin_fmaf(-lr, gt.y, as_f32(wq[1])));
    nw[2] = as_u32(__builtin_fmaf(-lr, gt.z, as_f32(wq[2])));
    nw[3] = as_u32(__builtin_fmaf(-lr, gt.w, as_f32(wq[3])));
    if (el >= lo && el + 4 <= hi) {
      if (out_of_place) st128_through_nt(rw, off, nw);
      else st128_through(rw, off, nw);
      st128(rgt, off, gv);          // empty descriptor when g~ is not wanted: dropped
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (el + r >= lo && el + r < hi) {
          st32(rw, off + 4u * r, nw[r]);
          st32(rgt, off + 4u * r, gv[r]);
        }
    }
  }

  // all pieces of wave-vector v, the sums read back from LDS rows in the coalesced (transposed) order
  __device__ __forceinline__ void finish_from_rows(int64_t e0, int v, const float* buf, const u32x4 (&wq)[EPV / 4],
                                                   uint32_t lo, uint32_t hi) const {
#pragma unroll
    for (int q = 0; q < EPV / 4; ++q) {
      const uint32_t m = (uint32_t)(q * kWave + lane) * 4u;       // element inside the wave-vector
      const float4 gt = *reinterpret_cast<const float4*>(buf + (m / EPV) * ROW + (m % EPV));
      finish_piece(e0, v, q, gt, wq[q], lo, hi);
    }
  }

  // transpose the sums of a tile into the coalesced shape and finish it
  __device__ __forceinline__ void update_store(int64_t e0, const float (&acc)[VPL][EPV],
                                               const u32x4 (&wv)[VPL][EPV / 4], uint32_t lo, uint32_t hi) const {
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      if constexpr (EPV > 4) {
        rows_to_lds(acc[v], tb);
        wave_lds_sync();
        finish_from_rows(e0, v, tb, wv[v], lo, hi);
        wave_lds_sync();
      } else {
        finish_piece(e0, v, 0, make_float4(acc[v][0], acc[v][1], acc[v][2], acc[v][3]), wv[v][0], lo, hi);
      }
    }
  }
};

// A wave owns `rounds` tiles: tile index = first tile of the workgroup + 4*round + wave.  The
// sums of the last HOLD of them are kept in registers, those of the one before in LDS (LH = 1), and
// all of them are written when the wave has finished reading.
// LAYERED (Sec. 4.5): the tiles are cut per layer (see LayerPlan); a tile takes the coefficient row
// of its layer, and only the elements of its layer are written.
// GROUPED (a wave owns more tiles than it can hold): the wave works through its tiles in groups of
// HOLD + LH rounds and writes each group in one burst of its own, instead of writing the early tiles one
// by one as they finish.  Fewer, larger write bursts disturb the other waves' reads less (ViT-B/16
// shape, bf16: 0.74 -> 0.67 ms; D = 350 M int8: 8.8 -> 8.5 ms).  It is a separate instantiation because
// the loop costs the single-group kernel registers it does not have.
template <int DT, int U, int VPL, int HOLD, int LH, bool LAYERED, bool GROUPED>
__device__ __forceinline__ void expand_body(PView P, const float* __restrict__ s, const float* w_in, float* w, float lr,
                                            float* __restrict__ g_tilde, int rounds, LayerPlan plan) {
  using X = Expander<DT, U, VPL, LAYERED>;
  constexpr int EPV = X::EPV;
  __shared__ float tbuf[4][kWave * X::ROW];
  __shared__ float lhold[LH ? 4 : 1][LH ? VPL : 1][LH ? kWave * X::ROW : 1];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t D = P.D;
  const int64_t ntiles = LAYERED ? (int64_t)plan.first[LAYERED ? plan.L : 0] : (D + X::TILE - 1) / X::TILE;
  // the number of per-layer tiles is known on the device only: there the tiles per wave are set here
  if constexpr (LAYERED) rounds = (int)((ntiles + 4 * (int64_t)gridDim.x - 1) / (4 * (int64_t)gridDim.x));
  const int64_t first = (int64_t)blockIdx.x * 4 * rounds + wave;
  const uint32_t w_bytes = (uint32_t)(D * 4);
  // bytes of one stored vector, rounded up to whole dwords: the range check drops a dword that
  // is only partly inside, and the tail bytes are padding of the same vector (ld >= D, ld % 128 == 0)
  const X x{P,
            lane,
            (uint32_t)((((D * X::S::kBitsPerElem + 7) >> 3) + 3) & ~(int64_t)3),
            (P.ld * X::S::kBitsPerElem) >> 3,
            kScaleSpanShift - P.block_shift,
            X::S::kScaled ? ((uint32_t)P.n << (kScaleSpanShift - P.block_shift)) * (uint32_t)X::S::kScaleBytes : 0u,
            make_rsrc(w, w_bytes),
            make_rsrc(g_tilde, g_tilde ? w_bytes : 0u),
            make_rsrc(w_in, w_bytes),
            w_in != w,
            lr,
            tbuf[wave]};

  // where tile t lies, which elements of it are written and which coefficients it takes.  The
  // tiles of a wave only move forward, so a layer cursor follows them.
  struct Where {
    int64_t e0;
    uint32_t lo, hi;
    const float* sv;
    float mm_a, mm_b;                   // min-max formats: the layer's a_l and b_l + bias * a_l
  };
  // (the plan is read again for every tile: keeping a layer's numbers in registers across the
  //  tiles costs registers this kernel does not have, and a tile is long enough to hide the loads)
  const int cur0 = LAYERED && first < ntiles ? layer_of_tile(plan, first) : 0;
  auto locate = [&](int64_t t, int& c) -> Where {
    if constexpr (LAYERED) {
      while (c < plan.L - 1 && plan.first[c + 1] <= t) ++c;
      const int64_t lo = plan.off[c];
      int64_t hi = plan.off[c + 1];
      hi = hi < D ? hi : D;
      const int64_t e0 = (lo & ~(int64_t)(kLayerAlign - 1)) + (t - plan.first[c]) * X::TILE;
      float ma = 1.0f, mb = 0.0f;
      if constexpr (kMinMax<DT>) {
        const float* ab = reinterpret_cast<const float*>(P.scales) + 2 * (int64_t)c;
        ma = ab[0];
        mb = ab[1] + kCodeBias<DT> * ma;
      }
      return Where{e0, (uint32_t)lo, (uint32_t)hi, s + (int64_t)c * P.n, ma, mb};
    } else {
      return Where{t * X::TILE, 0u, (uint32_t)D, s, 1.0f, 0.0f};
    }
  };
  int cur = cur0;                       // cursor of the reading phases

  if constexpr (GROUPED) {
    int cur_w = cur0;                   // cursor of the writing bursts (the same tiles again)
    // One group of rounds [r0, r0 + nr), nr <= HOLD + LH: the sums of the first round wait in LDS if the
    // registers cannot take all of them, the others stay in registers; then the wave writes them all.
    auto group = [&](int r0, int nr) {
      const int64_t t_lds = first + 4 * (int64_t)r0;
      const bool lds_tile = LH && nr > HOLD && t_lds < ntiles;
      if (lds_tile) {
        const Where at = locate(t_lds, cur);
        float acc[VPL][EPV];
        x.accumulate(at.e0, acc, at.sv, at.mm_a, at.mm_b);
#pragma unroll
        for (int v = 0; v < VPL; ++v) x.rows_to_lds(acc[v], lhold[wave][v]);
      }
      const int reg0 = (LH && nr > HOLD) ? r0 + 1 : r0;          // first round whose sums stay in registers
      float held[HOLD][VPL][EPV];
#pragma unroll
      for (int i = 0; i < HOLD; ++i) {
        const int64_t t = first + 4 * (int64_t)(reg0 + i);
        if (reg0 + i < r0 + nr && t < ntiles) {
          const Where at = locate(t, cur);
          x.accumulate(at.e0, held[i], at.sv, at.mm_a, at.mm_b);
        }
      }
      if (lds_tile) {
        const Where at = locate(t_lds, cur_w);
        u32x4 wv[VPL][EPV / 4];
        x.load_w(at.e0, wv);
        wave_lds_sync();
#pragma unroll
        for (int v = 0; v < VPL; ++v) x.finish_from_rows(at.e0, v, lhold[wave][v], wv[v], at.lo, at.hi);
        wave_lds_sync();                // the LDS rows are free for the next group
      }
#pragma unroll
      for (int i = 0; i < HOLD; ++i) {
        const int64_t t = first + 4 * (int64_t)(reg0 + i);
        if (reg0 + i < r0 + nr && t < ntiles) {
          const Where at = locate(t, cur_w);
          u32x4 wv[VPL][EPV / 4];
          x.load_w(at.e0, wv);
          x.update_store(at.e0, held[i], wv, at.lo, at.hi);
        }
      }
    };
    // the first group takes the remainder, so that every other group is a full burst
    constexpr int PH = HOLD + LH;
    int r0 = 0;
    if (rounds % PH != 0 && rounds > PH) {
      group(0, rounds % PH);
      r0 = rounds % PH;
    }
    for (; r0 < rounds; r0 += PH) group(r0, rounds - r0 < PH ? rounds - r0 : PH);
  } else {
    // ---- early rounds (only when a wave owns more tiles than it can hold): written as they finish
    const int early = rounds > HOLD + LH ? rounds - HOLD - LH : 0;
    for (int r = 0; r < early; ++r) {
      const int64_t t = first + 4 * (int64_t)r;
      if (t >= ntiles) break;
      const Where at = locate(t, cur);
      u32x4 wv[VPL][EPV / 4];
      x.load_w(at.e0, wv);                  // issued before the stream of P, consumed after it
      float acc[VPL][EPV];
      x.accumulate(at.e0, acc, at.sv, at.mm_a, at.mm_b);
      x.update_store(at.e0, acc, wv, at.lo, at.hi);
    }

    // ---- the round before the last HOLD ones: its sums wait in LDS ...
    const int64_t t_lds = first + 4 * (int64_t)early;
    const bool lds_tile = LH && rounds > HOLD && t_lds < ntiles;
    if (lds_tile) {
      const Where at = locate(t_lds, cur);
      float acc[VPL][EPV];
      x.accumulate(at.e0, acc, at.sv, at.mm_a, at.mm_b);
  #pragma unroll
      for (int v = 0; v < VPL; ++v) x.rows_to_lds(acc[v], lhold[wave][v]);
    }
    const int reg0 = (LH && rounds > HOLD) ? early + 1 : early;      // first round whose sums stay in registers

    // ---- ... the last rounds: their sums stay in registers ...
    float held[HOLD][VPL][EPV];
  #pragma unroll
    for (int i = 0; i < HOLD; ++i) {
      const int64_t t = first + 4 * (int64_t)(reg0 + i);
      if (reg0 + i < rounds && t < ntiles) {
        const Where at = locate(t, cur);
        x.accumulate(at.e0, held[i], at.sv, at.mm_a, at.mm_b);
      }
    }
    // ---- ... and everything is written in one burst once this wave has finished reading (the same
    //      tiles again, found with a cursor of its own)
    int cur_w = cur0;
    if (lds_tile) {
      const Where at = locate(t_lds, cur_w);
      u32x4 wv[VPL][EPV / 4];
      x.load_w(at.e0, wv);
      wave_lds_sync();
  #pragma unroll
      for (int v = 0; v < VPL; ++v) x.finish_from_rows(at.e0, v, lhold[wave][v], wv[v], at.lo, at.hi);
    }
  #pragma unroll
    for (int i = 0; i < HOLD; ++i) {
      const int64_t t = first + 4 * (int64_t)(reg0 + i);
      if (reg0 + i < rounds && t < ntiles) {
        const Where at = locate(t, cur_w);
        u32x4 wv[VPL][EPV / 4];
        x.load_w(at.e0, wv);
        x.update_store(at.e0, held[i], wv, at.lo, at.hi);
      }
    }
  }
}

template <int DT, int U, int VPL, int HOLD, int LH, bool LAYERED>
__global__ __launch_bounds__(256, 2) void expand_update_kernel(PView P, const float* __restrict__ s,
                                                               const float* w_in, float* w, float lr,
                                                               float* __restrict__ g_tilde, int rounds,
                                                               LayerPlan plan) {
  expand_body<DT, U, VPL, HOLD, LH, LAYERED, false>(P, s, w_in, w, lr, g_tilde, rounds, plan);
}
template <int DT, int U, int VPL, int HOLD, int LH, bool LAYERED>
__global__ __launch_bounds__(256, 2) void expand_update_grouped_kernel(PView P, const float* __restrict__ s,
                                                                       const float* w_in, float* w, float lr,
                                                                       float* __restrict__ g_tilde, int rounds,
                                                                       LayerPlan plan) {
  expand_body<DT, U, VPL, HOLD, LH, LAYERED, true>(P, s, w_in, w, lr, g_tilde, rounds, plan);
}

template <int DT, int U, int VPL, int HOLD, int LH, bool LAYERED>
static void launch_expand_cfg(const PView& P, const float* s, const float* w_in, float* w, float lr, float* g_tilde,
                              int max_grid, hipStream_t st, const void* plan_dev, int L) {
  constexpr int tile = kWave * VPL * Store<DT>::kEPV;
  LayerPlan plan{nullptr, nullptr, 1};
  const int64_t ntiles = (P.D + tile - 1) / tile;
  const int64_t rounds = (ntiles + 4 * (int64_t)max_grid - 1) / (4 * (int64_t)max_grid);   // tiles per wave
  int grid = (int)((ntiles + 4 * rounds - 1) / (4 * rounds));
  if constexpr (LAYERED) {
    plan = plan_view(plan_dev, L, tile);
    grid = max_grid;                  // the kernel divides the plan's tiles over the grid itself
  }
  // (the layer-wise kernel sets its rounds from the plan's tile count; the host's figure with one more tile
  //  per layer is an upper bound for it)
  const int64_t rounds_max = LAYERED ? (ntiles + L + 4 * (int64_t)grid - 1) / (4 * (int64_t)grid) : rounds;
  // (the grouped kernel holds one round less: its loop needs the registers)
  if (rounds_max > HOLD + LH)
    hipLaunchKernelGGL((expand_update_grouped_kernel<DT, U, VPL, HOLD - 1, LH, LAYERED>), dim3(grid), dim3(256), 0, st,
                       P, s, w_in, w, lr, g_tilde, (int)rounds, plan);
  else
    hipLaunchKernelGGL((expand_update_kernel<DT, U, VPL, HOLD, LH, LAYERED>), dim3(grid), dim3(256), 0, st, P, s, w_in,
                       w, lr, g_tilde, (int)rounds, plan);
}

// <U, VPL, HOLD, LH> per storage type: chosen by interleaved timing on MI355X at D = 25.6 M, n = 100
template <bool LAYERED>
static int launch_expand_any(const PView& P, int dtype, const float* s, const float* w_in, float* w, float lr,
                             float* g_tilde, int max_grid, hipStream_t st, const void* plan_dev, int L) {
  switch (dtype) {
    case TWA_F32: launch_expand_cfg<TWA_F32, 1, 8, 6, 1, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_BF16: launch_expand_cfg<TWA_BF16, 2, 4, 6, 1, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_I8: launch_expand_cfg<TWA_I8, 4, 2, 6, 1, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_I4: launch_expand_cfg<TWA_I4, 8, 1, 5, 0, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_U8MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U8MM, 4, 2, 6, 1, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
        break;
      }
      return TWA_ERR_DTYPE;
    case TWA_U4MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U4MM, 8, 1, 5, 0, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
        break;
      }
      return TWA_ERR_DTYPE;
    default: return TWA_ERR_DTYPE;
  }
  return hip_check(hipGetLastError());
}

int launch_expand_update(const PView& P, int dtype, const float* s, float* w, float lr, float* g_tilde, int max_grid,
                         hipStream_t st) {
  return launch_expand_any<false>(P, dtype, s, w, w, lr, g_tilde, max_grid, st, nullptr, 1);
}

// Layer-wise: s is L x n, row l holds the coefficients of layer l; `plan_dev` is the device plan.
// w_out = w_in - lr * g~ (w_in may be w_out: the in-place update).
int launch_expand_update_layers(const PView& P, int dtype, const float* s, const void* plan_dev, int L,
                                const float* w_in, float* w_out, float lr, float* g_tilde, int max_grid,
                                hipStream_t st) {
  return launch_expand_any<true>(P, dtype, s, w_in, w_out, lr, g_tilde, max_grid, st, plan_dev, L);
}

}  // namespace twa
