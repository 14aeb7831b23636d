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
// are over cost about what their size suggests.  A wave therefore keeps the finished sums of ALL
// its tiles (HOLD rounds in registers, one more in LDS) and writes them at the very end of the
// launch; a matrix too long for that is expanded by several launches, one run of tiles each.
#include <cstdint>

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
  float lr;
  bool want_gt;                                         // g~ is stored as well
  float* tb;                                            // this wave's LDS transpose buffer

  // sums of tile e0 over all basis vectors with the coefficients sv[0..n) (for I4 the bias / nibble
  // corrections are applied at the end)
  // Min-max formats (Sec. 4.6): mm_a scales every coefficient, and mm_b * sum_j s_j is added at the end
  // (mm_b = b_l + bias * a_l for codes stored relative to `bias`).
  // Layer-wise, [lo, hi) are the layer's elements: a lane whose elements all lie in front of the layer or
  // behind it reads at the end of the descriptor -- out-of-range loads return 0 and move no memory, so a
  // tile of a short layer costs the layer's bytes.  (The descriptors stay the same for every tile.)
  __device__ __forceinline__ void accumulate(int64_t e0, float (&acc)[VPL][EPV], const float* __restrict__ sv,
                                             float mm_a = 1.0f, float mm_b = 0.0f, uint32_t lo = 0u,
                                             uint32_t hi = 0u) const {
    const int n = P.n;
    uint32_t voff[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const uint32_t loc = (uint32_t)(v * kWave + lane) * EPV;     // element inside the tile
      voff[v] = (uint32_t)((((uint64_t)e0 + loc) * S::kBitsPerElem) >> 3);
      if constexpr (LAYERED) voff[v] = (e0 + loc + EPV <= (int64_t)lo || e0 + loc >= (int64_t)hi) ? col_bytes : voff[v];
    }
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
          raw[u][v] = load_codes<DT>(rc, voff[v]);
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

  // One coalesced 128-bit piece of wave-vector v is written: new weights (W) or g~.  Only the elements
  // [lo, hi) are written (the whole vector, or the tile's layer).
  template <bool W>
  __device__ __forceinline__ void put_piece(int64_t e0, int v, int q, const u32x4& val, uint32_t lo, uint32_t hi) const {
    const uint32_t el = piece(e0, v, q);
    const uint32_t off = el * 4u;
    if (el >= lo && el + 4 <= hi) {
      if constexpr (W) {
        st128_through_nt(rw, off, val);
      } else {
        st128(rgt, off, val);
      }
    } else {
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (el + r >= lo && el + r < hi) st32(W ? rw : rgt, off + 4u * r, val[r]);
    }
  }

  // w - lr * g~ for one piece; g~ itself is stored on the way if it is wanted
  __device__ __forceinline__ u32x4 new_piece(int64_t e0, int v, int q, float4 gt, const u32x4& wq, uint32_t lo,
                                             uint32_t hi) const {
    if (want_gt) put_piece<false>(e0, v, q, u32x4{as_u32(gt.x), as_u32(gt.y), as_u32(gt.z), as_u32(gt.w)}, lo, hi);
    u32x4 nw;
    nw[0] = as_u32(__builtin_fmaf(-lr, gt.x, as_f32(wq[0])));
    nw[1] = as_u32(__builtin_fmaf(-lr, gt.y, as_f32(wq[1])));
    nw[2] = as_u32(__builtin_fmaf(-lr, gt.z, as_f32(wq[2])));
    nw[3] = as_u32(__builtin_fmaf(-lr, gt.w, as_f32(wq[3])));
    return nw;
  }

  // The write burst has two phases, because the memory counter of a wave retires loads and stores in
  // the order of issue: a load of w issued after a (write-through) store waits for that store's
  // acknowledgement from memory.  Phase 1 turns the sums of every held tile into new weights IN the
  // registers that held the sums (loads of w only, nothing stored); phase 2 stores them all.

  // phase 1, tile in registers: acc <- w - lr * acc, in the coalesced (transposed) order of the pieces
  __device__ __forceinline__ void update_in_place(int64_t e0, float (&acc)[VPL][EPV], uint32_t lo, uint32_t hi) const {
    u32x4 wv[VPL][EPV / 4];
    load_w(e0, wv);
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      if constexpr (EPV > 4) {
        rows_to_lds(acc[v], tb);
        wave_lds_sync();
#pragma unroll
        for (int q = 0; q < EPV / 4; ++q) {
          const uint32_t m = (uint32_t)(q * kWave + lane) * 4u;       // element inside the wave-vector
          const float4 gt = *reinterpret_cast<const float4*>(tb + (m / EPV) * ROW + (m % EPV));
          const u32x4 nw = new_piece(e0, v, q, gt, wv[v][q], lo, hi);
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[v][4 * q + r] = as_f32(nw[r]);
        }
        wave_lds_sync();
      } else {
        const u32x4 nw = new_piece(e0, v, 0, make_float4(acc[v][0], acc[v][1], acc[v][2], acc[v][3]), wv[v][0], lo, hi);
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[v][r] = as_f32(nw[r]);
      }
    }
  }
  // phase 2, tile in registers
  __device__ __forceinline__ void store_tile(int64_t e0, const float (&acc)[VPL][EPV], uint32_t lo, uint32_t hi) const {
#pragma unroll
    for (int v = 0; v < VPL; ++v)
#pragma unroll
      for (int q = 0; q < EPV / 4; ++q)
        put_piece<true>(e0, v, q, u32x4{as_u32(acc[v][4 * q]), as_u32(acc[v][4 * q + 1]), as_u32(acc[v][4 * q + 2]),
                                        as_u32(acc[v][4 * q + 3])}, lo, hi);
  }

  // phase 1, tile whose sums wait in LDS rows: every lane replaces the pieces it reads by the new weights
  __device__ __forceinline__ void update_rows_in_place(int64_t e0, int v, float* buf, const u32x4 (&wq)[EPV / 4],
                                                       uint32_t lo, uint32_t hi) const {
#pragma unroll
    for (int q = 0; q < EPV / 4; ++q) {
      const uint32_t m = (uint32_t)(q * kWave + lane) * 4u;
      float4* at = reinterpret_cast<float4*>(buf + (m / EPV) * ROW + (m % EPV));
      const u32x4 nw = new_piece(e0, v, q, *at, wq[q], lo, hi);
      *at = make_float4(as_f32(nw[0]), as_f32(nw[1]), as_f32(nw[2]), as_f32(nw[3]));
    }
  }
  // phase 2 for it (the same lane reads what it wrote)
  __device__ __forceinline__ void store_rows(int64_t e0, int v, const float* buf, uint32_t lo, uint32_t hi) const {
#pragma unroll
    for (int q = 0; q < EPV / 4; ++q) {
      const uint32_t m = (uint32_t)(q * kWave + lane) * 4u;
      const float4 nw = *reinterpret_cast<const float4*>(buf + (m / EPV) * ROW + (m % EPV));
      put_piece<true>(e0, v, q, u32x4{as_u32(nw.x), as_u32(nw.y), as_u32(nw.z), as_u32(nw.w)}, lo, hi);
    }
  }
};

// Tiles per wave for a launch over R tiles on at most `max_grid` workgroups (4 waves each, two workgroups
// per compute unit): the workgroups run side by side, so the launch takes (workgroups per compute unit,
// rounded up) x (tiles per wave); the smallest such product wins, and of equal ones the one with more
// workgroups.  A full launch (R = 4 * most * max_grid) gets `most`.  Host and device agree by using this.
__host__ __device__ inline int pick_rounds(int64_t R, int max_grid, int most) {
  const int64_t cus = (max_grid + 1) / 2;
  int best = most;
  int64_t best_cost = INT64_MAX;
  for (int r = 1; r <= most; ++r) {
    const int64_t wgs = (R + 4 * r - 1) / (4 * r);
    if (wgs > max_grid) continue;
    const int64_t cost = ((wgs + cus - 1) / cus) * r;
    if (cost < best_cost) {
      best_cost = cost;
      best = r;
    }
  }
  return best;
}

// One launch covers the `chunk`-th run of 4 * (HOLD + LH) * max_grid tiles (the last run is shorter).  In it
// a wave owns `rounds` <= HOLD + LH tiles: tile index = first tile of the workgroup + 4*round + wave.  The
// sums of the last HOLD of them are kept in registers, those of the LH before in LDS, and all of
// them are written when the wave has finished reading.  (A matrix too long for that takes several
// launches, one after the other: see launch_expand_cfg.)
// LAYERED (Sec. 4.5): the tiles are cut per layer (see LayerPlan); a tile takes the coefficient row
// of its layer, and only the elements of its layer are written.
template <int DT, int U, int VPL, int HOLD, int LH, bool LAYERED>
__global__ __launch_bounds__(256, 2) void expand_update_kernel(PView P, const float* __restrict__ s,
                                                               const float* w_in, float* w, float lr,
                                                               float* __restrict__ g_tilde, int chunk,
                                                               int max_grid, LayerPlan plan) {
  using X = Expander<DT, U, VPL, LAYERED>;
  constexpr int EPV = X::EPV;
  __shared__ float tbuf[4][kWave * X::ROW];
  __shared__ float lhold[LH ? 4 : 1][LH ? VPL : 1][LH ? kWave * X::ROW : 1];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t D = P.D;
  if constexpr (LAYERED) {
    if (!plan_header_ok(plan.off, plan.L, D)) {           // not this call's plan: no table is read, nothing is expanded,
      if (blockIdx.x == 0 && threadIdx.x == 0 && chunk == 0) {      // and the first weight says so
        w[0] = __builtin_nanf("");
        if (g_tilde) g_tilde[0] = __builtin_nanf("");
      }
      return;
    }
  }
  const int64_t ntiles_all = LAYERED ? (int64_t)plan.first[LAYERED ? plan.L : 0] : (D + X::TILE - 1) / X::TILE;
  // the run of tiles of this launch, and the tiles per wave (set here, because the number of
  // per-layer tiles is known on the device only)
  constexpr int PH = HOLD + LH;
  const int64_t per_launch = 4 * (int64_t)PH * max_grid;
  const int64_t t_begin = (int64_t)chunk * per_launch;
  const int64_t t_end = t_begin + per_launch < ntiles_all ? t_begin + per_launch : ntiles_all;
  if (t_end <= t_begin) return;                                 // (the host sized the launches for an upper bound)
  const int rounds = pick_rounds(t_end - t_begin, max_grid, PH);
  const int64_t first = t_begin + (int64_t)blockIdx.x * 4 * rounds + wave;
  const uint32_t w_bytes = (uint32_t)(D * 4);
  // bytes of one stored vector, rounded up to whole dwords: the range check drops a dword that
  // is only partly inside, and the tail bytes are padding of the same vector (ld >= D, ld % 128 == 0)
  const X x{P,
            lane,
            stored_bytes<DT>(D),
            (P.ld * X::S::kBitsPerElem) >> 3,
            kScaleSpanShift - P.block_shift,
            X::S::kScaled ? ((uint32_t)P.n << (kScaleSpanShift - P.block_shift)) * (uint32_t)X::S::kScaleBytes : 0u,
            make_rsrc(w, w_bytes),
            make_rsrc(g_tilde, g_tilde ? w_bytes : 0u),
            make_rsrc(w_in, w_bytes),
            lr,
            g_tilde != nullptr,
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
  const int cur0 = LAYERED && first < t_end ? layer_of_tile(plan, first) : 0;
  auto locate = [&](int64_t t, int& c) -> Where {
    if constexpr (LAYERED) {
      // (tables that no kernel of this launch writes, the same entry for every lane: scalar fetches)
      while (c < plan.L - 1 && ld_plan(plan.first + c + 1) <= t) ++c;
      const int64_t lo = ld_plan(plan.off + c);
      int64_t hi = ld_plan(plan.off + c + 1);
      hi = hi < D ? hi : D;
      const int64_t e0 = (lo & ~(int64_t)(kLayerAlign - 1)) + (t - ld_plan(plan.first + c)) * X::TILE;
      float ma = 1.0f, mb = 0.0f;
      if constexpr (kMinMax<DT>) {
        const float* ab = reinterpret_cast<const float*>(P.scales) + 2 * (int64_t)c;
        ma = ld_plan(ab);
        mb = ld_plan(ab + 1) + P.code_bias * ma;
      }
      return Where{e0, (uint32_t)lo, (uint32_t)hi, s + (int64_t)c * P.n, ma, mb};
    } else {
      return Where{t * X::TILE, 0u, (uint32_t)D, s, 1.0f, 0.0f};
    }
  };

  // ---- reading: the sums of the first round(s) wait in LDS if the registers cannot take all rounds:
  //      one tile in `lhold`, and with LH = 2 one more, the very first, in the wave's transposition buffer
  //      (possible where that buffer is as large as a tile, VPL = 1) ...
  static_assert(LH <= 1 || (LH == 2 && VPL == 1), "a second LDS tile lives in the transposition buffer");
  int cur = cur0;
  const int nl = rounds > HOLD ? (rounds - HOLD < LH ? rounds - HOLD : LH) : 0;     // tiles that wait in LDS
  const int64_t t_lds = first + 4 * (int64_t)(nl > 0 ? nl - 1 : 0);
  const bool tb_tile = LH == 2 && nl == 2 && first < t_end;
  const bool lds_tile = LH >= 1 && nl >= 1 && t_lds < t_end;
  if (tb_tile) {
    const Where at = locate(first, cur);
    float acc[VPL][EPV];
    x.accumulate(at.e0, acc, at.sv, at.mm_a, at.mm_b, at.lo, at.hi);
    x.rows_to_lds(acc[0], tbuf[wave]);
  }
  if (lds_tile) {
    const Where at = locate(t_lds, cur);
    float acc[VPL][EPV];
    x.accumulate(at.e0, acc, at.sv, at.mm_a, at.mm_b, at.lo, at.hi);
#pragma unroll
    for (int v = 0; v < VPL; ++v) x.rows_to_lds(acc[v], lhold[wave][v]);
  }
  // ... those of the other rounds stay in registers.  (Every copy of the accumulation is ~5 KB of code and
  // the instruction cache holds 64 KB: one call site per phase, no more.)
  const int reg0 = nl;                                         // first round whose sums stay in registers
  // (The place of the NEXT tile is looked up before this tile is accumulated: layer-wise that is a chain of
  //  scalar loads from the plan, which then has a whole tile's time to arrive.)
  float held[HOLD][VPL][EPV];
  auto owned = [&](int i) { return i < HOLD && reg0 + i < rounds && first + 4 * (int64_t)(reg0 + i) < t_end; };
  Where ahead{0, 0u, 0u, nullptr, 0.0f, 0.0f};
  if (owned(0)) ahead = locate(first + 4 * (int64_t)reg0, cur);
#pragma unroll
  for (int i = 0; i < HOLD; ++i) {
    const Where at = ahead;
    if (owned(i + 1)) ahead = locate(first + 4 * (int64_t)(reg0 + i + 1), cur);
    if (owned(i)) x.accumulate(at.e0, held[i], at.sv, at.mm_a, at.mm_b, at.lo, at.hi);
  }
  // ---- the burst, phase 1: the new weights are formed where the sums were (the same tiles again, found
  //      with a cursor of their own) ...
  int cur_w = cur0;
  Where at_tb{0, 0u, 0u, nullptr, 0.0f, 0.0f}, at_lds{0, 0u, 0u, nullptr, 0.0f, 0.0f};
  if (tb_tile) {
    at_tb = locate(first, cur_w);
    u32x4 wv[VPL][EPV / 4];
    x.load_w(at_tb.e0, wv);
    wave_lds_sync();
    x.update_rows_in_place(at_tb.e0, 0, tbuf[wave], wv[0], at_tb.lo, at_tb.hi);
  }
  if (lds_tile) {
    at_lds = locate(t_lds, cur_w);
    u32x4 wv[VPL][EPV / 4];
    x.load_w(at_lds.e0, wv);
    wave_lds_sync();
#pragma unroll
    for (int v = 0; v < VPL; ++v) x.update_rows_in_place(at_lds.e0, v, lhold[wave][v], wv[v], at_lds.lo, at_lds.hi);
  }
  if (tb_tile) {
    // the tile in the transposition buffer has to leave before the register tiles are transposed: its
    // stores go out now (the one place where loads of w queue behind stores)
    wave_lds_sync();
    x.store_rows(at_tb.e0, 0, tbuf[wave], at_tb.lo, at_tb.hi);
    wave_lds_sync();
  }
  int cur_s = cur_w;                                           // (a third walk, for the stores)
#pragma unroll
  for (int i = 0; i < HOLD; ++i) {
    const int64_t t = first + 4 * (int64_t)(reg0 + i);
    if (reg0 + i < rounds && t < t_end) {
      const Where at = locate(t, cur_w);
      x.update_in_place(at.e0, held[i], at.lo, at.hi);
    }
  }
  // ---- ... phase 2: everything is stored
  if (lds_tile) {
    wave_lds_sync();
#pragma unroll
    for (int v = 0; v < VPL; ++v) x.store_rows(at_lds.e0, v, lhold[wave][v], at_lds.lo, at_lds.hi);
  }
#pragma unroll
  for (int i = 0; i < HOLD; ++i) {
    const int64_t t = first + 4 * (int64_t)(reg0 + i);
    if (reg0 + i < rounds && t < t_end) {
      const Where at = locate(t, cur_s);
      x.store_tile(at.e0, held[i], at.lo, at.hi);
    }
  }
}

// A launch holds at most HOLD + LH rounds of tiles per wave, i.e. 4 * (HOLD + LH) * grid tiles.  A longer
// matrix is cut into runs of that many tiles (and a shorter last one), one launch each, back to back on the
// stream: the kernel boundary is the one moment when nobody reads, and that is when the writes are cheap.
// Measured against one launch whose waves write a burst after every HOLD + LH rounds (the bursts of
// different waves drift apart and mix into the reads): D = 100 M, n = 100, int8: 1.93 -> 1.64 ms;
// ViT-B/16 shape, bf16: 0.69 -> 0.66 ms; D = 350 M, n = 128, int4: 4.8 -> 4.25 ms.
template <int DT, int U, int VPL, int HOLD, int LH, bool LAYERED>
static void launch_expand_cfg(const PView& P, const float* s, const float* w_in, float* w, float lr, float* g_tilde,
                              int max_grid, hipStream_t st, const void* plan_dev, int L) {
  constexpr int tile = kWave * VPL * Store<DT>::kEPV;
  constexpr int PH = HOLD + LH;
  LayerPlan plan{nullptr, nullptr, 1};
  if constexpr (LAYERED) plan = plan_view(plan_dev, L, tile);
  const int64_t ntiles = (P.D + tile - 1) / tile;
  // Layer-wise the kernel takes the number of tiles from the plan on the device.  A layer's tiles start on
  // the alignment grid, which is the tile size here, so the layers share at most one tile with each
  // neighbour: one more tile per layer is an upper bound, and the launches are sized for it.
  static_assert(!LAYERED || tile == kLayerAlign, "the bound of one extra tile per layer needs tiles of the layer alignment");
  const int64_t bound = LAYERED ? ntiles + L : ntiles;
  const int64_t per_launch = 4 * (int64_t)PH * max_grid;
  const int64_t K = (bound + per_launch - 1) / per_launch;
  for (int64_t k = 0; k < K; ++k) {
    int grid = max_grid;                 // (layer-wise the kernel divides the run itself; spare workgroups leave)
    if constexpr (!LAYERED) {
      const int64_t R = ntiles - k * per_launch < per_launch ? ntiles - k * per_launch : per_launch;
      const int r = pick_rounds(R, max_grid, PH);
      grid = (int)((R + 4 * r - 1) / (4 * r));
    }
    hipLaunchKernelGGL((expand_update_kernel<DT, U, VPL, HOLD, LH, LAYERED>), dim3(grid), dim3(256), 0, st, P, s, w_in,
                       w, lr, g_tilde, (int)k, max_grid, plan);
  }
}

// <U, VPL, HOLD, LH> per storage type: chosen by interleaved timing on MI355X at D = 25.6 M, n = 100
template <bool LAYERED>
static int launch_expand_any(const PView& P, int dtype, const float* s, const float* w_in, float* w, float lr,
                             float* g_tilde, int max_grid, hipStream_t st, const void* plan_dev, int L) {
  switch (dtype) {
    case TWA_F32: launch_expand_cfg<TWA_F32, 1, 8, 6, 1, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_BF16: launch_expand_cfg<TWA_BF16, 2, 4, 6, 1, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_I8: launch_expand_cfg<TWA_I8, 4, 2, 6, 1, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_I4: launch_expand_cfg<TWA_I4, 8, 1, 5, 2, LAYERED>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L); break;
    case TWA_U8MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U8MM, 4, 2, 6, 1, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
        break;
      }
      return TWA_ERR_DTYPE;
    case TWA_U16MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U16MM, 2, 4, 6, 1, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
        break;
      }
      return TWA_ERR_DTYPE;
    case TWA_U2MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U2MM, 8, 1, 5, 2, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
        break;
      }
      return TWA_ERR_DTYPE;
    case TWA_U1MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U1MM, 8, 1, 5, 2, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
        break;
      }
      return TWA_ERR_DTYPE;
    case TWA_U3MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U3MM, 8, 1, 5, 2, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
        break;
      }
      return TWA_ERR_DTYPE;
    case TWA_U4MM:
      if constexpr (LAYERED) {
        launch_expand_cfg<TWA_U4MM, 8, 1, 5, 2, true>(P, s, w_in, w, lr, g_tilde, max_grid, st, plan_dev, L);
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
