// s = P^T g  (arXiv 2205.13104, Sec. 4.2: the gradient w.r.t. the averaging coefficients is the
// model gradient projected on the basis).  A tall-skinny reduction over D that is bound by the
// one pass over the stored P, so the kernel is a pure HBM stream:
//
//   * a persistent grid sized so that every workgroup owns the SAME number of consecutive D-tiles
//     (only the last may own fewer): equal bytes per workgroup, so they all finish together;
//   * the 4 waves of a workgroup share the tile (same slice of g, kept in registers) and split
//     the n basis vectors between them, so a lane keeps <= 32 running sums in registers with
//     compile-time indices;
//   * every lane fetches 128 bits per load, a wave covers 1 KB contiguous of one basis vector;
//     int8 / bf16 are decoded in registers, 4-bit codes enter integer dot products as they are stored; the block
//     scale is applied once per (lane-vector, basis vector), never per element;
//   * all loads go through buffer descriptors: the ragged end of D and unused column slots
//     read zeros without memory traffic and without branches in the steady state;
//   * one cross-lane reduction per wave at the very end, per-workgroup partial sums in the
//     workspace, and a second tiny kernel adds them in a fixed order (fp64) -> deterministic.
#include <mutex>

#include "twa_device.h"
#include "twa_host.h"

namespace twa {

// ---- the 4-bit block codes in integers ---------------------------------------------------------------------
// Decoding a 4-bit code to a float and multiplying costs two vector instructions per element, and at 32 elements
// per 128-bit load the vector ALUs, not the memory stream, bound the kernel.  The integer dot product of eight
// 4-bit pairs (v_dot8_i32_i4) takes a dword of codes as it is stored (after one XOR that turns code + 8 into the
// two's complement nibble), so the gradient comes to it instead: each lane turns its 32-element slice of g into a
// fixed-point number per element, x_i = round_to_nearest_even(g_i / unit), unit = 2^(e-22) with 2^e the smallest
// power of two above the slice's largest |g_i| (|x_i| <= 2^22), written as six signed hexadecimal digits
// x_i = sum_k d_ik 16^k, d_ik in [-8, 7].  Then sum_i q_i x_i = sum_k 16^k sum_i q_i d_ik exactly, in 32-bit
// integers, and one conversion and two multiplications per (lane, basis vector) bring it back to a float.
// Error model: g is rounded to multiples of `unit` <= 2^-21 max|g_slice| (error <= unit / 2); products and sums
// of a slice are exact; the running sums over tiles are fp32 as for every other storage type.
// A slice that holds an infinity or a NaN gets unit = NaN, which every sum it enters inherits.
constexpr int kFixDigits = 6;

// out[k] = nibble k of y[0..7] gathered into one dword (nibble r of out[k] = nibble k of y[r]), k < 6:
// 16-bit halves, bytes, then nibbles change places.
__device__ __forceinline__ void gather_digits(const uint32_t (&y)[8], uint32_t (&out)[kFixDigits]) {
  uint32_t a[8], b[8];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    a[r] = __builtin_amdgcn_perm(y[r + 4], y[r], 0x05040100u);
    a[r + 4] = __builtin_amdgcn_perm(y[r + 4], y[r], 0x07060302u);
  }
#pragma unroll
  for (int h = 0; h < 8; h += 4) {
#pragma unroll
    for (int r = h; r < h + 2; ++r) {
      b[r] = __builtin_amdgcn_perm(a[r], a[r + 2], 0x02060004u);
      b[r + 2] = __builtin_amdgcn_perm(a[r], a[r + 2], 0x03070105u);
    }
  }
#pragma unroll
  for (int r = 0; r < kFixDigits; r += 2) {
    out[r] = (b[r] & 0x0f0f0f0fu) | ((b[r + 1] << 4) & 0xf0f0f0f0u);
    out[r + 1] = ((b[r] >> 4) & 0x0f0f0f0fu) | (b[r + 1] & 0xf0f0f0f0u);
  }
}

// Codes of 4 bits and fewer enter the dot products; the narrower ones are spread to one code per nibble first.
template <int DT>
constexpr bool kDotCodes = kNibbles<DT> || DT == TWA_U2MM || DT == TWA_U1MM || DT == TWA_U3MM;

// Which of the lane's 32 elements meets nibble r of the m-th dword of spread codes (see spread_codes).
template <int DT> __device__ __forceinline__ constexpr int slice_elem(int m, int r) {
  if constexpr (DT == TWA_U1MM) return 4 * r + m;                       // dword m holds bit m of every nibble of the word
  else if constexpr (DT == TWA_U2MM || DT == TWA_U3MM) return 16 * (m >> 1) + 2 * r + (m & 1);   // even / odd codes of word m/2
  else return 8 * m + r;                                                 // 4-bit codes: as stored
}

// The fixed-point digits of a lane's 32 gradient elements, in the nibble order of the spread codes (element
// slice_elem(m, r) in nibble r of dg[m][k]); returns `unit`.
template <int DT>
__device__ __forceinline__ float fixed_point_digits(const float (&g)[32], uint32_t (&dg)[4][kFixDigits]) {
  uint32_t amax = 0;                               // largest |g| as a bit pattern: NaN sorts above infinity
#pragma unroll
  for (int e = 0; e < 32; ++e) {
    const uint32_t ab = as_u32(g[e]) & 0x7fffffffu;
    amax = ab > amax ? ab : amax;
  }
  const uint32_t eb = amax >> 23;                  // biased exponent: max|g| < 2^(eb - 126)
  const uint32_t ex = eb < 22u ? 22u : eb;         // (below 2^-104 the unit stays 2^-126)
  const float up = as_f32((275u - ex) << 23);      // 2^(148 - ex) = 1 / unit
  const float unit = eb == 255u ? __builtin_nanf("") : as_f32((ex - 21u) << 23);
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    uint32_t y[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      // 1.5 * 2^23 + x: the low mantissa bits hold x (two's complement), rounded to nearest even by the FMA
      const uint32_t bits = as_u32(__builtin_fmaf(g[slice_elem<DT>(m, r)], up, 12582912.0f));
      // x + 0x888888 has the digits d_k + 8 in its nibbles; XOR 8 makes each the two's complement nibble of d_k
      y[r] = (bits + (0x00888888u - 0x4B400000u)) ^ 0x00888888u;
    }
    gather_digits(y, dg[m]);
  }
  return unit;
}

// One code per nibble, as signed 4-bit numbers, from what a lane loaded for one basis vector:
//   4 bits: the stored nibble is code + 8 (block codes) or the unsigned code c (min-max): XOR 8 gives code or c - 8;
//   2 bits: a word holds 16 codes, code j at bits 2j: the even ones and the odd ones make a dword each;
//   1 bit : the word holds 32 codes: bit s of every nibble makes dword s;
//   3 bits: words 0 and 1 hold the low two bits like the 2-bit layout, word 2 the high bit of element 16h + 4k + m at
//           bit 8k + m + 4h: for the even codes of word h (m = 0, 2) it moves to bit 2 of nibbles 2k, 2k + 1, for the odd
//           ones (m = 1, 3) likewise.
template <int DT> __device__ __forceinline__ void spread_codes(const u32x4& codes, int (&q)[4]) {
  if constexpr (kNibbles<DT>) {
#pragma unroll
    for (int m = 0; m < 4; ++m) q[m] = (int)(codes[m] ^ 0x88888888u);
  } else if constexpr (DT == TWA_U2MM) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      q[2 * h] = (int)(codes[h] & 0x33333333u);
      q[2 * h + 1] = (int)((codes[h] >> 2) & 0x33333333u);
    }
  } else if constexpr (DT == TWA_U1MM) {
#pragma unroll
    for (int m = 0; m < 4; ++m) q[m] = (int)((codes[0] >> m) & 0x11111111u);
  } else {
    static_assert(DT == TWA_U3MM, "codes of 4 bits and fewer");
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t t = codes[2] >> (4 * h);
      q[2 * h] = (int)((codes[h] & 0x33333333u) | ((t & 0x01010101u) << 2) | ((t & 0x04040404u) << 4));
      q[2 * h + 1] = (int)(((codes[h] >> 2) & 0x33333333u) | ((t & 0x02020202u) << 1) | ((t & 0x08080808u) << 3));
    }
  }
}

// sum_i q_i x_i for the 32 codes of one load against the digits of the lane's slice.
template <int DT>
__device__ __forceinline__ int dot_codes_fixed(const u32x4& codes, const uint32_t (&dg)[4][kFixDigits]) {
  int q[4];
  spread_codes<DT>(codes, q);
  // Horner over the digits, most significant first, in ONE accumulator (wrap-around in between is harmless:
  // the final value is below 2^31 in magnitude and the arithmetic is modulo 2^32)
  int v = 0;
#pragma unroll
  for (int k = kFixDigits - 1; k >= 0; --k) {
    if (k != kFixDigits - 1) v = (int)((uint32_t)v << 4);
#pragma unroll
    for (int m = 0; m < 4; ++m) v = __builtin_amdgcn_sdot8(q[m], (int)dg[m][k], v, false);
  }
  return v;
}

// KB = gradients handled together (1 or TWA_MAX_K slots), U = column slots per chunk,
// NCH = chunks, so a wave owns up to U*NCH basis vectors; VPL = 128-bit vectors per lane per
// basis vector and tile.
//
// LAYERED (Sec. 4.5, Alg. 1): every layer has its own n sums.  The tiles are cut per layer (see
// LayerPlan), so a tile belongs to one layer and the stream over P is the same as for the whole
// model; the gradient is read through a descriptor that ends with the layer, and the few elements in
// front of a layer's unaligned start are zeroed in that layer's first tile.  When the workgroup
// walks into the next layer it reduces its running sums and writes them to partial slot
// (workgroup + layer): along the walk both indices only grow, so the slot is unique, and the
// reduction kernel knows from the plan which workgroups contributed to a layer.
// SQUARES (with LAYERED, F32): no gradient; the sums are the squares of the CENTRED elements of the
// layer, sum_i ((W_ij - hi_i) - lo_i)^2 -- the squared norms that the layer-wise basis divides by
// (Sec. 4.1, 4.5).  The mean arrives as two binary32 words per element: `g` holds hi, `aux` lo.
// `aux` is the one extra buffer of a mode: written for the min-max formats (per-workgroup sums of the
// gradient, which the zero points b_l multiply), read in the squares mode (the mean's low words), unused else.
template <int DT, int KB, int U, int NCH, int VPL, bool LAYERED, bool SQUARES = false>
__device__ __forceinline__ void project_body(PView P, const float* __restrict__ g, int64_t ldg, int kvalid,
                                             float* __restrict__ partial, int cpw, int tiles_per_wg, LayerPlan plan,
                                             float* __restrict__ aux) {
  using S = Store<DT>;
  constexpr int EPV = S::kEPV;
  constexpr int TILE = kWave * VPL * EPV;
  constexpr int SLOTS = U * NCH;
  static_assert(!kDotCodes<DT>, "codes of 4 bits and fewer are projected by project_dot_kernel");
  static_assert(kScaleSpan % TILE == 0 || TILE % kScaleSpan == 0, "tiles and scale spans nest");
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  const int64_t D = P.D;
  if constexpr (LAYERED) {
    if (!plan_header_ok(plan.off, plan.L, D)) return;      // not this call's plan: the reduction kernel answers with NaN
  }
  const int64_t ntiles = LAYERED ? (int64_t)plan.first[LAYERED ? plan.L : 0] : (D + TILE - 1) / TILE;
  // every workgroup owns the same number of consecutive tiles (the last ones may own fewer); the
  // number of per-layer tiles is known on the device only, so there the split is made here
  if constexpr (LAYERED) tiles_per_wg = (int)((ntiles + gridDim.x - 1) / gridDim.x);
  const int64_t t0 = (int64_t)blockIdx.x * tiles_per_wg;
  int64_t t1 = t0 + tiles_per_wg;
  if (t1 > ntiles) t1 = ntiles;

  const int c0 = wave * cpw;
  int ncol = P.n - c0;
  ncol = ncol < 0 ? 0 : (ncol > cpw ? cpw : ncol);

  // bytes of one stored vector, rounded up to whole dwords: the range check drops a dword that
  // is only partly inside, and the tail bytes are padding of the same vector (ld >= D, ld % 128 == 0)
  const uint32_t col_bytes = stored_bytes<DT>(D);
  const int64_t ld_bytes = (P.ld * S::kBitsPerElem) >> 3;
  const int gshift = kScaleSpanShift - P.block_shift;            // log2(scales per span and vector)
  const uint32_t span_scale_bytes = S::kScaled ? ((uint32_t)P.n << gshift) * (uint32_t)S::kScaleBytes : 0u;

  float acc[SLOTS][KB];
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl)
#pragma unroll
    for (int c = 0; c < KB; ++c) acc[sl][c] = 0.0f;

  // min-max formats: the layer's sum of the gradient itself (the zero point b_l multiplies it)
  float gsum = 0.0f;
  // one reduction over the wave's lanes, then the partial sums of row `slot_row`
  auto flush = [&](int slot_row) {
    if constexpr (kMinMax<DT>) {
      const float tot = wave_sum_to_last_lane(gsum);
      if (wave == 0 && lane == kSumLane) aux[slot_row] = tot;
      gsum = 0.0f;
    }
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
#pragma unroll
      for (int c = 0; c < KB; ++c) {
        const float tot = wave_sum_to_last_lane(acc[sl][c]);
        if (lane == kSumLane && sl < ncol && c < kvalid)
          partial[((int64_t)slot_row * kvalid + c) * P.n + c0 + sl] = tot;
        if constexpr (LAYERED) acc[sl][c] = 0.0f;
      }
    }
  };

  LayerCursor lc{0, 0, 0, 0, 0};        // layer of the tile at hand
  if constexpr (LAYERED) {
    if (t0 < t1) lc.load(plan, layer_of_tile(plan, t0));
  }

  for (int64_t t = t0; t < t1; ++t) {
    int64_t e0 = t * TILE;
    uint32_t g_bytes = (uint32_t)(D * 4);
    uint32_t head = 0;                  // elements of this tile in front of its layer's first element
    uint32_t tail = TILE;               // elements of this tile up to its layer's end
    if constexpr (LAYERED) {
      if (lc.behind(plan, t)) {                                  // this tile starts the next (non-empty) layer
        flush((int)blockIdx.x + lc.cur);                         // a workgroup never holds a layer without tiles
        lc.seek(plan, t);
      }
      const int64_t hi = lc.hi < D ? lc.hi : D;
      e0 = lc.tile_start(t, TILE);
      g_bytes = (uint32_t)(hi * 4);                              // the gradient ends with the layer
      head = lc.lo > e0 ? (uint32_t)(lc.lo - e0 < TILE ? lc.lo - e0 : TILE) : 0u;
      tail = hi - e0 < TILE ? (uint32_t)(hi > e0 ? hi - e0 : 0) : (uint32_t)TILE;
    }
    // Where this lane's elements sit in a stored vector.  A tile of a short layer is mostly outside the
    // layer: a lane whose elements all lie in front of the layer or behind it reads at the end of the
    // descriptor instead -- out-of-range loads return 0 and move no memory, so such a tile costs the
    // layer's bytes, not a whole tile's.  (The descriptors themselves stay the same for every tile: ending
    // them with the layer made them loop-variant and cost the 1- and 2-bit kernels 15-28 %.)
    uint32_t voff[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const uint32_t loc = (uint32_t)(v * kWave + lane) * EPV;
      voff[v] = (uint32_t)((((uint64_t)e0 + loc) * S::kBitsPerElem) >> 3);
      if constexpr (LAYERED) {
        voff[v] = (loc + EPV <= head || loc >= tail) ? col_bytes : voff[v];
        asm volatile("" : "+v"(voff[v]));      // one register per vector, formed once per tile
      }
    }

    // ---- this lane's slice of the gradient(s); the descriptor ends at element D (at the end of
    //      the layer), and the range check is per dword, so elements past that end arrive as 0 --
    float gs[KB][VPL][EPV];
    float mean_hi[SQUARES ? VPL : 1][EPV], mean_lo[SQUARES ? VPL : 1][EPV];     // SQUARES: this lane's slice of the mean
#pragma unroll
    for (int c = 0; c < KB; ++c) {
      const rsrc_t rg = make_rsrc(g + (int64_t)c * ldg, c < kvalid ? g_bytes : 0u);
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        const uint32_t elem = (uint32_t)e0 + (uint32_t)(v * kWave + lane) * EPV;
        if constexpr (SQUARES) {
          const uint32_t rel = (uint32_t)(v * kWave + lane) * EPV;
#pragma unroll
          for (int e = 0; e < EPV; ++e) gs[c][v][e] = (rel + e >= head && rel + e < tail) ? 1.0f : 0.0f;
          const rsrc_t rl = make_rsrc(aux, g_bytes);
#pragma unroll
          for (int q = 0; q < EPV / 4; ++q) {
            const u32x4 h = ld128(rg, (elem + 4u * q) * 4u), l = ld128(rl, (elem + 4u * q) * 4u);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              mean_hi[v][4 * q + r] = as_f32(h[r]);
              mean_lo[v][4 * q + r] = as_f32(l[r]);
            }
          }
        } else {
#pragma unroll
          for (int q = 0; q < EPV / 4; ++q) {
            const u32x4 x = ld128(rg, (elem + 4u * q) * 4u);   // shared by the 4 waves: keep it cacheable
#pragma unroll
            for (int r = 0; r < 4; ++r) gs[c][v][4 * q + r] = as_f32(x[r]);
          }
        }
        if constexpr (LAYERED && !SQUARES) {
          if (head != 0) {                                   // first tile of a layer with an unaligned start
            const uint32_t rel = (uint32_t)(v * kWave + lane) * EPV;
#pragma unroll
            for (int e = 0; e < EPV; ++e) gs[c][v][e] = rel + e >= head ? gs[c][v][e] : 0.0f;
          }
        }
        if constexpr (kMinMax<DT>) {
          float sum = 0.0f;
#pragma unroll
          for (int e = 0; e < EPV; ++e) sum += gs[c][v][e];
          gsum += sum;
        }
      }
    }

    // ---- stream this wave's basis vectors over the tile ----------------------------------
    rsrc_t rs = make_rsrc(g, 0u);
    // scale spans one tile touches (per-layer tiles start on the same grid: kLayerAlign is a multiple of the span)
    constexpr int SPANS = TILE > kScaleSpan ? TILE / kScaleSpan : 1;
    static_assert(kLayerAlign % kScaleSpan == 0, "per-layer tiles keep the alignment of the scale spans");
    if constexpr (S::kScaled)
      rs = make_rsrc(P.scales + (e0 >> kScaleSpanShift) * (int64_t)span_scale_bytes, SPANS * span_scale_bytes);
    const uint32_t in_span = (uint32_t)e0 & (uint32_t)(kScaleSpan - 1);   // tile offset inside its first span
    // chunk ch = column slots [ch*U, (ch+1)*U): fetch (128-bit codes/values + block scales) ...
    auto load_chunk = [&](int ch, u32x4 (&raw)[U][VPL], float (&sc)[U][VPL]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int slot = ch * U + u;
        const bool valid = slot < ncol;
        const int col = valid ? c0 + slot : 0;
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
                valid ? ((((pos >> kScaleSpanShift) * (uint32_t)P.n + (uint32_t)col) << gshift) +
                         ((pos & (uint32_t)(kScaleSpan - 1)) >> P.block_shift)) * (uint32_t)S::kScaleBytes
                      : 0x7fffff00u;
            sc[u][v] = load_scale<DT>(rs, soff, P.gscale);
          } else {
            sc[u][v] = 1.0f;
          }
        }
      }
    };
    // ... and fold it into the running sums of its slots
    auto compute_chunk = [&](int ch, const u32x4 (&raw)[U][VPL], const float (&sc)[U][VPL]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int slot = ch * U + u;
#pragma unroll
        for (int v = 0; v < VPL; ++v) {
          float x[EPV];
          decode<DT>(raw[u][v], x);
          if constexpr (SQUARES) {
#pragma unroll
            for (int e = 0; e < EPV; ++e) x[e] = (x[e] - mean_hi[v][e]) - mean_lo[v][e];
          }
#pragma unroll
          for (int c = 0; c < KB; ++c) {
            if constexpr (S::kScaled) {
              float d = 0.0f;
#pragma unroll
              for (int e = 0; e < EPV; ++e) d = __builtin_fmaf(x[e], gs[c][v][e], d);
              acc[slot][c] = __builtin_fmaf(d, sc[u][v], acc[slot][c]);
            } else {
              float d = acc[slot][c];
#pragma unroll
              for (int e = 0; e < EPV; ++e) d = __builtin_fmaf(SQUARES ? x[e] * gs[c][v][e] : x[e], SQUARES ? x[e] : gs[c][v][e], d);
              acc[slot][c] = d;
            }
          }
        }
      }
    };
    // double buffered: the loads of chunk ch+1 are issued before chunk ch is consumed
    u32x4 rawA[U][VPL], rawB[U][VPL];
    float scA[U][VPL], scB[U][VPL];
    load_chunk(0, rawA, scA);
#pragma unroll
    for (int ch = 0; ch < NCH; ch += 2) {
      if (ch + 1 < NCH) load_chunk(ch + 1, rawB, scB);
      compute_chunk(ch, rawA, scA);
      if (ch + 2 < NCH) load_chunk(ch + 2, rawA, scA);
      if (ch + 1 < NCH) compute_chunk(ch + 1, rawB, scB);
    }
  }

  if constexpr (LAYERED) {
    if (t0 < t1) flush((int)blockIdx.x + lc.cur);
  } else {
    flush((int)blockIdx.x);
  }
}

// The kernels around the body differ in their register budget only, which decides how the compiler
// schedules the loads (measured at D = 25.6 M over n = 10 .. 128 and all storage types):
//   * whole model, many basis vectors per wave (5 or more chunks, n > 64): the compiler's default;
//   * whole model, few basis vectors per wave: exactly two waves per SIMD.  By default several of these
//     variants use the accumulation registers as well and run at ONE wave per SIMD (int8, n = 10: 0.129 ms
//     instead of 0.078 ms);
//   * layer-wise: two workgroups per compute unit (256 registers per lane), for the same reason.
template <int DT, int KB, int U, int NCH, int VPL>
__global__ __launch_bounds__(256) void project_kernel(PView P, const float* __restrict__ g, int64_t ldg, int kvalid,
                                                      float* __restrict__ partial, int cpw, int tiles_per_wg) {
  project_body<DT, KB, U, NCH, VPL, false, false>(P, g, ldg, kvalid, partial, cpw, tiles_per_wg,
                                                  LayerPlan{nullptr, nullptr, 1}, nullptr);
}
template <int DT, int KB, int U, int NCH, int VPL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void project_kernel_two_waves(
    PView P, const float* __restrict__ g, int64_t ldg, int kvalid, float* __restrict__ partial, int cpw,
    int tiles_per_wg) {
  project_body<DT, KB, U, NCH, VPL, false, false>(P, g, ldg, kvalid, partial, cpw, tiles_per_wg,
                                                  LayerPlan{nullptr, nullptr, 1}, nullptr);
}
template <int DT, int U, int NCH, int VPL, bool SQUARES>
__global__ __launch_bounds__(256, 2) void project_layers_kernel(PView P, const float* __restrict__ g,
                                                                float* __restrict__ partial, int cpw, LayerPlan plan,
                                                                float* __restrict__ aux) {
  project_body<DT, 1, U, NCH, VPL, true, SQUARES>(P, g, 0, 1, partial, cpw, 0, plan, aux);
}

// The projection on codes that enter the dot products (k = 1; 4-bit block codes, whole model or layer-wise; min-max
// codes of 4 bits and fewer, layer-wise), with the stream pipelined ACROSS tiles.  With 32 elements per lane and
// load a tile is at most 1 KB per basis vector, so the start of a tile -- fetch the slice of g, turn it into
// digits, fetch the first chunk of codes -- is a large part of the tile's time, and a wave that has nothing in
// flight meanwhile costs bandwidth (a pure-read kernel with this access pattern falls from 6.3 to 3.9 TB/s when
// its loads are not kept in flight).  Here the next tile's slice of g is fetched as soon as this tile's digits are
// formed (its registers are free then), and the next tile's first chunk of codes while this tile's last chunk is
// consumed.  Sums, reduction and partial-sum layout as in project_body.
// LAYERED: the tiles follow the layer plan as in project_body (a tile belongs to one layer; the gradient is read
// through a descriptor that ends with the layer; the elements in front of an unaligned layer start are zeroed; a
// lane wholly outside the layer reads nothing), and the place of the NEXT tile is worked out one tile ahead, on a
// copy of the layer cursor.  When the next tile belongs to another layer the running sums are reduced and written
// to partial slot (workgroup + layer) after this tile.
// KB = 2 (whole model only): two gradients, g and g + ldg, share one pass over the codes; their sums go to partial
// rows 2 * workgroup and 2 * workgroup + 1 (the layout the reduction of a batch expects).
template <int DT, int U, int NCH, bool LAYERED, int KB = 1>
__global__ __launch_bounds__(256, 2) void project_dot_kernel(PView P, const float* __restrict__ g, int64_t ldg,
                                                             float* __restrict__ partial, int cpw, int tiles_per_wg,
                                                             LayerPlan plan, float* __restrict__ aux) {
  using S = Store<DT>;
  constexpr int EPV = S::kEPV;
  constexpr int TILE = kWave * EPV;
  constexpr int SLOTS = U * NCH;
  static_assert(kDotCodes<DT> && EPV == 32 && TILE == kLayerAlign && TILE == kScaleSpan, "32 codes per lane, one span per tile");
  static_assert(NCH >= 2, "chunk 0 of the next tile is fetched while another chunk is consumed");
  static_assert(LAYERED || !kMinMax<DT>, "the min-max formats exist layer-wise only");
  static_assert(KB == 1 || (KB == 2 && !LAYERED), "gradients in pairs: whole model only");
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t D = P.D;
  int64_t ntiles = (D + TILE - 1) / TILE;
  if constexpr (LAYERED) {
    if (!plan_header_ok(plan.off, plan.L, D)) return;         // not this call's plan: the reduction kernel answers with NaN
    ntiles = (int64_t)plan.first[plan.L];                     // known on the device only: the split is made here
    tiles_per_wg = (int)((ntiles + gridDim.x - 1) / gridDim.x);
  }
  const int64_t t0 = (int64_t)blockIdx.x * tiles_per_wg;
  int64_t t1 = t0 + tiles_per_wg;
  if (t1 > ntiles) t1 = ntiles;
  if (t0 >= t1) return;              // layer-wise: a workgroup without tiles owns no partial slot (whole model: none exists)
  const int c0 = wave * cpw;
  int ncol = P.n - c0;
  ncol = ncol < 0 ? 0 : (ncol > cpw ? cpw : ncol);
  const uint32_t col_bytes = stored_bytes<DT>(D);
  const int64_t ld_bytes = (P.ld * S::kBitsPerElem) >> 3;
  const int gshift = kScaleSpanShift - P.block_shift;          // log2(scales per span and vector)
  const uint32_t span_scale_bytes = S::kScaled ? ((uint32_t)P.n << gshift) * (uint32_t)S::kScaleBytes : 0u;
  const uint32_t loc = (uint32_t)lane * EPV;                   // this lane's first element inside a tile

  // where a tile sits: first element of its grid cell, the part of the cell that belongs to the layer, the end of
  // the layer in the gradient, and the place of this lane's codes in a stored vector
  struct Place {
    int64_t e0;
    uint32_t head, tail, g_bytes, voff;
  };
  auto place = [&](const LayerCursor& c, int64_t t) {
    Place p;
    if constexpr (LAYERED) {
      const int64_t hi = c.hi < D ? c.hi : D;
      const int64_t e0 = c.tile_start(t, TILE);
      // the same for every lane; said so, or the descriptors built from these numbers are taken for lane-dependent
      // and every load through them is wrapped in a loop over the distinct values
      const auto uni = [](uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); };
      p.e0 = (int64_t)(((uint64_t)uni((uint32_t)((uint64_t)e0 >> 32)) << 32) | uni((uint32_t)e0));
      p.g_bytes = uni((uint32_t)(hi * 4));
      p.head = uni(c.lo > e0 ? (uint32_t)(c.lo - e0 < TILE ? c.lo - e0 : TILE) : 0u);
      p.tail = uni(hi - e0 < TILE ? (uint32_t)(hi > e0 ? hi - e0 : 0) : (uint32_t)TILE);
      p.voff = (loc + EPV <= p.head || loc >= p.tail) ? col_bytes : (uint32_t)((((uint64_t)p.e0 + loc) * S::kBitsPerElem) >> 3);
    } else {
      p.e0 = t * TILE;
      p.g_bytes = (uint32_t)(D * 4);                           // elements past D arrive as 0
      p.head = 0u;
      p.tail = (uint32_t)TILE;
      p.voff = (uint32_t)((((uint64_t)p.e0 + loc) * S::kBitsPerElem) >> 3);
    }
    return p;
  };

  float acc[SLOTS][KB];
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl)
#pragma unroll
    for (int c = 0; c < KB; ++c) acc[sl][c] = 0.0f;
  float gsum = 0.0f;                                           // min-max formats: the layer's sum of the gradient itself
  // one reduction over the wave's lanes, then the partial sums of row `slot_row`
  auto flush = [&](int slot_row) {
    if constexpr (kMinMax<DT>) {
      const float tot = wave_sum_to_last_lane(gsum);
      if (wave == 0 && lane == kSumLane) aux[slot_row] = tot;
      gsum = 0.0f;
    }
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
#pragma unroll
      for (int c = 0; c < KB; ++c) {
        const float tot = wave_sum_to_last_lane(acc[sl][c]);
        if (lane == kSumLane && sl < ncol) partial[((int64_t)slot_row * KB + c) * P.n + c0 + sl] = tot;
        acc[sl][c] = 0.0f;
      }
    }
  };

  float gs[KB][EPV];                                           // slice of g of the tile whose digits are formed next
  uint32_t gdig[KB][4][kFixDigits];
  float gunit[KB];
  // (`dead` = 0x80000000 puts every offset of a fetch outside its descriptor: a prefetch past the workgroup's last
  //  tile is issued like any other, returns zeros and moves no memory -- no branch in the pipeline)
  auto load_g = [&](const Place& p, uint32_t dead) {
    const uint32_t elem = (uint32_t)p.e0 + loc;
#pragma unroll
    for (int c = 0; c < KB; ++c) {
      const rsrc_t rg = make_rsrc(g + (int64_t)c * ldg, p.g_bytes);
#pragma unroll
      for (int q = 0; q < EPV / 4; ++q) {
        const u32x4 x = ld128(rg, ((elem + 4u * q) * 4u) | dead);    // shared by the 4 waves: keep it cacheable
#pragma unroll
        for (int r = 0; r < 4; ++r) gs[c][4 * q + r] = as_f32(x[r]);
      }
    }
  };
  // chunk ch of a tile: codes (and binary16 scale bits) of column slots [ch*U, (ch+1)*U)
  auto load_chunk = [&](const Place& p, int ch, uint32_t dead, u32x4 (&raw)[U], uint32_t (&sc)[U]) {
    rsrc_t rs = make_rsrc(g, 0u);
    if constexpr (S::kScaled) rs = make_rsrc(P.scales + (p.e0 >> kScaleSpanShift) * (int64_t)span_scale_bytes, span_scale_bytes);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int slot = ch * U + u;
      const bool valid = slot < ncol;
      const int col = valid ? c0 + slot : 0;
      const rsrc_t rc = make_rsrc(P.data + (int64_t)col * ld_bytes, valid ? col_bytes : 0u);
      raw[u] = load_codes<DT>(rc, p.voff | dead);
      if constexpr (S::kScaled) {
        // [vector][block in span]; an unused column slot reads far outside the range and gets 0
        const uint32_t soff = valid ? ((((uint32_t)col) << gshift) + (loc >> P.block_shift)) * (uint32_t)S::kScaleBytes : 0x7fffff00u;
        sc[u] = ld16(rs, soff | dead);
      } else {
        sc[u] = 0u;
      }
    }
  };
  auto compute_chunk = [&](int ch, const u32x4 (&raw)[U], const uint32_t (&sc)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int c = 0; c < KB; ++c) {
        const float d = (float)dot_codes_fixed<DT>(raw[u], gdig[c]) * gunit[c];
        if constexpr (S::kScaled) {
          const float scale = (float)__builtin_bit_cast(_Float16, (uint16_t)sc[u]) * P.gscale;
          acc[ch * U + u][c] = __builtin_fmaf(d, scale, acc[ch * U + u][c]);
        } else {
          acc[ch * U + u][c] += d;                              // min-max codes: a_l multiplies the finished sum
        }
      }
    }
  };
  // nothing may cross a fence: what consumes a load is a single XOR or mask, which the scheduler would otherwise
  // put, with its wait, right behind the load
  auto fence = [] { __builtin_amdgcn_sched_barrier(0); };

  LayerCursor lc{0, 0, 0, 0, 0};
  if constexpr (LAYERED) lc.load(plan, layer_of_tile(plan, t0));
  Place now = place(lc, t0);
  // Three code buffers: chunk 0 of a tile always sits in Z, chunks 1, 3, .. in X, chunks 2, 4, .. in Y, so that every
  // tile runs the same code (two buffers would change roles from tile to tile when NCH is odd, and the second copy
  // of the loop body costs the kernel its registers).  Z is free once chunk 0 is consumed: the next tile's chunk 0
  // is fetched into it while this tile's last chunk is consumed.
  u32x4 rawX[U], rawY[U], rawZ[U];
  uint32_t scX[U], scY[U], scZ[U];
  load_g(now, 0u);
  load_chunk(now, 0, 0u, rawZ, scZ);
  fence();
  for (int64_t t = t0; t < t1; ++t) {
    if constexpr (LAYERED) {
      if (now.head != 0) {                                      // first tile of a layer with an unaligned start
#pragma unroll
        for (int e = 0; e < EPV; ++e) gs[0][e] = loc + e >= now.head ? gs[0][e] : 0.0f;
      }
    }
    if constexpr (kMinMax<DT>) {
      float sum = 0.0f;
#pragma unroll
      for (int e = 0; e < EPV; ++e) sum += gs[0][e];
      gsum += sum;
    }
#pragma unroll
    for (int c = 0; c < KB; ++c) gunit[c] = fixed_point_digits<DT>(gs[c], gdig[c]);
    fence();
    // the next tile: its layer, its place, and whether the sums have to be handed over before it
    const bool more = t + 1 < t1;
    const uint32_t dead = more ? 0u : 0x80000000u;
    LayerCursor ln = lc;
    bool next_layer = false;
    if constexpr (LAYERED) {
      if (more && ln.behind(plan, t + 1)) {
        ln.seek(plan, t + 1);
        next_layer = true;
      }
    }
    const Place nxt = place(ln, more ? t + 1 : t);
    load_g(nxt, dead);                                          // gs is free: the digits are formed
    fence();
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      if (ch + 1 == NCH) load_chunk(nxt, 0, dead, rawZ, scZ);
      else if ((ch + 1) % 2 == 1) load_chunk(now, ch + 1, 0u, rawX, scX);
      else load_chunk(now, ch + 1, 0u, rawY, scY);
      fence();
      if (ch == 0) compute_chunk(ch, rawZ, scZ);
      else if (ch % 2 == 1) compute_chunk(ch, rawX, scX);
      else compute_chunk(ch, rawY, scY);
      fence();
    }
    if constexpr (LAYERED) {
      if (next_layer) flush((int)blockIdx.x + lc.cur);          // a workgroup never holds a layer without tiles
    }
    lc = ln;
    now = nxt;
  }
  flush(LAYERED ? (int)blockIdx.x + lc.cur : (int)blockIdx.x);
}

// S = P^T G for up to TWA_MAX_K gradients in ONE pass over P (up to 32 basis vectors per launch; not int4).
// The gradients are 44 % of the bytes at k = 8, n = 20, so they must not be fetched once per wave:
// the workgroup loads each tile of G once, coalesced, into a double-buffered LDS tile (the loads of
// tile t+1 are issued before tile t is consumed), and every wave reads its k slices from there.
// Columns are split over the 4 waves and streamed exactly as in project_kernel (VPL = 1).
template <int DT, int U, int NCH>
__global__ __launch_bounds__(256) void project_batched_kernel(PView P, const float* __restrict__ G, int64_t ldg,
                                                              int kvalid, float* __restrict__ partial, int cpw,
                                                              int tiles_per_wg, int col_begin, int col_end) {
  using S = Store<DT>;
  constexpr int KB = TWA_MAX_K;
  constexpr int EPV = S::kEPV;
  constexpr int TILE = kWave * EPV;
  constexpr int SLOTS = U * NCH;
  constexpr int F4 = TILE / 4;                       // 128-bit pieces per gradient and tile
  constexpr int NLD = KB * F4 / 256;                 // pieces each thread stages per tile
  static_assert(kScaleSpan % TILE == 0, "a tile lies inside one scale span");
  static_assert(F4 % kWave == 0 && (KB * F4) % 256 == 0, "staging pieces are wave-uniform in the gradient index");
  __shared__ float gl[2][KB][TILE];

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t D = P.D;
  const int64_t ntiles = (D + TILE - 1) / TILE;
  const int64_t t0 = (int64_t)blockIdx.x * tiles_per_wg;
  int64_t t1 = t0 + tiles_per_wg;
  if (t1 > ntiles) t1 = ntiles;

  // this launch serves the basis vectors [col_begin, col_end) (at most 32 of them: 4 waves x 8 slots)
  const int c0 = col_begin + wave * cpw;
  int ncol = col_end - c0;
  ncol = ncol < 0 ? 0 : (ncol > cpw ? cpw : ncol);
  const uint32_t col_bytes = stored_bytes<DT>(D);
  const int64_t ld_bytes = (P.ld * S::kBitsPerElem) >> 3;
  const int gshift = kScaleSpanShift - P.block_shift;
  const uint32_t span_scale_bytes = S::kScaled ? ((uint32_t)P.n << gshift) * (uint32_t)S::kScaleBytes : 0u;
  const uint32_t g_bytes = (uint32_t)(D * 4);

  // piece r of this thread: gradient (wave-uniform) and position inside the tile
  auto stage_load = [&](int64_t t, u32x4 (&pre)[NLD]) {
#pragma unroll
    for (int r = 0; r < NLD; ++r) {
      const int f = (int)threadIdx.x + 256 * r;
      const int c = __builtin_amdgcn_readfirstlane(f / F4);
      const int pos = f % F4;
      const rsrc_t rg = make_rsrc(G + (int64_t)c * ldg, c < kvalid ? g_bytes : 0u);   // past D and past k: zeros
      pre[r] = ld128(rg, ((uint32_t)(t * TILE) + 4u * (uint32_t)pos) * 4u);
    }
  };
  auto stage_store = [&](int buf, const u32x4 (&pre)[NLD]) {
#pragma unroll
    for (int r = 0; r < NLD; ++r) {
      const int f = (int)threadIdx.x + 256 * r;
      *reinterpret_cast<u32x4*>(&gl[buf][f / F4][4 * (f % F4)]) = pre[r];
    }
  };

  float acc[SLOTS][KB];
#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl)
#pragma unroll
    for (int c = 0; c < KB; ++c) acc[sl][c] = 0.0f;

  if (t0 < t1) {
    u32x4 pre[NLD];
    stage_load(t0, pre);
    stage_store(0, pre);
  }
  __syncthreads();

  for (int64_t t = t0; t < t1; ++t) {
    const int64_t e0 = t * TILE;
    const int cur = (int)(t - t0) & 1;
    const bool more = t + 1 < t1;                      // uniform
    u32x4 pre[NLD];
    if (more) stage_load(t + 1, pre);

    float gs[KB][EPV];
#pragma unroll
    for (int c = 0; c < KB; ++c)
#pragma unroll
      for (int q = 0; q < EPV / 4; ++q) {
        const float4 x = *reinterpret_cast<const float4*>(&gl[cur][c][lane * EPV + 4 * q]);
        gs[c][4 * q] = x.x; gs[c][4 * q + 1] = x.y; gs[c][4 * q + 2] = x.z; gs[c][4 * q + 3] = x.w;
      }

    rsrc_t rs = make_rsrc(G, 0u);
    if constexpr (S::kScaled)
      rs = make_rsrc(P.scales + (e0 >> kScaleSpanShift) * (int64_t)span_scale_bytes, span_scale_bytes);
    const uint32_t in_span = (uint32_t)e0 & (uint32_t)(kScaleSpan - 1);
    auto load_chunk = [&](int ch, u32x4 (&raw)[U], float (&sc)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int slot = ch * U + u;
        const bool valid = slot < ncol;
        const int col = valid ? c0 + slot : 0;
        const rsrc_t rc = make_rsrc(P.data + (int64_t)col * ld_bytes, valid ? col_bytes : 0u);
        const uint32_t loc = (uint32_t)lane * EPV;
        raw[u] = load_codes<DT>(rc, (uint32_t)((((uint64_t)e0 + loc) * S::kBitsPerElem) >> 3));
        if constexpr (S::kScaled) {
          const uint32_t soff = valid ? ((((uint32_t)col) << gshift) + ((in_span + loc) >> P.block_shift)) *
                                            (uint32_t)S::kScaleBytes
                                      : 0x7fffff00u;
          sc[u] = load_scale<DT>(rs, soff, P.gscale);
        } else {
          sc[u] = 1.0f;
        }
      }
    };
    auto compute_chunk = [&](int ch, const u32x4 (&raw)[U], const float (&sc)[U]) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int slot = ch * U + u;
        float x[EPV];
        decode<DT>(raw[u], x);
#pragma unroll
        for (int c = 0; c < KB; ++c) {
          if constexpr (S::kScaled) {
            float d = 0.0f;
#pragma unroll
            for (int e = 0; e < EPV; ++e) d = __builtin_fmaf(x[e], gs[c][e], d);
            acc[slot][c] = __builtin_fmaf(d, sc[u], acc[slot][c]);
          } else {
            float d = acc[slot][c];
#pragma unroll
            for (int e = 0; e < EPV; ++e) d = __builtin_fmaf(x[e], gs[c][e], d);
            acc[slot][c] = d;
          }
        }
      }
    };
    u32x4 rawA[U], rawB[U];
    float scA[U], scB[U];
    load_chunk(0, rawA, scA);
#pragma unroll
    for (int ch = 0; ch < NCH; ch += 2) {
      if (ch + 1 < NCH) load_chunk(ch + 1, rawB, scB);
      compute_chunk(ch, rawA, scA);
      if (ch + 2 < NCH) load_chunk(ch + 2, rawA, scA);
      if (ch + 1 < NCH) compute_chunk(ch + 1, rawB, scB);
    }

    if (more) stage_store(cur ^ 1, pre);
    __syncthreads();      // tile t+1 of G is in LDS; every wave is done reading tile t
  }

#pragma unroll
  for (int sl = 0; sl < SLOTS; ++sl) {
#pragma unroll
    for (int c = 0; c < KB; ++c) {
      const float tot = wave_sum_to_last_lane(acc[sl][c]);
      if (lane == kSumLane && sl < ncol && c < kvalid)
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

// Exact division of the tiles: every workgroup gets `tiles_per_wg` consecutive tiles.
static void divide_tiles(int64_t D, int tile, int max_grid, int* grid, int* tiles_per_wg) {
  const int64_t ntiles = (D + tile - 1) / tile;
  const int64_t per = (ntiles + max_grid - 1) / max_grid;
  *tiles_per_wg = (int)per;
  *grid = (int)((ntiles + per - 1) / per);
}

template <int DT, int KB, int VPL, bool LAYERED = false, bool SQUARES = false>
static int launch_project_dt(const PView& P, const float* g, int64_t ldg, int kvalid, float* partial, int max_grid,
                             int* grid_out, hipStream_t st, LayerPlan plan = LayerPlan{nullptr, nullptr, 1},
                             float* aux = nullptr) {
  const int cpw = (P.n + 3) / 4;
  constexpr int tile = kWave * VPL * Store<DT>::kEPV;
  int grid, tiles_per_wg;
  divide_tiles(P.D, tile, max_grid, &grid, &tiles_per_wg);
  if (LAYERED) grid = max_grid;      // the kernel divides the plan's tiles over the grid itself
  *grid_out = grid;
  // chunks of 4 column slots; 25 columns per wave (n = 97..100) divide exactly into 5 chunks of 5
#define TWA_LAUNCH(U_, NCH_)                                                                                  \
  do {                                                                                                        \
    if constexpr (kDotCodes<DT> && !SQUARES && (KB == 1 || (KB == 2 && !LAYERED)) && VPL == 1 && (NCH_) >= 2)   \
      hipLaunchKernelGGL((project_dot_kernel<DT, U_, NCH_, LAYERED, KB>), dim3(grid), dim3(256), 0, st, P, g,   \
                         ldg, partial, cpw, tiles_per_wg, plan, aux);                                         \
    else if constexpr (LAYERED)                                                                               \
      hipLaunchKernelGGL((project_layers_kernel<DT, U_, NCH_, VPL, SQUARES>), dim3(grid), dim3(256), 0, st, P, g, \
                         partial, cpw, plan, aux);                                                            \
    else if constexpr (NCH_ <= 4)                                                                             \
      hipLaunchKernelGGL((project_kernel_two_waves<DT, KB, U_, NCH_, VPL>), dim3(grid), dim3(256), 0, st, P, g, ldg, \
                         kvalid, partial, cpw, tiles_per_wg);                                                 \
    else                                                                                                      \
      hipLaunchKernelGGL((project_kernel<DT, KB, U_, NCH_, VPL>), dim3(grid), dim3(256), 0, st, P, g, ldg, kvalid, \
                         partial, cpw, tiles_per_wg);                                                         \
  } while (0)
  if constexpr (SQUARES) {
    // the slices of the two mean words take 32 registers more: chunks of 3 column slots keep the kernel
    // inside its register budget
    switch ((cpw + 2) / 3) {
      case 1: TWA_LAUNCH(3, 1); break;
      case 2: TWA_LAUNCH(3, 2); break;
      case 3: TWA_LAUNCH(3, 3); break;
      case 4: TWA_LAUNCH(3, 4); break;
      case 5: TWA_LAUNCH(3, 5); break;
      case 6: TWA_LAUNCH(3, 6); break;
      case 7: TWA_LAUNCH(3, 7); break;
      case 8: TWA_LAUNCH(3, 8); break;
      case 9: TWA_LAUNCH(3, 9); break;
      case 10: TWA_LAUNCH(3, 10); break;
      default: TWA_LAUNCH(3, 11); break;
    }
  } else {
    if (cpw == 25) {
      if constexpr (kDotCodes<DT> && KB == 2) TWA_LAUNCH(4, 7);      // (chunks of 5 do not fit the registers with two gradients)
      else TWA_LAUNCH(5, 5);
    } else {
      switch ((cpw + 3) / 4) {
        case 1:
          if constexpr (kDotCodes<DT> && !SQUARES && VPL == 1) TWA_LAUNCH(2, 2);   // (the pipelined kernel needs two chunks)
          else TWA_LAUNCH(4, 1);
          break;
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

// k == 1 path.  `partial` holds (at most max_grid)*n floats.
int launch_project(const PView& P, int dtype, const float* g, float* s, float* partial, int max_grid,
                   hipStream_t st) {
  int rc, grid = 0;
  switch (dtype) {
    case TWA_F32: rc = launch_project_dt<TWA_F32, 1, 4>(P, g, 0, 1, partial, max_grid, &grid, st); break;
    case TWA_BF16: rc = launch_project_dt<TWA_BF16, 1, 2>(P, g, 0, 1, partial, max_grid, &grid, st); break;
    case TWA_I8: rc = launch_project_dt<TWA_I8, 1, 2>(P, g, 0, 1, partial, max_grid, &grid, st); break;
    case TWA_I4: rc = launch_project_dt<TWA_I4, 1, 1>(P, g, 0, 1, partial, max_grid, &grid, st); break;
    default: return TWA_ERR_DTYPE;
  }
  if (rc != TWA_OK) return rc;
  hipLaunchKernelGGL(project_reduce_kernel, dim3(P.n), dim3(kWave), 0, st, partial, grid, P.n, s);
  return hip_check(hipGetLastError());
}

// What the layer-wise reduction does with a finished sum s: store it, and/or take the coefficient
// step of Alg. 1 with it, beta <- (1 - lr*lambda) beta - lr s ("update variables").
struct BetaStep {
  float* beta;          // NULL: no step
  float lr, lambda;
  __device__ __forceinline__ void finish(float* __restrict__ S, int64_t at, float s) const {
    if (S) S[at] = s;
    if (beta) beta[at] = __builtin_fmaf(-lr, s, (1.0f - lr * lambda) * beta[at]);
  }
};

// S[l][j] = sum of the partial slots (b + l) of the workgroups b that own tiles of layer l, accumulated
// in fp64 in a fixed order.  One block per layer; thread (q, j) adds the slots of every kRedWays-th
// workgroup for basis vector j (a long layer spans ~50 workgroups: one thread per vector alone would
// walk them one dependent load after the other), then the kRedWays sums are added in the order of q.
// The min-max formats (Sec. 4.6) finish with (P~^l)^T g^l = a_l * (C^l)^T g^l + (b_l + bias * a_l) * sum(g^l),
// where C holds the decoded codes (code - bias).
constexpr int kRedWays = 8;
template <bool MINMAX>
__global__ __launch_bounds__(TWA_MAX_N* kRedWays) void project_layers_reduce_kernel(
    const float* __restrict__ partial, const float* __restrict__ partial_g, int n, LayerPlan plan, int64_t D, int grid,
    const float* __restrict__ ab, float bias, float* __restrict__ S, BetaStep bs) {
  __shared__ double red[kRedWays][TWA_MAX_N];
  __shared__ double redg[kRedWays];
  const int l = blockIdx.x;
  const int j = threadIdx.x % TWA_MAX_N;
  const int q = threadIdx.x / TWA_MAX_N;
  if (!plan_header_ok(plan.off, plan.L, D)) {             // a plan of another layer table: no table is read
    if (q == 0 && j < n) bs.finish(S, (int64_t)l * n + j, __builtin_nanf(""));
    return;
  }
  const int ntiles = plan.first[plan.L];
  const int tiles_per_wg = ntiles > 0 ? (ntiles + grid - 1) / grid : 1;      // as in project_kernel
  const int32_t ta = plan.first[l], tb = plan.first[l + 1];                  // tiles [ta, tb)
  double a = 0.0, gs = 0.0;
  if (tb > ta && j < n) {
    const int b0 = ta / tiles_per_wg, b1 = (tb - 1) / tiles_per_wg;
    for (int b = b0 + q; b <= b1; b += kRedWays) {
      a += (double)partial[(int64_t)(b + l) * n + j];
      if (MINMAX && j == 0) gs += (double)partial_g[b + l];
    }
  }
  red[q][j] = a;
  if (MINMAX && j == 0) redg[q] = gs;
  __syncthreads();
  if (q != 0 || j >= n) return;
  double tot = 0.0, totg = 0.0;
#pragma unroll
  for (int r = 0; r < kRedWays; ++r) {
    tot += red[r][j];
    if (MINMAX) totg += redg[r];
  }
  if constexpr (MINMAX) {
    const double al = (double)ab[2 * l], bl = (double)ab[2 * l + 1];
    tot = al * tot + (bl + (double)bias * al) * totg;
  }
  bs.finish(S, (int64_t)l * n + j, (float)tot);
}

template <int DT, int VPL>
static int launch_project_layers_dt(const PView& P, const float* g, const void* plan_dev, int L, float* S,
                                    float* partial, int max_grid, hipStream_t st, BetaStep bs) {
  constexpr int tile = kWave * VPL * Store<DT>::kEPV;
  const LayerPlan plan = plan_view(plan_dev, L, tile);
  int grid = 0;
  float* partial_g = partial + ((size_t)kMaxGrid + (size_t)L) * P.n;        // min-max formats only
  int rc = launch_project_dt<DT, 1, VPL, true>(P, g, 0, 1, partial, max_grid, &grid, st, plan, partial_g);
  if (rc != TWA_OK) return rc;
  hipLaunchKernelGGL(project_layers_reduce_kernel<kMinMax<DT>>, dim3(L), dim3(TWA_MAX_N * kRedWays), 0, st, partial,
                     partial_g, P.n, plan, P.D, grid, reinterpret_cast<const float*>(P.scales),
                     kNibbles<DT> ? 8.0f : P.code_bias,   // (nibbles enter the dot products as code - 8)
                     S, bs);
  return hip_check(hipGetLastError());
}

// Per-layer squared norms of the centred vectors of an fp32 matrix:
// Q[l][j] = sum over layer l of ((P_ij - mean_hi_i) - mean_lo_i)^2.
int launch_layer_squares(const PView& P, const float* mean_hi, float* mean_lo, const void* plan_dev, int L, float* Q,
                         float* partial, int max_grid, hipStream_t st) {
  constexpr int tile = kWave * 4 * Store<TWA_F32>::kEPV;
  const LayerPlan plan = plan_view(plan_dev, L, tile);
  int grid = 0;
  int rc = launch_project_dt<TWA_F32, 1, 4, true, true>(P, mean_hi, 0, 1, partial, max_grid, &grid, st, plan, mean_lo);
  if (rc != TWA_OK) return rc;
  hipLaunchKernelGGL(project_layers_reduce_kernel<false>, dim3(L), dim3(TWA_MAX_N * kRedWays), 0, st, partial, nullptr,
                     P.n, plan, P.D, grid, nullptr, 0.0f, Q, BetaStep{nullptr, 0.0f, 0.0f});
  return hip_check(hipGetLastError());
}

// Layer-wise projection.  `partial` holds (max_grid + L) * (n + 1) floats.  S and/or beta (the fused
// coefficient step, beta <- (1 - lr*lambda) beta - lr s) receive the result.
int launch_project_layers(const PView& P, int dtype, const float* g, const void* plan_dev, int L, float* S,
                          float* beta, float lr, float lambda, float* partial, int max_grid, hipStream_t st) {
  const BetaStep bs{beta, lr, lambda};
  switch (dtype) {
    case TWA_F32: return launch_project_layers_dt<TWA_F32, 4>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_BF16: return launch_project_layers_dt<TWA_BF16, 2>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_I8: return launch_project_layers_dt<TWA_I8, 2>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_I4: return launch_project_layers_dt<TWA_I4, 1>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_U8MM: return launch_project_layers_dt<TWA_U8MM, 2>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_U4MM: return launch_project_layers_dt<TWA_U4MM, 1>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_U16MM: return launch_project_layers_dt<TWA_U16MM, 2>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_U2MM: return launch_project_layers_dt<TWA_U2MM, 1>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_U1MM: return launch_project_layers_dt<TWA_U1MM, 1>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    case TWA_U3MM: return launch_project_layers_dt<TWA_U3MM, 1>(P, g, plan_dev, L, S, partial, max_grid, st, bs);
    default: return TWA_ERR_DTYPE;
  }
}

// k > 1 gradients: one pass over P serves all k gradients (project_batched_kernel).  A launch takes up to 32
// basis vectors (4 waves x 8 column slots, k running sums each); a wider matrix is served in groups of 32 vectors,
// one launch each -- P is still read once in total, only the gradients are read once per group (n = 100, k = 8:
// 2.6 GB + 4 x 0.8 GB instead of the 8 x 2.7 GB of one launch per gradient).  The 4-bit codes are projected two
// gradients per pass (project_dot_kernel with KB = 2).
template <int DT>
static int launch_project_batched_dt(const PView& P, const float* g, int64_t ldg, int k, float* s, float* partial,
                                     int max_grid, hipStream_t st) {
  if constexpr (DT != TWA_I4) {
    int grid, tiles_per_wg;
    divide_tiles(P.D, kWave * Store<DT>::kEPV, max_grid, &grid, &tiles_per_wg);
    const int groups = (P.n + 31) / 32;
    const int per_group = (P.n + groups - 1) / groups;            // balanced: 100 vectors -> 4 x 25
    for (int col = 0; col < P.n; col += per_group) {
      const int col_end = col + per_group < P.n ? col + per_group : P.n;
      const int cpw = (col_end - col + 3) / 4;
#define TWA_LAUNCH_B(U_, NCH_)                                                                              \
  hipLaunchKernelGGL((project_batched_kernel<DT, U_, NCH_>), dim3(grid), dim3(256), 0, st, P, g, ldg, k, partial, \
                     cpw, tiles_per_wg, col, col_end)
      if (cpw <= 3) TWA_LAUNCH_B(3, 1);
      else if (cpw == 4) TWA_LAUNCH_B(4, 1);
      else if (cpw == 5) TWA_LAUNCH_B(5, 1);
      else if (cpw == 6) TWA_LAUNCH_B(3, 2);
      else TWA_LAUNCH_B(4, 2);
#undef TWA_LAUNCH_B
      int rc = hip_check(hipGetLastError());
      if (rc != TWA_OK) return rc;
    }
    hipLaunchKernelGGL(project_reduce_kernel, dim3(P.n * k), dim3(kWave), 0, st, partial, grid, P.n * k, s);
    return hip_check(hipGetLastError());
  }
  // the 4-bit codes: two gradients share a pass over P (their fixed-point digits take 50 registers together, which is
  // what the kernel has); an odd last one goes alone
  if constexpr (DT == TWA_I4) {
    const bool pairs = (P.n + 3) / 4 <= 28;       // (more than 28 basis vectors per wave: the pair kernel would spill)
    for (int c = 0; !pairs && c < k; ++c) {
      int rc = launch_project(P, DT, g + (int64_t)c * ldg, s + (int64_t)c * P.n, partial, max_grid, st);
      if (rc != TWA_OK) return rc;
    }
    if (!pairs) return TWA_OK;
    for (int c = 0; c + 1 < k; c += 2) {
      int grid = 0;
      int rc = launch_project_dt<TWA_I4, 2, 1>(P, g + (int64_t)c * ldg, ldg, 2, partial, max_grid, &grid, st);
      if (rc != TWA_OK) return rc;
      hipLaunchKernelGGL(project_reduce_kernel, dim3(P.n * 2), dim3(kWave), 0, st, partial, grid, P.n * 2,
                         s + (int64_t)c * P.n);
      rc = hip_check(hipGetLastError());
      if (rc != TWA_OK) return rc;
    }
    if (k & 1) return launch_project(P, DT, g + (int64_t)(k - 1) * ldg, s + (int64_t)(k - 1) * P.n, partial, max_grid, st);
  }
  return TWA_OK;
}

// ---- partial sums for callers that cannot allocate ------------------------------------------------
// The per-workgroup partial sums of a projection normally live in the caller's workspace.  For callers that
// cannot allocate one (code under stream capture, serving loops, harnesses that forbid it) the library
// keeps a fixed array in device memory: kNoAllocFloats floats per GPU, held until the process ends.  In host
// code the array's name is only a handle; its device address is asked for once per device (with that device
// current) and kept, and only that address is ever handed to a kernel.
constexpr size_t kNoAllocFloats = (size_t)kMaxGrid * TWA_NOALLOC_MAX_NK;         // 4 MiB
static __device__ __align__(256) float scratch[kNoAllocFloats];

int noalloc_partials(float** out, size_t* floats) {
  static std::mutex mu;
  static float* ptr[64] = {nullptr};
  int dev = 0;
  int rc = hip_check(hipGetDevice(&dev));
  if (rc != TWA_OK) return rc;
  if (dev < 0 || dev >= 64) return TWA_ERR_NO_DEVICE;
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    rc = hip_check(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (rc != TWA_OK) return rc;
    if (!p) return TWA_ERR_HIP;
    ptr[dev] = static_cast<float*>(p);
  }
  *out = ptr[dev];
  *floats = kNoAllocFloats;
  return TWA_OK;
}

int launch_project_batched(const PView& P, int dtype, const float* g, int64_t ldg, int k, float* s, float* partial,
                           int max_grid, hipStream_t st) {
  switch (dtype) {
    case TWA_F32: return launch_project_batched_dt<TWA_F32>(P, g, ldg, k, s, partial, max_grid, st);
    case TWA_BF16: return launch_project_batched_dt<TWA_BF16>(P, g, ldg, k, s, partial, max_grid, st);
    case TWA_I8: return launch_project_batched_dt<TWA_I8>(P, g, ldg, k, s, partial, max_grid, st);
    case TWA_I4: return launch_project_batched_dt<TWA_I4>(P, g, ldg, k, s, partial, max_grid, st);
    default: return TWA_ERR_DTYPE;
  }
}

}  // namespace twa
