// Device-side helpers shared by the gfx950 kernels: buffer-descriptor loads/stores and the
// in-register decoding of the four storage types of the projection matrix.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/twa.h"

namespace twa {

using u32x4 = unsigned int __attribute__((ext_vector_type(4)));
using u32x2 = unsigned int __attribute__((ext_vector_type(2)));
using u32x3 = unsigned int __attribute__((ext_vector_type(3)));
using rsrc_t = __amdgpu_buffer_rsrc_t;

constexpr int kWave = 64;

// Scales of the integer formats are stored "span interleaved": the scales of the blocks that cover
// elements [kScaleSpan*t, kScaleSpan*(t+1)) of vector j are contiguous, at scale index
// (t*n + j)*(kScaleSpan/block) + r.  A kernel tile of kScaleSpan elements then finds the scales of
// all n vectors in one contiguous run (n * 64 B for block 128) instead of n separate 64-byte pieces.
constexpr int kScaleSpan = 2048;
constexpr int kScaleSpanShift = 11;

// Raw (stride 0) buffer descriptor over [base, base+bytes).  A load whose byte offset lies
// outside the range returns 0 and moves no data; a store outside it is dropped.  Every
// streaming access in the hot kernels goes through such a descriptor, so ragged tails and
// unused column slots need no branches: they are given an empty range.
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 ld128(rsrc_t r, uint32_t voff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
}
// Same, with the non-temporal hint: for data that is streamed once per kernel (the stored P).
// Measured on MI355X: a pure read stream reaches ~7.1 TB/s with the hint and ~6.3 TB/s without.
__device__ __forceinline__ u32x4 ld128_stream(rsrc_t r, uint32_t voff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, /*nt*/ 2);
}
__device__ __forceinline__ uint32_t ld32(rsrc_t r, uint32_t voff) {
  return __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, 0, 0);
}
__device__ __forceinline__ uint32_t ld16(rsrc_t r, uint32_t voff) {
  return (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)voff, 0, 0);
}
__device__ __forceinline__ void st128(rsrc_t r, uint32_t voff, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)voff, 0, 0);
}
// Store of the burst of w at the end of the expand kernel: written through to memory (sc0 sc1) instead
// of lingering dirty in L2, and marked non-temporal.  Measured with the step (projection + expansion)
// repeated at D = 25.6 M .. 350 M: lines left behind by plain or merely written-through stores slow the
// NEXT kernel down, by 1.5 % of the step at D = 25.6 M and by 10 % at D = 100 M.
__device__ __forceinline__ void st128_through_nt(rsrc_t r, uint32_t voff, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)voff, 0, /*sc0*/ 1 | /*nt*/ 2 | /*sc1*/ 16);
}
__device__ __forceinline__ void st32(rsrc_t r, uint32_t voff, uint32_t v) {
  __builtin_amdgcn_raw_buffer_store_b32(v, r, (int)voff, 0, 0);
}

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// Storage traits.  One "vector" is what a lane fetches with one 128-bit load.
template <int DT> struct Store;
template <> struct Store<TWA_F32> {
  static constexpr int kEPV = 4;          // elements per 128-bit vector
  static constexpr int kBitsPerElem = 32;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
template <> struct Store<TWA_BF16> {
  static constexpr int kEPV = 8;
  static constexpr int kBitsPerElem = 16;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
template <> struct Store<TWA_I8> {
  static constexpr int kEPV = 16;
  static constexpr int kBitsPerElem = 8;
  static constexpr bool kScaled = true;
  static constexpr int kScaleBytes = 4;
};
template <> struct Store<TWA_I4> {
  static constexpr int kEPV = 32;
  static constexpr int kBitsPerElem = 4;
  static constexpr bool kScaled = true;
  static constexpr int kScaleBytes = 2;
};

// The paper's own format: unsigned codes, one (a, b) pair per layer, no per-block scales.  The
// stored bytes are those of I8 (c - 128) and I4 (nibbles), so they share the decoders.
template <> struct Store<TWA_U8MM> {
  static constexpr int kEPV = 16;
  static constexpr int kBitsPerElem = 8;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
template <> struct Store<TWA_U4MM> {
  static constexpr int kEPV = 32;
  static constexpr int kBitsPerElem = 4;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
template <> struct Store<TWA_U16MM> {
  static constexpr int kEPV = 8;
  static constexpr int kBitsPerElem = 16;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
// Two and one bit per code: a lane still owns 32 consecutive elements (as with nibbles), which are 8 or 4
// bytes, fetched with a 64- or 32-bit load.
template <> struct Store<TWA_U2MM> {
  static constexpr int kEPV = 32;
  static constexpr int kBitsPerElem = 2;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
template <> struct Store<TWA_U1MM> {
  static constexpr int kEPV = 32;
  static constexpr int kBitsPerElem = 1;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
// Three bits per code, packed exactly: a lane's 32 elements are 12 bytes, fetched with a 96-bit load.
template <> struct Store<TWA_U3MM> {
  static constexpr int kEPV = 32;
  static constexpr int kBitsPerElem = 3;
  static constexpr bool kScaled = false;
  static constexpr int kScaleBytes = 0;
};
template <int DT>
constexpr bool kMinMax = DT == TWA_U8MM || DT == TWA_U4MM || DT == TWA_U16MM || DT == TWA_U2MM || DT == TWA_U1MM ||
                         DT == TWA_U3MM;
template <int DT> constexpr bool kNibbles = DT == TWA_I4 || DT == TWA_U4MM;
// (The byte and word containers of the min-max formats hold c - 2^(B-1) for B-bit codes c: centred
// whatever B is, so that the fused dequantisation does not lose bits to cancellation.  The bias travels
// in the view, PView::code_bias.  Nibbles and narrower hold c itself.)

// Decode one 128-bit vector into kEPV "raw" floats: the stored value up to the per-block
// scale, and for I4 up to the bias and nibble position:
//   F32, BF16 : raw = value
//   I8        : raw = q
//   I4        : raw[e] = (q+8) for even e, 16*(q+8) for odd e   (elements e = 2*byte, 2*byte+1)
// Callers fold the 1/16 and the -8 into per-tile / per-block terms instead of per element.  (The expansion decodes
// nibbles this way; the projection takes them as integers, see twa_project.hip.)
template <int DT> __device__ __forceinline__ void decode(const u32x4& v, float* raw);

template <> __device__ __forceinline__ void decode<TWA_F32>(const u32x4& v, float* raw) {
#pragma unroll
  for (int q = 0; q < 4; ++q) raw[q] = as_f32(v[q]);
}
template <> __device__ __forceinline__ void decode<TWA_BF16>(const u32x4& v, float* raw) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    raw[2 * q] = as_f32(v[q] << 16);
    raw[2 * q + 1] = as_f32(v[q] & 0xffff0000u);
  }
}
template <> __device__ __forceinline__ void decode<TWA_I8>(const u32x4& v, float* raw) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const uint32_t w = v[q];
    raw[4 * q + 0] = (float)(int8_t)(w & 0xff);          // one sign-extending byte convert each
    raw[4 * q + 1] = (float)(int8_t)((w >> 8) & 0xff);
    raw[4 * q + 2] = (float)(int8_t)((w >> 16) & 0xff);
    raw[4 * q + 3] = (float)(int8_t)(w >> 24);
  }
}
template <> __device__ __forceinline__ void decode<TWA_I4>(const u32x4& v, float* raw) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    uint32_t lo = v[q] & 0x0f0f0f0fu;                     // even elements: q+8
    uint32_t hi = v[q] & 0xf0f0f0f0u;                     // odd elements: 16*(q+8)
    // keep the two masked words as they are: otherwise the optimiser re-derives every nibble
    // from v[q] with a bit-field extract of its own (3 instructions per element instead of 2)
    asm volatile("" : "+v"(lo), "+v"(hi));
    raw[8 * q + 0] = (float)(lo & 0xff);
    raw[8 * q + 1] = (float)(hi & 0xff);
    raw[8 * q + 2] = (float)((lo >> 8) & 0xff);
    raw[8 * q + 3] = (float)((hi >> 8) & 0xff);
    raw[8 * q + 4] = (float)((lo >> 16) & 0xff);
    raw[8 * q + 5] = (float)((hi >> 16) & 0xff);
    raw[8 * q + 6] = (float)(lo >> 24);
    raw[8 * q + 7] = (float)(hi >> 24);
  }
}

template <> __device__ __forceinline__ void decode<TWA_U8MM>(const u32x4& v, float* raw) { decode<TWA_I8>(v, raw); }
template <> __device__ __forceinline__ void decode<TWA_U4MM>(const u32x4& v, float* raw) { decode<TWA_I4>(v, raw); }
template <> __device__ __forceinline__ void decode<TWA_U16MM>(const u32x4& v, float* raw) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    raw[2 * q] = (float)(int16_t)(v[q] & 0xffffu);          // sign-extending converts of the two halves
    raw[2 * q + 1] = (float)((int32_t)v[q] >> 16);
  }
}

// B = 2: byte k of (w >> 2m) & 0x03030303 is element 4k + m of the 16 a dword holds.
template <> __device__ __forceinline__ void decode<TWA_U2MM>(const u32x4& v, float* raw) {
#pragma unroll
  for (int q = 0; q < 2; ++q) {
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      uint32_t t = (v[q] >> (2 * m)) & 0x03030303u;
      asm volatile("" : "+v"(t));                          // keep the masked word: one byte convert per element
      raw[16 * q + 0 + m] = (float)(t & 0xff);
      raw[16 * q + 4 + m] = (float)((t >> 8) & 0xff);
      raw[16 * q + 8 + m] = (float)((t >> 16) & 0xff);
      raw[16 * q + 12 + m] = (float)(t >> 24);
    }
  }
}
// B = 1: byte k of (w >> m) & 0x01010101 is element 8k + m of the 32 a dword holds.
template <> __device__ __forceinline__ void decode<TWA_U1MM>(const u32x4& v, float* raw) {
#pragma unroll
  for (int m = 0; m < 8; ++m) {
    uint32_t t = (v[0] >> m) & 0x01010101u;
    asm volatile("" : "+v"(t));
    raw[0 + m] = (float)(t & 0xff);
    raw[8 + m] = (float)((t >> 8) & 0xff);
    raw[16 + m] = (float)((t >> 16) & 0xff);
    raw[24 + m] = (float)(t >> 24);
  }
}

// B = 3: words 0 and 1 hold the low two bits like U2MM, word 2 the high bits, placed so that
// (w2 >> (m + 4h)) & 0x01010101 has the high bit of element 16h + 4k + m in byte k -- the element whose low
// part (w_h >> 2m) & 0x03030303 has in byte k.
template <> __device__ __forceinline__ void decode<TWA_U3MM>(const u32x4& v, float* raw) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const uint32_t hi = (v[2] >> (m + 4 * h)) & 0x01010101u;
      uint32_t t = ((v[h] >> (2 * m)) & 0x03030303u) | (hi << 2);
      asm volatile("" : "+v"(t));                          // keep the combined word: one byte convert per element
      raw[16 * h + 0 + m] = (float)(t & 0xff);
      raw[16 * h + 4 + m] = (float)((t >> 8) & 0xff);
      raw[16 * h + 8 + m] = (float)((t >> 16) & 0xff);
      raw[16 * h + 12 + m] = (float)(t >> 24);
    }
  }
}

// Bytes of a stored vector that hold its first `elems` elements, rounded up to whole dwords (the range check of a
// descriptor drops a dword that is only partly inside).  The 3-bit type is packed in groups of 32 elements whose
// third word carries a bit of every element of the group: whole groups.
template <int DT> __device__ __forceinline__ uint32_t stored_bytes(int64_t elems) {
  if constexpr (DT == TWA_U3MM) return (uint32_t)(((elems + 31) >> 5) * 12);
  return (uint32_t)((((elems * Store<DT>::kBitsPerElem + 7) >> 3) + 3) & ~(int64_t)3);
}

// The kEPV stored elements of one lane, streamed: 128 bits for most types, 64 or 32 for the 2- and 1-bit
// codes (the unused words of the result are zero and never read).
template <int DT> __device__ __forceinline__ u32x4 load_codes(rsrc_t r, uint32_t voff) {
  constexpr int kBits = Store<DT>::kEPV * Store<DT>::kBitsPerElem;
  static_assert(kBits == 128 || kBits == 96 || kBits == 64 || kBits == 32, "a lane's elements are one load");
  if constexpr (kBits == 128) {
    return ld128_stream(r, voff);
  } else if constexpr (kBits == 96) {
    const u32x3 t = __builtin_amdgcn_raw_buffer_load_b96(r, (int)voff, 0, /*nt*/ 2);
    return u32x4{t[0], t[1], t[2], 0u};
  } else if constexpr (kBits == 64) {
    const u32x2 t = __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, 0, /*nt*/ 2);
    return u32x4{t[0], t[1], 0u, 0u};
  } else {
    return u32x4{__builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, 0, /*nt*/ 2), 0u, 0u, 0u};
  }
}

// Scale of one block as a float (binary16 scales are widened and multiplied by gscale).
template <int DT> __device__ __forceinline__ float load_scale(rsrc_t r, uint32_t voff, float gscale) {
  if constexpr (DT == TWA_I8) {
    return as_f32(ld32(r, voff));
  } else if constexpr (DT == TWA_I4) {
    const uint16_t h = (uint16_t)ld16(r, voff);
    return (float)__builtin_bit_cast(_Float16, h) * gscale;
  } else {
    return 1.0f;
  }
}

// Sum over the 64 lanes of a wave with data-parallel-primitive adds instead of cross-lane shuffles
// (no LDS traffic, a few cycles per step): an inclusive scan inside each row of 16 lanes (row_shr 1, 2, 4, 8; lanes
// without a source add 0), then row_bcast:15 hands each row total to the next row (rows 1 and 3)
// and row_bcast:31 hands the total of the first half to the second.  LANE 63 ends with the sum of
// all 64 lanes; the other lanes hold partial sums.  Fixed order: identical bits on every call.
constexpr int kSumLane = 63;
__device__ __forceinline__ float wave_sum_to_last_lane(float x) {
#define TWA_DPP_ADD(ctrl, rows)                                                                              \
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), ctrl, rows, 0xf, false))
  TWA_DPP_ADD(0x111, 0xf);
  TWA_DPP_ADD(0x112, 0xf);
  TWA_DPP_ADD(0x114, 0xf);
  TWA_DPP_ADD(0x118, 0xf);
  TWA_DPP_ADD(0x142, 0xa);
  TWA_DPP_ADD(0x143, 0xc);
#undef TWA_DPP_ADD
  return x;
}
// Sum of a double over the 64 lanes, same order on every call; result valid in every lane.
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, kWave);
  return x;
}

// View of a stored matrix passed to kernels by value.
struct PView {
  const uint8_t* data;
  const uint8_t* scales;
  int64_t D;
  int64_t ld;
  int32_t n;
  int32_t block_shift;   // log2(block)
  float gscale;
  float code_bias;       // TWA_U8MM, TWA_U16MM: 2^(B-1), what the stored integer lacks of the code; else 0
};

// Layer-wise processing (Sec. 4.5): the tiles of the step kernels are cut per layer.  Layer l =
// elements [off[l], off[l+1]) is covered by tiles of T elements that start at its first element
// rounded down to kLayerAlign, so a tile belongs to one layer; the elements of a tile that lie
// outside its layer (before the start in the layer's first tile, past the end in its last) are
// masked.  first[l] = index of the first tile of layer l in the global numbering, first[L] = the
// number of tiles.  The plan is built on the device from the caller's offsets, which it clamps into
// a non-decreasing table inside [0, D]: the kernels can trust it.
constexpr int kLayerAlign = 2048;        // elements (= kScaleSpan = the larger tile): the tiles stay on the grid of
                                         // the whole-model kernels, so loads stay aligned to memory lines and a
                                         // tile's scales stay one contiguous run; a grid cell that holds a layer
                                         // boundary simply is a tile of each layer it meets
struct LayerPlan {
  const int64_t* off;      // L+1 clamped offsets
  const int32_t* first;    // L+1 tile indices for the tile size of the kernel at hand
  int32_t L;
};
// The plan buffer starts with a 16-byte header {magic, L, D (64 bit)} written by the kernel that builds the
// plan; off[] follows it directly.  A caller may hand a step call a plan that was built for another layer
// count or vector length (the host cannot see into device memory): every kernel that reads plan tables
// compares the header with its own L and D FIRST and, on a mismatch, reads no table at all and poisons its
// output with NaN instead (the tables would be read at the wrong places, and tile counts taken from there
// could carry stores out of the workspace).
constexpr uint32_t kPlanMagic = 0x50415754u;
constexpr int kPlanHeaderBytes = 16;
__device__ __forceinline__ bool plan_header_ok(const int64_t* off, int L, int64_t D) {
  const int32_t* h = reinterpret_cast<const int32_t*>(off) - kPlanHeaderBytes / 4;
  return (uint32_t)h[0] == kPlanMagic && h[1] == L && *reinterpret_cast<const int64_t*>(h + 2) == D;
}
// The plan tables are written by an earlier launch, never by the kernels that walk them, and every lane reads the
// same entry: they are fetched as constants, i.e. through the scalar cache.  As ordinary global loads they went
// through the vector memory path, and waiting for one meant waiting for every load the wave had in flight (the
// counter is in order) -- which drains a pipelined stream at every look at the plan.
template <typename T> __device__ __forceinline__ T ld_plan(const T* p) {
  return *(const __attribute__((address_space(4))) T*)(p);
}
// Largest l in [0, L-1] with first[l] <= t: the layer that owns tile t (empty layers own none).
__device__ __forceinline__ int layer_of_tile(const LayerPlan& plan, int64_t t) {
  int a = 0, b = plan.L - 1;
  while (a < b) {
    const int mid = (a + b + 1) >> 1;
    if (ld_plan(plan.first + mid) <= t) a = mid; else b = mid - 1;
  }
  return a;
}

// Cursor over the layers for a walk through increasing tile indices.  The layer's numbers are kept in
// registers and re-read only when the walk enters another layer, so finding a tile's place costs
// no memory access (a dependent scalar load in front of every tile cost 5 % of the projection).
struct LayerCursor {
  int cur;
  int32_t first_cur, first_next;     // tiles [first_cur, first_next) belong to layer cur
  int64_t lo, hi;                    // its elements
  __device__ __forceinline__ void load(const LayerPlan& plan, int l) {
    cur = l;
    first_cur = ld_plan(plan.first + l);
    first_next = ld_plan(plan.first + l + 1);
    lo = ld_plan(plan.off + l);
    hi = ld_plan(plan.off + l + 1);
  }
  // true if tile t lies in a later layer than the cursor (the caller may want to act before moving on)
  __device__ __forceinline__ bool behind(const LayerPlan& plan, int64_t t) const {
    return cur < plan.L - 1 && first_next <= t;
  }
  __device__ __forceinline__ void seek(const LayerPlan& plan, int64_t t) {
    while (behind(plan, t)) load(plan, cur + 1);
  }
  // first element of tile t of the cursor's layer
  __device__ __forceinline__ int64_t tile_start(int64_t t, int tile) const {
    return (lo & ~(int64_t)(kLayerAlign - 1)) + (t - first_cur) * tile;
  }
};

// Balanced split of `total` units over `parts` workers: worker w owns [lo, hi).
__device__ __forceinline__ void split_range(int64_t total, int parts, int w, int64_t& lo, int64_t& hi) {
  lo = total * (int64_t)w / parts;
  hi = total * (int64_t)(w + 1) / parts;
}

// Wave-local ordering of LDS traffic: every lane's earlier LDS writes are visible to every lane's
// later LDS reads of the same wave (no workgroup barrier: waves run different trip counts).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace twa
