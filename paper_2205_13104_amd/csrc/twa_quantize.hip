// Low-bit storage of the projection matrix (arXiv 2205.13104, Sec. 4.6: P is kept as B-bit
// integer codes plus scaling factors).  Grouping: symmetric absmax per block of `block`
// consecutive elements of one basis vector (the benchmark configuration's format); every step
// is a single correctly rounded binary32 operation, so codes and scales are unique bit for bit:
//     amax = max|p|, scale = amax / qmax, [I4: h = binary16(scale / gscale), e = float(h)*gscale]
//     inv = 1 / e,  q = clamp(rint(p * inv), -qmax, qmax)   (rint: ties to even)
// One-time work, bound by reading the fp32 matrix once.  A lane handles EL consecutive
// elements, the block's absmax is a shuffle reduction over block/EL lanes, and each lane
// writes one packed dword of codes, so reads and writes are fully coalesced.
#include <math.h>

#include "twa_device.h"
#include "twa_host.h"

namespace twa {

// max over groups of `lanes` consecutive lanes (lanes: power of two <= 64)
__device__ __forceinline__ float group_max(float x, int lanes) {
#pragma unroll
  for (int m = 1; m < kWave; m <<= 1)
    if (m < lanes) x = fmaxf(x, __shfl_xor(x, m, kWave));
  return x;
}

__device__ __forceinline__ int code_of(float p, float inv, float qmax) {
  float r = __builtin_rintf(p * inv);      // v_rndne_f32: round half to even
  r = fminf(fmaxf(r, -qmax), qmax);
  return (int)r;
}

// Each lane: EL = 4 (I8) or 8 (I4) consecutive fp32 elements -> one dword of codes.
template <int DT>
__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ P, int64_t D, int64_t ldp,
                                                       uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
                                                       int64_t ld, int block_shift, float gscale, float inv_gscale,
                                                       int n) {
  constexpr int EL = (DT == TWA_I8) ? 4 : 8;
  constexpr float QMAX = (DT == TWA_I8) ? 127.0f : 7.0f;
  const int j = blockIdx.y;
  const int lanes_per_block = (1 << block_shift) / EL;
  const int64_t nvec = ld / EL;                 // lane-vectors per basis vector (padding included)
  const int gshift = kScaleSpanShift - block_shift;      // log2(blocks per scale span)
  const float* p = P + (int64_t)j * ldp;
  uint32_t* out = reinterpret_cast<uint32_t*>(codes + (((int64_t)j * ld * Store<DT>::kBitsPerElem) >> 3));
  for (int64_t vec = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; vec < (nvec + kWave - 1) / kWave * kWave;
       vec += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i0 = vec * EL;
    float x[EL];
#pragma unroll
    for (int e = 0; e < EL; e += 4) {
      if (i0 + e + 4 <= D) {
        const float4 t = *reinterpret_cast<const float4*>(p + i0 + e);
        x[e] = t.x; x[e + 1] = t.y; x[e + 2] = t.z; x[e + 3] = t.w;
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) x[e + r] = (i0 + e + r < D) ? p[i0 + e + r] : 0.0f;
      }
    }
    float amax = 0.0f;
#pragma unroll
    for (int e = 0; e < EL; ++e) amax = fmaxf(amax, fabsf(x[e]));
    amax = group_max(amax, lanes_per_block);
    const float scale = amax / QMAX;
    float eff = scale;
    uint16_t hbits = 0;
    if constexpr (DT == TWA_I4) {
      const _Float16 h = (_Float16)(scale * inv_gscale);   // exact power-of-two scaling, then RNE to binary16
      hbits = __builtin_bit_cast(uint16_t, h);
      eff = (float)h * gscale;
    }
    const bool live = eff != 0.0f;
    const float inv = live ? 1.0f / eff : 0.0f;
    uint32_t word = 0;
    if constexpr (DT == TWA_I8) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int q = live ? code_of(x[e], inv, QMAX) : 0;
        word |= ((uint32_t)q & 0xffu) << (8 * e);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int q = live ? code_of(x[e], inv, QMAX) : 0;
        word |= ((uint32_t)(q + 8) & 0xfu) << (4 * e);
      }
    }
    if (vec < nvec) {
      out[vec] = word;
      if ((vec & (lanes_per_block - 1)) == 0) {
        // span-interleaved: the scales of one 2048-element span of all n vectors are contiguous
        const int64_t b = i0 >> block_shift;
        const int64_t idx = ((((b >> gshift) * n + j)) << gshift) + (b & (((int64_t)1 << gshift) - 1));
        if constexpr (DT == TWA_I8)
          reinterpret_cast<float*>(scales)[idx] = scale;
        else
          reinterpret_cast<uint16_t*>(scales)[idx] = hbits;
      }
    }
  }
}

// F32 copy / BF16 round-to-nearest-even, 4 elements per lane, padding zeroed.
template <int DT>
__global__ __launch_bounds__(256) void convert_kernel(const float* __restrict__ P, int64_t D, int64_t ldp,
                                                      uint8_t* __restrict__ dst, int64_t ld) {
  const int j = blockIdx.y;
  const float* p = P + (int64_t)j * ldp;
  const int64_t nvec = ld / 4;
  for (int64_t vec = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; vec < nvec;
       vec += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i0 = vec * 4;
    float x[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) x[r] = (i0 + r < D) ? p[i0 + r] : 0.0f;
    if constexpr (DT == TWA_F32) {
      float4 t = {x[0], x[1], x[2], x[3]};
      *reinterpret_cast<float4*>(reinterpret_cast<float*>(dst) + (int64_t)j * ld + i0) = t;
    } else {
      uint32_t h[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t u = as_u32(x[r]);
        if ((u & 0x7fffffffu) > 0x7f800000u) {
          h[r] = (u >> 16) | 0x40u;                       // keep NaN a NaN
        } else {
          const uint32_t keep = u >> 16, rem = u & 0xffffu;
          h[r] = keep + ((rem > 0x8000u || (rem == 0x8000u && (keep & 1u))) ? 1u : 0u);
        }
      }
      uint2 t = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
      *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(dst) + (int64_t)j * ld + i0) = t;
    }
  }
}

// Largest |p| over the logical elements, as the bit pattern of a non-negative float
// (unsigned order == float order), combined with an atomic max: order independent.
__global__ __launch_bounds__(256) void absmax_kernel(const float* __restrict__ P, int64_t D, int64_t ldp,
                                                     unsigned int* __restrict__ out) {
  const int j = blockIdx.y;
  const float* p = P + (int64_t)j * ldp;
  float m = 0.0f;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < D; i += (int64_t)gridDim.x * blockDim.x)
    m = fmaxf(m, fabsf(p[i]));
#pragma unroll
  for (int k = 32; k >= 1; k >>= 1) m = fmaxf(m, __shfl_xor(m, k, kWave));
  if ((threadIdx.x & (kWave - 1)) == 0) atomicMax(out, as_u32(m));
}

__global__ void zero_word_kernel(unsigned int* p) { *p = 0u; }

static int grid_x_for(int64_t work_items, int n) {
  int64_t gx = (work_items + 255) / 256;
  const int64_t cap = 4096 / (n > 0 ? n : 1) + 8;    // a few thousand workgroups in total
  if (gx > cap) gx = cap;
  if (gx < 1) gx = 1;
  return (int)gx;
}

int launch_absmax(const float* P, int64_t D, int n, int64_t ldp, float* out_dev, bool accumulate, hipStream_t st) {
  if (!accumulate)
    hipLaunchKernelGGL(zero_word_kernel, dim3(1), dim3(1), 0, st, reinterpret_cast<unsigned int*>(out_dev));
  hipLaunchKernelGGL(absmax_kernel, dim3(grid_x_for(D, n), n), dim3(256), 0, st, P, D, ldp,
                     reinterpret_cast<unsigned int*>(out_dev));
  return hip_check(hipGetLastError());
}

int launch_quantize(const float* P, int64_t D, int n, int64_t ldp, const twa_pmat& out, hipStream_t st) {
  int shift = 0;
  while ((1 << shift) < out.block) ++shift;
  uint8_t* data = static_cast<uint8_t*>(out.data);
  uint8_t* scales = static_cast<uint8_t*>(out.scales);
  switch (out.dtype) {
    case TWA_F32:
      hipLaunchKernelGGL((convert_kernel<TWA_F32>), dim3(grid_x_for(out.ld / 4, n), n), dim3(256), 0, st, P, D, ldp,
                         data, out.ld);
      break;
    case TWA_BF16:
      hipLaunchKernelGGL((convert_kernel<TWA_BF16>), dim3(grid_x_for(out.ld / 4, n), n), dim3(256), 0, st, P, D, ldp,
                         data, out.ld);
      break;
    case TWA_I8:
      hipLaunchKernelGGL((quantize_kernel<TWA_I8>), dim3(grid_x_for(out.ld / 4, n), n), dim3(256), 0, st, P, D, ldp,
                         data, scales, out.ld, shift, 1.0f, 1.0f, n);
      break;
    case TWA_I4:
      hipLaunchKernelGGL((quantize_kernel<TWA_I4>), dim3(grid_x_for(out.ld / 8, n), n), dim3(256), 0, st, P, D, ldp,
                         data, scales, out.ld, shift, out.gscale, 1.0f / out.gscale, n);
      break;
    default:
      return TWA_ERR_DTYPE;
  }
  return hip_check(hipGetLastError());
}

}  // namespace twa
