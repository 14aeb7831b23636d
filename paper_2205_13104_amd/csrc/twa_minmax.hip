// The paper's own quantiser of the projection matrix (arXiv 2205.13104, Sec. 4.6): uniform min-max
// codes with ONE scaling and zero factor per layer, shared by all n basis vectors:
//     a_l = (max - min)/(2^B - 1),  b_l = min,  c = round((p - b_l)/a_l) in [0, 2^B - 1].
// One-time work in three small steps, each bound by one pass over the fp32 matrix or less:
//   1. layer_minmax_kernel   minimum and maximum of every layer over all vectors.  Workgroups walk
//      the per-layer tiles of the plan; a wave reduces what it saw of a layer and merges it with
//      integer atomics on an order-preserving key of the float (min and max do not depend on the
//      order, so the result is deterministic);
//   2. layer_factors_kernel  (a_l, b_l): binary32 for the stored matrix, a_l also in fp64 for step 3;
//   3. minmax_codes_kernel   the codes, in fp64 with ties to even like the definition's oracle
//      (a constant layer, a_l = 0, gets c = 0), packed into dwords.
#include <math.h>

#include "twa_device.h"
#include "twa_host.h"

namespace twa {

// order-preserving map float -> uint32 (larger float <=> larger key)
__device__ __forceinline__ uint32_t key_of(float f) {
  const uint32_t u = as_u32(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_of(uint32_t k) {
  return as_f32((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ __launch_bounds__(256) void minmax_init_kernel(uint32_t* __restrict__ keys, int L) {
  const int l = blockIdx.x * 256 + threadIdx.x;
  if (l < L) {
    keys[2 * l] = 0xffffffffu;        // running minimum
    keys[2 * l + 1] = 0u;             // running maximum
  }
}

// Tiles of 2048 elements: a thread owns 8 consecutive elements of the tile, for every vector.
__global__ __launch_bounds__(256) void layer_minmax_kernel(const float* __restrict__ P, int64_t D, int n, int64_t ldp,
                                                           LayerPlan plan, uint32_t* __restrict__ keys) {
  constexpr int TILE = 2048;
  if (!plan_header_ok(plan.off, plan.L, D)) return;      // not this call's plan: layer_factors_kernel answers with NaN
  const int ntiles = plan.first[plan.L];
  const int per = (ntiles + gridDim.x - 1) / gridDim.x;
  const int t0 = blockIdx.x * per;
  const int t1 = t0 + per < ntiles ? t0 + per : ntiles;
  if (t0 >= t1) return;
  const uint32_t bytes = (uint32_t)(D * 4);
  LayerCursor lc{0, 0, 0, 0, 0};
  lc.load(plan, layer_of_tile(plan, t0));
  float mn = INFINITY, mx = -INFINITY;
  auto merge = [&](int layer) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      mn = fminf(mn, __shfl_xor(mn, m, kWave));
      mx = fmaxf(mx, __shfl_xor(mx, m, kWave));
    }
    if ((threadIdx.x & (kWave - 1)) == 0 && mn <= mx) {
      atomicMin(&keys[2 * layer], key_of(mn));
      atomicMax(&keys[2 * layer + 1], key_of(mx));
    }
    mn = INFINITY;
    mx = -INFINITY;
  };
  for (int t = t0; t < t1; ++t) {
    if (lc.behind(plan, t)) {
      merge(lc.cur);
      lc.seek(plan, t);
    }
    const int64_t hi = lc.hi < D ? lc.hi : D;
    const int64_t i0 = lc.tile_start(t, TILE) + 8 * (int64_t)threadIdx.x;
    for (int j = 0; j < n; ++j) {
      const rsrc_t rc = make_rsrc(P + (int64_t)j * ldp, bytes);
      const u32x4 x0 = ld128_stream(rc, (uint32_t)i0 * 4u), x1 = ld128_stream(rc, (uint32_t)i0 * 4u + 16u);
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const float v = as_f32(r < 4 ? x0[r] : x1[r - 4]);
        if (i0 + r >= lc.lo && i0 + r < hi) {
          mn = fminf(mn, v);
          mx = fmaxf(mx, v);
        }
      }
    }
  }
  merge(lc.cur);
}

// ab[2l] = (float)a_l, ab[2l+1] = b_l; a64[l] = a_l in fp64 and ra64[l] = 1 / a_l (0 for a_l = 0).  An empty
// layer gets (0, 0).
__global__ __launch_bounds__(256) void layer_factors_kernel(const uint32_t* __restrict__ keys, int L, double levels,
                                                            float* __restrict__ ab, double* __restrict__ a64,
                                                            double* __restrict__ ra64, const int64_t* __restrict__ off,
                                                            int64_t D) {
  const int l = blockIdx.x * 256 + threadIdx.x;
  if (l >= L) return;
  if (!plan_header_ok(off, L, D)) {                      // a plan of another layer table: every factor says so
    ab[2 * l] = ab[2 * l + 1] = __builtin_nanf("");
    a64[l] = ra64[l] = __builtin_nan("");
    return;
  }
  const uint32_t kmin = keys[2 * l], kmax = keys[2 * l + 1];
  double a = 0.0;
  float b = 0.0f;
  if (kmin <= kmax) {                       // the layer has elements
    const float mn = float_of(kmin), mx = float_of(kmax);
    a = ((double)mx - (double)mn) / levels;
    b = mn;
  }
  ab[2 * l] = (float)a;
  ab[2 * l + 1] = b;
  a64[l] = a;
  ra64[l] = a > 0.0 ? 1.0 / a : 0.0;
}

// A thread packs WPT * EL consecutive elements of one vector into WPT dwords; a dword
// holds EL elements: 2 words or 4 bytes holding c - half (half = 2^(B-1): centred whatever B is), or 8
// nibbles, 16 two-bit or 32 one-bit codes c (element e of the dword at bit e * width).  The layer of the
// first element is found by bisection, once per thread and trip; after that the thread only watches for the
// next boundary.
template <int DT, int WPT>
__global__ __launch_bounds__(256) void minmax_codes_kernel(const float* __restrict__ P, int64_t D, int64_t ldp,
                                                           uint8_t* __restrict__ codes, int64_t ld,
                                                           const int64_t* __restrict__ off, int L,
                                                           const float* __restrict__ ab,
                                                           const double* __restrict__ a64,
                                                           const double* __restrict__ ra64, double levels,
                                                           uint32_t half) {
  constexpr int BITS = Store<DT>::kBitsPerElem;
  constexpr int EL = 32 / BITS;                 // elements per dword
  if (!plan_header_ok(off, L, D)) return;       // (the factors are NaN already; no table is read)
  const int j = blockIdx.y;
  const int64_t nquad = ld / (WPT * EL);        // groups of WPT dwords per vector (ld is a multiple of 2048)
  const float* p = P + (int64_t)j * ldp;
  uint32_t* out = reinterpret_cast<uint32_t*>(codes + (((int64_t)j * ld * BITS) >> 3));
  uint32_t pad = 0;                             // padding: code 0
  if constexpr (DT == TWA_U8MM) pad = ((0u - half) & 0xffu) * 0x01010101u;
  if constexpr (DT == TWA_U16MM) pad = ((0u - half) & 0xffffu) * 0x00010001u;
  for (int64_t quad = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; quad < nquad;
       quad += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i0 = quad * WPT * EL;
    uint32_t words[WPT];
#pragma unroll
    for (int w = 0; w < WPT; ++w) words[w] = pad;
    if (i0 < D) {
      int lo = 0, hi = L - 1;                   // largest l with off[l] <= i0
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (off[mid] <= i0) lo = mid; else hi = mid - 1;
      }
      int l = lo;
      int64_t next = l < L - 1 ? off[l + 1] : D;         // first element of the following layer
      double a = a64[l], ra = ra64[l], b = (double)ab[2 * l + 1];
#pragma unroll
      for (int w = 0; w < WPT; ++w) {
        uint32_t word = 0;
#pragma unroll
        for (int e4 = 0; e4 < EL; e4 += 4) {
          const int64_t i4 = i0 + w * EL + e4;
          float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
          if constexpr (EL >= 4) {
            if (i4 + 4 <= D) {
              const float4 t = *reinterpret_cast<const float4*>(p + i4);
              v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) v[r] = i4 + r < D ? p[i4 + r] : 0.0f;
            }
          } else {
#pragma unroll
            for (int r = 0; r < EL; ++r) v[r] = i4 + r < D ? p[i4 + r] : 0.0f;
          }
#pragma unroll
          for (int r = 0; r < (EL < 4 ? EL : 4); ++r) {
            const int64_t i = i4 + r;
            uint32_t c = 0;
            if (i < D) {
              if (i >= next) {                               // into the next layer that has elements
                while (l < L - 1 && off[l + 1] <= i) ++l;
                next = l < L - 1 ? off[l + 1] : D;
                a = a64[l];
                ra = ra64[l];
                b = (double)ab[2 * l + 1];
              }
              // c = rint((p - b) / a) with the quotient in fp64, as the definition says.  p - b is exact in
              // fp64; times 1/a it is within a few ulp (< 1e-10) of the quotient, so the two round to the same
              // integer unless the product lies that close to a tie; only then (a few elements in a million)
              // the quotient itself decides.
              const double t = (double)v[r] - b;
              const double x = t * ra;
              double q = rint(x);
              if (fabs(fabs(x - q) - 0.5) < 1e-6) q = rint(t / a);      // (a = 0: x = 0, q = 0, never here)
              q = q < 0.0 ? 0.0 : (q > levels ? levels : q);
              c = (uint32_t)q;
            }
            const int e = e4 + r;
            if constexpr (DT == TWA_U16MM) word |= ((c - half) & 0xffffu) << (16 * e);      // two's complement int16
            else if constexpr (DT == TWA_U8MM) word |= ((c - half) & 0xffu) << (8 * e);       // two's complement int8
            else word |= (c & ((1u << BITS) - 1u)) << (BITS * e);                            // low bits first
          }
        }
        words[w] = word;
      }
    }
    if constexpr (WPT == 4) {
      *reinterpret_cast<u32x4*>(out + 4 * quad) = u32x4{words[0], words[1], words[2], words[3]};
    } else {
#pragma unroll
      for (int w = 0; w < WPT; ++w) out[quad * WPT + w] = words[w];
    }
  }
}

// B = 3, packed exactly: a thread owns a group of 32 consecutive elements = three dwords.  Element
// e = 16h + 4k + m of the group has its two low bits in word h at bits 2(4k+m).., its high bit in word 2 at
// bit 8k + m + 4h (the layout the step kernels' decoder lines up with byte lanes).  Same arithmetic as above.
__global__ __launch_bounds__(256) void minmax_codes3_kernel(const float* __restrict__ P, int64_t D, int64_t ldp,
                                                            uint8_t* __restrict__ codes, int64_t ld,
                                                            const int64_t* __restrict__ off, int L,
                                                            const float* __restrict__ ab,
                                                            const double* __restrict__ a64,
                                                            const double* __restrict__ ra64, double levels) {
  if (!plan_header_ok(off, L, D)) return;       // (the factors are NaN already; no table is read)
  const int j = blockIdx.y;
  const int64_t ngroups = ld / 32;
  const float* p = P + (int64_t)j * ldp;
  uint32_t* out = reinterpret_cast<uint32_t*>(codes + (((int64_t)j * ld * 3) >> 3));
  for (int64_t grp = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; grp < ngroups;
       grp += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i0 = grp * 32;
    uint32_t w0 = 0, w1 = 0, w2 = 0;                 // padding: code 0
    if (i0 < D) {
      int lo = 0, hi = L - 1;                        // largest l with off[l] <= i0
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (off[mid] <= i0) lo = mid; else hi = mid - 1;
      }
      int l = lo;
      int64_t next = l < L - 1 ? off[l + 1] : D;
      double a = a64[l], ra = ra64[l], b = (double)ab[2 * l + 1];
#pragma unroll
      for (int e4 = 0; e4 < 32; e4 += 4) {
        const int64_t i4 = i0 + e4;
        float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (i4 + 4 <= D) {
          const float4 t = *reinterpret_cast<const float4*>(p + i4);
          v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        } else {
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = i4 + r < D ? p[i4 + r] : 0.0f;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int64_t i = i4 + r;
          uint32_t c = 0;
          if (i < D) {
            if (i >= next) {
              while (l < L - 1 && off[l + 1] <= i) ++l;
              next = l < L - 1 ? off[l + 1] : D;
              a = a64[l];
              ra = ra64[l];
              b = (double)ab[2 * l + 1];
            }
            const double t = (double)v[r] - b;
            const double x = t * ra;
            double q = rint(x);
            if (fabs(fabs(x - q) - 0.5) < 1e-6) q = rint(t / a);
            q = q < 0.0 ? 0.0 : (q > levels ? levels : q);
            c = (uint32_t)q;
          }
          const int e = e4 + r;                      // compile-time after unrolling
          const int h = e >> 4, f = e & 15, k = f >> 2, m = f & 3;
          if (h == 0) w0 |= (c & 3u) << (2 * f); else w1 |= (c & 3u) << (2 * f);
          w2 |= ((c >> 2) & 1u) << (8 * k + m + 4 * h);
        }
      }
    }
    out[3 * grp] = w0;
    out[3 * grp + 1] = w1;
    out[3 * grp + 2] = w2;
  }
}

size_t minmax_workspace_bytes(int L) { return (size_t)L * (2 * sizeof(uint32_t) + 2 * sizeof(double)); }

int launch_quantize_minmax(const float* P, int64_t D, int n, int64_t ldp, const void* plan_dev, int L, int dtype,
                           int bits, uint8_t* codes, int64_t ld, float* ab, void* ws, hipStream_t st) {
  double* a64 = static_cast<double*>(ws);                         // 8-byte aligned first
  double* ra64 = a64 + L;
  uint32_t* keys = reinterpret_cast<uint32_t*>(ra64 + L);
  const LayerPlan plan = plan_view(plan_dev, L, 2048);
  const double levels = (double)((1 << bits) - 1);              // codes 0 .. 2^B - 1, whatever the container
  const int lgrid = (L + 255) / 256;
  hipLaunchKernelGGL(minmax_init_kernel, dim3(lgrid), dim3(256), 0, st, keys, L);
  const int cus = device_cus();
  hipLaunchKernelGGL(layer_minmax_kernel, dim3(cus * 4), dim3(256), 0, st, P, D, n, ldp, plan, keys);
  hipLaunchKernelGGL(layer_factors_kernel, dim3(lgrid), dim3(256), 0, st, keys, L, levels, ab, a64, ra64, plan.off, D);
  const int el = dtype == TWA_U16MM ? 2 : dtype == TWA_U8MM ? 4 : dtype == TWA_U4MM ? 8 : dtype == TWA_U2MM ? 16 : 32;
  // dwords of codes a thread writes per trip, per container: measured at the ResNet-50 shape (code pass in ms
  // for 1 / 2 / 4 dwords: 16 bits 11.2 / 7.7 / 6.8, 8 bits 5.9 / 3.9 / 3.3, 4 bits 3.7 / 3.1 / 4.5,
  // 2 bits 3.0 / 4.5 / 4.4, 1 bit 4.5 / 4.3 / 3.9)
  const int wpt = dtype == TWA_U4MM ? 2 : dtype == TWA_U2MM ? 1 : 4;
  const int64_t ngroups = ld / (wpt * el);
  int gx = (int)((ngroups + 255) / 256);
  if (gx > cus * 8) gx = cus * 8;
#define TWA_CODES(DT_, WPT_)                                                                                       \
  hipLaunchKernelGGL((minmax_codes_kernel<DT_, WPT_>), dim3(gx, n), dim3(256), 0, st, P, D, ldp, codes, ld, plan.off, L, \
                     ab, a64, ra64, levels, 1u << (bits - 1))
  if (dtype == TWA_U3MM) {
    const int64_t ng = ld / 32;
    int g3 = (int)((ng + 255) / 256);
    if (g3 > cus * 8) g3 = cus * 8;
    hipLaunchKernelGGL(minmax_codes3_kernel, dim3(g3, n), dim3(256), 0, st, P, D, ldp, codes, ld, plan.off, L, ab, a64,
                       ra64, levels);
    return hip_check(hipGetLastError());
  }
  switch (dtype) {
    case TWA_U16MM: TWA_CODES(TWA_U16MM, 4); break;
    case TWA_U8MM: TWA_CODES(TWA_U8MM, 4); break;
    case TWA_U4MM: TWA_CODES(TWA_U4MM, 2); break;
    case TWA_U2MM: TWA_CODES(TWA_U2MM, 1); break;
    default: TWA_CODES(TWA_U1MM, 4); break;
  }
#undef TWA_CODES
  return hip_check(hipGetLastError());
}

}  // namespace twa
