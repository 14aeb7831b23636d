// Plan of the layer-wise step (arXiv 2205.13104, Sec. 4.5: one block of the basis and one set of
// coefficients per layer).  The step kernels cut their tiles per layer, so that a tile never meets
// two layers and the stream over P stays the branch-free one of the whole-model step; this file
// turns the caller's table of layer offsets into what those kernels need:
//   header          {magic, L, D}: 16 bytes the step kernels compare with their own arguments
//   off[L+1]        the offsets, clamped into a non-decreasing table with off[0] = 0, off[L] = D
//   first2048[L+1]  index of the first tile of every layer for tiles of 2048 elements
//   first1024[L+1]  the same for tiles of 1024 elements
// Layer l = [off[l], off[l+1]) is covered by tiles that start at off[l] rounded down to
// kLayerAlign elements; an empty layer has no tile.
#include "twa_device.h"
#include "twa_host.h"

namespace twa {

constexpr int kPlanThreads = 256;

__device__ __forceinline__ int32_t tiles_of(int64_t lo, int64_t hi, int tile) {
  if (hi <= lo) return 0;
  const int64_t a = lo & ~(int64_t)(kLayerAlign - 1);
  return (int32_t)((hi - a + tile - 1) / tile);
}

// One workgroup.  Thread i owns the chunk of consecutive layers [i*chunk, (i+1)*chunk).
__global__ __launch_bounds__(kPlanThreads) void layer_plan_kernel(const int64_t* __restrict__ layer_off, int L, int64_t D,
                                                                  int64_t* __restrict__ off, int32_t* __restrict__ f2048,
                                                                  int32_t* __restrict__ f1024) {
  __shared__ int64_t s_max[kPlanThreads];
  __shared__ int32_t s_a[kPlanThreads], s_b[kPlanThreads];
  const int i = threadIdx.x;
  if (i == 0) {                                        // the header the step kernels check (see plan_header_ok)
    int32_t* h = reinterpret_cast<int32_t*>(off) - kPlanHeaderBytes / 4;
    h[0] = (int32_t)kPlanMagic;
    h[1] = L;
    *reinterpret_cast<int64_t*>(h + 2) = D;
  }
  const int chunk = (L + 1 + kPlanThreads - 1) / kPlanThreads;
  const int q0 = i * chunk;
  const int q1 = q0 + chunk < L + 1 ? q0 + chunk : L + 1;

  // ---- offsets: running maximum of the values clamped to [0, D]; ends pinned to 0 and D ----------
  auto clamped = [&](int q) -> int64_t {
    if (q == 0) return 0;
    if (q == L) return D;
    const int64_t v = layer_off[q];
    return v < 0 ? 0 : (v > D ? D : v);
  };
  int64_t m = 0;
  for (int q = q0; q < q1; ++q) { const int64_t v = clamped(q); m = v > m ? v : m; }
  s_max[i] = m;
  __syncthreads();
  int64_t run = 0;                                   // maximum over the chunks before this one
  for (int k = 0; k < i; ++k) run = s_max[k] > run ? s_max[k] : run;
  for (int q = q0; q < q1; ++q) {
    const int64_t v = clamped(q);
    run = v > run ? v : run;
    off[q] = q == L ? D : run;                       // (run <= D always)
  }
  __threadfence_block();
  __syncthreads();

  // ---- tiles per layer, exclusive prefix sums ------------------------------------------------------
  int32_t a = 0, b = 0;
  for (int q = q0; q < q1 && q < L; ++q) {
    a += tiles_of(off[q], off[q + 1], 2048);
    b += tiles_of(off[q], off[q + 1], 1024);
  }
  s_a[i] = a;
  s_b[i] = b;
  __syncthreads();
  int32_t pa = 0, pb = 0;
  for (int k = 0; k < i; ++k) { pa += s_a[k]; pb += s_b[k]; }
  for (int q = q0; q < q1; ++q) {
    f2048[q] = pa;
    f1024[q] = pb;
    if (q < L) {
      pa += tiles_of(off[q], off[q + 1], 2048);
      pb += tiles_of(off[q], off[q + 1], 1024);
    }
  }
}

size_t layer_plan_bytes(int L) { return kPlanHeaderBytes + (size_t)(L + 1) * (sizeof(int64_t) + 2 * sizeof(int32_t)); }

LayerPlan plan_view(const void* plan_dev, int L, int tile) {
  const int64_t* off = reinterpret_cast<const int64_t*>(static_cast<const uint8_t*>(plan_dev) + kPlanHeaderBytes);
  const int32_t* f2048 = reinterpret_cast<const int32_t*>(off + L + 1);
  const int32_t* f1024 = f2048 + L + 1;
  return LayerPlan{off, tile == 2048 ? f2048 : f1024, L};
}

int launch_layer_plan(const int64_t* layer_off, int L, int64_t D, void* plan_dev, hipStream_t st) {
  int64_t* off = reinterpret_cast<int64_t*>(static_cast<uint8_t*>(plan_dev) + kPlanHeaderBytes);
  int32_t* f2048 = reinterpret_cast<int32_t*>(off + L + 1);
  int32_t* f1024 = f2048 + L + 1;
  hipLaunchKernelGGL(layer_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, layer_off, L, D, off, f2048, f1024);
  return hip_check(hipGetLastError());
}

// Measurement aid: one plain pass of non-temporal 128-bit reads over a buffer, 64 KB per workgroup in the
// order of the workgroup index -- the read ceiling of the device a benchmark runs on.  The XOR of the
// words read goes to `sink` only if it has one improbable value, so the loads cannot be dropped.
__global__ __launch_bounds__(256) void read_probe_kernel(const u32x4* __restrict__ p, int64_t nvec, uint32_t* sink) {
  constexpr int64_t kPer = 65536 / 16;                     // 128-bit words per workgroup
  const int64_t v0 = (int64_t)blockIdx.x * kPer;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int64_t i = v0 + threadIdx.x; i < v0 + kPer && i < nvec; i += 256) acc ^= __builtin_nontemporal_load(p + i);
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) *sink = 1u;
}

int launch_read_probe(const void* buf, size_t bytes, uint32_t* sink, hipStream_t st) {
  const int64_t nvec = (int64_t)(bytes / 16);
  const int64_t grid = (nvec + 4095) / 4096;
  hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)grid), dim3(256), 0, st, static_cast<const u32x4*>(buf), nvec,
                     sink);
  return hip_check(hipGetLastError());
}

}  // namespace twa
