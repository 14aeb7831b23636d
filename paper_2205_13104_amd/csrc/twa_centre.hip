// The paper's default basis (arXiv 2205.13104, Sec. 4.1, the extraction of base vectors, and
// Sec. 4.5, its layer-wise form; Alg. 1, first steps):
//   wbar = (1/n) sum_j w_j ,   e_j^l = (w_j^l - wbar^l) / || w_j^l - wbar^l ||_2 .
// One-time work that is bound by a few passes over the n x D checkpoint matrix:
//   1. mean_kernel          reads W, writes wbar (the sum is kept in fp64; besides the fp32 mean its
//                           rounding error is kept too, so that the later steps subtract the mean to
//                           almost fp64 accuracy: layers that hardly move between checkpoints have
//                           |w_j - wbar| << |wbar| and would otherwise lose most of their digits);
//   2. the per-layer squared norms of c = (W - wbar_hi) - wbar_lo, centred in registers (the layer-wise
//      projection kernel in its squares mode);
//   3. rinv_kernel          1/norm per (layer, vector), 0 for a zero vector; the norms if wanted;
//   4. centre_scale_kernel  E_ij = c_ij * 1/norm of (layer of i, j), zero padding; may run in place.
// W is read three times and E written once; the centred matrix is never stored unscaled.
#include "twa_device.h"
#include "twa_host.h"

namespace twa {

constexpr int kEltThreads = 256;

// 4 consecutive elements per thread; `grid` workgroups stride over the D elements.
__global__ __launch_bounds__(kEltThreads) void mean_kernel(const float* __restrict__ W, int64_t D, int n, int64_t ldw,
                                                           float* __restrict__ wbar, float* __restrict__ wbar_lo) {
  const uint32_t bytes = (uint32_t)(D * 4);
  const rsrc_t ro = make_rsrc(wbar, bytes), rl = make_rsrc(wbar_lo, bytes);
  const int64_t nvec = (D + 3) / 4;
  for (int64_t q = (int64_t)blockIdx.x * kEltThreads + threadIdx.x; q < nvec; q += (int64_t)gridDim.x * kEltThreads) {
    double a[4] = {0.0, 0.0, 0.0, 0.0};
    for (int j = 0; j < n; ++j) {
      const u32x4 x = ld128_stream(make_rsrc(W + (int64_t)j * ldw, bytes), (uint32_t)q * 16u);   // past D: zeros
#pragma unroll
      for (int r = 0; r < 4; ++r) a[r] += (double)as_f32(x[r]);
    }
    u32x4 hi, lo;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const double m = a[r] / (double)n;
      const float h = (float)m;
      hi[r] = as_u32(h);
      lo[r] = as_u32((float)(m - (double)h));
    }
    // a 128-bit store is range-checked dword by dword: the ragged end is cut off
    st128(ro, (uint32_t)q * 16u, hi);
    st128(rl, (uint32_t)q * 16u, lo);
  }
}

// rinv[l][j] = 1/sqrt(Q[l][j]) (0 where Q is 0); norms[l][j] = sqrt(Q[l][j]) if wanted.
__global__ __launch_bounds__(kEltThreads) void rinv_kernel(const float* __restrict__ Q, int64_t count,
                                                           float* __restrict__ rinv, float* __restrict__ norms) {
  const int64_t q = (int64_t)blockIdx.x * kEltThreads + threadIdx.x;
  if (q >= count) return;
  const double v = (double)Q[q];
  const double r = sqrt(v);
  rinv[q] = v > 0.0 ? (float)(1.0 / r) : 0.0f;
  if (norms) norms[q] = (float)r;
}

// E[j][i] = ((W[j][i] - hi[i]) - lo[i]) * rinv[layer of i][j] for i < D, 0 for D <= i < lde  (E may be W).
// 4 consecutive elements per thread; the layer of the first one by bisection, the others follow.
__global__ __launch_bounds__(kEltThreads) void centre_scale_kernel(const float* W, int64_t D, int n, int64_t ldw,
                                                                   const float* __restrict__ wbar,
                                                                   const float* __restrict__ wbar_lo, float* E,
                                                                   int64_t lde, const int64_t* __restrict__ off, int L,
                                                                   const float* __restrict__ rinv) {
  if (!plan_header_ok(off, L, D)) {             // not this call's plan: no table is read; the norms are NaN already,
    if (blockIdx.x == 0 && threadIdx.x == 0) E[0] = __builtin_nanf("");      // and the basis says so too
    return;
  }
  const uint32_t bytes = (uint32_t)(D * 4);
  const rsrc_t rh = make_rsrc(wbar, bytes), rl = make_rsrc(wbar_lo, bytes);
  const int64_t nvec = lde / 4;
  for (int64_t q = (int64_t)blockIdx.x * kEltThreads + threadIdx.x; q < nvec; q += (int64_t)gridDim.x * kEltThreads) {
    const int64_t i0 = 4 * q;
    int a = 0, b = L - 1;                       // largest l with off[l] <= i0
    while (a < b) {
      const int mid = (a + b + 1) >> 1;
      if (off[mid] <= i0) a = mid; else b = mid - 1;
    }
    int lay[4];
    int l = a;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      while (l < L - 1 && off[l + 1] <= i0 + r) ++l;
      lay[r] = l;
    }
    const u32x4 h = ld128(rh, (uint32_t)q * 16u), lo = ld128(rl, (uint32_t)q * 16u);      // past D: zeros
    for (int j = 0; j < n; ++j) {
      const u32x4 x = ld128_stream(make_rsrc(W + (int64_t)j * ldw, bytes), (uint32_t)q * 16u);
      u32x4 y;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float c = (as_f32(x[r]) - as_f32(h[r])) - as_f32(lo[r]);
        y[r] = i0 + r < D ? as_u32(c * rinv[(int64_t)lay[r] * n + j]) : 0u;
      }
      *reinterpret_cast<u32x4*>(E + (int64_t)j * lde + i0) = y;
    }
  }
}

// beta <- (1 - lr*lambda) beta - lr * s   (Alg. 1, "update variables")
__global__ __launch_bounds__(kEltThreads) void beta_update_kernel(float* __restrict__ beta, const float* __restrict__ s,
                                                                  int64_t count, float lr, float lambda) {
  const int64_t q = (int64_t)blockIdx.x * kEltThreads + threadIdx.x;
  if (q >= count) return;
  const float keep = 1.0f - lr * lambda;
  beta[q] = __builtin_fmaf(-lr, s[q], keep * beta[q]);
}

// The coefficient step with the base optimiser (Sec. 5.1), one coefficient per thread.
//   KIND 0  heavy-ball momentum:  d = s + lambda beta;  m <- mu m + d;  beta <- beta - lr m
//   KIND 1  Adam (decay as an L2 term), KIND 2 AdamW (decoupled decay):
//           m <- mu m + (1 - mu) d;  v <- beta2 v + (1 - beta2) d^2;
//           beta <- beta - lr (m / bias1) / (sqrt(v / bias2) + eps),  bias1 = 1 - mu^t, bias2 = 1 - beta2^t
template <int KIND>
__global__ __launch_bounds__(kEltThreads) void beta_optim_kernel(float* __restrict__ beta, const float* __restrict__ s,
                                                                 float* __restrict__ m, float* __restrict__ v,
                                                                 int64_t count, float lr, float lambda, float mu,
                                                                 float beta2, float eps, float bias1, float bias2) {
  const int64_t q = (int64_t)blockIdx.x * kEltThreads + threadIdx.x;
  if (q >= count) return;
  float b = beta[q];
  if constexpr (KIND == 0) {
    const float d = __builtin_fmaf(lambda, b, s[q]);
    const float mq = __builtin_fmaf(mu, m[q], d);
    m[q] = mq;
    beta[q] = __builtin_fmaf(-lr, mq, b);
  } else {
    float d = s[q];
    if constexpr (KIND == 1) d = __builtin_fmaf(lambda, b, d);
    else b *= 1.0f - lr * lambda;
    const float mq = __builtin_fmaf(mu, m[q], (1.0f - mu) * d);
    const float vq = __builtin_fmaf(beta2, v[q], (1.0f - beta2) * d * d);
    m[q] = mq;
    v[q] = vq;
    beta[q] = b - lr * (mq / bias1) / (__builtin_sqrtf(vq / bias2) + eps);
  }
}

static int elt_grid(int64_t nvec) {
  const int64_t want = (nvec + kEltThreads - 1) / kEltThreads;
  const int cap = device_cus() * 8;
  return (int)(want < cap ? (want > 0 ? want : 1) : cap);
}

// Workspace layout: wbar_lo [D rounded up to 4 floats] | Q [L*n] | rinv [L*n] | partial sums of the squares kernel.
size_t centre_workspace_bytes(int64_t D, int n, int L) {
  const size_t lo = (size_t)((D + 3) / 4 * 4) * sizeof(float);
  return lo + 2 * (size_t)L * n * sizeof(float) + ((size_t)kMaxGrid + (size_t)L) * n * sizeof(float);
}

int launch_centre_normalise(const float* W, int64_t D, int n, int64_t ldw, const void* plan_dev, int L, float* wbar,
                            float* E, int64_t lde, float* norms, void* ws, int max_grid, hipStream_t st) {
  float* wbar_lo = static_cast<float*>(ws);
  float* Q = wbar_lo + (D + 3) / 4 * 4;
  float* rinv = Q + (size_t)L * n;
  float* partial = rinv + (size_t)L * n;
  hipLaunchKernelGGL(mean_kernel, dim3(elt_grid((D + 3) / 4)), dim3(kEltThreads), 0, st, W, D, n, ldw, wbar, wbar_lo);
  int rc = hip_check(hipGetLastError());
  if (rc != TWA_OK) return rc;
  // the squared norms are taken from W centred on the fly, and the centred matrix is written once,
  // already scaled: four passes over the n x D matrix (three reads, one write) instead of six
  PView v{reinterpret_cast<const uint8_t*>(W), nullptr, D, ldw, n, 0, 1.0f, 0.0f};
  rc = launch_layer_squares(v, wbar, wbar_lo, plan_dev, L, Q, partial, max_grid, st);
  if (rc != TWA_OK) return rc;
  const int64_t count = (int64_t)L * n;
  hipLaunchKernelGGL(rinv_kernel, dim3((unsigned)((count + kEltThreads - 1) / kEltThreads)), dim3(kEltThreads), 0, st, Q,
                     count, rinv, norms);
  const LayerPlan plan = plan_view(plan_dev, L, 2048);
  hipLaunchKernelGGL(centre_scale_kernel, dim3(elt_grid(lde / 4)), dim3(kEltThreads), 0, st, W, D, n, ldw, wbar, wbar_lo,
                     E, lde, plan.off, L, rinv);
  return hip_check(hipGetLastError());
}

int launch_beta_update(float* beta, const float* s, int64_t count, float lr, float lambda, hipStream_t st) {
  hipLaunchKernelGGL(beta_update_kernel, dim3((unsigned)((count + kEltThreads - 1) / kEltThreads)), dim3(kEltThreads), 0,
                     st, beta, s, count, lr, lambda);
  return hip_check(hipGetLastError());
}

int launch_beta_optim(int kind, float* beta, const float* s, float* m, float* v, int64_t count, float lr, float lambda,
                      float mu, float beta2, float eps, float bias1, float bias2, hipStream_t st) {
  const dim3 grid((unsigned)((count + kEltThreads - 1) / kEltThreads)), block(kEltThreads);
  if (kind == TWA_OPT_MOMENTUM)
    hipLaunchKernelGGL(beta_optim_kernel<0>, grid, block, 0, st, beta, s, m, v, count, lr, lambda, mu, beta2, eps, bias1, bias2);
  else if (kind == TWA_OPT_ADAM)
    hipLaunchKernelGGL(beta_optim_kernel<1>, grid, block, 0, st, beta, s, m, v, count, lr, lambda, mu, beta2, eps, bias1, bias2);
  else
    hipLaunchKernelGGL(beta_optim_kernel<2>, grid, block, 0, st, beta, s, m, v, count, lr, lambda, mu, beta2, eps, bias1, bias2);
  return hip_check(hipGetLastError());
}

}  // namespace twa
