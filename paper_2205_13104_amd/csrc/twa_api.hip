// C-ABI entry points (include/twa.h): argument validation on the host, dispatch to the gfx950
// kernels, and the small fp64 host algebra of CholeskyQR2 (n <= 128).
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <initializer_list>
#include <mutex>
#include <vector>

#include "twa_device.h"
#include "twa_host.h"

namespace twa {

static thread_local int g_last_hip_error = 0;

int hip_check(hipError_t e) {
  if (e == hipSuccess) return TWA_OK;
  g_last_hip_error = (int)e;
  return (e == hipErrorNoDevice || e == hipErrorInvalidDevice) ? TWA_ERR_NO_DEVICE : TWA_ERR_HIP;
}

int device_cus() {
  static std::mutex mu;
  static int cus[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -1;
  std::lock_guard<std::mutex> lk(mu);
  if (cus[dev] == 0) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return -1;
    cus[dev] = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : -1;
  }
  return cus[dev];
}

// Launch-geometry knobs (twa_set_launch_knob): process-wide, 0 = the library's own choice.
static std::atomic<int> g_knob[TWA_KNOB_COUNT];
int launch_knob(int which) { return (which >= 0 && which < TWA_KNOB_COUNT) ? g_knob[which].load(std::memory_order_relaxed) : 0; }

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool pow2(int x) { return x > 0 && (x & (x - 1)) == 0; }
static bool scaled(int dtype) { return dtype == TWA_I8 || dtype == TWA_I4; }
static bool minmax(int dtype) {
  return dtype == TWA_U8MM || dtype == TWA_U4MM || dtype == TWA_U16MM || dtype == TWA_U2MM || dtype == TWA_U1MM ||
         dtype == TWA_U3MM;
}
static int bits_of(int dtype) {
  switch (dtype) {
    case TWA_F32: return 32;
    case TWA_BF16: return 16;
    case TWA_I8: return 8;
    case TWA_I4: return 4;
    case TWA_U8MM: return 8;
    case TWA_U4MM: return 4;
    case TWA_U16MM: return 16;
    case TWA_U2MM: return 2;
    case TWA_U1MM: return 1;
    case TWA_U3MM: return 3;
    default: return 0;
  }
}

static int64_t ld_multiple(int dtype) { return scaled(dtype) || minmax(dtype) ? TWA_SCALE_SPAN : TWA_LD_MULTIPLE; }

static int check_dims(int64_t D, int32_t n, int64_t ld, int dtype) {
  const int bits = bits_of(dtype);
  if (D <= 0 || n <= 0 || n > TWA_MAX_N || ld < D) return TWA_ERR_SHAPE;
  // byte offsets inside a stored vector, g and w are 32-bit, and "one access past the end" must not wrap
  constexpr int64_t kOffsetLimit = ((int64_t)1 << 32) - 64;
  if ((D * (int64_t)bits + 7) / 8 >= kOffsetLimit) return TWA_ERR_SHAPE;
  if (D * 4 >= kOffsetLimit) return TWA_ERR_SHAPE;                 // g and w are fp32 vectors of length D
  if (ld % ld_multiple(dtype) != 0) return TWA_ERR_ALIGN;
  return TWA_OK;
}

// Validate a descriptor and turn it into the kernel-side view.
static int view_of(const twa_pmat* P, PView* v) {
  if (!P) return TWA_ERR_NULL;
  const int bits = bits_of(P->dtype);
  if (bits == 0) return TWA_ERR_DTYPE;
  if (!P->data) return TWA_ERR_NULL;
  int rc = check_dims(P->D, P->n, P->ld, P->dtype);
  if (rc != TWA_OK) return rc;
  if (!aligned16(P->data)) return TWA_ERR_ALIGN;
  int shift = 0;
  float gscale = 1.0f;
  float code_bias = 0.0f;
  if (minmax(P->dtype)) {
    if (!P->scales) return TWA_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(P->scales) & 7u) return TWA_ERR_ALIGN;
    if (P->dtype == TWA_U8MM || P->dtype == TWA_U16MM) {
      // `block` holds B, the bits of the codes (0: as many as the container has); the container holds c - 2^(B-1)
      const int B = P->block ? P->block : bits;
      if (B < 1 || B > bits) return TWA_ERR_SHAPE;
      code_bias = (float)(1 << (B - 1));
    }
  }
  if (scaled(P->dtype)) {
    if (!P->scales) return TWA_ERR_NULL;
    if (!aligned16(P->scales)) return TWA_ERR_ALIGN;
    if (!pow2(P->block) || P->block < 32 || P->block > 256) return TWA_ERR_SHAPE;
    if (P->ld % P->block != 0) return TWA_ERR_ALIGN;
    while ((1 << shift) < P->block) ++shift;
    if (P->dtype == TWA_I4) {
      int ex = 0;
      if (!(P->gscale > 0.0f) || !isfinite(P->gscale) || frexpf(P->gscale, &ex) != 0.5f) return TWA_ERR_SHAPE;
      gscale = P->gscale;
    }
  }
  v->data = static_cast<const uint8_t*>(P->data);
  v->scales = static_cast<const uint8_t*>(P->scales);
  v->D = P->D;
  v->ld = P->ld;
  v->n = P->n;
  v->block_shift = shift;
  v->gscale = gscale;
  v->code_bias = code_bias;
  return TWA_OK;
}

// Upper bound of a persistent grid: `per_cu_x4`/4 workgroups per compute unit (a multiple of a
// quarter), or the caller's absolute value of the launch knob `knob` when one is set.
static int persistent_grid(int knob, int per_cu_x4) {
  const int cus = device_cus();
  if (cus <= 0) return -1;
  int64_t g = launch_knob(knob);
  if (g <= 0) g = (int64_t)cus * per_cu_x4 / 4;
  if (g > kMaxGrid) g = kMaxGrid;
  if (g < 1) g = 1;
  return (int)g;
}

// ---- fp64 host algebra for CholeskyQR2 (row-major n x n) --------------------------------------

// G = R^T R with R upper triangular, diag > 0.  Returns -1 or the index of the first pivot that
// is <= tol * (largest diagonal entry of G).
static int cholesky_upper(const std::vector<double>& G, int n, double tol, std::vector<double>& R) {
  R.assign((size_t)n * n, 0.0);
  double dmax = 0.0;
  for (int i = 0; i < n; ++i) dmax = fmax(dmax, G[(size_t)i * n + i]);
  for (int j = 0; j < n; ++j) {
    double d = G[(size_t)j * n + j];
    for (int k = 0; k < j; ++k) d -= R[(size_t)k * n + j] * R[(size_t)k * n + j];
    if (!(d > tol * dmax)) return j;
    const double rjj = sqrt(d);
    R[(size_t)j * n + j] = rjj;
    for (int i = j + 1; i < n; ++i) {
      double v = G[(size_t)j * n + i];
      for (int k = 0; k < j; ++k) v -= R[(size_t)k * n + j] * R[(size_t)k * n + i];
      R[(size_t)j * n + i] = v / rjj;
    }
  }
  return -1;
}

// X = R^-1 (upper triangular) by back substitution, column by column.
static void invert_upper(const std::vector<double>& R, int n, std::vector<double>& X) {
  X.assign((size_t)n * n, 0.0);
  for (int j = 0; j < n; ++j) {
    X[(size_t)j * n + j] = 1.0 / R[(size_t)j * n + j];
    for (int i = j - 1; i >= 0; --i) {
      double v = 0.0;
      for (int k = i + 1; k <= j; ++k) v += R[(size_t)i * n + k] * X[(size_t)k * n + j];
      X[(size_t)i * n + j] = -v / R[(size_t)i * n + i];
    }
  }
}


// One power of two for all binary16 scales of a matrix whose largest entry is amax: the largest scale, amax / 7,
// lands in [2^14, 2^15).
float gscale_of(float amax) {
  const float smax = amax / 7.0f;
  if (!(smax > 0.0f) || !isfinite(smax)) return 1.0f;
  int ex = 0;
  (void)frexpf(smax, &ex);                    // smax = m * 2^ex, m in [0.5, 1)
  return ldexpf(1.0f, ex - 1 - 14);
}

}  // namespace twa

using namespace twa;

extern "C" {

int twa_version(void) { return 100; }

const char* twa_strerror(int status) {
  switch (status) {
    case TWA_OK: return "success";
    case TWA_ERR_NULL: return "a required pointer is NULL";
    case TWA_ERR_SHAPE: return "D, n, k, ld, block or gscale out of range";
    case TWA_ERR_ALIGN: return "pointer not 16-byte aligned, or ld not a multiple of 128 (fp32, bf16) / 2048 (int8, int4)";
    case TWA_ERR_DTYPE: return "unknown or unsupported storage type";
    case TWA_ERR_WORKSPACE: return "workspace missing or too small";
    case TWA_ERR_RANK: return "checkpoints are numerically linearly dependent";
    case TWA_ERR_HIP: return "a HIP runtime call failed";
    case TWA_ERR_NO_DEVICE: return "no usable GPU device";
    case TWA_ERR_LIMIT: return "size beyond the fixed device array of an entry point that allocates nothing";
    default: return "unknown status";
  }
}

int twa_last_hip_error(void) { return g_last_hip_error; }

int twa_set_launch_knob(int32_t knob, int32_t value) {
  if (knob < 0 || knob >= TWA_KNOB_COUNT) return TWA_ERR_DTYPE;
  if (value < 0 || value > kMaxGrid) return TWA_ERR_SHAPE;
  g_knob[knob].store(value, std::memory_order_relaxed);
  return TWA_OK;
}

int twa_pmat_bytes(int32_t dtype, int64_t D, int32_t n, int32_t block, int64_t* ld, size_t* data_bytes,
                   size_t* scale_bytes) {
  if (!ld || !data_bytes || !scale_bytes) return TWA_ERR_NULL;
  const int bits = bits_of(dtype);
  if (bits == 0) return TWA_ERR_DTYPE;
  if (D <= 0 || n <= 0 || n > TWA_MAX_N) return TWA_ERR_SHAPE;
  if (scaled(dtype) && (!pow2(block) || block < 32 || block > 256)) return TWA_ERR_SHAPE;
  const int64_t mult = ld_multiple(dtype);
  const int64_t l = (D + mult - 1) / mult * mult;
  int rc = check_dims(D, n, l, dtype);
  if (rc != TWA_OK) return rc;
  *ld = l;
  *data_bytes = (size_t)n * (size_t)l * (size_t)bits / 8;
  *scale_bytes = scaled(dtype) ? (size_t)n * (size_t)(l / block) * (dtype == TWA_I8 ? 4 : 2) : 0;
  return TWA_OK;
}

int twa_project_workspace_bytes(int32_t n, int32_t k, size_t* bytes) {
  if (!bytes) return TWA_ERR_NULL;
  if (n <= 0 || n > TWA_MAX_N || k <= 0 || k > TWA_MAX_K) return TWA_ERR_SHAPE;
  *bytes = (size_t)kMaxGrid * (size_t)n * (size_t)k * sizeof(float);
  return TWA_OK;
}

static constexpr int kGramMaxGrid = 512;

int twa_build_basis_workspace_bytes(int32_t n, size_t* bytes) {
  if (!bytes) return TWA_ERR_NULL;
  if (n <= 0 || n > TWA_MAX_N) return TWA_ERR_SHAPE;
  const size_t NP = (size_t)(n + 15) / 16 * 16;
  // per-workgroup partial Gram matrices + the reduced Gram matrix + R^-1 in fp32
  *bytes = (size_t)kGramMaxGrid * NP * NP * sizeof(double) + NP * NP * sizeof(double) + NP * NP * sizeof(float);
  return TWA_OK;
}

int twa_project(const twa_pmat* P, const float* g, int32_t k, int64_t ldg, float* s, void* ws, size_t ws_bytes,
                void* stream) {
  PView v;
  int rc = view_of(P, &v);
  if (rc != TWA_OK) return rc;
  if (!g || !s) return TWA_ERR_NULL;
  if (k <= 0 || k > TWA_MAX_K) return TWA_ERR_SHAPE;
  if (k > 1 && (ldg < v.D || (ldg & 3) != 0)) return TWA_ERR_SHAPE;
  if (!aligned16(g) || (reinterpret_cast<uintptr_t>(s) & 3u)) return TWA_ERR_ALIGN;
  size_t need = 0;
  twa_project_workspace_bytes(v.n, k, &need);
  if (!ws || ws_bytes < need) return TWA_ERR_WORKSPACE;
  if (!aligned16(ws)) return TWA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int grid = persistent_grid(TWA_KNOB_PROJECT_GRID, 8);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  float* partial = static_cast<float*>(ws);
  if (k == 1) return launch_project(v, P->dtype, g, s, partial, grid, st);
  return launch_project_batched(v, P->dtype, g, ldg, k, s, partial, grid, st);
}

int twa_project_noalloc(const twa_pmat* P, const float* g, int32_t k, int64_t ldg, float* s, void* stream) {
  PView v;
  int rc = view_of(P, &v);
  if (rc != TWA_OK) return rc;
  if (!g || !s) return TWA_ERR_NULL;
  if (k <= 0 || k > TWA_MAX_K) return TWA_ERR_SHAPE;
  if ((int64_t)v.n * k > TWA_NOALLOC_MAX_NK) return TWA_ERR_LIMIT;      // beyond the fixed array: said on the host
  if (k > 1 && (ldg < v.D || (ldg & 3) != 0)) return TWA_ERR_SHAPE;
  if (!aligned16(g) || (reinterpret_cast<uintptr_t>(s) & 3u)) return TWA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int grid = persistent_grid(TWA_KNOB_PROJECT_GRID, 8);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  float* partial = nullptr;
  size_t floats = 0;
  rc = noalloc_partials(&partial, &floats);
  if (rc != TWA_OK) return rc;
  if ((size_t)grid * (size_t)v.n * (size_t)k > floats) return TWA_ERR_LIMIT;
  if (k == 1) return launch_project(v, P->dtype, g, s, partial, grid, st);
  return launch_project_batched(v, P->dtype, g, ldg, k, s, partial, grid, st);
}

int twa_expand_update(const twa_pmat* P, const float* s, float* w, float lr, float* g_tilde, void* stream) {
  PView v;
  int rc = view_of(P, &v);
  if (rc != TWA_OK) return rc;
  if (!s || !w) return TWA_ERR_NULL;
  if (!aligned16(w) || (g_tilde && !aligned16(g_tilde)) || (reinterpret_cast<uintptr_t>(s) & 3u))
    return TWA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int grid = persistent_grid(TWA_KNOB_EXPAND_GRID, 8);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  return launch_expand_update(v, P->dtype, s, w, lr, g_tilde, grid, st);
}

int twa_project_layers_workspace_bytes(int32_t n, int32_t L, size_t* bytes) {
  if (!bytes) return TWA_ERR_NULL;
  if (n <= 0 || n > TWA_MAX_N || L <= 0 || L > TWA_MAX_LAYERS) return TWA_ERR_SHAPE;
  // partial sums per (workgroup + layer) slot: n coefficients, and one more number for the min-max formats
  *bytes = ((size_t)kMaxGrid + (size_t)L) * ((size_t)n + 1) * sizeof(float);
  return TWA_OK;
}

int twa_layer_plan_bytes(int32_t L, size_t* bytes) {
  if (!bytes) return TWA_ERR_NULL;
  if (L <= 0 || L > TWA_MAX_LAYERS) return TWA_ERR_SHAPE;
  *bytes = layer_plan_bytes(L);
  return TWA_OK;
}

int twa_layer_plan(const int64_t* layer_off, int32_t L, int64_t D, void* plan, size_t plan_bytes, void* stream) {
  if (!layer_off || !plan) return TWA_ERR_NULL;
  if (L <= 0 || L > TWA_MAX_LAYERS) return TWA_ERR_SHAPE;
  int rc = check_dims(D, 1, (D + TWA_LD_MULTIPLE - 1) / TWA_LD_MULTIPLE * TWA_LD_MULTIPLE, TWA_F32);
  if (rc != TWA_OK) return rc;
  if (plan_bytes < layer_plan_bytes(L)) return TWA_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(layer_off) & 7u) || (reinterpret_cast<uintptr_t>(plan) & 7u)) return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  return launch_layer_plan(layer_off, L, D, plan, static_cast<hipStream_t>(stream));
}

static int check_plan(const void* plan, int32_t L) {
  if (!plan) return TWA_ERR_NULL;
  if (L <= 0 || L > TWA_MAX_LAYERS) return TWA_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(plan) & 7u) return TWA_ERR_ALIGN;
  return TWA_OK;
}

static int project_layers_common(const twa_pmat* P, const float* g, const void* plan, int32_t L, float* S, float* beta,
                                 float lr, float lambda, void* ws, size_t ws_bytes, void* stream) {
  PView v;
  int rc = view_of(P, &v);
  if (rc != TWA_OK) return rc;
  if (!g || (!S && !beta)) return TWA_ERR_NULL;
  rc = check_plan(plan, L);
  if (rc != TWA_OK) return rc;
  if (!aligned16(g) || (reinterpret_cast<uintptr_t>(S) & 3u) || (reinterpret_cast<uintptr_t>(beta) & 3u))
    return TWA_ERR_ALIGN;
  size_t need = 0;
  twa_project_layers_workspace_bytes(v.n, L, &need);
  if (!ws || ws_bytes < need) return TWA_ERR_WORKSPACE;
  if (!aligned16(ws)) return TWA_ERR_ALIGN;
  const int grid = persistent_grid(TWA_KNOB_PROJECT_GRID, 8);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  return launch_project_layers(v, P->dtype, g, plan, L, S, beta, lr, lambda, static_cast<float*>(ws), grid,
                               static_cast<hipStream_t>(stream));
}

int twa_project_layers(const twa_pmat* P, const float* g, const void* plan, int32_t L, float* S, void* ws,
                       size_t ws_bytes, void* stream) {
  if (!S) return TWA_ERR_NULL;
  return project_layers_common(P, g, plan, L, S, nullptr, 0.0f, 0.0f, ws, ws_bytes, stream);
}

int twa_beta_step(const twa_pmat* P, const float* g, const void* plan, int32_t L, float* beta, float lr, float lambda,
                  float* S, void* ws, size_t ws_bytes, void* stream) {
  if (!beta) return TWA_ERR_NULL;
  return project_layers_common(P, g, plan, L, S, beta, lr, lambda, ws, ws_bytes, stream);
}

int twa_expand_update_layers(const twa_pmat* P, const float* S, const void* plan, int32_t L, float* w, float lr,
                             float* g_tilde, void* stream) {
  PView v;
  int rc = view_of(P, &v);
  if (rc != TWA_OK) return rc;
  if (!S || !w) return TWA_ERR_NULL;
  rc = check_plan(plan, L);
  if (rc != TWA_OK) return rc;
  if (!aligned16(w) || (g_tilde && !aligned16(g_tilde)) || (reinterpret_cast<uintptr_t>(S) & 3u))
    return TWA_ERR_ALIGN;
  const int grid = persistent_grid(TWA_KNOB_EXPAND_GRID, 8);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  return launch_expand_update_layers(v, P->dtype, S, plan, L, w, w, lr, g_tilde, grid,
                                     static_cast<hipStream_t>(stream));
}

int twa_weights_from_beta(const twa_pmat* P, const float* beta, const void* plan, int32_t L, const float* wbar,
                          float* w, void* stream) {
  PView v;
  int rc = view_of(P, &v);
  if (rc != TWA_OK) return rc;
  if (!beta || !wbar || !w) return TWA_ERR_NULL;
  rc = check_plan(plan, L);
  if (rc != TWA_OK) return rc;
  if (!aligned16(w) || !aligned16(wbar) || (reinterpret_cast<uintptr_t>(beta) & 3u)) return TWA_ERR_ALIGN;
  const int grid = persistent_grid(TWA_KNOB_EXPAND_GRID, 8);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  // w = wbar - (-1) * (P beta): the expansion kernel with the mean as the weights it reads
  return launch_expand_update_layers(v, P->dtype, beta, plan, L, wbar, w, -1.0f, nullptr, grid,
                                     static_cast<hipStream_t>(stream));
}

int twa_beta_update(float* beta, const float* s, int64_t count, float lr, float lambda, void* stream) {
  if (!beta || !s) return TWA_ERR_NULL;
  if (count <= 0 || count > (int64_t)TWA_MAX_LAYERS * TWA_MAX_N) return TWA_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(beta) & 3u) || (reinterpret_cast<uintptr_t>(s) & 3u)) return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  return launch_beta_update(beta, s, count, lr, lambda, static_cast<hipStream_t>(stream));
}

int twa_beta_optim(const twa_optim* opt, float* beta, const float* s, float* m, float* v, int64_t count, void* stream) {
  if (!opt || !beta || !s || !m) return TWA_ERR_NULL;
  if (opt->kind != TWA_OPT_MOMENTUM && opt->kind != TWA_OPT_ADAM && opt->kind != TWA_OPT_ADAMW) return TWA_ERR_DTYPE;
  const bool adam = opt->kind != TWA_OPT_MOMENTUM;
  if (adam && !v) return TWA_ERR_NULL;
  if (count <= 0 || count > (int64_t)TWA_MAX_LAYERS * TWA_MAX_N) return TWA_ERR_SHAPE;
  if (!(opt->mu >= 0.0f && opt->mu < 1.0f)) return TWA_ERR_SHAPE;
  if (adam && (opt->t < 1 || !(opt->beta2 >= 0.0f && opt->beta2 < 1.0f) || !(opt->eps >= 0.0f))) return TWA_ERR_SHAPE;
  for (const void* p : {(const void*)beta, (const void*)s, (const void*)m, (const void*)v})
    if (reinterpret_cast<uintptr_t>(p) & 3u) return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  float bias1 = 1.0f, bias2 = 1.0f;
  if (adam) {
    bias1 = (float)(1.0 - pow((double)opt->mu, (double)opt->t));
    bias2 = (float)(1.0 - pow((double)opt->beta2, (double)opt->t));
  }
  return launch_beta_optim(opt->kind, beta, s, m, v, count, opt->lr, opt->lambda, opt->mu, opt->beta2, opt->eps, bias1,
                           bias2, static_cast<hipStream_t>(stream));
}

int twa_quantize_minmax_workspace_bytes(int32_t L, size_t* bytes) {
  if (!bytes) return TWA_ERR_NULL;
  if (L <= 0 || L > TWA_MAX_LAYERS) return TWA_ERR_SHAPE;
  *bytes = minmax_workspace_bytes(L);
  return TWA_OK;
}

int twa_quantize_minmax(const float* P, int64_t D, int32_t n, int64_t ldp, const void* plan, int32_t L, int32_t bits,
                        twa_pmat* out, void* ws, size_t ws_bytes, void* stream) {
  if (!P || !out || !out->data || !out->scales) return TWA_ERR_NULL;
  if (!minmax(out->dtype)) return TWA_ERR_DTYPE;
  if (bits < 1 || bits > bits_of(out->dtype)) return TWA_ERR_SHAPE;
  if (out->D != D || out->n != n) return TWA_ERR_SHAPE;
  int rc = check_dims(D, n, ldp, TWA_F32);
  if (rc != TWA_OK) return rc;
  rc = check_dims(D, n, out->ld, out->dtype);
  if (rc != TWA_OK) return rc;
  rc = check_plan(plan, L);
  if (rc != TWA_OK) return rc;
  if (!aligned16(P) || !aligned16(out->data) || (reinterpret_cast<uintptr_t>(out->scales) & 7u)) return TWA_ERR_ALIGN;
  if (!ws || ws_bytes < minmax_workspace_bytes(L)) return TWA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 7u) return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  out->block = bits;                       // the descriptor remembers B (the byte and word containers need it)
  return launch_quantize_minmax(P, D, n, ldp, plan, L, out->dtype, bits, static_cast<uint8_t*>(out->data), out->ld,
                                static_cast<float*>(out->scales), ws, static_cast<hipStream_t>(stream));
}

int twa_centre_normalise_workspace_bytes(int64_t D, int32_t n, int32_t L, size_t* bytes) {
  if (!bytes) return TWA_ERR_NULL;
  if (D <= 0 || n <= 0 || n > TWA_MAX_N || L <= 0 || L > TWA_MAX_LAYERS) return TWA_ERR_SHAPE;
  *bytes = centre_workspace_bytes(D, n, L);
  return TWA_OK;
}

int twa_centre_normalise(const float* W, int64_t D, int32_t n, int64_t ldw, const void* plan, int32_t L, float* wbar,
                         float* E, int64_t lde, float* norms, void* ws, size_t ws_bytes, void* stream) {
  if (!W || !wbar || !E) return TWA_ERR_NULL;
  int rc = check_dims(D, n, ldw, TWA_F32);
  if (rc != TWA_OK) return rc;
  rc = check_dims(D, n, lde, TWA_F32);
  if (rc != TWA_OK) return rc;
  rc = check_plan(plan, L);
  if (rc != TWA_OK) return rc;
  if (!aligned16(W) || !aligned16(E) || !aligned16(wbar) || (norms && (reinterpret_cast<uintptr_t>(norms) & 3u)))
    return TWA_ERR_ALIGN;
  if (E != W) {                              // in place, or apart: no partial overlap
    const char* a = reinterpret_cast<const char*>(W);
    const char* b = reinterpret_cast<const char*>(E);
    const size_t wa = (size_t)n * ldw * 4, eb = (size_t)n * lde * 4;
    if (a < b + eb && b < a + wa) return TWA_ERR_SHAPE;
  } else if (lde != ldw) {
    return TWA_ERR_SHAPE;
  }
  if (!ws || ws_bytes < centre_workspace_bytes(D, n, L)) return TWA_ERR_WORKSPACE;
  if (!aligned16(ws)) return TWA_ERR_ALIGN;
  const int grid = persistent_grid(TWA_KNOB_PROJECT_GRID, 8);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  return launch_centre_normalise(W, D, n, ldw, plan, L, wbar, E, lde, norms, ws, grid, static_cast<hipStream_t>(stream));
}

int twa_quantize(const float* P, int64_t D, int32_t n, int64_t ldp, twa_pmat* out, void* stream) {
  if (!P || !out || !out->data) return TWA_ERR_NULL;
  const int bits = bits_of(out->dtype);
  if (bits == 0) return TWA_ERR_DTYPE;
  if (out->D != D || out->n != n) return TWA_ERR_SHAPE;
  int rc = check_dims(D, n, ldp, TWA_F32);
  if (rc != TWA_OK) return rc;
  rc = check_dims(D, n, out->ld, out->dtype);
  if (rc != TWA_OK) return rc;
  if (!aligned16(P) || !aligned16(out->data)) return TWA_ERR_ALIGN;
  if (scaled(out->dtype)) {
    if (!out->scales) return TWA_ERR_NULL;
    if (!aligned16(out->scales)) return TWA_ERR_ALIGN;
    if (!pow2(out->block) || out->block < 32 || out->block > 256) return TWA_ERR_SHAPE;
    if (out->ld % out->block != 0) return TWA_ERR_ALIGN;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (out->dtype == TWA_I4) {
    if (out->gscale == 0.0f) {
      // largest block scale = (largest |p|) / 7: find it, then pick the power of two that puts
      // the largest binary16 scale in [2^14, 2^15).  The first word of the code buffer is scratch.
      float* tmp = static_cast<float*>(out->data);
      rc = launch_absmax(P, D, n, ldp, tmp, false, st);
      if (rc != TWA_OK) return rc;
      float amax = 0.0f;
      rc = hip_check(hipMemcpyAsync(&amax, tmp, sizeof(float), hipMemcpyDeviceToHost, st));
      if (rc != TWA_OK) return rc;
      rc = hip_check(hipStreamSynchronize(st));
      if (rc != TWA_OK) return rc;
      out->gscale = gscale_of(amax);
    } else {
      int ex = 0;
      if (!(out->gscale > 0.0f) || !isfinite(out->gscale) || frexpf(out->gscale, &ex) != 0.5f) return TWA_ERR_SHAPE;
    }
  }
  return launch_quantize(P, D, n, ldp, *out, st);
}

// Workgroups of the two basis kernels for a run of `rows` rows.
static int basis_grid(int64_t rows) {
  const int cus = device_cus();
  if (cus <= 0) return -1;
  const int64_t nchunks = (rows + 63) / 64;
  const int per_cu = launch_knob(TWA_KNOB_BASIS_WGS_PER_CU);
  int grid = cus * (per_cu > 0 ? per_cu : 2);
  if (grid > kGramMaxGrid) grid = kGramMaxGrid;
  if (grid > nchunks) grid = (int)nchunks;
  return grid;
}

// Gram matrix (device, NP x NP doubles, upper blocks) -> host: R with G = R^T R, and R^-1 as NP x NP floats
// on the device.  Synchronises the stream twice.  Returns TWA_ERR_RANK with *bad = index of the failing pivot.
static int factor_gram(const double* gram_dev, int n, float* rinv_dev, std::vector<double>& R, int* bad,
                       hipStream_t st) {
  const int NP = (n + 15) / 16 * 16;
  std::vector<double> gram_pad((size_t)NP * NP), G((size_t)n * n), X;
  std::vector<float> rinv_pad((size_t)NP * NP, 0.0f);
  int rc = hip_check(hipMemcpyAsync(gram_pad.data(), gram_dev, sizeof(double) * NP * NP, hipMemcpyDeviceToHost, st));
  if (rc != TWA_OK) return rc;
  rc = hip_check(hipStreamSynchronize(st));
  if (rc != TWA_OK) return rc;
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < n; ++j)
      G[(size_t)i * n + j] = (j >= i) ? gram_pad[(size_t)i * NP + j] : gram_pad[(size_t)j * NP + i];
  *bad = cholesky_upper(G, n, 1e-12, R);
  if (*bad >= 0) return TWA_ERR_RANK;
  invert_upper(R, n, X);
  for (int i = 0; i < n; ++i)
    for (int j = i; j < n; ++j) rinv_pad[(size_t)i * NP + j] = (float)X[(size_t)i * n + j];
  rc = hip_check(hipMemcpyAsync(rinv_dev, rinv_pad.data(), sizeof(float) * NP * NP, hipMemcpyHostToDevice, st));
  if (rc != TWA_OK) return rc;
  return hip_check(hipStreamSynchronize(st));     // rinv_pad leaves scope
}

// Rtot <- R * Rtot (both n x n upper triangular, row major):  W = Q1 Rtot, Q1 = P R  ->  W = P (R Rtot)
static void compose_upper(const std::vector<double>& R, std::vector<double>& Rtot, int n) {
  std::vector<double> T((size_t)n * n, 0.0);
  for (int i = 0; i < n; ++i)
    for (int j = i; j < n; ++j) {
      double v = 0.0;
      for (int k = i; k <= j; ++k) v += R[(size_t)i * n + k] * Rtot[(size_t)k * n + j];
      T[(size_t)i * n + j] = v;
    }
  Rtot.swap(T);
}

int twa_build_basis(const float* W, int64_t D, int32_t n, int64_t ldw, float* P, int64_t ldp, double* R_host,
                    void* ws, size_t ws_bytes, void* stream) {
  if (!W || !P) return TWA_ERR_NULL;
  int rc = check_dims(D, n, ldw, TWA_F32);
  if (rc != TWA_OK) return rc;
  rc = check_dims(D, n, ldp, TWA_F32);
  if (rc != TWA_OK) return rc;
  if (n > D) return TWA_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(P)) return TWA_ERR_ALIGN;
  if (static_cast<const void*>(W) == static_cast<const void*>(P) && ldw != ldp) return TWA_ERR_SHAPE;
  size_t need = 0;
  twa_build_basis_workspace_bytes(n, &need);
  if (!ws || ws_bytes < need) return TWA_ERR_WORKSPACE;
  if (!aligned16(ws)) return TWA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);

  const int NP = (n + 15) / 16 * 16;
  const int grid = basis_grid(D);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  double* partial = static_cast<double*>(ws);
  double* gram_dev = partial + (size_t)kGramMaxGrid * NP * NP;
  float* rinv_dev = reinterpret_cast<float*>(gram_dev + (size_t)NP * NP);

  std::vector<double> R, Rtot;
  const float* src = W;
  int64_t lds = ldw;
  for (int pass = 0; pass < 2; ++pass) {
    rc = launch_gram(src, D, n, lds, partial, grid, gram_dev, false, /*orthonormal_input=*/pass == 1, st);
    if (rc != TWA_OK) return rc;
    int bad = -1;
    rc = factor_gram(gram_dev, n, rinv_dev, R, &bad, st);
    if (rc == TWA_ERR_RANK && R_host) R_host[0] = (double)bad;
    if (rc != TWA_OK) return rc;
    rc = launch_apply_rinv(src, lds, P, ldp, D, n, rinv_dev, grid, true, st);
    if (rc != TWA_OK) return rc;
    if (pass == 0) Rtot = R;
    else compose_upper(R, Rtot, n);
    src = P;
    lds = ldp;
  }
  if (R_host) memcpy(R_host, Rtot.data(), sizeof(double) * (size_t)n * n);
  return TWA_OK;
}

int twa_build_basis_async(const float* W, int64_t D, int32_t n, int64_t ldw, float* P, int64_t ldp, double* R,
                          int32_t* status, void* ws, size_t ws_bytes, void* stream) {
  if (!W || !P || !status) return TWA_ERR_NULL;
  int rc = check_dims(D, n, ldw, TWA_F32);
  if (rc != TWA_OK) return rc;
  rc = check_dims(D, n, ldp, TWA_F32);
  if (rc != TWA_OK) return rc;
  if (n > D) return TWA_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(P) || (reinterpret_cast<uintptr_t>(R) & 7u) || (reinterpret_cast<uintptr_t>(status) & 3u))
    return TWA_ERR_ALIGN;
  if (static_cast<const void*>(W) == static_cast<const void*>(P) && ldw != ldp) return TWA_ERR_SHAPE;
  size_t need = 0;
  twa_build_basis_workspace_bytes(n, &need);
  if (!ws || ws_bytes < need) return TWA_ERR_WORKSPACE;
  if (!aligned16(ws)) return TWA_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int NP = (n + 15) / 16 * 16;
  const int grid = basis_grid(D);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  double* partial = static_cast<double*>(ws);
  double* gram_dev = partial + (size_t)kGramMaxGrid * NP * NP;
  float* rinv_dev = reinterpret_cast<float*>(gram_dev + (size_t)NP * NP);
  // between a pass's reduction and the next pass's Gram kernel the partial sums are dead: room for two n x n matrices
  double* r_pass = partial;
  double* scratch = partial + (size_t)n * n;
  rc = launch_zero_status(status, st);
  if (rc != TWA_OK) return rc;
  const float* src = W;
  int64_t lds = ldw;
  for (int pass = 0; pass < 2; ++pass) {
    rc = launch_gram(src, D, n, lds, partial, grid, gram_dev, false, /*orthonormal_input=*/pass == 1, st);
    if (rc != TWA_OK) return rc;
    rc = launch_gram_factor(gram_dev, n, rinv_dev, R ? (pass == 0 ? R : r_pass) : nullptr, status, st);
    if (rc != TWA_OK) return rc;
    if (R && pass == 1) {
      rc = launch_compose_upper(r_pass, R, scratch, n, st);
      if (rc != TWA_OK) return rc;
    }
    rc = launch_apply_rinv(src, lds, P, ldp, D, n, rinv_dev, grid, true, st);
    if (rc != TWA_OK) return rc;
    src = P;
    lds = ldp;
  }
  return TWA_OK;
}

int twa_gram_factor_async(const double* gram, int32_t n, float* rinv, double* R, int32_t* status, void* stream) {
  if (!gram || !rinv || !status) return TWA_ERR_NULL;
  if (n <= 0 || n > TWA_MAX_N) return TWA_ERR_SHAPE;
  if (!aligned16(gram) || !aligned16(rinv) || (reinterpret_cast<uintptr_t>(R) & 7u) || (reinterpret_cast<uintptr_t>(status) & 3u))
    return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  return launch_gram_factor(gram, n, rinv, R, status, static_cast<hipStream_t>(stream));
}

// ---- measurement aid: a plain non-temporal read pass (no other entry point calls it) ------------

int twa_probe_read(const void* buf, size_t bytes, uint32_t* sink, void* stream) {
  if (!buf || !sink) return TWA_ERR_NULL;
  if (bytes < 16 || bytes / 65536 >= ((size_t)1 << 31)) return TWA_ERR_SHAPE;
  if (!aligned16(buf) || (reinterpret_cast<uintptr_t>(sink) & 3u)) return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  return launch_read_probe(buf, bytes, sink, static_cast<hipStream_t>(stream));
}

// ---- the same construction for checkpoints whose rows arrive in panels -------------------------

int twa_basis_state_bytes(int32_t n, size_t* gram_bytes, size_t* rinv_bytes, size_t* ws_bytes) {
  if (!gram_bytes || !rinv_bytes || !ws_bytes) return TWA_ERR_NULL;
  if (n <= 0 || n > TWA_MAX_N) return TWA_ERR_SHAPE;
  const size_t NP = (size_t)(n + 15) / 16 * 16;
  *gram_bytes = NP * NP * sizeof(double);
  *rinv_bytes = NP * NP * sizeof(float);
  *ws_bytes = (size_t)kGramMaxGrid * NP * NP * sizeof(double);
  return TWA_OK;
}

static int check_panel(const float* W, int64_t rows, int32_t n, int64_t ldw) {
  if (!W) return TWA_ERR_NULL;
  if (rows <= 0 || n <= 0 || n > TWA_MAX_N || ldw < rows || rows * 4 >= ((int64_t)1 << 32)) return TWA_ERR_SHAPE;
  if (!aligned16(W) || ldw % 4 != 0) return TWA_ERR_ALIGN;
  return TWA_OK;
}

int twa_gram_accumulate(const float* W, int64_t rows, int32_t n, int64_t ldw, double* gram, int32_t accumulate,
                        void* ws, size_t ws_bytes, void* stream) {
  int rc = check_panel(W, rows, n, ldw);
  if (rc != TWA_OK) return rc;
  if (!gram) return TWA_ERR_NULL;
  if (accumulate & ~(TWA_GRAM_ADD | TWA_GRAM_ORTHONORMAL_INPUT)) return TWA_ERR_SHAPE;
  size_t gb = 0, rb = 0, wb = 0;
  twa_basis_state_bytes(n, &gb, &rb, &wb);
  if (!ws || ws_bytes < wb) return TWA_ERR_WORKSPACE;
  if (!aligned16(ws) || !aligned16(gram)) return TWA_ERR_ALIGN;
  const int grid = basis_grid(rows);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  return launch_gram(W, rows, n, ldw, static_cast<double*>(ws), grid, gram, (accumulate & TWA_GRAM_ADD) != 0,
                     (accumulate & TWA_GRAM_ORTHONORMAL_INPUT) != 0, static_cast<hipStream_t>(stream));
}

int twa_gram_factor(const double* gram, int32_t n, float* rinv, double* R_host, int32_t compose, void* stream) {
  if (!gram || !rinv) return TWA_ERR_NULL;
  if (n <= 0 || n > TWA_MAX_N) return TWA_ERR_SHAPE;
  if (compose && !R_host) return TWA_ERR_NULL;
  if (!aligned16(gram) || !aligned16(rinv)) return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  std::vector<double> R;
  int bad = -1;
  int rc = factor_gram(gram, n, rinv, R, &bad, static_cast<hipStream_t>(stream));
  if (rc == TWA_ERR_RANK && R_host) R_host[0] = (double)bad;
  if (rc != TWA_OK) return rc;
  if (R_host) {
    if (compose) {
      std::vector<double> Rtot(R_host, R_host + (size_t)n * n);
      compose_upper(R, Rtot, n);
      memcpy(R_host, Rtot.data(), sizeof(double) * (size_t)n * n);
    } else {
      memcpy(R_host, R.data(), sizeof(double) * (size_t)n * n);
    }
  }
  return TWA_OK;
}

int twa_apply_rinv(const float* W, int64_t rows, int32_t n, int64_t ldw, const float* rinv, float* P, int64_t ldp,
                   void* stream) {
  int rc = check_panel(W, rows, n, ldw);
  if (rc != TWA_OK) return rc;
  if (!rinv || !P) return TWA_ERR_NULL;
  if (ldp < rows) return TWA_ERR_SHAPE;
  if (!aligned16(P) || !aligned16(rinv) || ldp % 4 != 0) return TWA_ERR_ALIGN;
  if (static_cast<const void*>(W) == static_cast<const void*>(P) && ldw != ldp) return TWA_ERR_SHAPE;
  const int grid = basis_grid(rows);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  return launch_apply_rinv(W, ldw, P, ldp, rows, n, rinv, grid, false, static_cast<hipStream_t>(stream));
}

float twa_gscale_for_absmax(float amax) { return gscale_of(amax); }

int twa_absmax_accumulate(const float* X, int64_t rows, int32_t n, int64_t ld, float* amax, int32_t accumulate,
                          void* stream) {
  int rc = check_panel(X, rows, n, ld);
  if (rc != TWA_OK) return rc;
  if (!amax) return TWA_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(amax) & 3u) return TWA_ERR_ALIGN;
  if (device_cus() <= 0) return TWA_ERR_NO_DEVICE;
  return launch_absmax(X, rows, n, ld, amax, accumulate != 0, static_cast<hipStream_t>(stream));
}

int twa_apply_rinv_quantize(const float* W, int64_t rows, int32_t n, int64_t ldw, const float* rinv, const twa_pmat* out,
                            int64_t row0, void* stream) {
  int rc = check_panel(W, rows, n, ldw);
  if (rc != TWA_OK) return rc;
  if (!rinv || !out || !out->data) return TWA_ERR_NULL;
  const int dt = out->dtype;
  if (dt != TWA_F32 && dt != TWA_BF16 && dt != TWA_I8 && dt != TWA_I4) return TWA_ERR_DTYPE;
  if (out->n != n) return TWA_ERR_SHAPE;
  rc = check_dims(out->D, n, out->ld, dt);
  if (rc != TWA_OK) return rc;
  if (row0 < 0 || row0 + rows > out->D) return TWA_ERR_SHAPE;
  const bool last = row0 + rows == out->D;
  // panels meet on the grid of the scale spans, so that no quantisation block straddles two panels
  if (row0 % TWA_SCALE_SPAN != 0 || (!last && rows % TWA_SCALE_SPAN != 0)) return TWA_ERR_ALIGN;
  if (!aligned16(rinv) || !aligned16(out->data)) return TWA_ERR_ALIGN;
  if (scaled(dt)) {
    if (!out->scales) return TWA_ERR_NULL;
    if (!aligned16(out->scales)) return TWA_ERR_ALIGN;
    if (!pow2(out->block) || out->block < 32 || out->block > 128) return TWA_ERR_SHAPE;    // a block spans two tiles at most
    if (dt == TWA_I4) {
      int ex = 0;
      if (!(out->gscale > 0.0f) || !isfinite(out->gscale) || frexpf(out->gscale, &ex) != 0.5f) return TWA_ERR_SHAPE;
    }
  }
  {  // the stored matrix must not overlap the panel it is made from
    const char* a = reinterpret_cast<const char*>(W);
    const char* b = reinterpret_cast<const char*>(out->data);
    const size_t wa = ((size_t)(n - 1) * ldw + rows) * 4, ob = (size_t)n * out->ld * bits_of(dt) / 8;
    const bool same_f32 = dt == TWA_F32 && static_cast<const void*>(W) == static_cast<const void*>(static_cast<const float*>(out->data) + row0) && ldw == out->ld;
    if (!same_f32 && a < b + ob && b < a + wa) return TWA_ERR_SHAPE;
  }
  const int grid = basis_grid(rows);
  if (grid <= 0) return TWA_ERR_NO_DEVICE;
  return launch_apply_rinv_store(W, ldw, rows, n, rinv, *out, row0, last, grid, static_cast<hipStream_t>(stream));
}

}  // extern "C"
