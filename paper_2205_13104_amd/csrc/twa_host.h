// Host-side plumbing shared by the translation units of the library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/twa.h"

namespace twa {

struct PView;

// Records a failing hipError_t for twa_last_hip_error() and maps it to a twa_status.
int hip_check(hipError_t e);

// Number of compute units of the current device (cached per device); <= 0 on failure.
int device_cus();

// Upper bound of any persistent grid the library launches (sizes the workspaces).
constexpr int kMaxGrid = 2048;

// Current value of a launch knob (TWA_KNOB_*, set with twa_set_launch_knob); 0 = the library's own choice.
int launch_knob(int which);

// Kernel launchers (defined next to their kernels).
// `max_grid`: upper bound of the persistent grid; the launchers pick the largest grid below it
// that divides the tiles evenly.
int launch_project(const PView& P, int dtype, const float* g, float* s, float* partial, int max_grid,
                   hipStream_t st);
int launch_project_batched(const PView& P, int dtype, const float* g, int64_t ldg, int k, float* s, float* partial,
                           int max_grid, hipStream_t st);
int launch_expand_update(const PView& P, int dtype, const float* s, float* w, float lr, float* g_tilde, int max_grid,
                         hipStream_t st);
// Device address and size of the library's own array of partial sums on the current device (no allocation).
int noalloc_partials(float** out, size_t* floats);
// Layer-wise step: the device plan (see twa_layers.hip) and the kernels that use it.
struct LayerPlan;
size_t layer_plan_bytes(int L);
LayerPlan plan_view(const void* plan_dev, int L, int tile);
int launch_layer_plan(const int64_t* layer_off, int L, int64_t D, void* plan_dev, hipStream_t st);
int launch_project_layers(const PView& P, int dtype, const float* g, const void* plan_dev, int L, float* S,
                          float* beta, float lr, float lambda, float* partial, int max_grid, hipStream_t st);
int launch_expand_update_layers(const PView& P, int dtype, const float* s, const void* plan_dev, int L,
                                const float* w_in, float* w_out, float lr, float* g_tilde, int max_grid,
                                hipStream_t st);
int launch_layer_squares(const PView& P, const float* mean_hi, float* mean_lo, const void* plan_dev, int L, float* Q,
                         float* partial, int max_grid, hipStream_t st);
size_t centre_workspace_bytes(int64_t D, int n, int L);
int launch_centre_normalise(const float* W, int64_t D, int n, int64_t ldw, const void* plan_dev, int L, float* wbar,
                            float* E, int64_t lde, float* norms, void* ws, int max_grid, hipStream_t st);
size_t minmax_workspace_bytes(int L);
int launch_quantize_minmax(const float* P, int64_t D, int n, int64_t ldp, const void* plan_dev, int L, int dtype,
                           int bits, uint8_t* codes, int64_t ld, float* ab, void* ws, hipStream_t st);
int launch_beta_update(float* beta, const float* s, int64_t count, float lr, float lambda, hipStream_t st);
// bias1 = 1 - mu^t, bias2 = 1 - beta2^t (formed on the host in double)
int launch_beta_optim(int kind, float* beta, const float* s, float* m, float* v, int64_t count, float lr, float lambda,
                      float mu, float beta2, float eps, float bias1, float bias2, hipStream_t st);
int launch_quantize(const float* P, int64_t D, int n, int64_t ldp, const twa_pmat& out, hipStream_t st);
int launch_absmax(const float* P, int64_t D, int n, int64_t ldp, float* out_dev, bool accumulate, hipStream_t st);
int launch_gram(const float* W, int64_t D, int n, int64_t ldw, double* partial, int grid, double* gram,
                bool accumulate, bool orthonormal_input, hipStream_t st);
int launch_apply_rinv(const float* W, int64_t ldw, float* Q, int64_t ldq, int64_t D, int n, const float* rinv_dev,
                      int grid, bool zero_padding, hipStream_t st);

int launch_zero_status(int* status, hipStream_t st);
int launch_gram_factor(const double* gram, int n, float* rinv, double* Rout, int* status, hipStream_t st);
int launch_compose_upper(const double* R, double* Rtot, double* T, int n, hipStream_t st);
int launch_apply_rinv_store(const float* W, int64_t ldw, int64_t rows, int n, const float* rinv_dev, const twa_pmat& out,
                            int64_t row0, bool last, int grid, hipStream_t st);

int launch_read_probe(const void* buf, size_t bytes, uint32_t* sink, hipStream_t st);

}  // namespace twa
