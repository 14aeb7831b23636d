/*
 * Driver of the fp64 oracle for a build with -fsanitize=address,undefined (test infrastructure, CPU only):
 * every exported function of oracle/twa_oracle.c is called on small inputs whose buffers are heap blocks of
 * EXACTLY the documented sizes, so that an access one element past an end, a misaligned access or a signed
 * overflow in the oracle aborts the run.  The values are checked elsewhere; here only a few sums keep the
 * calls from being optimised away.  Exit status 0 = every call returned its expected status.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  int32_t dtype, n;
  int64_t D, ld;
  const void* data;
  const void* scales;
  int32_t block;
  float gscale;
  const int64_t* layer_off;
  int32_t L;
} orc_pmat;

int twa_oracle_threads(void);
void twa_oracle_set_threads(int t);
uint16_t twa_oracle_f32_to_f16(float f);
float twa_oracle_f16_to_f32(uint16_t h);
uint16_t twa_oracle_f32_to_bf16(float f);
float twa_oracle_bf16_to_f32(uint16_t b);
int twa_oracle_dequant(const orc_pmat* P, double* out, int64_t ldo);
int twa_oracle_project(const orc_pmat* P, const double* G, int32_t k, int64_t ldg, double* S);
int twa_oracle_expand_update(const orc_pmat* P, const double* s, double* w, double eta, double* g_tilde);
int twa_oracle_build_basis(const double* W, int64_t D, int32_t n, int64_t ldw, double* P, int64_t ldp, double* R,
                           double rank_tol, int32_t* bad);
int twa_oracle_centre_normalise(const double* W, int64_t D, int32_t n, int64_t ldw, double* E, int64_t lde, double* wbar);
int twa_oracle_project_layers(const orc_pmat* P, const double* g, const int64_t* off, int32_t L, double* S);
int twa_oracle_expand_update_layers(const orc_pmat* P, const double* S, const int64_t* off, int32_t L, double* w, double eta,
                                    double* g_tilde);
int twa_oracle_beta_step(double* beta, const double* s, int64_t count, double eta, double lambda);
int twa_oracle_beta_optim(int32_t kind, double* beta, const double* s, double* m, double* v, int64_t count, double eta,
                          double lambda, double mu_or_b1, double b2, double eps, int32_t t);
int twa_oracle_weights_from_beta(const orc_pmat* P, const double* beta, const int64_t* off, int32_t L, const double* wbar,
                                 double* w);
int twa_oracle_centre_normalise_layers(const double* W, int64_t D, int32_t n, int64_t ldw, const int64_t* off, int32_t L,
                                       double* E, int64_t lde, double* wbar, double* nrm);
int twa_oracle_quantize_i8(const float* P, int64_t D, int32_t n, int64_t ldp, int8_t* codes, int64_t ldc, float* scales,
                           int32_t block);
float twa_oracle_gscale_i4(const float* P, int64_t D, int32_t n, int64_t ldp);
int twa_oracle_quantize_i4(const float* P, int64_t D, int32_t n, int64_t ldp, uint8_t* codes, int64_t ldc,
                           uint16_t* scales, int32_t block, float gscale);
int twa_oracle_to_bf16(const float* P, int64_t D, int32_t n, int64_t ldp, uint16_t* out, int64_t ldo);
int twa_oracle_quantize_minmax(const double* P, int64_t D, int32_t n, int64_t ldp, int32_t B, const int64_t* layer_off,
                               int32_t L, uint16_t* codes, int64_t ldc, double* a_out, double* b_out);

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double rnd(void) {                       /* uniform in (-1, 1), a plain xorshift */
  rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
  return (double)(rng_state >> 11) / 4503599627370496.0 - 1.0;
}
static int fails = 0;
#define EXPECT(call, want) do { int rc_ = (call); if (rc_ != (want)) { printf("FAIL %s -> %d (want %d)\n", #call, rc_, (want)); ++fails; } } while (0)
#define NEW(type, count) ((type*)malloc(sizeof(type) * (size_t)(count)))

/* the step operators over one stored matrix: whole model, layer-wise, coefficient form */
static double run_steps(const orc_pmat* P, const int64_t* off, int32_t L) {
  const int64_t D = P->D;
  const int32_t n = P->n, k = 3;
  double* G = NEW(double, k * D); double* S = NEW(double, k * n); double* w = NEW(double, D); double* gt = NEW(double, D);
  double* dense = NEW(double, (int64_t)n * D); double* SL = NEW(double, (int64_t)L * n); double* wbar = NEW(double, D);
  for (int64_t i = 0; i < k * D; ++i) G[i] = rnd();
  for (int64_t i = 0; i < D; ++i) { w[i] = rnd(); wbar[i] = rnd(); }
  EXPECT(twa_oracle_dequant(P, dense, D), 0);
  EXPECT(twa_oracle_project(P, G, k, D, S), 0);
  EXPECT(twa_oracle_expand_update(P, S, w, 0.1, gt), 0);
  EXPECT(twa_oracle_expand_update(P, S + n, w, 0.1, NULL), 0);
  EXPECT(twa_oracle_project_layers(P, G, off, L, SL), 0);
  EXPECT(twa_oracle_expand_update_layers(P, SL, off, L, w, 0.1, gt), 0);
  EXPECT(twa_oracle_weights_from_beta(P, SL, off, L, wbar, w), 0);
  double acc = dense[(int64_t)n * D - 1] + S[k * n - 1] + w[D - 1] + gt[D - 1] + SL[(int64_t)L * n - 1];
  free(G); free(S); free(w); free(gt); free(dense); free(SL); free(wbar);
  return acc;
}

int main(void) {
  twa_oracle_set_threads(2);
  double sink = (double)twa_oracle_threads();
  for (int i = 0; i < 70000; i += 13) sink += twa_oracle_f16_to_f32((uint16_t)i) == 0.0f;
  const float specials[] = {0.0f, -0.0f, 1.0f, 65504.0f, 65520.0f, 1e-8f, 6e-8f, 6.1e-5f, -3.3e4f, INFINITY, -INFINITY, NAN, 3e38f};
  for (size_t i = 0; i < sizeof(specials) / sizeof(specials[0]); ++i)
    sink += twa_oracle_f32_to_f16(specials[i]) + twa_oracle_f32_to_bf16(specials[i]) + (twa_oracle_bf16_to_f32((uint16_t)(i * 977)) > 0);

  /* shapes: ragged D, padded leading dimensions, layers with an empty one and a one-element one */
  const int64_t D = 333, ld = 384;               /* ld: a multiple of 128 and of 64 */
  const int32_t n = 5, L = 5;
  const int64_t off[6] = {0, 100, 100, 101, 300, 333};

  /* ---- basis construction: fine, then dependent checkpoints */
  double* W = NEW(double, n * ld); double* P = NEW(double, n * ld); double* R = NEW(double, n * n);
  for (int64_t i = 0; i < n * ld; ++i) W[i] = rnd();
  int32_t bad = -1;
  EXPECT(twa_oracle_build_basis(W, D, n, ld, P, ld, R, 1e-6, &bad), 0);
  EXPECT(twa_oracle_build_basis(W, D, n, ld, P, ld, NULL, 1e-6, NULL), 0);
  for (int64_t i = 0; i < D; ++i) W[3 * ld + i] = 2.0 * W[0 * ld + i] - W[1 * ld + i];
  EXPECT(twa_oracle_build_basis(W, D, n, ld, P, ld, R, 1e-6, &bad), -6);
  if (bad != 3) { printf("FAIL rank error names column %d\n", bad); ++fails; }
  EXPECT(twa_oracle_build_basis(W, 3, n, ld, P, ld, R, 1e-6, &bad), -1);      /* n > D */
  for (int64_t i = 0; i < n * ld; ++i) W[i] = rnd();

  /* ---- the default basis, whole model and layer-wise */
  double* E = NEW(double, n * ld); double* wbar = NEW(double, D); double* nrm = NEW(double, L * n);
  EXPECT(twa_oracle_centre_normalise(W, D, n, ld, E, ld, wbar), 0);
  EXPECT(twa_oracle_centre_normalise_layers(W, D, n, ld, off, L, E, ld, wbar, nrm), 0);
  EXPECT(twa_oracle_centre_normalise_layers(W, D, n, ld, off, L, E, ld, wbar, NULL), 0);
  sink += E[n * ld - 1] + wbar[D - 1] + nrm[L * n - 1];

  /* ---- stored forms of the same matrix */
  float* P32 = NEW(float, n * ld);
  for (int64_t i = 0; i < n * ld; ++i) P32[i] = (float)(rnd() / 18.0);
  for (int64_t i = 128; i < 256; ++i) P32[2 * ld + i] = 0.0f;                /* an all-zero block */
  orc_pmat pm;
  memset(&pm, 0, sizeof(pm));
  pm.n = n; pm.D = D; pm.ld = ld; pm.gscale = 1.0f;
  {                                                                          /* fp64 and fp32 values */
    pm.dtype = -1; pm.data = E; sink += run_steps(&pm, off, L);
    pm.dtype = 0; pm.data = P32; sink += run_steps(&pm, off, L);
  }
  {                                                                          /* bfloat16 */
    uint16_t* b = NEW(uint16_t, n * ld);
    EXPECT(twa_oracle_to_bf16(P32, D, n, ld, b, ld), 0);
    pm.dtype = 1; pm.data = b; sink += run_steps(&pm, off, L);
    free(b);
  }
  {                                                                          /* int8, blocks of 128 */
    int8_t* c = NEW(int8_t, n * ld); float* sc = NEW(float, n * (ld / 128));
    EXPECT(twa_oracle_quantize_i8(P32, D, n, ld, c, ld, sc, 128), 0);
    EXPECT(twa_oracle_quantize_i8(P32, D, n, ld, c, ld, sc, 100), -1);        /* ldc % block */
    pm.dtype = 2; pm.data = c; pm.scales = sc; pm.block = 128; sink += run_steps(&pm, off, L);
    free(c); free(sc);
  }
  {                                                                          /* int4, blocks of 64, binary16 scales */
    uint8_t* c = NEW(uint8_t, n * ld / 2); uint16_t* sc = NEW(uint16_t, n * (ld / 64));
    const float gs = twa_oracle_gscale_i4(P32, D, n, ld);
    EXPECT(twa_oracle_quantize_i4(P32, D, n, ld, c, ld, sc, 64, gs), 0);
    EXPECT(twa_oracle_quantize_i4(P32, D, n, ld, c, ld, sc, 64, 0.0f), -1);
    pm.dtype = 3; pm.data = c; pm.scales = sc; pm.block = 64; pm.gscale = gs; sink += run_steps(&pm, off, L);
    pm.gscale = 1.0f;
    free(c); free(sc);
  }
  for (int32_t B = 1; B <= 16; B += (B < 4 ? 1 : 4)) {                       /* the paper's min-max codes: 1, 2, 3, 4, 8, 12, 16 bits */
    uint16_t* c = NEW(uint16_t, n * D); double* a = NEW(double, L); double* b = NEW(double, L); float* ab = NEW(float, 2 * L);
    EXPECT(twa_oracle_quantize_minmax(E, D, n, ld, B, off, L, c, D, a, b), 0);
    for (int32_t l = 0; l < L; ++l) { ab[2 * l] = (float)a[l]; ab[2 * l + 1] = (float)b[l]; }
    pm.dtype = 4; pm.data = c; pm.scales = ab; pm.ld = D; pm.layer_off = off; pm.L = L; sink += run_steps(&pm, off, L);
    pm.ld = ld; pm.layer_off = NULL; pm.L = 0;
    free(c); free(a); free(b); free(ab);
  }
  EXPECT(twa_oracle_quantize_minmax(E, D, n, ld, 17, off, L, NULL, D, NULL, NULL), -1);

  /* ---- coefficient steps */
  const int64_t count = (int64_t)L * n;
  double* beta = NEW(double, count); double* s = NEW(double, count); double* m = NEW(double, count); double* v = NEW(double, count);
  for (int64_t q = 0; q < count; ++q) { beta[q] = rnd(); s[q] = rnd(); m[q] = 0.0; v[q] = 0.0; }
  EXPECT(twa_oracle_beta_step(beta, s, count, 0.1, 1e-4), 0);
  EXPECT(twa_oracle_beta_optim(0, beta, s, m, NULL, count, 0.1, 1e-4, 0.9, 0.0, 0.0, 1), 0);
  EXPECT(twa_oracle_beta_optim(1, beta, s, m, v, count, 0.1, 1e-4, 0.9, 0.999, 1e-8, 1), 0);
  EXPECT(twa_oracle_beta_optim(2, beta, s, m, v, count, 0.1, 1e-4, 0.9, 0.999, 1e-8, 2), 0);
  EXPECT(twa_oracle_beta_optim(1, beta, s, m, NULL, count, 0.1, 1e-4, 0.9, 0.999, 1e-8, 1), -1);
  sink += beta[count - 1] + m[count - 1] + v[count - 1];

  free(W); free(P); free(R); free(E); free(wbar); free(nrm); free(P32); free(beta); free(s); free(m); free(v);
  printf("oracle under the sanitizers: %d unexpected statuses (checksum %.6g)\n", fails, sink);
  return fails ? 1 : 0;
}
