/*
 * twa_oracle.c -- slow, plain, fp64 CPU oracle for the projected-gradient step of
 * Trainable Weight Averaging (arXiv 2205.13104).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the test-suite, the smoke check
 * and the benchmark's "cpu_baseline" leg may build, load or call it.  It shares no code,
 * header, table or helper with the HIP library; it is written from the paper's
 * definitions so that a reader can check it against the paper by eye.
 *
 * Data layout (a storage convention, not arithmetic): every D x n matrix is "basis
 * major": basis vector / checkpoint j (0-based) is a contiguous run, element (i, j)
 * lives at a[j*ld + i], 0 <= i < D <= ld.  Elements i in [D, ld) are padding.
 *
 * What is computed, and where the paper defines it:
 *   twa_oracle_build_basis   Sec. 3 (solution set U = span{w_i}) and Sec. 4.1 (second
 *                            construction: orthogonalise the w_i one after another in
 *                            checkpoint order).  Result: the unique thin QR factor
 *                            W = P R, P^T P = I, R upper triangular, diag(R) > 0,
 *                            by Householder reflections in fp64.
 *   twa_oracle_project       Sec. 4.2, chain rule: dL/dbeta = P^T g.
 *   twa_oracle_expand_update Sec. 4.2, weight-space form of the update rule with
 *                            lambda = 0:  w <- w - eta * P (P^T g); here the n-vector
 *                            s stands for P^T g (or whatever the base optimiser made
 *                            of it) and the call forms g~ = P s and w -= eta g~.
 *   twa_oracle_quantize_*    Sec. 4.6 stores P as B-bit integer codes plus scaling
 *                            factors.  The grouping used here is the benchmark
 *                            configuration's: symmetric absmax per block of `block`
 *                            consecutive elements of ONE basis vector, round half to
 *                            even, codes in [-qmax, qmax].  The paper's own grouping
 *                            (one (a, b) pair per layer, min/max, Eq. of Sec. 4.6) is
 *                            twa_oracle_quantize_minmax.
 *   twa_oracle_centre_normalise  Sec. 4.1 first construction (mean removal and
 *                            normalisation), kept as a reference for that variant.
 *
 * Precision: all floating point is IEEE binary64, evaluated in the order written.
 * The quantiser is an ENCODING whose arithmetic is fixed in binary32 (see the recipe
 * above twa_oracle_quantize_i8); each binary32 operation of the recipe is evaluated
 * here as the binary64 operation rounded once to float, which yields the identical
 * result for * and / (53 >= 2*24 + 2), so the codes are unique and comparable bit for
 * bit.
 *
 * Threads: loops over independent outputs (the n dot products of a projection, the D
 * elements of an expansion) are split over OpenMP threads; no sum is re-associated.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_RANK (-6)
#define ORC_ERR_NOMEM (-8)

enum { ORC_F64 = -1, ORC_F32 = 0, ORC_BF16 = 1, ORC_I8 = 2, ORC_I4 = 3, ORC_MM = 4 };

int twa_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void twa_oracle_set_threads(int t) {
#ifdef _OPENMP
  if (t > 0) omp_set_num_threads(t);
#else
  (void)t;
#endif
}

/* ------------------------------------------------------------------------- */
/* binary16 / bfloat16 <-> binary32, written out from the IEEE 754 definitions */
/* ------------------------------------------------------------------------- */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* binary32 -> binary16, round to nearest, ties to even; overflow -> inf. */
uint16_t twa_oracle_f32_to_f16(float f) {
  uint32_t u = f32_bits(f);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
  uint32_t a = u & 0x7fffffffu;
  if (a >= 0x7f800000u) return (uint16_t)(sign | (a > 0x7f800000u ? 0x7e00u : 0x7c00u));
  /* value = m * 2^(e-150) with m the 24-bit significand (implicit bit restored) */
  int e = (int)(a >> 23);
  uint32_t m = a & 0x7fffffu;
  if (e == 0) return sign;              /* binary32 subnormal: < 2^-126, rounds to 0 */
  m |= 0x800000u;
  /* target: binary16 normal needs exponent e-127 in [-14, 15]; quantum 2^(E-10) */
  int E = e - 127;
  int shift;                             /* number of low bits of m to drop */
  if (E >= -14) shift = 13;              /* normal: keep 11 bits */
  else shift = 13 + (-14 - E);           /* subnormal: quantum fixed at 2^-24 */
  if (shift > 25) return sign;           /* below half of the smallest subnormal */
  uint32_t keep = m >> shift;
  uint32_t rem = m & ((1u << shift) - 1u);
  uint32_t half = 1u << (shift - 1);
  if (rem > half || (rem == half && (keep & 1u))) keep += 1u;
  uint32_t h;
  if (E >= -14) {
    /* keep has 11 bits (or 12 after a carry); fold the implicit bit into the exponent */
    h = ((uint32_t)(E + 15) << 10) + (keep - 0x400u);
  } else {
    h = keep;                            /* a carry into 0x400 lands on the smallest normal */
  }
  if (h >= 0x7c00u) h = 0x7c00u;
  return (uint16_t)(sign | h);
}

float twa_oracle_f16_to_f32(uint16_t h) {
  int sign = (h >> 15) & 1;
  int e = (h >> 10) & 0x1f;
  int m = h & 0x3ff;
  double v;
  if (e == 0) v = ldexp((double)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = ldexp((double)(m + 1024), e - 25);
  return (float)(sign ? -v : v);
}

/* binary32 -> bfloat16, round to nearest, ties to even. */
uint16_t twa_oracle_f32_to_bf16(float f) {
  uint32_t u = f32_bits(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  uint32_t keep = u >> 16, rem = u & 0xffffu;
  if (rem > 0x8000u || (rem == 0x8000u && (keep & 1u))) keep += 1u;
  return (uint16_t)keep;
}

float twa_oracle_bf16_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }

/* ------------------------------------------------------------------------- */
/* stored projection matrix, as the oracle sees it                            */
/* ------------------------------------------------------------------------- */

typedef struct {
  int32_t dtype;        /* ORC_F64 / ORC_F32 / ORC_BF16 / ORC_I8 / ORC_I4 */
  int32_t n;
  int64_t D;
  int64_t ld;           /* elements between consecutive basis vectors */
  const void* data;     /* values, or codes (I4: two per byte, even element in the low nibble, stored q+8) */
  const void* scales;   /* [n][ld/block]: float (I8) or binary16 bits (I4) */
  int32_t block;
  float gscale;         /* power-of-two multiplier of the binary16 scales (I4) */
  /* ORC_MM only (Sec. 4.6, the paper's own format): data = one uint16 code per element,
     scales = L pairs of floats (a_l, b_l), value = a_l * code + b_l for the elements of layer l */
  const int64_t* layer_off;
  int32_t L;
} orc_pmat;

/* The value of stored element (i, j), exactly, as a double. */
static double deq(const orc_pmat* P, int64_t i, int32_t j) {
  switch (P->dtype) {
    case ORC_F64: return ((const double*)P->data)[(int64_t)j * P->ld + i];
    case ORC_F32: return (double)((const float*)P->data)[(int64_t)j * P->ld + i];
    case ORC_BF16:
      return (double)twa_oracle_bf16_to_f32(((const uint16_t*)P->data)[(int64_t)j * P->ld + i]);
    case ORC_I8: {
      int64_t nblk = P->ld / P->block;
      double sc = (double)((const float*)P->scales)[(int64_t)j * nblk + i / P->block];
      return sc * (double)((const int8_t*)P->data)[(int64_t)j * P->ld + i];
    }
    case ORC_MM: {
      int32_t l = 0, hi = P->L - 1;                              /* bisection: the last layer that starts at or before i */
      while (l < hi) {
        int32_t mid = (l + hi + 1) / 2;
        if (P->layer_off[mid] <= i) l = mid; else hi = mid - 1;
      }
      const float* ab = (const float*)P->scales + 2 * (int64_t)l;
      return (double)ab[0] * (double)((const uint16_t*)P->data)[(int64_t)j * P->ld + i] + (double)ab[1];
    }
    case ORC_I4: {
      int64_t nblk = P->ld / P->block;
      uint16_t h = ((const uint16_t*)P->scales)[(int64_t)j * nblk + i / P->block];
      double sc = (double)twa_oracle_f16_to_f32(h) * (double)P->gscale;
      uint8_t byte = ((const uint8_t*)P->data)[((int64_t)j * P->ld + i) >> 1];
      int q = (int)((i & 1) ? (byte >> 4) : (byte & 0xf)) - 8;
      return sc * (double)q;
    }
  }
  return NAN;
}

/* Widen a stored matrix to plain doubles: out[j*ldo + i] = value of element (i, j). */
int twa_oracle_dequant(const orc_pmat* P, double* out, int64_t ldo) {
  if (!P || !out || ldo < P->D) return ORC_ERR_ARG;
  for (int32_t j = 0; j < P->n; ++j)
    for (int64_t i = 0; i < P->D; ++i) out[(int64_t)j * ldo + i] = deq(P, i, j);
  return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.2: s = P^T g  (k gradients at once: S[c][j] = sum_i P_ij G[c][i])   */
/* ------------------------------------------------------------------------- */
int twa_oracle_project(const orc_pmat* P, const double* G, int32_t k, int64_t ldg, double* S) {
  if (!P || !G || !S || k <= 0 || ldg < P->D) return ORC_ERR_ARG;
  const int32_t n = P->n;
  const int64_t D = P->D;
#pragma omp parallel for collapse(2) schedule(static)
  for (int32_t c = 0; c < k; ++c)
    for (int32_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (int64_t i = 0; i < D; ++i) acc += deq(P, i, j) * G[(int64_t)c * ldg + i];
      S[(int64_t)c * n + j] = acc;
    }
  return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.2: g~ = P s ;  w <- w - eta g~   (lambda = 0)                        */
/* g_tilde may be NULL.                                                       */
/* ------------------------------------------------------------------------- */
int twa_oracle_expand_update(const orc_pmat* P, const double* s, double* w, double eta,
                             double* g_tilde) {
  if (!P || !s || !w) return ORC_ERR_ARG;
  const int32_t n = P->n;
  const int64_t D = P->D;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < D; ++i) {
    double gt = 0.0;
    for (int32_t j = 0; j < n; ++j) gt += deq(P, i, j) * s[j];
    if (g_tilde) g_tilde[i] = gt;
    w[i] = w[i] - eta * gt;
  }
  return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.1 (orthogonalisation variant): thin QR of W by Householder.         */
/*   W: D x n basis-major doubles (read only), ldw >= D                       */
/*   P: D x n basis-major doubles (out), ldp >= D                             */
/*   R: n x n row-major doubles (out, may be NULL), R[a*n+b], zero below diag */
/* Error ORC_ERR_RANK if some |R_kk| <= rank_tol * max_j ||w_j||; then *bad   */
/* (if given) holds the 0-based index of the first such column.               */
/* ------------------------------------------------------------------------- */
int twa_oracle_build_basis(const double* W, int64_t D, int32_t n, int64_t ldw, double* P,
                           int64_t ldp, double* R, double rank_tol, int32_t* bad) {
  if (!W || !P || D <= 0 || n <= 0 || ldw < D || ldp < D || (int64_t)n > D) return ORC_ERR_ARG;
  double* A = (double*)malloc(sizeof(double) * (size_t)D * (size_t)n);   /* working copy; ends as reflectors */
  double* Rr = (double*)calloc((size_t)n * (size_t)n, sizeof(double));
  double* beta = (double*)malloc(sizeof(double) * (size_t)n);
  if (!A || !Rr || !beta) { free(A); free(Rr); free(beta); return ORC_ERR_NOMEM; }
  double maxnorm = 0.0;
  for (int32_t j = 0; j < n; ++j) {
    double ss = 0.0;
    for (int64_t i = 0; i < D; ++i) { double x = W[(int64_t)j * ldw + i]; A[(int64_t)j * D + i] = x; ss += x * x; }
    if (sqrt(ss) > maxnorm) maxnorm = sqrt(ss);
  }
  int rc = ORC_OK;
  /* Forward sweep: reflector k maps column k (rows k..D-1) onto alpha e_k. */
  for (int32_t k = 0; k < n; ++k) {
    double* x = A + (int64_t)k * D;
    double ss = 0.0;
    for (int64_t i = k; i < D; ++i) ss += x[i] * x[i];
    double nrm = sqrt(ss);
    if (!(nrm > rank_tol * maxnorm)) { rc = ORC_ERR_RANK; if (bad) *bad = k; break; }
    double alpha = (x[k] >= 0.0) ? -nrm : nrm;
    /* v = x - alpha e_k, stored in place in rows k..D-1 of column k */
    for (int32_t a = 0; a < k; ++a) Rr[a * n + k] = x[a];
    Rr[k * n + k] = alpha;
    x[k] -= alpha;
    double vv = 0.0;
    for (int64_t i = k; i < D; ++i) vv += x[i] * x[i];
    beta[k] = (vv > 0.0) ? 2.0 / vv : 0.0;
    /* apply H_k = I - beta v v^T to the remaining columns */
#pragma omp parallel for schedule(static)
    for (int32_t j = k + 1; j < n; ++j) {
      double* y = A + (int64_t)j * D;
      double dot = 0.0;
      for (int64_t i = k; i < D; ++i) dot += x[i] * y[i];
      double t = beta[k] * dot;
      for (int64_t i = k; i < D; ++i) y[i] -= t * x[i];
    }
  }
  if (rc == ORC_OK) {
    /* Q = H_0 H_1 ... H_{n-1} [I_n; 0]: apply the reflectors in reverse to unit vectors. */
#pragma omp parallel for schedule(static)
    for (int32_t j = 0; j < n; ++j) {
      double* q = P + (int64_t)j * ldp;
      for (int64_t i = 0; i < D; ++i) q[i] = 0.0;
      q[j] = 1.0;
      for (int32_t k = n - 1; k >= 0; --k) {
        const double* v = A + (int64_t)k * D;
        double dot = 0.0;
        for (int64_t i = k; i < D; ++i) dot += v[i] * q[i];
        double t = beta[k] * dot;
        for (int64_t i = k; i < D; ++i) q[i] -= t * v[i];
      }
    }
    /* make diag(R) positive: flip row k of R together with column k of Q */
    for (int32_t k = 0; k < n; ++k)
      if (Rr[k * n + k] < 0.0) {
        for (int32_t b = k; b < n; ++b) Rr[k * n + b] = -Rr[k * n + b];
        double* q = P + (int64_t)k * ldp;
        for (int64_t i = 0; i < D; ++i) q[i] = -q[i];
      }
    for (int32_t j = 0; j < n; ++j)
      for (int64_t i = D; i < ldp; ++i) P[(int64_t)j * ldp + i] = 0.0;
    if (R) memcpy(R, Rr, sizeof(double) * (size_t)n * (size_t)n);
  }
  free(A); free(Rr); free(beta);
  return rc;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.1 (default construction): wbar = mean_i w_i; e_i = (w_i - wbar)/||.|| */
/* ------------------------------------------------------------------------- */
int twa_oracle_centre_normalise(const double* W, int64_t D, int32_t n, int64_t ldw, double* E,
                                int64_t lde, double* wbar) {
  if (!W || !E || !wbar || D <= 0 || n <= 0 || ldw < D || lde < D) return ORC_ERR_ARG;
  for (int64_t i = 0; i < D; ++i) {
    double m = 0.0;
    for (int32_t j = 0; j < n; ++j) m += W[(int64_t)j * ldw + i];
    wbar[i] = m / (double)n;
  }
  for (int32_t j = 0; j < n; ++j) {
    double ss = 0.0;
    for (int64_t i = 0; i < D; ++i) { double d = W[(int64_t)j * ldw + i] - wbar[i]; ss += d * d; }
    double nrm = sqrt(ss);
    for (int64_t i = 0; i < D; ++i)
      E[(int64_t)j * lde + i] = (nrm > 0.0) ? (W[(int64_t)j * ldw + i] - wbar[i]) / nrm : 0.0;
    for (int64_t i = D; i < lde; ++i) E[(int64_t)j * lde + i] = 0.0;
  }
  return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.5 (layer-wise processing) and Alg. 1.  The D parameters are cut     */
/* into L consecutive groups; layer l covers elements [off[l], off[l+1]),     */
/* off[0] = 0, off[L] = D, empty layers allowed.  Every layer has its own     */
/* block P^l (rows off[l]..off[l+1] of the stored matrix) and its own n       */
/* coefficients, kept as row l of an L x n array.                             */
/* ------------------------------------------------------------------------- */
static int layers_ok(const int64_t* off, int32_t L, int64_t D) {
  if (!off || L < 1 || off[0] != 0 || off[L] != D) return 0;
  for (int32_t l = 0; l < L; ++l) if (off[l + 1] < off[l]) return 0;
  return 1;
}

/* Alg. 1, coefficient gradient of layer l:  S[l][j] = sum_{i in layer l} P_ij g_i */
int twa_oracle_project_layers(const orc_pmat* P, const double* g, const int64_t* off, int32_t L,
                              double* S) {
  if (!P || !g || !S || !layers_ok(off, L, P->D)) return ORC_ERR_ARG;
  const int32_t n = P->n;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int32_t l = 0; l < L; ++l)
    for (int32_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (int64_t i = off[l]; i < off[l + 1]; ++i) acc += deq(P, i, j) * g[i];
      S[(int64_t)l * n + j] = acc;
    }
  return ORC_OK;
}

/* Weight-space form of the layer-wise step with lambda = 0:                  */
/*   g~_i = sum_j P_ij S[l(i)][j] ;  w_i <- w_i - eta g~_i                     */
int twa_oracle_expand_update_layers(const orc_pmat* P, const double* S, const int64_t* off, int32_t L,
                                    double* w, double eta, double* g_tilde) {
  if (!P || !S || !w || !layers_ok(off, L, P->D)) return ORC_ERR_ARG;
  const int32_t n = P->n;
  for (int32_t l = 0; l < L; ++l) {
    const double* sl = S + (int64_t)l * n;
#pragma omp parallel for schedule(static)
    for (int64_t i = off[l]; i < off[l + 1]; ++i) {
      double gt = 0.0;
      for (int32_t j = 0; j < n; ++j) gt += deq(P, i, j) * sl[j];
      if (g_tilde) g_tilde[i] = gt;
      w[i] = w[i] - eta * gt;
    }
  }
  return ORC_OK;
}

/* Alg. 1, "update variables":  beta <- (1 - eta*lambda) beta - eta s   (count = L*n entries) */
int twa_oracle_beta_step(double* beta, const double* s, int64_t count, double eta, double lambda) {
  if (!beta || !s || count < 0) return ORC_ERR_ARG;
  for (int64_t q = 0; q < count; ++q) beta[q] = (1.0 - eta * lambda) * beta[q] - eta * s[q];
  return ORC_OK;
}

/* The coefficient step with the base optimiser in place of plain gradient descent (Sec. 5.1: the base
 * optimiser of the run is applied to the coefficients; the paper's runs use SGD with momentum, Adam and
 * AdamW).  The optimisers are the published ones, written out on the count = L*n coefficients:
 *   kind 0, heavy-ball momentum:   d = s + lambda beta;  m <- mu m + d;  beta <- beta - eta m
 *                                  (mu = 0 is Alg. 1's own step)
 *   kind 1, Adam, decay as an L2 term:   d = s + lambda beta
 *   kind 2, AdamW, decoupled decay:      beta <- (1 - eta lambda) beta first;  d = s
 *     then for both:  m <- b1 m + (1 - b1) d;  v <- b2 v + (1 - b2) d^2;
 *                     beta <- beta - eta (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps),   t = 1, 2, ...
 * m (and v) are the caller's state, zero before the first step. */
int twa_oracle_beta_optim(int32_t kind, double* beta, const double* s, double* m, double* v, int64_t count,
                          double eta, double lambda, double mu_or_b1, double b2, double eps, int32_t t) {
  if (!beta || !s || !m || count < 0 || kind < 0 || kind > 2) return ORC_ERR_ARG;
  if (kind != 0 && (!v || t < 1)) return ORC_ERR_ARG;
  for (int64_t q = 0; q < count; ++q) {
    if (kind == 0) {
      const double d = s[q] + lambda * beta[q];
      m[q] = mu_or_b1 * m[q] + d;
      beta[q] -= eta * m[q];
    } else {
      double d = s[q];
      if (kind == 1) d += lambda * beta[q];
      else beta[q] *= 1.0 - eta * lambda;
      m[q] = mu_or_b1 * m[q] + (1.0 - mu_or_b1) * d;
      v[q] = b2 * v[q] + (1.0 - b2) * d * d;
      const double mhat = m[q] / (1.0 - pow(mu_or_b1, (double)t));
      const double vhat = v[q] / (1.0 - pow(b2, (double)t));
      beta[q] -= eta * mhat / (sqrt(vhat) + eps);
    }
  }
  return ORC_OK;
}

/* Alg. 1, "update weights":  w^l = wbar^l + P^l beta^l */
int twa_oracle_weights_from_beta(const orc_pmat* P, const double* beta, const int64_t* off, int32_t L,
                                 const double* wbar, double* w) {
  if (!P || !beta || !wbar || !w || !layers_ok(off, L, P->D)) return ORC_ERR_ARG;
  const int32_t n = P->n;
  for (int32_t l = 0; l < L; ++l) {
    const double* bl = beta + (int64_t)l * n;
#pragma omp parallel for schedule(static)
    for (int64_t i = off[l]; i < off[l + 1]; ++i) {
      double acc = 0.0;
      for (int32_t j = 0; j < n; ++j) acc += deq(P, i, j) * bl[j];
      w[i] = wbar[i] + acc;
    }
  }
  return ORC_OK;
}

/* Sec. 4.5, layer-wise basis:  wbar = mean_i w_i ;                            */
/*   e_i^l = (w_i^l - wbar^l) / ||w_i^l - wbar^l||_2 .                          */
/* A (layer, checkpoint) pair whose centred part is exactly zero gives a zero  */
/* vector (the paper does not say; a zero direction changes nothing).          */
/* nrm (may be NULL) receives the L x n norms.                                 */
int twa_oracle_centre_normalise_layers(const double* W, int64_t D, int32_t n, int64_t ldw,
                                       const int64_t* off, int32_t L, double* E, int64_t lde,
                                       double* wbar, double* nrm) {
  if (!W || !E || !wbar || D <= 0 || n <= 0 || ldw < D || lde < D || !layers_ok(off, L, D)) return ORC_ERR_ARG;
  for (int64_t i = 0; i < D; ++i) {
    double m = 0.0;
    for (int32_t j = 0; j < n; ++j) m += W[(int64_t)j * ldw + i];
    wbar[i] = m / (double)n;
  }
  for (int32_t l = 0; l < L; ++l)
    for (int32_t j = 0; j < n; ++j) {
      double ss = 0.0;
      for (int64_t i = off[l]; i < off[l + 1]; ++i) { double d = W[(int64_t)j * ldw + i] - wbar[i]; ss += d * d; }
      const double nr = sqrt(ss);
      if (nrm) nrm[(int64_t)l * n + j] = nr;
      for (int64_t i = off[l]; i < off[l + 1]; ++i)
        E[(int64_t)j * lde + i] = (nr > 0.0) ? (W[(int64_t)j * ldw + i] - wbar[i]) / nr : 0.0;
    }
  for (int32_t j = 0; j < n; ++j)
    for (int64_t i = D; i < lde; ++i) E[(int64_t)j * lde + i] = 0.0;
  return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Block-absmax quantiser.  Recipe (every step one correctly rounded binary32 */
/* operation; f(.) below = "round the exact result once to binary32"):        */
/*   block b of vector j = elements i in [b*block, min((b+1)*block, D))       */
/*   amax   = max |p_i| over the block                                         */
/*   scale  = f(amax / qmax)                     qmax = 127 (I8) or 7 (I4)     */
/*   I8: stored scale = scale, effective scale e = scale                       */
/*   I4: stored h = binary16_rne(f(scale / gscale)), e = float(h) * gscale     */
/*   e == 0  ->  every code of the block is 0                                  */
/*   inv    = f(1 / e)                                                         */
/*   q_i    = clamp(round_half_even(f(p_i * inv)), -qmax, +qmax)               */
/*   padding elements i in [D, ld): code 0; blocks wholly in padding: scale 0  */
/* ------------------------------------------------------------------------- */
static int code_of(float p, float inv, int qmax) {
  float t = (float)((double)p * (double)inv);
  double r = nearbyint((double)t);         /* default rounding mode: ties to even */
  if (r > (double)qmax) r = (double)qmax;
  if (r < -(double)qmax) r = -(double)qmax;
  return (int)r;
}

static float block_amax(const float* p, int64_t lo, int64_t hi) {
  float amax = 0.0f;
  for (int64_t i = lo; i < hi; ++i) { float a = fabsf(p[i]); if (a > amax) amax = a; }
  return amax;
}

int twa_oracle_quantize_i8(const float* P, int64_t D, int32_t n, int64_t ldp, int8_t* codes,
                           int64_t ldc, float* scales, int32_t block) {
  if (!P || !codes || !scales || D <= 0 || n <= 0 || block <= 0 || ldp < D || ldc < D || ldc % block)
    return ORC_ERR_ARG;
  const int64_t nblk = ldc / block;
#pragma omp parallel for schedule(static)
  for (int32_t j = 0; j < n; ++j) {
    const float* p = P + (int64_t)j * ldp;
    for (int64_t b = 0; b < nblk; ++b) {
      int64_t lo = b * block, hi = lo + block;
      int64_t hid = hi < D ? hi : D;
      float amax = (lo < D) ? block_amax(p, lo, hid) : 0.0f;
      float scale = (float)((double)amax / 127.0);
      scales[(int64_t)j * nblk + b] = scale;
      float inv = (scale != 0.0f) ? (float)(1.0 / (double)scale) : 0.0f;
      for (int64_t i = lo; i < hi; ++i)
        codes[(int64_t)j * ldc + i] = (int8_t)((i < D && scale != 0.0f) ? code_of(p[i], inv, 127) : 0);
    }
  }
  return ORC_OK;
}

/* Power-of-two multiplier that keeps every binary16 scale normal:            */
/*   gscale = 2^(floor(log2(max over blocks of f(amax/7))) - 14), 1 if P == 0. */
float twa_oracle_gscale_i4(const float* P, int64_t D, int32_t n, int64_t ldp) {
  float amax = 0.0f;
  for (int32_t j = 0; j < n; ++j) {
    float a = block_amax(P + (int64_t)j * ldp, 0, D);
    if (a > amax) amax = a;
  }
  float smax = (float)((double)amax / 7.0);
  if (!(smax > 0.0f)) return 1.0f;
  int ex;
  (void)frexp((double)smax, &ex);          /* smax = m * 2^ex, m in [0.5, 1) -> floor(log2) = ex-1 */
  return (float)ldexp(1.0, ex - 1 - 14);
}

int twa_oracle_quantize_i4(const float* P, int64_t D, int32_t n, int64_t ldp, uint8_t* codes,
                           int64_t ldc, uint16_t* scales, int32_t block, float gscale) {
  if (!P || !codes || !scales || D <= 0 || n <= 0 || block <= 0 || (block & 1) || ldp < D || ldc < D ||
      ldc % block || !(gscale > 0.0f))
    return ORC_ERR_ARG;
  const int64_t nblk = ldc / block;
#pragma omp parallel for schedule(static)
  for (int32_t j = 0; j < n; ++j) {
    const float* p = P + (int64_t)j * ldp;
    for (int64_t b = 0; b < nblk; ++b) {
      int64_t lo = b * block, hi = lo + block;
      int64_t hid = hi < D ? hi : D;
      float amax = (lo < D) ? block_amax(p, lo, hid) : 0.0f;
      float scale = (float)((double)amax / 7.0);
      uint16_t h = twa_oracle_f32_to_f16((float)((double)scale / (double)gscale));
      scales[(int64_t)j * nblk + b] = h;
      float eff = (float)((double)twa_oracle_f16_to_f32(h) * (double)gscale);
      float inv = (eff != 0.0f) ? (float)(1.0 / (double)eff) : 0.0f;
      for (int64_t i = lo; i < hi; i += 2) {
        int q0 = (i < D && eff != 0.0f) ? code_of(p[i], inv, 7) : 0;
        int q1 = (i + 1 < D && eff != 0.0f) ? code_of(p[i + 1], inv, 7) : 0;
        codes[((int64_t)j * ldc + i) >> 1] = (uint8_t)((q0 + 8) | ((q1 + 8) << 4));
      }
    }
  }
  return ORC_OK;
}

int twa_oracle_to_bf16(const float* P, int64_t D, int32_t n, int64_t ldp, uint16_t* out, int64_t ldo) {
  if (!P || !out || D <= 0 || n <= 0 || ldp < D || ldo < D) return ORC_ERR_ARG;
  for (int32_t j = 0; j < n; ++j) {
    for (int64_t i = 0; i < D; ++i) out[(int64_t)j * ldo + i] = twa_oracle_f32_to_bf16(P[(int64_t)j * ldp + i]);
    for (int64_t i = D; i < ldo; ++i) out[(int64_t)j * ldo + i] = 0;
  }
  return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Sec. 4.6, the paper's own quantiser: one (a, b) per layer, shared by all n */
/* basis vectors:  a = (max - min)/(2^B - 1), b = min,                        */
/*   code = round((p - b)/a) in {0 .. 2^B - 1},   p~ = a*code + b.            */
/* Evaluated in fp64; ties to even (the paper names no tie rule); a == 0      */
/* (constant layer) gives code 0.  layer_off has L+1 entries, layer l covers  */
/* elements [layer_off[l], layer_off[l+1]).  codes: one uint16 per element.   */
/* ------------------------------------------------------------------------- */
int twa_oracle_quantize_minmax(const double* P, int64_t D, int32_t n, int64_t ldp, int32_t B,
                               const int64_t* layer_off, int32_t L, uint16_t* codes, int64_t ldc,
                               double* a_out, double* b_out) {
  if (!P || !layer_off || !codes || !a_out || !b_out || B < 1 || B > 16 || L < 1 || ldp < D || ldc < D)
    return ORC_ERR_ARG;
  if (layer_off[0] != 0 || layer_off[L] != D) return ORC_ERR_ARG;
  const double levels = (double)((1u << B) - 1u);
  for (int32_t l = 0; l < L; ++l) {
    int64_t lo = layer_off[l], hi = layer_off[l + 1];
    if (hi < lo) return ORC_ERR_ARG;
    if (hi == lo) { a_out[l] = 0.0; b_out[l] = 0.0; continue; }      /* an empty layer has nothing to store */
    double mn = INFINITY, mx = -INFINITY;
    for (int32_t j = 0; j < n; ++j)
      for (int64_t i = lo; i < hi; ++i) {
        double v = P[(int64_t)j * ldp + i];
        if (v < mn) mn = v;
        if (v > mx) mx = v;
      }
    double a = (mx - mn) / levels, b = mn;
    a_out[l] = a; b_out[l] = b;
    for (int32_t j = 0; j < n; ++j)
      for (int64_t i = lo; i < hi; ++i) {
        double c = (a > 0.0) ? nearbyint((P[(int64_t)j * ldp + i] - b) / a) : 0.0;
        if (c < 0.0) c = 0.0;
        if (c > levels) c = levels;
        codes[(int64_t)j * ldc + i] = (uint16_t)c;
      }
  }
  return ORC_OK;
}
