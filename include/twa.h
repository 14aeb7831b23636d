/*
 * twa.h -- C ABI of the MI355X (gfx950) library for the projected-gradient step of
 * Trainable Weight Averaging (arXiv 2205.13104).
 *
 * The paper trains the n coefficients of a weighted average of n checkpoints
 * w_1..w_n in R^D by ordinary gradient descent restricted to U = span{w_i} (Sec. 3):
 * with P = [e_1 .. e_n] a basis of U (Sec. 4.1) each iteration computes
 *     s  = P^T g                      (Sec. 4.2, gradient w.r.t. the coefficients)
 *     g~ = P s ,  w <- w - eta g~     (Sec. 4.2, weight-space form of the update, lambda = 0)
 * and P may be kept as low-bit integer codes plus scaling factors (Sec. 4.6).
 * This library provides exactly those operations, plus the one-time construction of an
 * orthonormal P from the checkpoints (the orthogonalisation variant of Sec. 4.1).
 *
 * Conventions common to every entry point
 *   - Plain C types only.  Every pointer is a DEVICE pointer unless its name ends in
 *     _host.  The caller owns every buffer; the library never frees or keeps them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on it and return without synchronising, except where stated.
 *   - Matrices are "basis major": vector j (0-based) of a D x n matrix is the contiguous
 *     run x[j*ld .. j*ld + D), ld >= D.  Elements [D, ld) of each run are padding.
 *   - Return value: TWA_OK (0) or a negative twa_status.  Argument errors are detected on
 *     the host before anything is enqueued (no GPU needed to get them).
 *   - Device base pointers must be 16-byte aligned; `ld` is a multiple of TWA_LD_MULTIPLE
 *     (fp32, bf16) or of TWA_SCALE_SPAN (every integer-code type) elements.  Padding elements must hold finite
 *     values (the library's own producers write zeros there).
 *   - Limits: 1 <= n <= TWA_MAX_N, 1 <= k <= TWA_MAX_K, 1 <= D, and D * (bytes per stored
 *     element) < 2^32 for one vector (D <= 1.07e9 for fp32).
 */
#ifndef TWA_H_
#define TWA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TWA_MAX_N 128
#define TWA_MAX_K 8
#define TWA_LD_MULTIPLE 128   /* ld of fp32 / bf16 matrices is a multiple of this many elements   */
#define TWA_SCALE_SPAN 2048   /* ld of integer-code matrices is a multiple of this many elements  */

typedef enum twa_status {
  TWA_OK = 0,
  TWA_ERR_NULL = -1,      /* a required pointer is NULL                                        */
  TWA_ERR_SHAPE = -2,     /* D, n, k, ld or block out of range                                 */
  TWA_ERR_ALIGN = -3,     /* pointer not 16-byte aligned, or ld not a multiple of 128 / 2048   */
  TWA_ERR_DTYPE = -4,     /* unknown storage type, or one the call does not accept             */
  TWA_ERR_WORKSPACE = -5, /* workspace missing or smaller than the query reports               */
  TWA_ERR_RANK = -6,      /* checkpoints numerically linearly dependent (build_basis)          */
  TWA_ERR_HIP = -7,       /* a HIP runtime call failed; see twa_last_hip_error()               */
  TWA_ERR_NO_DEVICE = -8, /* no usable gfx950 device                                           */
  TWA_ERR_LIMIT = -9      /* size beyond the fixed device array of twa_project_noalloc         */
} twa_status;

/* Storage type of a projection matrix. */
typedef enum twa_dtype {
  TWA_F32 = 0,  /* IEEE binary32 values                                                        */
  TWA_BF16 = 1, /* bfloat16 values (binary32 rounded to nearest even to 16 bits)               */
  TWA_I8 = 2,   /* int8 codes q in [-127,127] + one binary32 scale per block: value = scale*q  */
  TWA_I4 = 3,   /* 4-bit codes q in [-7,7], two per byte (element i in the LOW nibble when i is
                   even), stored offset-binary as q+8; one binary16 scale h per block:
                   value = (float(h) * gscale) * q                                             */
  /* The paper's own format (Sec. 4.6): unsigned B-bit codes c in [0, 2^B - 1] and ONE pair of
     binary32 factors (a_l, b_l) per layer, shared by all n vectors: value = a_l * c + b_l.
     `scales` of the descriptor points to the 2L floats a_0, b_0, a_1, b_1, ...; `block` and
     `gscale` are ignored.  Only the layer-wise calls accept these (with the plan of the same
     layer table the matrix was quantised with).                                               */
  TWA_U8MM = 4, /* B <= 8: the byte holds c - 2^(B-1) as a two's-complement int8; the descriptor's
                   `block` field carries B (0 means 8)                                           */
  TWA_U4MM = 5, /* B = 4: two codes per byte, element i in the LOW nibble when i is even         */
  TWA_U16MM = 6, /* B <= 16: the 16-bit word holds c - 2^(B-1) as an int16; `block` carries B (0: 16) */
  TWA_U2MM = 7,  /* B = 2: four codes per byte, element i in bits 2*(i mod 4) .. 2*(i mod 4)+1    */
  TWA_U1MM = 8,  /* B = 1: eight codes per byte, element i in bit i mod 8                         */
  TWA_U3MM = 9   /* B = 3 in exactly 3 bits: every 32 consecutive elements are three 32-bit words.
                    Element e = 16h + 4k + m of the group (h in 0..1, k in 0..3, m in 0..3) has its
                    two LOW bits in word h at bits 2(4k+m) .. 2(4k+m)+1 -- words 0 and 1 are the
                    TWA_U2MM layout of c mod 4 -- and its HIGH bit in word 2 at bit 8k + m + 4h, so
                    that one shift and mask of word 2 lines four high bits up with four byte lanes of
                    low parts                                                                       */
} twa_dtype;

/*
 * Descriptor of a stored projection matrix P (Sec. 4.2: P = [e_1 .. e_n]; Sec. 4.6 for the
 * integer forms).  Filled by the caller; passed by pointer; never retained.
 *   data   : n runs of `ld` elements (F32: 4 B, BF16: 2 B, I8: 1 B, I4: 1/2 B per element; the min-max
 *            types: their container width, see twa_dtype).
 *   scales : one scale per block; I8: float, I4: binary16 bits (uint16_t); NULL for F32/BF16.
 *            Block b of vector j covers elements [b*block, min((b+1)*block, D)) of THAT
 *            vector.  Storage is "span interleaved": with G = TWA_SCALE_SPAN/block, the scale
 *            of block b of vector j sits at index ((b / G) * n + j) * G + (b % G), i.e. an
 *            array [ld/TWA_SCALE_SPAN][n][G].  The G scales that cover one 2048-element span
 *            are contiguous and the spans of all n vectors follow each other, so a kernel tile
 *            reads the scales of all vectors in one contiguous run.  (The paper keeps one
 *            scale pair per layer, Sec. 4.6; the per-block grouping is the finer-grained form
 *            of the benchmark configuration.)
 *   block  : power of two in {32, 64, 128, 256} (I8, I4); ignored for F32/BF16.  For TWA_U8MM and
 *            TWA_U16MM: B, the bits of the codes (0 = the container's width); ignored by the
 *            narrower min-max types.
 *   gscale : I4 only: a power of two multiplying every binary16 scale so that the scales of
 *            a matrix with tiny entries (|p| ~ D^-1/2) stay normal binary16 numbers.
 */
typedef struct twa_pmat {
  int32_t dtype;   /* twa_dtype */
  int32_t n;
  int64_t D;
  int64_t ld;
  void* data;
  void* scales;
  int32_t block;
  float gscale;
} twa_pmat;

/* Library version (major*10000 + minor*100 + patch). */
int twa_version(void);

/* Static, NUL-terminated description of a status code. */
const char* twa_strerror(int status);

/* hipError_t value of the most recent failing HIP call made by this library in the calling
 * thread (0 if none). */
int twa_last_hip_error(void);

/*
 * Launch geometry, for tests and tuning runs only.  The library reads NO environment variable and keeps no
 * other state between calls; these three process-wide integers are the one exception, and they change the
 * launch geometry only -- never which operation is computed.  0 (the initial value) leaves the choice to the
 * library.  The reduction order of twa_project[_layers] follows the grid, so the bits of its result are
 * reproducible for a given knob value, not across values.  Set them while no call of the library is in flight.
 *   TWA_KNOB_PROJECT_GRID      upper bound of the workgroups of the projection kernels (also the squares pass of
 *                              twa_centre_normalise)             1 .. 2048
 *   TWA_KNOB_EXPAND_GRID       upper bound of the workgroups of the expansion kernels          1 .. 2048
 *   TWA_KNOB_BASIS_WGS_PER_CU  workgroups per compute unit of the Gram / apply kernels (default 2)
 * Errors: TWA_ERR_DTYPE (unknown knob), TWA_ERR_SHAPE (value < 0 or > 2048).
 */
#define TWA_KNOB_PROJECT_GRID 0
#define TWA_KNOB_EXPAND_GRID 1
#define TWA_KNOB_BASIS_WGS_PER_CU 2
#define TWA_KNOB_COUNT 3
int twa_set_launch_knob(int32_t knob, int32_t value);

/*
 * Sizes of the buffers that hold an n-vector matrix of logical length D in storage `dtype`.
 * Writes the smallest admissible ld, and the byte sizes of `data` and `scales` for that ld
 * (scale_bytes = 0 for F32/BF16).  Matches the paper's memory table (Sec. 4.6): 4nD bytes at
 * 32 bits, nBD/8 bytes of codes at B bits.  Pure host arithmetic.
 */
int twa_pmat_bytes(int32_t dtype, int64_t D, int32_t n, int32_t block, int64_t* ld,
                   size_t* data_bytes, size_t* scale_bytes);

/* Workspace (device bytes) needed by twa_project for n vectors and k gradients. */
int twa_project_workspace_bytes(int32_t n, int32_t k, size_t* bytes);

/* Workspace (device bytes) needed by twa_build_basis for n checkpoints. */
int twa_build_basis_workspace_bytes(int32_t n, size_t* bytes);

/*
 * Orthonormal basis of span{w_1..w_n}  (Sec. 3, solution set U; Sec. 4.1, construction by
 * orthogonalising the checkpoints in their given order).
 *   W  [in]  n checkpoints, fp32, basis major with stride ldw.
 *   P  [out] n orthonormal vectors, fp32, stride ldp; W = P R with R upper triangular and
 *            diag(R) > 0, so p_1 = w_1/||w_1|| and span(P) = span(W).  P may alias W (then
 *            ldp == ldw): the checkpoints are overwritten in place.  Padding is zeroed.
 *   R_host [out, HOST, optional] n*n doubles, row major, R[a*n + b] (zero below diagonal).
 *   ws, ws_bytes  device workspace of at least twa_build_basis_workspace_bytes(n).
 * Method: CholeskyQR2 -- twice { Gram matrix accumulated in fp64 on the matrix cores,
 * Cholesky factor in fp64 on the host, P <- P R^-1 in fp32 }; in the second round, whose input is
 * orthonormal to ~1e-4 already, the products of a 64-row tile are formed and summed in fp32 matrix
 * instructions and the tiles' sums added in fp64.  SYNCHRONISES `stream` twice
 * (the n x n Gram matrix travels to the host).  On TWA_ERR_RANK (a Cholesky pivot <=
 * 1e-12 * largest diagonal entry) R_host[0], if given, holds the 0-based index of the
 * offending checkpoint and P is unspecified.
 */
int twa_build_basis(const float* W, int64_t D, int32_t n, int64_t ldw, float* P, int64_t ldp,
                    double* R_host, void* ws, size_t ws_bytes, void* stream);

/*
 * twa_build_basis that never synchronises: the two n x n Cholesky factorisations, the triangular inverses and the
 * product R = R_2 R_1 run on the device (one workgroup, fp64, the operations of the host routines in their order:
 * P and R come out bit for bit as from twa_build_basis).  The call only enqueues on `stream`, so it can be captured
 * into a HIP graph together with what follows it (twa_quantize, the step calls).
 *   R      [out, optional, DEVICE] n*n doubles, row major, zero below the diagonal.
 *   status [out, DEVICE] one int32: 0 when the stream reaches the end of the call's work, or 1 + the 0-based index
 *          of the checkpoint at which a Cholesky pivot was <= 1e-12 * the largest diagonal entry (the condition of
 *          TWA_ERR_RANK); in that case P and the upper triangle of R are filled with NaN.  The library sets it to 0 first.
 * Other arguments, workspace and argument errors as for twa_build_basis.
 */
int twa_build_basis_async(const float* W, int64_t D, int32_t n, int64_t ldw, float* P, int64_t ldp, double* R,
                          int32_t* status, void* ws, size_t ws_bytes, void* stream);

/*
 * The same construction for checkpoints whose rows arrive in panels (a matrix that is generated, read or
 * kept elsewhere piece by piece: the benchmark's largest configuration streams 16 M-row panels).  A panel
 * is rows [r0, r0 + rows) of all n vectors: pointer W + r0 with the matrix' stride.  One pass of
 * CholeskyQR is
 *     for every panel:  twa_gram_accumulate   G += W_panel^T W_panel   (fp64; `accumulate` bit 0 clear on the first)
 *     once:             twa_gram_factor       G = R^T R on the host, R^-1 to the device (synchronises)
 *     for every panel:  twa_apply_rinv        P_panel = W_panel R^-1   (may overwrite W_panel)
 * and twa_build_basis is two such passes (the second over P) with R = R_2 R_1 -- `compose` = 1 in the
 * second twa_gram_factor forms that product in R_host.
 *   gram, rinv, ws  device buffers of the sizes twa_basis_state_bytes reports (contents opaque).
 *   W, P            fp32, 16-byte aligned, strides multiples of 4 elements and >= rows.  Elements outside
 *                   the panel are neither read nor written (padding of P is the caller's to zero).
 *   R_host          n*n doubles, row major, upper triangular; optional unless compose = 1.
 *   accumulate      flags: TWA_GRAM_ADD (1) adds to what `gram` holds, else it is overwritten;
 *                   TWA_GRAM_ORTHONORMAL_INPUT (2) says that the panel belongs to a matrix that is orthonormal
 *                   to ~1e-4 already (the second pass): its products are then formed by fp32 matrix
 *                   instructions per 64-row tile and the tiles summed in fp64, at twice the rate.
 * Errors as for twa_build_basis; on TWA_ERR_RANK R_host[0] holds the index of the dependent checkpoint.
 */
#define TWA_GRAM_ADD 1
#define TWA_GRAM_ORTHONORMAL_INPUT 2
int twa_basis_state_bytes(int32_t n, size_t* gram_bytes, size_t* rinv_bytes, size_t* ws_bytes);
int twa_gram_accumulate(const float* W, int64_t rows, int32_t n, int64_t ldw, double* gram, int32_t accumulate,
                        void* ws, size_t ws_bytes, void* stream);
int twa_gram_factor(const double* gram, int32_t n, float* rinv, double* R_host, int32_t compose, void* stream);
int twa_apply_rinv(const float* W, int64_t rows, int32_t n, int64_t ldw, const float* rinv, float* P, int64_t ldp,
                   void* stream);
/* twa_gram_factor on the device, without synchronising: rinv <- R^-1 of the accumulated Gram matrix, R [optional,
 * DEVICE, n*n doubles] <- R of THIS pass (the caller multiplies the passes' factors if it wants their product).
 * status [DEVICE, int32]: left alone on success, set to 1 + the index of the dependent checkpoint (and rinv, R to
 * NaN) if it still holds 0 and a pivot fails: zero it before the first pass. */
int twa_gram_factor_async(const double* gram, int32_t n, float* rinv, double* R, int32_t* status, void* stream);

/*
 * twa_apply_rinv with the result stored straight in the form `out` describes -- the second pass of the construction
 * fused with twa_quantize (Sec. 4.1 and Sec. 4.6: the fp32 projection matrix is the memory burden; this way it is
 * never written, the checkpoints' rows may be produced panel by panel into a small staging buffer and only the
 * low-bit matrix is kept).  Values and codes are those of twa_apply_rinv followed by twa_quantize, bit for bit.
 *   W    [in]  panel of the matrix after the FIRST pass: rows [row0, row0 + rows) of all n vectors (pointer to the
 *              panel's first row, stride ldw).
 *   rinv [in]  R^-1 of the second pass, from twa_gram_factor.
 *   out  [in]  descriptor of the WHOLE stored matrix (D, n, ld, data, scales, block, gscale), dtype TWA_F32,
 *              TWA_BF16, TWA_I8 or TWA_I4; block <= 128.  TWA_I4 needs out->gscale > 0 (a power of two): the
 *              largest scale of the whole matrix cannot be known from one panel.  Any value that keeps the binary16
 *              scales normal will do; twa_gscale_for_absmax(largest |entry| after the first pass, found with
 *              twa_absmax_accumulate) is the value twa_quantize itself would choose up to the 1e-4 by which the
 *              second pass moves the entries.
 *   row0       first row of the panel in the whole matrix, a multiple of TWA_SCALE_SPAN; rows must be one too except
 *              in the last panel (row0 + rows == out->D), whose call also writes the padding [D, ld): zeros, code 0,
 *              scale 0.
 * The stored matrix must not overlap W (except TWA_F32 exactly in place).  Asynchronous on `stream`.
 */
int twa_apply_rinv_quantize(const float* W, int64_t rows, int32_t n, int64_t ldw, const float* rinv, const twa_pmat* out,
                            int64_t row0, void* stream);

/* amax[0] = max(|X_ij|) over a panel (combined with what amax[0] holds when accumulate != 0; the value is a
 * non-negative binary32 number).  amax: device, 4 bytes.  Asynchronous on `stream`. */
int twa_absmax_accumulate(const float* X, int64_t rows, int32_t n, int64_t ld, float* amax, int32_t accumulate,
                          void* stream);

/* The power of two twa_quantize chooses for the binary16 scales of a TWA_I4 matrix whose largest |entry| is amax:
 * 2^(floor(log2(amax / 7)) - 14), 1 for amax == 0.  Host arithmetic. */
float twa_gscale_for_absmax(float amax);

/*
 * Store an fp32 matrix in the form described by `out`  (Sec. 4.6: P as B-bit integers plus
 * scaling factors).  `out->dtype, n, D, ld, data, scales, block` are preset by the caller;
 * buffers sized per twa_pmat_bytes.  Exact recipe (each step ONE correctly rounded binary32
 * operation, so the result is unique bit for bit), per block of one vector:
 *     amax  = max |p_i| over the block's elements with i < D
 *     scale = amax / qmax                         qmax = 127 (I8), 7 (I4)
 *     I8: stored scale = effective scale e = scale
 *     I4: stored h = binary16(scale / gscale) (round to nearest even), e = float(h) * gscale
 *     e == 0 -> all codes of the block are 0;   inv = 1 / e
 *     q_i   = clamp(round_half_to_even(p_i * inv), -qmax, qmax)
 *   Padding elements [D, ld) get code 0, blocks wholly in the padding get scale 0.
 *   BF16: round to nearest even; F32: copy.  Padding is zeroed.
 * I4 and out->gscale == 0: the library first finds the largest block scale, sets
 *   out->gscale = 2^(floor(log2(max scale)) - 14) (1 if P == 0) and SYNCHRONISES `stream`
 *   once to do so; with out->gscale > 0 (a power of two) nothing synchronises.
 */
int twa_quantize(const float* P, int64_t D, int32_t n, int64_t ldp, twa_pmat* out, void* stream);

/*
 * s = P^T g for k gradients  (Sec. 4.2: the gradient w.r.t. the coefficients is the model
 * gradient projected on the basis).
 *   g  [in]  k gradients, fp32, gradient c at g[c*ldg .. c*ldg + D)  (ldg ignored if k == 1;
 *            otherwise a multiple of 4 and >= D).
 *   s  [out] k*n floats, s[c*n + j] = sum_i value(P)_ij * g_c[i].
 *   ws, ws_bytes  device workspace of at least twa_project_workspace_bytes(n, k).
 * fp32 arithmetic; the reduction order is fixed, so repeated calls give identical bits.
 * TWA_I4 (and, in the layer-wise calls, the min-max formats of 4 bits and fewer) computes the products in
 * integers: every 32 consecutive elements of g (slices starting at
 * multiples of 32) are first rounded to nearest even multiples of unit = 2^(e-22), 2^e being the
 * smallest power of two above the slice's largest |g_i| (unit >= 2^-126) -- an error of at most
 * unit/2 <= 2^-22 max|g_slice| per element -- and the products with the codes and their sums over
 * a slice are then exact; the sums over slices are fp32 as for the other types.  A slice that
 * holds an infinity or a NaN makes every coefficient NaN.  (Layer-wise, the elements of a slice that
 * belong to another layer count as zeros.)
 */
int twa_project(const twa_pmat* P, const float* g, int32_t k, int64_t ldg, float* s, void* ws,
                size_t ws_bytes, void* stream);

/*
 * twa_project for callers that cannot allocate: code under stream capture into a HIP graph, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, kernels, arithmetic and bits as twa_project, without
 * the workspace: the per-workgroup partial sums go to a fixed array in device memory that belongs to the
 * library (TWA_NOALLOC_SCRATCH_BYTES per GPU the entry point is used on, held until the process ends).  The
 * call allocates and frees nothing (no hipMalloc, no hipFree, no allocating library routine).
 *   Limit: n * k <= TWA_NOALLOC_MAX_NK, else TWA_ERR_LIMIT (checked on the host before anything is enqueued).
 *   The array keeps the previous call's contents; nothing in it has to start at zero, because every slot the
 *   final reduction reads is written by the same call first.
 *   Every call on one GPU uses that GPU's one array: calls that overlap on a GPU (two streams, two threads)
 *   race and give wrong sums; calls on one stream are ordered and safe.  The first call on a device looks the
 *   array's address up (no allocation, but a runtime query: make it outside stream capture).
 */
#define TWA_NOALLOC_MAX_NK 512
#define TWA_NOALLOC_SCRATCH_BYTES (2048u * TWA_NOALLOC_MAX_NK * 4u)   /* 4 MiB */
int twa_project_noalloc(const twa_pmat* P, const float* g, int32_t k, int64_t ldg, float* s, void* stream);

/*
 * g~ = P s ; w <- w - lr * g~   (Sec. 4.2, weight-space form of the update rule, lambda = 0;
 * Alg. 1 "update weights").  The caller may put any n coefficients in `s` (for instance
 * P^T g after momentum or Adam, as the paper applies a base optimiser to the coefficients).
 *   s  [in]     n floats (device).
 *   w  [in/out] D floats, updated in place.
 *   g_tilde [out, optional] D floats receiving g~ (NULL: not stored).
 */
int twa_expand_update(const twa_pmat* P, const float* s, float* w, float lr, float* g_tilde,
                      void* stream);

/*
 * Layer-wise processing (Sec. 4.5; Alg. 1, the loop over l = 1..L).  The D parameters are cut
 * into L consecutive layers, layer l = elements [layer_off[l], layer_off[l+1]); every layer has its
 * own block P^l (those rows of the stored matrix) and its own n coefficients, so the coefficient
 * arrays are L x n (row l = layer l).  The stored matrix, its dtype and its scale blocks are the
 * same as in the whole-model calls: layers need not be aligned to anything, and a quantisation block
 * may straddle a boundary.
 *
 * The layer table is turned ONCE into a device-side plan (the layers of a model do not change
 * during training); the step calls take the plan.  In the plan the kernels' tiles are cut per layer,
 * so a tile never meets two layers and the stream over P is the branch-free one of the whole-model
 * step, at the price of at most one extra tile per layer.
 */
#define TWA_MAX_LAYERS 65536

/* Bytes of the device buffer that holds a plan for L layers. */
int twa_layer_plan_bytes(int32_t L, size_t* bytes);

/*
 * Build the plan.
 *   layer_off [in]  L+1 int64 values in DEVICE memory: layer_off[0] = 0, non-decreasing (empty layers
 *                   allowed), layer_off[L] = D.  The table is read on the device only; a table that
 *                   breaks these rules is clamped into one that keeps them (unspecified layers, but
 *                   no access out of range later on).
 *   plan [out]      device buffer of at least twa_layer_plan_bytes(L), 8-byte aligned; it must stay
 *                   intact as long as step calls use it, and is valid for any stored matrix with
 *                   the same D (every dtype).
 * 1 <= L <= TWA_MAX_LAYERS.  Asynchronous on `stream`.
 * The plan carries the L and D it was built for.  The host cannot see into it, so a call that is handed a
 * plan of another layer count or vector length still returns TWA_OK; on the device every kernel compares the
 * plan's L and D with its own before it reads a table and, if they differ, touches nothing else and marks
 * its result instead: twa_project_layers / twa_beta_step fill S (and beta) with NaN, twa_expand_update_layers /
 * twa_weights_from_beta set w[0] (and g_tilde[0]) to NaN and leave the rest alone, twa_quantize_minmax writes
 * NaN factors, twa_centre_normalise NaN norms and E[0] = NaN.
 */
int twa_layer_plan(const int64_t* layer_off, int32_t L, int64_t D, void* plan, size_t plan_bytes, void* stream);

/* Workspace (device bytes) needed by twa_project_layers for n vectors and L layers. */
int twa_project_layers_workspace_bytes(int32_t n, int32_t L, size_t* bytes);

/*
 * S[l][j] = sum over the elements i of layer l of value(P)_ij * g[i]   (Alg. 1: (P^l)^T g^l).
 *   g    [in]  D floats (device).      S [out] L*n floats (device); the row of an empty layer is 0.
 *   plan [in]  built by twa_layer_plan with the same L and D = P->D.
 *   ws, ws_bytes  device workspace of at least twa_project_layers_workspace_bytes(n, L).
 * Same pass over P, same arithmetic and the same fixed reduction order as twa_project.
 */
int twa_project_layers(const twa_pmat* P, const float* g, const void* plan, int32_t L, float* S, void* ws,
                       size_t ws_bytes, void* stream);

/*
 * g~_i = sum_j value(P)_ij * S[l(i)][j] ; w <- w - lr * g~   (Alg. 1 with lambda = 0 in weight
 * space; l(i) = the layer of element i).
 *   S  [in]     L*n floats (device).     w [in/out] D floats.     g_tilde [out, optional] D floats.
 */
int twa_expand_update_layers(const twa_pmat* P, const float* S, const void* plan, int32_t L, float* w, float lr,
                             float* g_tilde, void* stream);

/*
 * Quantise an fp32 matrix into the paper's own format (Sec. 4.6): per layer l, over ALL n vectors,
 *     a_l = (max - min) / (2^B - 1),  b_l = min,  c = round((p - b_l) / a_l)  in [0, 2^B - 1],
 * evaluated in fp64 with ties to even (the paper names no tie rule); a_l = 0 (a constant layer)
 * gives c = 0; the factors are stored rounded to binary32 (b_l exactly).  The stored value is
 * within a_l/2 of p.
 *   bits [in]     B: 1 with out->dtype TWA_U1MM, 1..2 with TWA_U2MM, 1..3 with TWA_U3MM, 1..4 with TWA_U4MM,
 *                 1..8 with TWA_U8MM, 1..16 with TWA_U16MM.  Each of the widths 1, 2, 3, 4, 8 and 16 has a
 *                 container of exactly that many bits per code.  Codes of fewer bits than
 *                 the container holds are stored in it (same values and factors as B-bit storage would
 *                 give, without the extra saving of memory); bytes and words hold them centred,
 *                 c - 2^(B-1), so that the fused dequantisation loses no bits to cancellation.
 *   out  [in/out] one of the TWA_U*MM types; data and scales (2L floats) allocated by the caller;
 *                 on return out->block = B, which the step calls read from the descriptor
 *                 (twa_pmat_bytes gives ld and the data size; it reports 0 scale bytes for these
 *                 types since it does not know L).
 *   ws, ws_bytes  device workspace of at least twa_quantize_minmax_workspace_bytes(L).
 */
int twa_quantize_minmax_workspace_bytes(int32_t L, size_t* bytes);
int twa_quantize_minmax(const float* P, int64_t D, int32_t n, int64_t ldp, const void* plan, int32_t L,
                        int32_t bits, twa_pmat* out, void* ws, size_t ws_bytes, void* stream);

/*
 * The paper's default basis and the coefficient form of the step (Sec. 4.1, extraction of base
 * vectors; Sec. 4.3, initialisation; Sec. 4.5; Alg. 1).  With one layer (L = 1) these are the
 * whole-model forms.
 */

/* Workspace (device bytes) needed by twa_centre_normalise. */
int twa_centre_normalise_workspace_bytes(int64_t D, int32_t n, int32_t L, size_t* bytes);

/*
 * wbar = (1/n) sum_j w_j ;  e_j^l = (w_j^l - wbar^l) / ||w_j^l - wbar^l||_2   for every layer l
 * (Sec. 4.1 / 4.5).  The vectors of a layer are NOT orthogonal and sum to zero after scaling by their
 * norms (rank <= n-1 per layer); a (layer, checkpoint) pair whose centred part is exactly zero gives
 * a zero vector (the paper does not say; a zero direction changes nothing).
 *   W     [in]  n checkpoints, fp32, checkpoint j at W[j*ldw .. j*ldw + D).
 *   wbar  [out] D floats: the mean (the SWA point the averaging starts from, Sec. 4.3); the sum is
 *               accumulated in fp64 in checkpoint order and rounded once.
 *   E     [out] n vectors with leading dimension lde, padding zeroed; E == W (lde == ldw) works
 *               in place, any other overlap is an error.  Feed it to twa_quantize.
 *   norms [out, optional] L*n floats: ||w_j^l - wbar^l||_2.
 *   ws, ws_bytes  device workspace of at least twa_centre_normalise_workspace_bytes(D, n, L).
 * Asynchronous on `stream`; a few passes over W.
 */
int twa_centre_normalise(const float* W, int64_t D, int32_t n, int64_t ldw, const void* plan, int32_t L, float* wbar,
                         float* E, int64_t lde, float* norms, void* ws, size_t ws_bytes, void* stream);

/*
 * beta <- (1 - lr*lambda) * beta - lr * s   (Alg. 1, "update variables"; `count` = L*n entries).
 * `s` is what twa_project_layers returned, or that after the caller's momentum / Adam.  The decay
 * acts on the coefficients, i.e. on w - wbar.
 */
int twa_beta_update(float* beta, const float* s, int64_t count, float lr, float lambda, void* stream);

/*
 * The coefficient step with the run's base optimiser in place of plain gradient descent (Sec. 5.1: the
 * base optimiser is applied to the coefficients; the paper's runs use SGD with momentum, Adam and AdamW).
 * On the `count` = L*n coefficients, with s from twa_project_layers:
 *   TWA_OPT_MOMENTUM  d = s + lambda*beta;  m <- mu*m + d;  beta <- beta - lr*m      (mu = 0: Alg. 1's own step)
 *   TWA_OPT_ADAM      d = s + lambda*beta                      (decay as an L2 term)
 *   TWA_OPT_ADAMW     beta <- (1 - lr*lambda)*beta first;  d = s   (decoupled decay)
 *     then for both   m <- mu*m + (1-mu)*d;  v <- beta2*v + (1-beta2)*d*d;
 *                     beta <- beta - lr * (m / (1 - mu^t)) / (sqrt(v / (1 - beta2^t)) + eps)
 *   m, v [in/out] device, `count` floats each: the optimiser's state, zero before the first step
 *                 (v is not used by TWA_OPT_MOMENTUM and may be NULL there).
 *   t             Adam / AdamW: number of this step, counted from 1.
 * Errors: TWA_ERR_NULL; TWA_ERR_DTYPE (unknown kind); TWA_ERR_SHAPE (count out of range, t < 1, mu or
 * beta2 outside [0, 1), eps < 0).  Asynchronous on `stream`; fp32 arithmetic.
 */
#define TWA_OPT_MOMENTUM 0
#define TWA_OPT_ADAM 1
#define TWA_OPT_ADAMW 2
typedef struct {
  int32_t kind;  /* TWA_OPT_* */
  float lr;      /* eta */
  float lambda;  /* weight decay */
  float mu;      /* heavy-ball factor (momentum), beta_1 (Adam, AdamW) */
  float beta2;   /* Adam, AdamW */
  float eps;     /* Adam, AdamW */
  int32_t t;     /* Adam, AdamW: step number from 1 */
} twa_optim;
int twa_beta_optim(const twa_optim* opt, float* beta, const float* s, float* m, float* v, int64_t count, void* stream);

/*
 * Both "update variables" steps of Alg. 1 in one call: s = (P^l)^T g^l for every layer, then
 * beta <- (1 - lr*lambda) * beta - lr * s, the second inside the reduction kernel of the first (one
 * launch less than twa_project_layers + twa_beta_update).
 *   beta [in/out] L*n floats.   S [out, optional] L*n floats receiving s (NULL: not stored).
 *   ws, ws_bytes  as for twa_project_layers.
 */
int twa_beta_step(const twa_pmat* P, const float* g, const void* plan, int32_t L, float* beta, float lr, float lambda,
                  float* S, void* ws, size_t ws_bytes, void* stream);

/*
 * w^l = wbar^l + P^l beta^l   (Alg. 1, "update weights"; Sec. 4.3).  The same pass over P as
 * twa_expand_update_layers.
 *   beta [in] L*n floats.   wbar [in] D floats.   w [out] D floats (may be wbar's buffer).
 */
int twa_weights_from_beta(const twa_pmat* P, const float* beta, const void* plan, int32_t L, const float* wbar,
                          float* w, void* stream);

/*
 * Measurement aid, NO part of the method and never called by any other entry point: one plain pass of non-temporal 128-bit reads over `bytes` bytes
 * (rounded down to 16) of `buf`, for callers that want the read ceiling of the device they run on next
 * to the rates of the step kernels (the benchmark reports both).
 *   buf  [in]  device, 16-byte aligned.     sink [out] device, 4 bytes; left alone in practice.
 */
int twa_probe_read(const void* buf, size_t bytes, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TWA_H_ */
