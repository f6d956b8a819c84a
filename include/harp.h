/*
 * libharp -- HARP structured orthogonal processors on AMD MI355X (gfx950).
 *
 * A HARP processor (paper Sec. 3, Eq. (6)-(8), Alg. 1) is a product of m sparse
 * block-orthogonal stride stages under a Mixed-Radix schedule b = (b_0..b_{m-1}),
 * prod b_t = d, together with a +-1 sign vector sigma (Sec. 3, the random sign
 * diagonals; Assumption 1(iv)).  With s_t = prod_{j<t} b_j and g_t = d / (b_t s_t),
 * stage t takes, for every alpha < g_t and beta < s_t, the b_t coordinates
 *
 *        alpha * b_t * s_t + r * s_t + beta,      r = 0 .. b_t - 1     (App. A, Lemma 1)
 *
 * as a row vector v and replaces them by v * K_t[c], c = alpha * s_t + beta, where
 * K_t[c] is a dense b_t x b_t block (Alg. 1, the step that views the stage's kernels per
 * group and stride offset).  Stage 0 is
 * applied to the data first (Alg. 1 loop order).  The processor's matrix U is defined by
 *
 *        apply(x) = x U = T(x .* sigma),        T = stage_{m-1} o ... o stage_0,
 *
 * so U = diag(sigma) T, and apply_transpose(x) = x U^T = (x T^T) .* sigma (stages in
 * reverse order, each block transposed).  With orthogonal blocks U is orthogonal and
 * apply_transpose inverts apply; with arbitrary blocks both are still the linear maps
 * just stated.  Conventions the paper leaves open and this library fixes: the row
 * vector is on the left of the block, blocks are numbered alpha-major, and the signs
 * act on the input coordinates of apply.
 *
 * All entry points return a status code; none throws or aborts.  The launch entry points
 * (harp_apply, harp_apply_transpose, harp_apply_noalloc, harp_rotate_weight(_inverse),
 * harp_grad_blocks) only enqueue work on the caller's stream and never wait for the device;
 * the plan constructors copy their images with blocking copies, and the first call of a
 * split program on a stream allocates its intermediate (see harp_apply).  Argument errors
 * are detected before any HIP call.  A plan is immutable
 * after creation and may be used concurrently from several host threads and streams.
 */
#ifndef HARP_H_
#define HARP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct harp_plan harp_plan_t; /* opaque */

typedef enum {
  HARP_OK = 0,
  HARP_ERR_INVALID_ARG = 1,    /* NULL pointer, negative size, leading dim < d, bad enum    */
  HARP_ERR_BAD_SCHEDULE = 2,   /* m < 1, some b_t < 2, or prod b_t != d   (Eq. (6))         */
  HARP_ERR_NOT_ORTHOGONAL = 3, /* HARP_VALIDATE_ORTHO set and a block fails K^T K = I       */
  HARP_ERR_UNSUPPORTED = 4,    /* radix > HARP_MAX_RADIX, or d too long for the on-chip tile */
  HARP_ERR_OOM = 5,            /* host or device allocation failed                           */
  HARP_ERR_DEVICE = 6          /* any other HIP runtime failure (including: no device)       */
} harp_status_t;

typedef enum {
  HARP_F32 = 0, /* X, Y hold IEEE binary32                                                   */
  HARP_BF16 = 1 /* X, Y hold bfloat16; arithmetic is fp32, one round-to-nearest-even at store */
} harp_dtype_t;

/* flags for harp_plan_create */
enum {
  HARP_VALIDATE_ORTHO = 1u,  /* reject blocks with max |K^T K - I| > 1e-5 (checked in float64) */
  HARP_BLOCKS_ON_DEVICE = 2u, /* blocks[t] and signs are device pointers (copied back to build) */
  /* harp_plan_create_from_theta_int8 only: also keep the int8 codes on the device and rebuild
   * the blocks inside the kernel for the stages that have such a kernel (see there) */
  HARP_THETA_IN_KERNEL = 4u,
  /* keep every intermediate of this plan in float32: split programs (harp_apply) and the
   * workspace of harp_rotate_weight otherwise carry bf16 callers' data between launches as
   * half-precision values with one power-of-two scale per 16 coordinates (see harp_rotate_weight) */
  HARP_F32_INTERMEDIATES = 8u
};

/* kernel selection, for tests and tuning (harp_plan_set_algo) */
typedef enum {
  HARP_ALGO_AUTO = 0,    /* fastest kernel that supports the plan                             */
  HARP_ALGO_GENERIC = 1, /* every stage through the runtime-radix code path                   */
  HARP_ALGO_FUSED = 2,   /* radix-specialised passes, whole rows on chip                      */
  HARP_ALGO_SPLIT = 3    /* low digits (product <= 4096) fused on chip per row chunk, each pass on
                            the digits above streamed through a float32 intermediate owned
                            by the plan (see harp_apply)                                       */
} harp_algo_t;

#define HARP_MAX_RADIX 64
#define HARP_MAX_STAGES 64

/*
 * Create a processor (Eq. (6)-(8); Alg. 1 REQUIRE lines).
 *   out      receives the plan; untouched on failure.
 *   d        transformed dimension, >= 2.
 *   m        number of stages, 1 .. HARP_MAX_STAGES.
 *   radices  m host ints, each >= 2 (<= HARP_MAX_RADIX), product == d.
 *   blocks   m host pointers (device pointers with HARP_BLOCKS_ON_DEVICE); blocks[t]
 *            holds D_t = d / b_t blocks of b_t * b_t float32, block c row-major:
 *            blocks[t][c*b*b + r*b + r2] = K_t[c][r][r2], used as  v'[r2] = sum_r v[r] K[r][r2].
 *   signs    d int8 values in {+1, -1}, or NULL for all +1.
 *   flags    OR of HARP_VALIDATE_ORTHO, HARP_BLOCKS_ON_DEVICE, HARP_F32_INTERMEDIATES.
 * The plan copies everything it needs into device memory it owns (on the current HIP
 * device); the caller's arrays may be freed on return.
 */
harp_status_t harp_plan_create(harp_plan_t **out, int64_t d, int32_t m, const int32_t *radices,
                               const float *const *blocks, const int8_t *signs, uint32_t flags);

/* Release the plan and its device memory.  NULL is accepted.  The caller must ensure
 * no launch using the plan is still in flight. */
harp_status_t harp_plan_destroy(harp_plan_t *plan);

/*
 * Y[n,d] = X[n,d] * U  (Alg. 1 on every row, signs first).
 *   X, Y     caller-owned DEVICE pointers, row-major, leading dimensions ldx, ldy in
 *            elements (>= d).  Y may be exactly X with ldy == ldx (in place); any other
 *            overlap is undefined.
 *   n        number of rows, >= 0 (0 is a no-op returning HARP_OK).
 *   dt       element type of both X and Y.
 *   stream   a hipStream_t passed as void* (NULL = the default stream).  The call only
 *            enqueues work on it.
 * Plans whose rows are longer than 4096 coordinates, and plans in which a stage of radix >= 9
 * follows stages of radix <= 8 with a product that is a multiple of 16 and at least 64 (a
 * leftover prime at the end of the schedule), and -- for forward calls with n >= 512 -- plans of
 * radix-2 stages followed by one radix-3 stage, run in two or more launches through a
 * float32 intermediate of at most 128 MB that the plan allocates (hipMalloc) the first time
 * it is used on a stream and keeps, one per stream, until harp_plan_destroy.  That first
 * call may therefore block; inside a stream capture it returns HARP_ERR_UNSUPPORTED instead
 * (run the plan once on the stream before capturing).  HARP_ERR_OOM if it cannot be had.
 * Arithmetic is float32 with one rounding at a bf16 store, with one exception: when dt is
 * HARP_BF16, a stage of radix 9..64 of such a plan runs on the matrix cores with every float32
 * operand split into two bf16 terms (x_hi K_hi + x_lo K_hi + x_hi K_lo accumulated in float32,
 * about 16 significant bits per product -- below the bf16 rounding of the result).  For
 * HARP_F32 callers that stage runs on the float32 matrix instruction with unsplit operands
 * (float32 products and sums, in another order than the vector path).  Setting the
 * environment variable HARP_NO_MFMA=1 selects the float32 vector path for every caller.
 * Second exception, HARP_BF16 callers only: when every block of the plan is orthogonal and the
 * stages above the on-chip chunk have radix 2 .. 8, the intermediate between the launches holds
 * half-precision values with one power-of-two scale per 16 coordinates instead of float32 (each
 * value within 2^-12 of itself or 2^-25 of the largest of its 16 neighbours: an eighth of the
 * rounding of the bf16 result); HARP_F32_INTERMEDIATES at plan creation keeps float32.  A
 * transposed call whose one stage above a 4096-chunk has radix 2, 3 or 5 (d = 8192, 12288,
 * 20480) runs in one launch without any intermediate when Y is not X.
 */
harp_status_t harp_apply(const harp_plan_t *plan, const void *X, int64_t ldx, void *Y,
                         int64_t ldy, int64_t n, harp_dtype_t dt, void *stream);

/* Y[n,d] = X[n,d] * U^T  (the stages in reverse order with transposed blocks, signs last;
 * the inverse of harp_apply when the blocks are orthogonal).  Same argument rules. */
harp_status_t harp_apply_transpose(const harp_plan_t *plan, const void *X, int64_t ldx, void *Y,
                                   int64_t ldy, int64_t n, harp_dtype_t dt, void *stream);

/*
 * harp_apply (transpose == 0) or harp_apply_transpose (transpose == 1) for callers that cannot
 * allocate device memory: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and bit-identical results, but the call never
 * allocates, frees or synchronises: the float32 intermediate that a plan of two or more launches
 * needs (see harp_apply) is a 32 MiB array that belongs to the loaded library itself -- one per
 * GPU, held until the process ends -- instead of a buffer the plan allocates.  A batch whose
 * intermediate n * d * 4 bytes exceeds that array is refused with HARP_ERR_UNSUPPORTED
 * (harp_apply_noalloc_max_rows gives the limit for a plan; plans that run in one launch use no
 * intermediate and take any n).  The plan's device must be the current device
 * (HARP_ERR_INVALID_ARG otherwise).  Every call on a GPU shares that GPU's one array, so two
 * calls that overlap in time on one GPU -- different streams or host threads -- race on it:
 * order them on one stream.  Nothing in the array has to start at zero (a call writes every
 * element before it reads it), so it is never cleared.
 */
harp_status_t harp_apply_noalloc(const harp_plan_t *plan, const void *X, int64_t ldx, void *Y,
                                 int64_t ldy, int64_t n, harp_dtype_t dt, int32_t transpose,
                                 void *stream);
/* Largest n harp_apply_noalloc accepts for this plan (INT64_MAX when the plan needs no
 * intermediate); -1 for NULL. */
int64_t harp_apply_noalloc_max_rows(const harp_plan_t *plan);

/*
 * Two-sided change of basis of a weight matrix (Sec. 2):  Wout = U_U^T * W * U_V,
 * W and Wout [d_out, d_in] row-major DEVICE arrays with leading dimensions ldw, ldo.
 * plan_U (dimension d_out) and plan_V (dimension d_in) may each be NULL = identity on
 * that side; if both are NULL, d_out and d_in say how much to copy.  With plan_U given,
 * d_out must equal its dimension, likewise d_in for plan_V.  Wout may be exactly W.
 * workspace: device scratch of at least the size reported by
 * harp_rotate_weight_workspace_size (may be NULL when that size is 0).
 * The inverse map  W = U_U * Wout * U_V^T  is harp_rotate_weight_inverse.
 * Arithmetic is float32 and the result is rounded once, at the last store.  Between the launches
 * of a call the matrix lies in the workspace as float32 -- or, for HARP_BF16 matrices between
 * processors whose blocks are all orthogonal (checked at plan creation), with d_in a multiple
 * of 128 and 16-byte aligned workspace, as half-precision values with one power-of-two scale
 * per 16 consecutive columns of a row: each of the at most three trips then changes an entry by at
 * most 2^-12 of itself (or 2^-25 of the largest of its 16 neighbours), an eighth of the rounding
 * the bf16 result receives anyway.  That error is relative to the entry between the launches,
 * i.e. to the scale of its column while plan_U's stages are still to come; HARP_F32_INTERMEDIATES
 * on either plan keeps the workspace in float32.
 */
harp_status_t harp_rotate_weight_workspace_size(const harp_plan_t *plan_U,
                                                const harp_plan_t *plan_V, int64_t d_out,
                                                int64_t d_in, harp_dtype_t dt, size_t *bytes);
harp_status_t harp_rotate_weight(const harp_plan_t *plan_U, const harp_plan_t *plan_V,
                                 const void *W, int64_t ldw, void *Wout, int64_t ldo,
                                 int64_t d_out, int64_t d_in, harp_dtype_t dt, void *workspace,
                                 size_t workspace_bytes, void *stream);
harp_status_t harp_rotate_weight_inverse(const harp_plan_t *plan_U, const harp_plan_t *plan_V,
                                         const void *W, int64_t ldw, void *Wout, int64_t ldo,
                                         int64_t d_out, int64_t d_in, harp_dtype_t dt,
                                         void *workspace, size_t workspace_bytes, void *stream);

/* Base mixer G_b of a stage's block kernels (Sec. 3, "Hadamard-preconditioned block kernels"). */
typedef enum {
  HARP_MIXER_IDENTITY = 0, /* G = I: the block is Q(theta) itself                              */
  HARP_MIXER_HADAMARD = 1, /* normalised Sylvester Hadamard matrix; power-of-two radices only  */
  HARP_MIXER_CUSTOM = 2    /* the b x b row-major matrix mixers[t] (host), e.g. the QR fallback
                              of a fixed Gaussian matrix the paper uses for other radices, whose
                              seed it does not publish                                         */
} harp_mixer_t;

/*
 * Block kernels from the rotation parameters: B_{t,c} = Q(theta_{t,c}) G_{b_t} (Sec. 3, block
 * definition), in the layout harp_plan_create takes.  Host only, computed in float64.
 *   theta        m host pointers or NULL (= all zero).  theta[t] is NULL (zeros: Q = I, the
 *                paper's initialisation) or D_t * b_t (b_t - 1) / 2 floats, block c first:
 *                for radix 2 the angle of [[cos, -sin], [sin, cos]]; for larger radices the
 *                strict upper triangle, row by row ((0,1), (0,2), ..., (1,2), ...), of the
 *                skew-symmetric A in the Cayley map Q = (I + A)^{-1} (I - A).
 *   mixer_kinds  m harp_mixer_t values, or NULL for HARP_MIXER_HADAMARD at every stage.
 *   mixers       m host pointers (read for HARP_MIXER_CUSTOM stages only), or NULL.
 *   blocks_out   m host buffers of D_t * b_t * b_t floats each, written.
 * The matrix product is taken as printed (Q on the left of G); the block then acts on row
 * vectors like any other (harp_plan_create).  HARP_ERR_INVALID_ARG for a Hadamard mixer at
 * a radix that is not a power of two, a missing custom mixer or a non-finite parameter.
 */
harp_status_t harp_blocks_from_theta(int64_t d, int32_t m, const int32_t *radices,
                                     const float *const *theta, const int32_t *mixer_kinds,
                                     const float *const *mixers, float *const *blocks_out);

/* harp_blocks_from_theta followed by harp_plan_create (flags: HARP_VALIDATE_ORTHO only). With
 * theta == NULL, Hadamard mixers and a power-of-two schedule the plan is the randomized
 * Hadamard transform diag(signs) H_d / sqrt(d) (Sec. 3, "Exact initialization"). */
harp_status_t harp_plan_create_from_theta(harp_plan_t **out, int64_t d, int32_t m,
                                          const int32_t *radices, const float *const *theta,
                                          const int32_t *mixer_kinds, const float *const *mixers,
                                          const int8_t *signs, uint32_t flags);

/*
 * Gradient through Y = X U for fitting (the update of the layerwise fitting procedure,
 * appendix "Layerwise fitting of HARP for a linear layer", differentiates the rotated weights
 * with respect to the processors' parameters; this is the chain rule through Algorithm 1).
 * With x_0 = X diag(signs), x_{t+1} = stage_t(x_t) and G = dL/dY:
 *     dK[t][c][r][r2] = sum over the n rows of  x_t[i(c, r)] * g_{t+1}[i(c, r2)],
 *     g_t = g_{t+1} through stage t with every block transposed,   g_m = G,
 *     dX = g_0 diag(signs)  (= G U^T),
 * i(c, r) = the r-th coordinate of block c of stage t.  The blocks need not be orthogonal.
 * The gradient for the two-sided rotation follows by calling this with X = W (plan_V) and
 * with X = (W V)^T (plan_U).
 *   X, G   device, [n, d] row-major, element type dt, leading dimensions ldx, ldg >= d.
 *   dK     host array of m DEVICE pointers; dK[t] receives D_t * b_t * b_t float32 values in
 *          the layout of harp_plan_create's blocks[t] (overwritten; zeros when n == 0).
 *   dX     device, [n, d] of type dt with leading dimension lddx, or NULL to skip it.
 *   workspace  device memory of at least harp_grad_blocks_workspace_size bytes (up to m + 2
 *          float32 copies of the batch plus partial sums); may be NULL when that size is 0.
 * Float32 arithmetic; the sum over rows is taken in a fixed order (bit-reproducible for the same
 * n).  Asynchronous on `stream`.  Every radix up to HARP_MAX_RADIX; stages of radix above 8 run
 * on a plain one-value-per-thread kernel.
 */
harp_status_t harp_grad_blocks_workspace_size(const harp_plan_t *plan, int64_t n, size_t *bytes);
harp_status_t harp_grad_blocks(const harp_plan_t *plan, const void *X, int64_t ldx, const void *G,
                               int64_t ldg, int64_t n, harp_dtype_t dt, float *const *dK, void *dX,
                               int64_t lddx, void *workspace, size_t workspace_bytes,
                               void *stream);

/*
 * Int8 storage of the rotation parameters (Sec. 3, "Parameter quantization for deployment";
 * appendix "Int8 storage of HARP parameters").  Per block c of stage t the p_t = b_t (b_t-1)/2
 * parameters a (the strict upper triangle of the Cayley matrix, or the one Givens angle for
 * radix 2; layout of theta[t] as in harp_blocks_from_theta) get one scale
 *     s_{t,c} = max |a| / 127        and codes        q = round(a / s_{t,c}).
 * The arithmetic that decides a code is float32 with ties to even; a block whose parameters
 * are all zero gets s = 0 and codes 0 (the appendix leaves 0/0 open).  Reconstruction is
 * a ~ s q in float32.  Host only; every pointer is a host pointer and must not be NULL.
 *   codes[t]   D_t * p_t int8 values in [-127, 127];   scales[t]   D_t floats (>= 0).
 * harp_theta_dequantize_int8 returns HARP_ERR_INVALID_ARG for a code of -128 or a negative or
 * non-finite scale, harp_theta_quantize_int8 for a non-finite parameter.
 * harp_plan_create_from_theta_int8 = dequantize, then harp_plan_create_from_theta: by default
 * the orthogonal blocks are rebuilt once, when the plan is created (most kernels keep a
 * block's values on chip for a whole launch, so rebuilding them per launch would save no
 * traffic).
 * With HARP_THETA_IN_KERNEL the plan also keeps the codes, scales and sign bits on the device
 * (b_t (b_t-1)/2 + 5 bytes per block instead of 4 b_t^2), and harp_apply / harp_apply_transpose
 * rebuild the blocks at run time (the run-time reconstruction of the same appendix) wherever a
 * kernel for it exists: chains of equal radix 4 or 8 with the
 * Hadamard or the identity mixer, on rows or row chunks of 4^k / 8^k <= 4096 coordinates (the
 * paper's default radix-8 schedules).  Each thread dequantizes its block's codes (s q in
 * float32), inverts I + A by Gauss-Jordan elimination in float32 registers (no pivoting is
 * needed: I + A is positive definite for skew-symmetric A), forms Q = 2 (I + A)^{-1} - I,
 * applies the mixer and the signs.  The rebuilt block differs from the float64 one by about
 * 5e-7 for |a| <= 1 and 2e-5 for |a| ~ 10, so the float32 tolerance of the other paths holds
 * for moderate parameters only.  Other stages of such a plan, harp_rotate_weight and
 * harp_grad_blocks use the blocks built at plan creation.  harp_plan_theta_in_kernel reports
 * whether a plan carries the run-time image (1) or not (0; -1 for NULL).
 */
harp_status_t harp_theta_quantize_int8(int64_t d, int32_t m, const int32_t *radices,
                                       const float *const *theta, int8_t *const *codes_out,
                                       float *const *scales_out);
harp_status_t harp_theta_dequantize_int8(int64_t d, int32_t m, const int32_t *radices,
                                         const int8_t *const *codes, const float *const *scales,
                                         float *const *theta_out);
harp_status_t harp_plan_create_from_theta_int8(harp_plan_t **out, int64_t d, int32_t m,
                                               const int32_t *radices, const int8_t *const *codes,
                                               const float *const *scales,
                                               const int32_t *mixer_kinds,
                                               const float *const *mixers, const int8_t *signs,
                                               uint32_t flags);
int32_t harp_plan_theta_in_kernel(const harp_plan_t *plan);

/*
 * Kronecker fallback (Sec. 3, "Mixed-Radix dimensions and Kronecker fallback", the equation
 * T_d = (H~_K / sqrt(K)) (x) T_{n2}): expands a processor T_{n2} on n2 coordinates and a
 * Hadamard-like table H~_K (K x K row-major, entries +-1, H~ H~^T = K I) into the schedule and
 * blocks of the equivalent Mixed-Radix processor on d = K n2 coordinates: every stage of
 * T_{n2} repeated for each of the K slices (tied parameters), then one stage of radix K at
 * stride n2 whose blocks all equal H~_K / sqrt(K).  With x viewed as a K x n2 array (index
 * k n2 + j) the result acts as x -> x (H~_K / sqrt(K) (x) T_{n2}).  Host only.
 *   radices_out  m2 + 1 ints, written.
 *   blocks_out   m2 + 1 host buffers: stage t < m2: K n2 b_t floats; stage m2: n2 K K floats.
 * Pass the result to harp_plan_create with d = K n2, m = m2 + 1.  HARP_ERR_INVALID_ARG for a
 * table entry other than +-1, HARP_ERR_NOT_ORTHOGONAL if H~ H~^T != K I, HARP_ERR_UNSUPPORTED
 * for K > HARP_MAX_RADIX.
 */
harp_status_t harp_kronecker_blocks(int32_t K, const float *table, int64_t n2, int32_t m2,
                                    const int32_t *radices2, const float *const *blocks2,
                                    int32_t *radices_out, float *const *blocks_out);

/*
 * The same processor as a plan whose parameters stay tied (the point of the Kronecker fallback:
 * one T_{n2} serves all K slices, and the last stage is one table).  Arguments as for
 * harp_kronecker_blocks; signs: d = K n2 values in {+1, -1} or NULL; flags: HARP_VALIDATE_ORTHO
 * only.  The plan equals harp_plan_create on the expansion (same apply / apply_transpose), but
 * when the slices are radix-2 chains of 256, 512 or 1024 coordinates in the two-shear form and
 * 9 <= K <= HARP_MAX_RADIX, its device image holds ONE slice's stage parameters and ONE K x K
 * table (parameter volume divided by K; harp_plan_param_bytes reports it, harp_plan_tied_slices
 * returns K), read by every slice modulo the slice length, and the signs are applied inside the
 * first (apply) or last (apply_transpose) kernel instead of being folded into the parameters.
 * Such a plan has the two-launch program only: X and Y must be 16-byte aligned with leading
 * dimensions that are multiples of 8 (HARP_ERR_UNSUPPORTED otherwise), harp_plan_set_algo
 * accepts HARP_ALGO_AUTO and HARP_ALGO_SPLIT, it cannot be plan_U of a column-mode weight
 * rotation (the transposing path is taken) and has no block gradients.  For every other shape
 * the call falls back to the expanded plan (harp_plan_tied_slices returns 0).
 */
harp_status_t harp_plan_create_kronecker(harp_plan_t **out, int32_t K, const float *table,
                                         int64_t n2, int32_t m2, const int32_t *radices2,
                                         const float *const *blocks2, const int8_t *signs,
                                         uint32_t flags);

/* Greedy Mixed-Radix schedule (appendix Alg. 2): peel b_base while it divides d, then the
 * factors min(b_max, r) .. 2 in decreasing order, then any leftover as one last stage.
 * out_radices must hold HARP_MAX_STAGES ints.  Host only; no HIP call. */
harp_status_t harp_greedy_schedule(int64_t d, int32_t b_base, int32_t b_max, int32_t *out_radices,
                                   int32_t *out_m);

/* Introspection and tuning. */
int64_t harp_plan_dim(const harp_plan_t *plan);          /* d, or -1 for NULL            */
int32_t harp_plan_num_stages(const harp_plan_t *plan);   /* m, or -1 for NULL            */
int32_t harp_plan_tied_slices(const harp_plan_t *plan);  /* K of a tied Kronecker plan, 0 for
                                                            any other plan, -1 for NULL     */
/* Eq. (13): number of free rotation parameters sum_t d (b_t - 1) / 2; -1 for NULL. */
int64_t harp_plan_param_count(const harp_plan_t *plan);
/* Bytes of stage parameters one launch reads from device memory (per row tile). */
int64_t harp_plan_param_bytes(const harp_plan_t *plan);
/* Choose the kernel family for later launches of this plan (not thread-safe against
 * concurrent launches).  HARP_ERR_UNSUPPORTED leaves the previous choice in place. */
harp_status_t harp_plan_set_algo(harp_plan_t *plan, harp_algo_t algo);
/* Rows per workgroup tile for later launches; 0 restores the automatic choice.  Kernels that
 * keep the whole tile in the 160 KB LDS clamp the value to what fits. */
harp_status_t harp_plan_set_rows_per_tile(harp_plan_t *plan, int32_t rows);
/* Short name of the kernel path harp_apply would take for n rows (static string). */
const char *harp_plan_kernel_name(const harp_plan_t *plan, int64_t n, harp_dtype_t dt);

const char *harp_status_string(harp_status_t status);
const char *harp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HARP_H_ */
