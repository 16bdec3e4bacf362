/*
 * libsfb: the data-parallel hot path of Sufficient Factor Broadcasting on one
 * MI355X (gfx950).
 *
 * For a matrix-parameterised model  min_W (1/N) sum_i f_i(W a_i) + h(W),
 * W in R^{J x D} (Section 2, problem (P)), the stochastic gradient of one
 * sample is the rank-1 matrix u v^T with u = d f / d(W a), v = a (Section 2.1,
 * "Proximal SGD").  A worker (Section 3)
 *   1. computes the sufficient factors (SFs) of its mini-batch,
 *   2. receives the SFs of its peers,
 *   3. reconstructs and applies  W <- W - eta * sum_i u_i v_i^T  over all of them,
 *   4. applies the proximal operator of h.
 * This library is steps 1, 3 and 4; step 2 is the caller's (peer SF blocks are
 * simply more rows of U and V).
 *
 * Conventions
 *   - Row-major, dense, no padding: W[J][D] fp32; X[B][D]; U[N][J]; V[N][D]
 *     (one SF per row: the layout in which SFs are buffered and sent,
 *     Section 4.2).
 *   - Every data pointer is a DEVICE pointer owned by the caller and must be
 *     16-byte aligned.  The library allocates and frees no device memory; the
 *     scratch it needs is the workspace the caller sets.
 *   - Every call only enqueues kernels on the context's stream and returns; no
 *     host synchronisation.  Results are valid once the caller has synchronised
 *     that stream.  Calls on one context are ordered; a context must not be used
 *     from two host threads at once.
 *   - Return value: 0 on success, a negative sfb_status otherwise.  Nothing is
 *     enqueued when an argument check fails.  Labels outside [0, J) are a caller
 *     bug and are not checked on the device.
 *   - The library never divides by the mini-batch size: the 1/K of Section 3
 *     ("Mini-batch proximal SGD") is folded into eta by the caller.
 */
#ifndef SFB_H
#define SFB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sfb_ctx sfb_ctx; /* opaque: device id, stream, workspace, last HIP error */

typedef enum { SFB_MLR = 0, SFB_DML = 1, SFB_SC = 2 } sfb_model;
typedef enum { SFB_F32 = 0, SFB_BF16 = 1 } sfb_dtype;
typedef enum { SFB_PROX_PROJECT = 0, SFB_PROX_NORMALIZE = 1 } sfb_prox_mode;

typedef enum {
    SFB_OK = 0,
    SFB_EINVAL = -1, /* null pointer, bad shape, bad enum, misaligned pointer, unsupported dtype mix */
    SFB_ENOWS = -2,  /* workspace missing or smaller than sfb_workspace_bytes() */
    SFB_EHIP = -3,   /* a HIP call failed; sfb_last_hip_error() has the code */
    SFB_ETOOBIG = -4 /* sfb_apply_static: the scratch this shape needs exceeds SFB_STATIC_SCRATCH_BYTES */
} sfb_status;

/* One mini-batch.  Pointers are device pointers; the struct itself is host memory. */
typedef struct {
    const void* X;       /* [B][D] of in_dtype.  MLR: features.  DML: first points.  SC: samples. */
    const void* Y;       /* MLR: int32 labels [B] in [0,J).  DML: second points [B][D] of in_dtype.  SC: NULL. */
    const int8_t* sim;   /* DML: +1 similar / -1 dissimilar, [B].  Otherwise NULL. */
    int64_t B;           /* samples (pairs) in the batch, >= 0 */
    int32_t in_dtype;    /* sfb_dtype of X (and of DML's Y) */
    int32_t sf_dtype;    /* sfb_dtype of the U and V outputs */
    float lambda;        /* SC: l1 weight */
    int32_t ista_iters;  /* SC: ISTA iterations */
    int32_t power_iters; /* SC: power iterations for the step size 1/L (>= 1) */
    float margin;        /* DML: hinge margin */
} sfb_batch;

/* Creates a context bound to HIP device `device_id` and to `hip_stream`
 * (a hipStream_t passed as void*; NULL = the device's default stream). */
int sfb_create(sfb_ctx** out, int device_id, void* hip_stream);
int sfb_destroy(sfb_ctx* ctx);

/* Bytes of device scratch sfb_compute_sf needs for this model/shape/batch
 * (0 is possible; negative sfb_status on bad arguments). */
int64_t sfb_workspace_bytes(int32_t model, int64_t J, int64_t D, const sfb_batch* batch);
/* Bytes of device scratch sfb_apply needs (0 for fp32 factors; bf16 factors
 * are transposed into it).  sfb_prox_rows needs none.  One workspace of the
 * larger size serves both calls: its contents do not outlive a call. */
int64_t sfb_apply_workspace_bytes(int64_t J, int64_t D, int64_t N, int32_t sf_dtype);

/*
 * Optional bf16 working copy ("shadow") of one parameter matrix, for the bf16
 * multiclass-logistic path: fp32 master weights W plus a bf16 copy, laid out
 * in the blocks the forward contraction streams, that it reads instead of W
 * (half the bytes, every request a whole cache line; the layout inside the
 * buffer is the library's business).  sfb_shadow_attach converts W
 * into the caller-allocated buffer (sfb_shadow_bytes, 256-byte aligned; the
 * library never frees it) and remembers (W, J, D).  While attached,
 *   - sfb_compute_sf(SFB_MLR, bf16) on that W reads the copy and needs
 *     sfb_shadow_bytes less workspace;
 *   - sfb_apply and sfb_prox_rows on that W keep the copy current (sfb_apply
 *     relies on it being current on entry: it rewrites only the entries whose
 *     bf16 value changes);
 *   - any other modification of W by the caller must be followed by another
 *     sfb_shadow_attach (a refresh), otherwise the copy is stale.
 * Without an attached copy the bf16 path converts W into the workspace on every
 * sfb_compute_sf call: same results, one more pass over W.
 */
int64_t sfb_shadow_bytes(int64_t J, int64_t D);
int sfb_shadow_attach(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, void* dev_ptr, int64_t bytes);
int sfb_shadow_detach(sfb_ctx* ctx);

/*
 * Optional split storage of one parameter matrix, for the bf16 multiclass-logistic
 * path (instead of a working copy, not in addition to one).  The fp32 word of every
 * element is kept as two 16-bit halves in two separate planes, the halves of
 * word = bits + 0x8000 (modulo 2^32): hi = word >> 16, which is the value rounded to
 * bf16 (to nearest, ties away from zero), and lo = word & 0xffff; bits = ((hi << 16)
 * | lo) - 0x8000, exactly.  Inside
 * the buffer the planes are laid out for the two kernels that stream them (hi in
 * blocks of 256 rows x 64 columns, lo in tiles of 256 x 256, each block one
 * contiguous piece); the layout is the library's business, the caller only provides
 * sfb_split_bytes bytes.  The forward contraction reads the hi plane as its bf16
 * operand; sfb_apply reads both planes and writes the lo plane, and the hi plane
 * only where the update moves a value across a bf16 rounding boundary (6 to 8 bytes
 * per element against 8 to 10 for the fp32 array plus working copy), with the same
 * fp32 arithmetic and the same resulting bits.
 * sfb_split_attach converts W into the caller-allocated buffer (sfb_split_bytes,
 * 256-byte aligned; never freed by the library) and remembers (W, J, D).  While
 * attached, the planes ARE the parameters and the fp32 array W is a stale
 * snapshot: sfb_compute_sf(SFB_MLR, bf16), sfb_mlr_sf_csr(bf16) and sfb_apply /
 * sfb_apply_signed / sfb_apply_csr with bf16 factors on that W work on the planes
 * (W itself is neither read nor written); every other call that would read or write
 * the fp32 array of that W returns SFB_EINVAL.  sfb_split_export writes the current
 * parameters back into W (the matrix stays attached); sfb_split_detach forgets the
 * planes without exporting.  A second sfb_split_attach of the same W re-converts it.
 */
int64_t sfb_split_bytes(int64_t J, int64_t D);
int sfb_split_attach(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, void* dev_ptr, int64_t bytes);
int sfb_split_export(sfb_ctx* ctx, float* W);
int sfb_split_detach(sfb_ctx* ctx);

/* Hands the context a caller-allocated device buffer (256-byte aligned) to use
 * as scratch until replaced.  The library never frees it.  Its contents are
 * undefined after any call. */
int sfb_set_workspace(sfb_ctx* ctx, void* dev_ptr, int64_t bytes);

/*
 * Sufficient factors of one mini-batch at parameters W (Section 2.1: u is the
 * derivative of f with respect to W a, v = a).  Outputs U [B][J], V [B][D] of
 * batch->sf_dtype.
 *
 *   SFB_MLR (Section 1; Figure 2): multiclass logistic loss.
 *       u_i = softmax(W x_i) - onehot(y_i),  v_i = x_i.
 *       If V is NULL or V == X nothing is written for V (the caller passes X as
 *       V to sfb_apply).  in_dtype F32 -> sf_dtype F32; in_dtype BF16 ->
 *       sf_dtype BF16 (W is rounded to bf16 on the fly, fp32 accumulate).
 *   SFB_DML (Section 2, "Distance metric learning"): a_i = x_i - y_i, q_i = W a_i.
 *       similar pair: f = ||q||^2, u = 2 q.  dissimilar pair: f = max(0, margin - ||q||^2),
 *       u = -2 q if ||q||^2 < margin (strictly) else 0.  v_i = a_i.
 *       Rows of U of inactive pairs are zero (shapes stay static); *n_active
 *       (device int32, may be NULL) receives the number of pairs with u != 0.
 *       fp32 only.  Here J is the latent dimension (rows of W).
 *   SFB_SC (Section 2, "Sparse coding"; Figure 3): rows of W are basis vectors;
 *       the code a_i minimises 1/2||x_i - W^T a||^2 + lambda||a||_1 approximately by
 *       ista_iters ISTA iterations from a = 0 with step 1/L, L = the norm estimate
 *       after power_iters power iterations on W^T W started from the constant
 *       unit vector.  u_i = a_i, v_i = x_i - W^T a_i; the descent step is
 *       sfb_apply with NEGATIVE eta (W += |eta| U^T V).  fp32 only.
 *
 * W, X, Y are not modified.
 */
int sfb_compute_sf(sfb_ctx* ctx, int32_t model, const float* W, int64_t J, int64_t D,
                   const sfb_batch* batch, void* U, void* V, int32_t* n_active);

/*
 * Reconstructs and applies the summed rank-1 updates of N sufficient-factor
 * pairs (Section 3: W_p <- W_p - sum_q u_q v_q^T; Section 2.1: W <- W - eta dW):
 *       W[j][d] <- W[j][d] - eta * sum_{i<N} U[i][j] * V[i][d].
 * U [N][J] and V [N][D] are of sf_dtype (local and peer SF blocks concatenated
 * by rows, or one call per block: the results agree to rounding).  The
 * accumulation is fp32; each element of W is read and written exactly once by
 * exactly one workgroup, so the result is bit-reproducible.  eta may be
 * negative.  N == 0 is a no-op.  U and V are not modified.  Needs the workspace
 * of sfb_apply_workspace_bytes (SFB_ENOWS otherwise).
 */
int sfb_apply(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V,
              int64_t N, int32_t sf_dtype, float eta);

/*
 * sfb_apply for callers that cannot allocate device memory and therefore cannot
 * hand the library a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the
 * same resulting bits as sfb_apply; the scratch (U^T and V^T of bf16 factors,
 * the k-split partial sums of fp32 factors) lives in a static device array of
 * SFB_STATIC_SCRATCH_BYTES inside the library instead of the context's workspace,
 * which is neither needed nor touched.  Each GPU the library runs on holds its
 * own copy of that array until the process ends; sfb_create resolves its address
 * on the context's device.  The call allocates and frees nothing.
 *   - Shapes whose scratch (sfb_apply_workspace_bytes) exceeds the array are
 *     refused with SFB_ETOOBIG; nothing is enqueued.
 *   - All contexts of one GPU share the array, and it keeps the last call's
 *     contents (every call overwrites all it reads): calls that overlap in time
 *     on one GPU - two streams, two host threads - race on it.  Calls on one
 *     stream are ordered and safe.
 *   - Other status codes as for sfb_apply; SFB_EHIP if the array's address could
 *     not be resolved when the context was created.
 */
#define SFB_STATIC_SCRATCH_BYTES (32u << 20)
int sfb_apply_static(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V,
                     int64_t N, int32_t sf_dtype, float eta);

/*
 * The same with one coefficient per factor pair, for updates that are a short
 * signed sum of outer products ("Low-rank Extensions" of Section 2.1: the
 * rank-2 update u1 v1^T - u2 v2^T of a restricted Boltzmann machine, the rank-3
 * BFGS update alpha u u^T - beta (u v^T + v u^T)):
 *       W[j][d] <- W[j][d] - eta * sum_{i<N} coef[i] * U[i][j] * V[i][d].
 * coef is a device array of N floats (16-byte aligned).  The coefficient is
 * folded into a scaled copy of V (fp32: exactly one extra rounding per element;
 * bf16: c * v is rounded to bf16, which is exact for c = +-1).  Needs the
 * workspace of sfb_apply_signed_workspace_bytes.
 */
int64_t sfb_apply_signed_workspace_bytes(int64_t J, int64_t D, int64_t N, int32_t sf_dtype);
int sfb_apply_signed(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const void* V,
                     const float* coef, int64_t N, int32_t sf_dtype, float eta);

/*
 * Sparse samples and sparse second factors (Section 5, experimental setup: the
 * data are sparse, hence so are the factors v_i = x_i and the update matrices,
 * and this is used to cut communication and computation).  A block of rows in
 * compressed sparse row form, all three arrays in device memory (16-byte
 * aligned) and owned by the caller:
 *   indptr  [rows + 1]  indptr[0] = 0, non-decreasing, indptr[rows] = nnz;
 *   indices [nnz]       column of each stored entry, in [0, cols), strictly
 *                       increasing within a row;
 *   values  [nnz]       of `dtype` (fp32, or bf16 as raw 16-bit words).
 * This is the form in which a sparse factor block is buffered and would be
 * sent: nnz * (4 + element size) + 8 * (rows + 1) bytes instead of rows * cols
 * elements.  The two calls below take it as it is.
 *
 * sfb_mlr_sf_csr computes the logits W x_i by one of two routes, chosen from
 * nnz, B, J and D (sfb_set_csr_route overrides the choice):
 *   - over the stored entries only (work proportional to nnz * J, W read once;
 *     the route of tf-idf-like data with a fraction of a per cent of non-zeros),
 *   - or, where that would be slower (about one per cent of non-zeros and more
 *     at a batch of a thousand samples), as the dense matrix product of the
 *     dense entry point, whose aligned operand is written straight from the
 *     CSR rows (no dense X in the caller's memory).
 * sfb_apply_csr always writes its dense operand from the CSR rows and runs the
 * dense contraction: with hundreds of factor pairs every column of W is touched
 * by some pair, and the read-modify-write of W is the cost either way.
 *
 * A stored entry with a column outside [0, cols) or a row range outside
 * [0, nnz] is ignored (nothing is written out of bounds); a row with repeated
 * columns gives an unspecified result for that row (one of the repeated values
 * on the dense route, their sum on the other).  sfb_csr_check verifies the
 * format on the device.
 */
typedef struct {
    const int64_t* indptr;
    const int32_t* indices;
    const void* values;
    int64_t rows, cols, nnz;
    int32_t dtype; /* sfb_dtype of values */
} sfb_csr;

/* Counts the violations of the format above into *violations (host memory).
 * Unlike the other calls this one waits for the stream.  Uses the first 256
 * bytes of the workspace (SFB_ENOWS if there is none). */
int sfb_csr_check(sfb_ctx* ctx, const sfb_csr* m, int64_t* violations);

/* sfb_compute_sf(SFB_MLR) for samples given as CSR rows (X->rows = B,
 * X->cols = D): U [B][J] of X->dtype receives softmax(W x_i) - onehot(y_i);
 * the second factors are the rows of X themselves.  y: int32 labels [B]. */
int64_t sfb_mlr_sf_csr_workspace_bytes(int64_t J, int64_t D, int64_t B, int32_t dtype);
int sfb_mlr_sf_csr(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, const sfb_csr* X, const int32_t* y, void* U);
/* Route of sfb_mlr_sf_csr on this context: 0 = chosen per call (the default), 1 = always the dense product,
 * 2 = always over the stored entries (shapes that route cannot take still go the dense way).  For
 * measurements and tests; results agree to rounding (different summation order). */
int sfb_set_csr_route(sfb_ctx* ctx, int route);

/* sfb_apply / sfb_apply_signed with the second factors given as CSR rows
 * (V->rows = N, V->cols = D, U [N][J] of V->dtype; coef may be NULL):
 *       W[j][d] <- W[j][d] - eta * sum_i coef[i] * U[i][j] * V[i][d]. */
int64_t sfb_apply_csr_workspace_bytes(int64_t J, int64_t D, int64_t N, int32_t sf_dtype);
int sfb_apply_csr(sfb_ctx* ctx, float* W, int64_t J, int64_t D, const void* U, const sfb_csr* V, const float* coef,
                  float eta);

/*
 * Stochastic dual coordinate ascent for l2-regularised multiclass logistic
 * regression (Section 2.1, "Stochastic DCA"; the L2-MLR model of Section 5):
 *   (P)  min_W (1/N) sum_i f_i(W a_i) + (lambda/2) ||W||_F^2,  f_i the logistic loss,
 *   (D)  min_U (1/N) sum_i f_i^*(-u_i) + h^*(Z),  Z = (1/N) U A^T,  W = grad h^*(Z) = Z / lambda.
 * The dual variable of a sample is held as the simplex point p_i = onehot(y_i) - u_i
 * (start: u_i = 0, i.e. p_i = onehot(y_i)); f_i^*(-u_i) is the negative entropy of p_i.
 *
 * sfb_sdca_mlr_sf computes, for a mini-batch and all at the same W, each sample's
 * coordinate step du_i = u_i - argmin_u (D): with z = W a_i, c = ||a_i||^2 / (lambda N),
 *       log p_j + c p_j = z_j + c P[i][j] - nu   for every class j,   sum_j p_j = 1
 * (solved to fp32 accuracy), then  dU[i] = beta (p - P[i])  and  P[i] += dU[i].
 * (dU[i], a_i) is the sufficient-factor pair of the step: the caller applies
 *       Z <- Z - (1/N) sum_i dU[i] a_i^T     as sfb_apply(Z, dU, X, eta = 1/N)
 * over its own and its peers' pairs, and then W <- grad h^*(Z) with
 * sfb_dual_to_primal_l2 (or, equivalently for this h, applies the pairs to W
 * directly with eta = 1 / (lambda N)).  The 1/N, which the text leaves out of the
 * update of Z, is what keeps Z = (1/N) U A^T.  beta in (0, 1] scales all steps of a
 * mini-batch (1 = the sequential algorithm when B = 1); P stays in the simplex.
 * X [B][D], P [B][J], dU [B][J], W [J][D] fp32 device arrays; N = samples in (P).
 * Needs the workspace of sfb_sdca_workspace_bytes.
 */
int64_t sfb_sdca_workspace_bytes(int64_t J, int64_t D, int64_t B);
int sfb_sdca_mlr_sf(sfb_ctx* ctx, const float* W, int64_t J, int64_t D, const float* X, int64_t B, float* P,
                    float lambda, int64_t N, float beta, float* dU);
/* W[j][d] = Z[j][d] / lambda (W may be Z itself).  Keeps an attached bf16 copy of W current. */
int sfb_dual_to_primal_l2(sfb_ctx* ctx, const float* Z, float* W, int64_t J, int64_t D, float lambda);

/*
 * Proximal operator of sparse coding's norm constraint (Figure 3, "prox"), on
 * the rows of W (the basis vectors in this library's orientation):
 *   SFB_PROX_PROJECT:   w_j <- w_j / ||w_j||  if ||w_j|| > 1, else unchanged;
 *   SFB_PROX_NORMALIZE: w_j <- w_j / ||w_j||  if ||w_j|| > 0.
 */
int sfb_prox_rows(sfb_ctx* ctx, float* W, int64_t J, int64_t D, int32_t mode);

/* Static description of a status code. */
const char* sfb_strerror(int code);
/* hipError_t (as int) of the last failed HIP call on this context, 0 if none. */
int sfb_last_hip_error(const sfb_ctx* ctx);
/* Library version, "major.minor". */
const char* sfb_version(void);
/*
 * Optional per-kernel timing for benchmarks.  When enabled, each kernel launch
 * of the context is bracketed by two HIP events recorded on the context's
 * stream (a fixed pool of 4096 pairs; launches beyond it are not timed).
 * sfb_profile_collect synchronises the stream, sums the elapsed time per kernel
 * group since the last collect into `out` (at most max_entries entries, *count
 * of them filled; `name` points to static storage) and empties the pool.  It
 * returns SFB_ENOWS if launches were dropped because the pool was full.
 * Keep it disabled (the default) while the stream is being captured into a HIP
 * graph: with it disabled every call enqueues kernels and device-to-device
 * copies only and can be captured and replayed.
 */
typedef struct {
    const char* name;
    int32_t launches;
    float total_ms;
} sfb_kernel_time;
int sfb_profile_enable(sfb_ctx* ctx, int on);
int sfb_profile_collect(sfb_ctx* ctx, sfb_kernel_time* out, int max_entries, int* count);

/*
 * Bound of the only in-kernel wait of the library (per context).  For rows of
 * 65536 classes or more the softmax of the bf16 multiclass-logistic path is
 * computed by several workgroups per row, each keeping its part of the row in
 * registers so that the logits are read once; they exchange one (max, sum) pair
 * per row through the workspace.  A workgroup polls a partner's pair at most
 * `polls` times (about a microsecond each; default 1000, restored by a negative
 * argument) and then computes that pair itself from the logits, so the result
 * never depends on which workgroups are on the chip together; 0 makes every
 * workgroup do so at once (same results; meant for tests of that path).
 * sfb_wait_fallbacks waits for the context's stream and reports how many pairs
 * workgroups have computed themselves in this way on the context's device since
 * the library was loaded (all contexts of the device together): each costs a
 * second read of the partner's part of the row, so a count that grows in
 * normal operation says that kernels of other streams keep partners off the chip.
 */
int sfb_set_wait_limit(sfb_ctx* ctx, int polls);
int sfb_wait_fallbacks(sfb_ctx* ctx, int64_t* count);

#ifdef __cplusplus
}
#endif
#endif /* SFB_H */
