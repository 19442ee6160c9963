/*
 * aser.h - C ABI of the MI355X (gfx950) implementation of ASER's per-linear-layer
 * calibration path (arXiv 2411.07762, "ASER: Activation Smoothing and Error Reconstruction
 * for Large Language Model Quantization").
 *
 * The calls follow the loop body of Algorithm 1 for one layer y = W x:
 *
 *   aser_gram_accumulate    G += X_c^T X_c over token chunks              (Eq. 5, Alg. 1)
 *   aser_smooth_outliers    outlier set I_f and smoothing diagonal m      (Sec. 4.2, Eq. 10-11)
 *   aser_quantize_rtn       Q(W_s) and the target T = W M - Q(W_s)        (Eq. 12, Sec. 3.1)
 *   aser_smoothed_weight,   the same stage around a weight quantizer of the caller's: W_s out,
 *   aser_quant_target       T = W M - W_q in                              (Sec. 4.1, closing remark)
 *   aser_whiten             S = chol(M^-1 G M^-1)                         (Eq. 5, Alg. 1)
 *   aser_error_reconstruct  rank-r SVD of T S, L_A = U_r Sigma_r,
 *                           L_B = V_r^T S^-1                              (Eq. 6, Sec. 4.1)
 *   aser_quantize_act_rtn   per-token RTN of X M^-1 (evaluation only)     (Sec. 5.1)
 *   aser_calibrate_layers   Algorithm 1's loop over the layers of a model, several layers in flight on
 *                           contexts and streams of their own (layers are independent once their inputs
 *                           are stored)                                    (Alg. 1, loop over the layers W^l)
 *
 * Orientation.  The paper stores activations as (in x tokens) and writes the Gram matrix
 * X X^T.  This library stores activations tokens x in (N x n, row-major, channel
 * contiguous); the same n x n matrix is then G = X^T X.  W is m x n (out x in), row-major.
 *
 * Conventions.
 *   - Every matrix pointer is a DEVICE pointer owned by the caller; the library never
 *     allocates, frees or retains caller-visible buffers.  Scratch memory comes from the
 *     workspace bound with aser_set_workspace (device memory, 256-byte aligned).
 *   - Row-major with explicit leading dimensions in ELEMENTS (ld >= number of columns).
 *   - All work is enqueued on the hipStream_t given to aser_create.  Calls are asynchronous
 *     unless they return a host scalar (aser_whiten's info, aser_error_reconstruct's err and
 *     n_iter), in which case they synchronise that stream before returning.
 *   - Every call returns an aser_status.  Arguments are validated on the host before any
 *     HIP call is made; on error nothing has been enqueued.  No exception or abort crosses
 *     the ABI.  aser_last_error(ctx) returns a text for the last failing call on ctx.
 *   - One GPU, one stream per context; calls on one context must not overlap.
 */
#ifndef ASER_H
#define ASER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct aser_ctx aser_ctx;

typedef enum aser_status {
    ASER_OK = 0,
    ASER_ERR_INVALID_ARG = 1,   /* null pointer, bad enum, bad alignment                 */
    ASER_ERR_SHAPE = 2,         /* non-positive size, ld < cols, f > n, r > min(m, n) ... */
    ASER_ERR_DTYPE = 3,         /* unsupported dtype / bit width                          */
    ASER_ERR_NOT_SPD = 4,       /* Cholesky met a non-positive pivot                      */
    ASER_ERR_NO_CONVERGE = 5,   /* the subspace iteration's orthogonalisation broke down  */
    ASER_ERR_WORKSPACE = 6,     /* workspace missing or too small                         */
    ASER_ERR_HIP = 7            /* a HIP runtime call failed                              */
} aser_status;

typedef enum aser_dtype { ASER_DTYPE_BF16 = 0, ASER_DTYPE_F32 = 1 } aser_dtype;

typedef enum aser_code_layout {
    ASER_CODES_INT8 = 0,        /* one int8 per weight, row pitch n bytes                     */
    ASER_CODES_INT4_PACKED = 1  /* two's-complement nibbles, even column in the low nibble,
                                   row pitch n/2 bytes; n must be even; needs bits == 4       */
} aser_code_layout;

/* Options of the truncated SVD.  Zero in any field selects its default. */
typedef struct aser_svd_opts {
    int32_t block;      /* subspace width b (multiple of 32, r <= b <= 128); default: the
                           smallest multiple of 32 that is >= min(2 r, 128) and >= r        */
    int32_t max_iter;   /* number of subspace iterations (A A^T applications); default 9, 12 when max(m, n) > 8192,
                           30 when block < 2 r */
    uint32_t seed;      /* seed of the random start block; default 1                       */
} aser_svd_opts;

/* How fp32 operands enter the bf16 MFMA products of aser_whiten, aser_error_reconstruct and the
 * fp32-input form of aser_gram_accumulate (bf16 activations are always multiplied exactly). */
typedef enum aser_precision {
    ASER_PRECISION_AUTO = 0,    /* default: EXACT for small problems (n <= 1024 for the Gram matrix and the
                                   whitening, m n <= 2^20 for the reconstruction), FAST otherwise         */
    ASER_PRECISION_FAST = 1,    /* x = hi + lo (bf16), three products per fp32 product, about 2^-16       */
    ASER_PRECISION_EXACT = 2    /* x = hi + mid + lo, six products, about 2^-24; about twice the time     */
} aser_precision;

const char* aser_status_string(int status);

/* Creates a context bound to `device` and to `hip_stream` (a hipStream_t, may be NULL for
 * the default stream).  No HIP call is made until the first compute call. */
int aser_create(aser_ctx** out, int device, void* hip_stream);
int aser_destroy(aser_ctx* ctx);
const char* aser_last_error(const aser_ctx* ctx);

/* Chooses the product form for later calls on ctx (see aser_precision). */
int aser_set_precision(aser_ctx* ctx, int precision);

/* Binds `bytes` of device memory at `dev_ptr` (256-byte aligned) as scratch space; `bytes` is rounded
 * down to a multiple of 256.  The caller keeps ownership and must keep it alive while calls on ctx may
 * use it, and until this call has returned when it replaces another workspace (status words that an
 * asynchronous call left in the old one are fetched first, and reported as this call's status). */
int aser_set_workspace(aser_ctx* ctx, void* dev_ptr, size_t bytes);

/* Workspace needed by the calls below for a layer of m x n with rank r (opts may be NULL).
 * aser_gram_accumulate and aser_quantize_rtn need none. */
size_t aser_workspace_bytes(int64_t m, int64_t n, int32_t r, const aser_svd_opts* opts);

/* Stage 1 (Eq. 5; Alg. 1 "Cholesky decomposition on (M^-1 X)(M^-1 X)^T" needs X X^T).
 * Accumulates one chunk of calibration tokens into caller-zeroed running sums:
 *     G[i][j]    += sum_t X[t][i] * X[t][j]        for i >= j   (fp32)
 *     abs_sum[i] += sum_t |X[t][i]|                             (fp64, may be NULL)
 *     *count     += rows                                        (device int64, may be NULL)
 * X: rows x n, dtype x_dtype (bf16 or fp32), leading dimension ldx.  G: n x n fp32, ldg.
 * Only the lower triangle of G (i >= j) is defined afterwards; entries above the diagonal
 * may or may not have been touched.  bf16 inputs are multiplied exactly and accumulated in
 * fp32; fp32 inputs are split into two bf16 terms (three MFMA products per term pair,
 * relative error about 2^-16 per product).  Partial sums are added with fp32 atomics, so
 * G is reproducible only up to summation order.  rows == 0 is a no-op. */
int aser_gram_accumulate(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                         float* G, int64_t ldg, double* abs_sum, int64_t* count);

/* Stage 2 (Sec. 4.2, Eq. 10, Eq. 11; Alg. 1 "Compute m_i = Xbar_i / Xbar_min for i in I_f").
 *     Xbar_i = abs_sum[i] / *count,  Wbar_i = mean_o |W[o][i]|,  score_i = Xbar_i * Wbar_i  (fp64)
 *     idx    = the f channels with the largest score, in descending score order, ties
 *              resolved towards the lower channel index
 *     mdiag  = Xbar_i / min_{j in I_f} Xbar_j for i in I_f, else 1                   (fp32, n)
 *     W_o    = W[:, idx] * mdiag[idx]   (m x f, row-major, ld = f; may be NULL)
 *     score  = the n scores (fp64; may be NULL)
 * f == 0 is the branch without activation smoothing: mdiag = 1, idx untouched.
 * Channels whose score is NaN or infinite are never selected.  If fewer than f channels remain (no
 * tokens accumulated, NaN/Inf in X or W), the left-over entries of idx are -1 (every consumer of idx in
 * this library skips entries outside [0, n)), and the next synchronising call on this context
 * (aser_whiten with info, aser_error_reconstruct, aser_set_workspace) returns ASER_ERR_INVALID_ARG.
 * Never synchronises.  Needs workspace (aser_workspace_bytes). */
int aser_smooth_outliers(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                         const double* abs_sum, const int64_t* count, int32_t f,
                         int32_t* idx, float* mdiag, float* W_o, double* score);

/* aser_smooth_outliers for callers that cannot allocate device memory and so have no workspace to bind:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results, same deferred report; the scratch (two fp64 arrays of n entries and a status word) lives
 * in a static device array of 512.25 KiB that each GPU the library runs on holds until the process ends.
 * n <= 32768, else ASER_ERR_SHAPE; the context's device index must be below 16.  Makes no hipMalloc,
 * hipFree or other allocating call; memory is cleared by kernels, not by memset nodes.  All calls on one
 * GPU share that GPU's array: calls that overlap on one GPU (two streams, two contexts) race; calls in
 * stream order on one stream do not. */
int aser_smooth_outliers_noalloc(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                 const double* abs_sum, const int64_t* count, int32_t f,
                                 int32_t* idx, float* mdiag, float* W_o, double* score);

/* Stage 3 (Sec. 3.1 E_q = W - W_q; Eq. 12; per-channel RTN, Sec. 5.1).
 * W_s = W with the idx columns set to zero.  Per output row o, in IEEE fp32:
 *     scale_o = max_j |W_s[o][j]| / qmax,  qmax = 2^(bits-1) - 1   (1 if the row is zero)
 *     code    = clamp(rint_half_even(W_s[o][j] / scale_o), -qmax, qmax)
 *     T[o][j] = W[o][j] * mdiag[j] - code * scale_o       ( = E_q + W_o of Eq. 12 )
 * codes: layout as aser_code_layout; scales: m fp32; T: m x n fp32, ldt (may be NULL).
 * idx/mdiag may be NULL when f == 0.  bits is 4 or 8. */
int aser_quantize_rtn(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                      const int32_t* idx, const float* mdiag, int32_t f, int32_t bits, int32_t layout,
                      void* codes, float* scales, float* T, int64_t ldt);

/* Stage 3 with another weight quantizer (Sec. 4.1, closing remark: the reconstruction builds on any
 * weight-only quantizer, not only RTN).  The caller's quantizer runs between these two calls, on the device:
 *     aser_smoothed_weight:  W_s[o][j] = 0 for j in idx, else W[o][j]          (what Alg. 1 quantizes)
 *     aser_quant_target:     T[o][j]   = W[o][j] * mdiag[j] - Wq[o][j]         (one fused multiply-add, fp32)
 * Wq is the dequantized result of that quantizer on W_s (m x n fp32, ldq).  W X = (Wq + T)(M^-1 X) holds
 * whatever Wq is; where Wq keeps the idx columns at zero, T = E_q + W_o as in Eq. 12, and T then goes to
 * aser_error_reconstruct like the T of aser_quantize_rtn.  W_s: m x n fp32, ldws, must not overlap W.
 * T: m x n fp32, ldt; T may be Wq itself (in place, same leading dimension).  idx may be NULL when f == 0
 * (W_s = W); entries of idx outside [0, n) are skipped.  mdiag may be NULL (M = I).  Never synchronise,
 * need no workspace. */
int aser_smoothed_weight(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                         const int32_t* idx, int32_t f, float* Ws, int64_t ldws);
int aser_quant_target(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw, const float* mdiag,
                      const float* Wq, int64_t ldq, float* T, int64_t ldt);

/* Stage 4a (Eq. 5: S^-1 X X^T S^-T = I, S by Cholesky decomposition; Alg. 1 uses M^-1 X).
 *     G'[i][j] = G[i][j] / (mdiag[i] * mdiag[j])  (+ damp * mean(diag G') on the diagonal)
 *     S = lower Cholesky factor, S S^T = G'
 * Reads the lower triangle of G (n x n, ldg); writes S (n x n, lds) with zeros above the
 * diagonal.  S may alias G (in place).  mdiag may be NULL (M = I).  damp >= 0, normally 0.
 * *info (host): 0, or the 1-based index of the first non-positive pivot, in which case
 * ASER_ERR_NOT_SPD is returned and S is unspecified; the call then synchronises the stream.
 * info == NULL: the call stays asynchronous; a non-positive pivot is then reported (as
 * ASER_ERR_NOT_SPD) by the next aser_error_reconstruct or aser_set_workspace on this context,
 * whose result is unspecified in that case.  Needs workspace. */
int aser_whiten(aser_ctx* ctx, const float* G, int64_t ldg, int64_t n, const float* mdiag, float damp,
                float* S, int64_t lds, int32_t* info);

/* Stage 4b/4c (Eq. 6; Sec. 4.1 L_A = U_r Sigma_r, L_B = V_r^T S^-1; Alg. 1 last lines).
 * Rank-r truncated SVD of A = T S: blocked subspace iteration with Rayleigh-Ritz, or, for small layers,
 * a dense solver (see "Solver" below).
 *     L_A   = U_r Sigma_r                  (m x r, ld = r)
 *     L_B   = V_r^T S^-1                   (r x n, ld = n), evaluated as Sigma_r^-1 U_r^T T,
 *             which is the same matrix because V_r^T = Sigma_r^-1 U_r^T T S
 *     sigma = the r Ritz singular values, descending (fp32, device)
 *     *err  (host, may be NULL) = ||A - U_r U_r^T A||_F evaluated as an explicit residual: the
 *             whitened layer-output error ||(T - L_A L_B) S||_F of Eq. 8
 *     *n_iter (host, may be NULL) = subspace iterations performed
 * T: m x n fp32 (ldt); S: n x n fp32 lower triangular with zeros above the diagonal (lds).
 * 0 < r <= min(m, n, 256); for the subspace iteration (r <= 128) a multiple of 32 must also lie in
 * [r, min(m, n, 128)] (the subspace width; e.g. r = 40 needs min(m, n) >= 64), else ASER_ERR_SHAPE.
 * r > 128 always takes the dense solver below, which then needs min(m, n) <= 16384.
 * Synchronises the stream.
 * idx, f: the outlier set I_f of aser_smooth_outliers (f device int32 entries; f == 0: none, idx may be
 * NULL).  Those columns of T hold the unquantized W_o of Eq. 12 and dwarf the quantization error in the
 * other columns, so they become the first columns of the start block, ahead of the random ones: the
 * orthogonalisation then works on a graded block instead of columns that all mix the largest and the
 * smallest wanted singular directions.  The result does not depend on them otherwise; entries outside
 * [0, n) are ignored.  A caller that has outlier columns in T and passes f = 0 gets
 * ASER_ERR_NO_CONVERGE once sigma_1 / sigma_b passes a few hundred.
 * Solver.  Layers with m n <= 2^20 (default options, precision mode not FAST), and every call with r > 128
 * (the widest subspace block is 128: tens to hundreds of milliseconds on layers of thousands of channels,
 * against milliseconds for the iteration), take a dense fp64 solver:
 * every eigenvalue of the Gram matrix of the shorter side of T S (Householder tridiagonalisation,
 * bisection), the eigenvectors of the r largest (inverse iteration), *err from the tail of the spectrum;
 * idx, f and the block-width rule do not apply, *n_iter is 0.  Larger layers, and any call with
 * opts->max_iter or opts->block set, run the subspace iteration for a fixed number of iterations
 * (aser_svd_plan reports it) without a residual test: the excess of the whitened error over the optimum
 * shrinks by about 0.47 per iteration on quantization-error spectra (measured 2e-5 relative after the
 * default count on every workload shape named in the bench, 1e-6 on int8 layers of 2048 channels).
 * Its products carry about 2^-16 relative error (2^-24 in the EXACT mode), so a whitened error below
 * about 1e-3 of ||T S||_F is resolved to fewer than four digits there; such residuals were only met on
 * layers of a few hundred channels, which the dense solver takes.
 * ASER_ERR_NO_CONVERGE: a pivot of a block Gram matrix was not positive.
 * Reports (as ASER_ERR_NOT_SPD / ASER_ERR_INVALID_ARG) what an asynchronous aser_whiten or an
 * aser_smooth_outliers on this context has left pending.  Needs workspace. */
int aser_error_reconstruct(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt,
                           const float* S, int64_t lds, int32_t r, const int32_t* idx, int32_t f,
                           const aser_svd_opts* opts,
                           float* L_A, float* L_B, float* sigma, double* err, int32_t* n_iter);

/* aser_error_reconstruct in two halves, for callers that keep several layers in flight on several contexts
 * (Algorithm 1's loop over layers: once the activations are stored a layer reads nothing of another).
 * aser_error_reconstruct_enqueue validates and enqueues everything, including the copy of the status block
 * to pinned host memory, and returns without waiting for the device: same arguments, same results in the
 * same buffers.  aser_finish waits for the context's stream and returns what aser_error_reconstruct
 * returns: its status (with what asynchronous calls left pending), *err and *n_iter (host, may be NULL).
 * Everything aser_error_reconstruct_enqueue and the stage calls before it enqueue is kernels and one
 * device-to-host copy into pinned memory (no memset nodes, no allocation, no host wait), so a layer's five
 * stages can be captured into a HIP graph on the context's stream after one eager pass (which sets function
 * attributes and allocates the pinned status block); a replay leaves the squared whitened error as the double
 * at byte 16 of the last 256 bytes of the workspace.
 * Between the two, the context accepts no other call that synchronises or rebinds the workspace
 * (ASER_ERR_INVALID_ARG), and the workspace and all buffers of the layer stay untouched by the caller. */
int aser_error_reconstruct_enqueue(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt,
                                   const float* S, int64_t lds, int32_t r, const int32_t* idx, int32_t f,
                                   const aser_svd_opts* opts, float* L_A, float* L_B, float* sigma);
int aser_finish(aser_ctx* ctx, double* err, int32_t* n_iter);

/* One layer of Algorithm 1's loop, as the five stage calls take it: every pointer is a DEVICE pointer with the
 * meaning, layout and alignment documented at the stage call that consumes it; the last three fields are
 * written by aser_calibrate_layers on the HOST. */
typedef struct aser_layer_desc {
    /* stage 1, aser_gram_accumulate.  X == NULL: G, abs_sum and count already hold the finished statistics
     * of this layer's input when aser_calibrate_layers is called (layers that share an input: accumulate
     * once, before the call).  clear_stats != 0 (with X): G (n x n, ldg), abs_sum and count are cleared first.
     * Intermediates that the caller does not keep may be NULL and then live in the context's workspace for
     * the time the layer is in flight: G (with X given; abs_sum and count are then taken from there too and
     * cleared), T, S.  The workspace must then hold aser_layer_workspace_bytes(layer).
     * stats_from (below) == j + 1 > 0: this layer reads the input of layers[j], an EARLIER layer of the same call
     * that accumulates its statistics in this call (X given; G, abs_sum and count in buffers of its own, not left
     * to the workspace): X, G, abs_sum and count of this descriptor are ignored, those of layers[j] are used once
     * its Gram update has run (q, k, v of an attention block; gate and up of an MLP).  0: none. */
    const void* X; int32_t x_dtype; int32_t clear_stats; int64_t rows; int64_t ldx;
    float* G; int64_t ldg; double* abs_sum; int64_t* count;
    /* stage 2, aser_smooth_outliers */
    const float* W; int64_t m; int64_t n; int64_t ldw; int32_t f; int32_t bits;
    int32_t* idx; float* mdiag;
    /* stage 3, aser_quantize_rtn */
    int32_t layout; int32_t r; void* codes; float* scales; float* T; int64_t ldt;
    /* stage 4, aser_whiten (asynchronous form) and aser_error_reconstruct */
    float damp; int32_t stats_from; float* S; int64_t lds;
    const aser_svd_opts* opts; float* L_A; float* L_B; float* sigma;
    /* results (host) */
    double err; int32_t n_iter; int32_t status;
} aser_layer_desc;

/* Algorithm 1's loop over layers with up to n_ctx (<= 64) layers in flight.  Layers are started in the order
 * given, each on a context that is free or, when all are busy, on the first one whose stream has drained
 * (every context has its own stream and its own workspace of at least aser_layer_workspace_bytes of EVERY layer);
 * the five stages of a layer are enqueued without a host wait.  The dependent chain of small launches that
 * bounds one layer (whitening, subspace iteration) leaves most of the device idle, and the chains of the
 * other layers run there; give long layers first.
 * Per layer: layers[k].status, .err, .n_iter as aser_error_reconstruct returns them (a layer whose
 * arguments are refused is skipped, the others still run); the text of a layer's failure stays in
 * aser_last_error of its context until that context's next layer.  Returns ASER_OK when every layer did,
 * else the first status that was not; ASER_ERR_INVALID_ARG for null arguments or n_ctx outside [1, 64].
 * Layers in flight together must not share output buffers; inputs (X, W, finished statistics) may be
 * shared.  Layers on one input (stats_from): the owner's Gram update is followed by an event on its stream and
 * the others' streams wait for that event before their first launch, so they start as soon as the statistics
 * are there and run beside the owner's later stages; a layer whose owner was refused gets ASER_ERR_INVALID_ARG.
 * Host code runs on the calling thread only. */
int aser_calibrate_layers(aser_ctx* const* ctxs, int32_t n_ctx, aser_layer_desc* layers, int32_t n_layers);
/* Workspace a context needs for this layer: aser_workspace_bytes of its shape plus the intermediates left NULL. */
size_t aser_layer_workspace_bytes(const aser_layer_desc* layer);

/* Streams for aser_calibrate_layers.  A process has few hardware queues (four by default; the environment variable
 * GPU_MAX_HW_QUEUES, read when the HIP runtime initialises, sets another count) and the runtime maps
 * every stream to one of them; two streams on the same queue run one after the other, however independent their
 * work.  From `n_candidates` streams (hipStream_t, created by the caller, idle) this picks up to `want` that
 * run concurrently with one another: chosen[0 .. *n_chosen) are indices into `candidates` (HOST arrays).
 * It times a delay kernel of one wavefront (about 0.2 ms, bounded) on a candidate alone and next to each
 * stream already chosen; a candidate whose pair takes as long as two in a row shares a queue and is passed over.
 * Synchronises the candidate streams; a few milliseconds per candidate.  ASER_ERR_INVALID_ARG, ASER_ERR_HIP. */
int aser_pick_concurrent_streams(int32_t device, void* const* candidates, int32_t n_candidates, int32_t want,
                                 int32_t* chosen, int32_t* n_chosen);

/* The subspace width and the iteration count aser_error_reconstruct will use for this shape and these
 * options (either pointer may be NULL); both 0 for r > 128, which the dense solver takes.  ASER_ERR_SHAPE
 * where aser_error_reconstruct would refuse. */
int aser_svd_plan(int64_t m, int64_t n, int32_t r, const aser_svd_opts* opts, int32_t* block, int32_t* iters);

/* All min(m, n) singular values of T S, descending, as fp64 (S == NULL: of T itself): the spectrum that
 * Eq. 9 sums over, that Eq. 3-4 take the entropy of and whose largest values Sec. 3.2 plots for the
 * weight error (S == NULL) and for the activation-weight error (S the whitening factor; E_q S and E_q X
 * have the same singular values because S S^T = X X^T).
 * T: m x n fp32 (ldt); S: n x n fp32 lower triangular (lds) or NULL; sigma: DEVICE, min(m, n) doubles.
 * The product T S carries about 2^-16 relative error per term; behind it everything is fp64 (Gram matrix
 * of the shorter side, Householder tridiagonalisation, bisection), so a singular value is off by at most
 * about 1e-5 of the mean singular value plus 1e-7 of the largest.  min(m, n) <= 16384.
 * Asynchronous.  Needs aser_spectrum_workspace_bytes(m, n, S != NULL) bytes of workspace. */
size_t aser_spectrum_workspace_bytes(int64_t m, int64_t n, int32_t with_s);
int aser_singular_values(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt,
                         const float* S, int64_t lds, double* sigma);

/* Rank from the threshold alpha (Eq. 9; Algorithm 1 "r <- ..." line): the largest r with
 * (sigma_1 + ... + sigma_r) / (sigma_1 + ... + sigma_k) < alpha, strictly, and at least 1.
 * sigma: DEVICE, k doubles, descending (aser_singular_values).  0 < alpha < 1.
 * *r (host) receives the rank; stats (host, 3 doubles, may be NULL) receives the sum of all singular
 * values and the cumulative shares at r and at r + 1, between which alpha lies (how far the decision is
 * from flipping).  Synchronises the stream.  Needs a bound workspace (any size). */
int aser_select_rank(aser_ctx* ctx, const double* sigma, int64_t k, double alpha, int32_t* r, double* stats);

/* Effective rank (Eq. 3, Eq. 4): exp(-sum_k p_k ln p_k) with p_k = sigma_k / sum_i sigma_i + eps.
 * sigma: DEVICE, k doubles; eps >= 0 (the paper does not give its value; 1e-12 keeps ln finite for
 * zero singular values); *erank: host.  Synchronises the stream.  Needs a bound workspace (any size). */
int aser_effective_rank(aser_ctx* ctx, const double* sigma, int64_t k, double eps, double* erank);

/* Per-token activation quantizer of the W4A8 setting (Sec. 5.1 "per-token for activations").
 * It does not feed L_A / L_B; it serves the layer-output error under activation quantization.
 *     X'[t][i] = X[t][i] / mdiag[i]  (IEEE fp32),  s_t = max_i |X'[t][i]| / qmax  (1 if zero)
 *     codes[t][i] = clamp(rint_half_even(X'[t][i] / s_t), -qmax, qmax)     (int8, ld = n)
 * mdiag may be NULL (M = I).  bits in [2, 8]. */
int aser_quantize_act_rtn(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                          const float* mdiag, int32_t bits, int8_t* codes, float* scales);

/* Remaining layer-output error of the quantized, compensated layer on a sample of tokens (the metric
 * of the paper's per-layer error figure, Sec. 5.3: ||W X - W~ X_q||_F; Sec. 5.1 for the quantizers):
 *     *err      = || X W^T - X'_q W~^T ||_F,   *ref_norm (may be NULL) = || X W^T ||_F
 * with X' = X M^-1 (Eq. 10), X'_q the per-token RTN image of X' at act_bits bits, dequantized
 * (act_bits == 0: X'_q = X', weights only), and W~ = deq(codes, scales) + L_A L_B (end of Sec. 4.2;
 * r == 0: the RTN baseline without compensation, L_A and L_B may then be NULL).  Both branches of the
 * compensated layer read the same quantized activations.
 * W: m x n fp32 (ldw); X: rows x n, bf16 or fp32 (ldx); mdiag: n fp32 or NULL; codes / layout / scales as
 * written by aser_quantize_rtn; L_A: m x r (ld r), L_B: r x n (ld n); act_bits: 0 or 2..8.  All DEVICE
 * pointers; err, ref_norm: host.  fp32-class products (about 2^-16 relative per term, random signs):
 * *err is resolved to about 1e-5 ||X W^T||_F.  Synchronises the stream.
 * Needs aser_output_error_workspace_bytes(m, n, rows, r) bytes of workspace. */
size_t aser_output_error_workspace_bytes(int64_t m, int64_t n, int64_t rows, int32_t r);
int aser_layer_output_error(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                            const void* X, int x_dtype, int64_t rows, int64_t ldx, const float* mdiag,
                            const void* codes, int32_t layout, const float* scales,
                            const float* L_A, const float* L_B, int32_t r, int32_t act_bits,
                            double* err, double* ref_norm);

/* The compensated layer at inference (end of Sec. 4.2: W_q X + L_A L_B X; Sec. 5.3 overhead analysis),
 * tokens x channels orientation, integer MFMA for the quantized product:
 *     Y[t][o] = s_t c_o sum_i xq[t][i] wq[o][i] + sum_k P[t][k] L_A[o][k],   P[t][k] = s_t sum_i xq[t][i] L_B[k][i]
 * x_codes (rows x n int8, pitch n) and x_scales (rows): per-token codes of X M^-1 from aser_quantize_act_rtn;
 * w_codes / layout / w_scales (m): from aser_quantize_rtn (int8 pitch n, or packed int4 pitch n / 2);
 * L_A: m x r (ld r), L_B: r x n (ld n), fp32; r == 0: no compensation (L_A, L_B may be NULL);
 * Y: rows x m fp32 (ldy).  All DEVICE pointers; codes 16-byte aligned.  n % 32 == 0, r <= 128.
 * The integer sums are exact.  lowrank_split != 0: the rank-r branch runs at fp32-class accuracy (bf16
 * hi + lo terms, about 2^-16 relative per product); 0: its factors are rounded to bf16 once, as an
 * inference kernel that stores them in 16 bits would (about 2^-9 relative per factor).
 * Asynchronous.  Needs aser_forward_workspace_bytes(rows, n, m, r) bytes of workspace when r > 0. */
size_t aser_forward_workspace_bytes(int64_t rows, int64_t n, int64_t m, int32_t r);
int aser_compensated_forward(aser_ctx* ctx, const int8_t* x_codes, const float* x_scales, int64_t rows, int64_t n,
                             const void* w_codes, int32_t layout, const float* w_scales, int64_t m,
                             const float* L_A, const float* L_B, int32_t r, int32_t lowrank_split,
                             float* Y, int64_t ldy);

/* Measurement aid (not a step of the method; bench.py reports it next to the nominal peaks): the rate, in
 * 10^12 operations per second, that a loop of nothing but MFMA instructions reaches on the device, with
 * `workgroups_per_cu` (1 .. 4) workgroups of four wavefronts per compute unit and `iters` rounds of 16
 * instructions per wavefront.  kind 0: v_mfma_f32_32x32x16_bf16, kind 1: v_mfma_i32_32x32x32_i8.  The hot
 * kernels of this library hold 256 accumulator registers per lane and so run one workgroup per compute unit.
 * kind 2 (bf16) and kind 3 (int8): the same instructions with the operand traffic of a 256 x 256 tile with
 * 64-byte K steps around them and nothing else (32 KB of LDS-direct loads per step and workgroup from a 32 MiB
 * operand image that the call writes, 16 fragment reads per wavefront, one barrier); workgroups_per_cu must
 * be 1.  Needs 256 KiB of workspace per workgroup_per_cu, kinds 2 and 3 another 32 MiB; synchronises the
 * stream.  Errors: ASER_ERR_INVALID_ARG (kind, null), ASER_ERR_SHAPE, ASER_ERR_WORKSPACE. */
int aser_mfma_rate_probe(aser_ctx* ctx, int32_t kind, int32_t workgroups_per_cu, int32_t iters, double* tops);

#ifdef __cplusplus
}
#endif
#endif /* ASER_H */
