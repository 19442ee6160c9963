// Internal declarations shared by the translation units of libaser.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdio.h>
#include <string.h>

#include "aser.h"

struct aser_ctx {
    int device;
    hipStream_t stream;
    void* ws;
    size_t ws_bytes;
    bool device_ready;
    int precision;       // aser_precision: how fp32 operands enter the MFMA products
    // aser_whiten without a host `info` leaves its pivot flag on the device (last 256 bytes of the
    // workspace) and does not synchronise; the next synchronising call reads it.
    int32_t* pending_info_dev;
    // aser_smooth_outliers never synchronises; when fewer than f channels have a usable score its
    // selection kernel raises the word behind the pivot flag, which the next synchronising call reads.
    int32_t* pending_sel_dev;
    // 64 bytes of pinned host memory (allocated with the first compute call): every synchronising call brings
    // the status block at the head of the workspace tail to the host in one copy.
    void* host_status;
    // aser_error_reconstruct_enqueue has left its status copy in flight; aser_finish waits for it
    bool rec_pending;
    bool rec_exact;      // the dense solver ran (no orthogonalisation flag to look at)
    int32_t rec_iters;
    int share;           // layers in flight on the device next to this context's (1: alone); see aser_split_k_parts
    char err[256];
};

// Bytes at the end of the bound workspace.  The first 32 are the status block that a synchronising call copies
// to the host in one piece: the whitening's pivot flag (word 0), the outlier selection's "no usable candidate"
// flag (word 1), the pivot flag of the Cholesky-QR steps of aser_error_reconstruct (word 2) and, at byte 16,
// the squared whitened error as a double.  Bytes 64 .. 135 carry the scalar results of aser_select_rank and
// aser_effective_rank.
static const size_t kAserWsTail = 256;
struct AserStatusBlock {
    int32_t pivot, sel, qr, pad;
    double res2;
    double spare;
};
static inline AserStatusBlock* aser_status_dev(const aser_ctx* ctx) {
    return (AserStatusBlock*)((char*)ctx->ws + ctx->ws_bytes - kAserWsTail);
}

// Host copies of the deferred status words; INT_MAX / 0 mean "nothing pending or nothing wrong".
struct AserPending {
    int32_t pivot;
    int32_t sel;
    int32_t qr;        // word 2 as it is
    double res2;       // the double at byte 16 as it is
};
// Enqueues the one copy of the status block, waits for the stream, and fills *p (words nobody has pending read
// as "nothing wrong"); aser_report_pending then clears the pending state and turns a raised word into a status.
int aser_sync_status(aser_ctx* ctx, AserPending* p);
// The two halves of aser_sync_status: the copy alone (asynchronous), and the wait with the read-out.
int aser_enqueue_status_copy(aser_ctx* ctx);
int aser_wait_status(aser_ctx* ctx, AserPending* p);
int aser_report_pending(aser_ctx* ctx, const AserPending& p, const char* who);
int aser_set_i32(aser_ctx* ctx, int32_t* p, int32_t v);

#define ASER_FAIL(ctx, code, ...)                                   \
    do {                                                            \
        if (ctx) snprintf((ctx)->err, sizeof((ctx)->err), __VA_ARGS__); \
        return (code);                                              \
    } while (0)

#define ASER_HIP(ctx, call)                                                              \
    do {                                                                                 \
        hipError_t e__ = (call);                                                         \
        if (e__ != hipSuccess) ASER_FAIL(ctx, ASER_ERR_HIP, "%s: %s", #call, hipGetErrorString(e__)); \
    } while (0)

#define ASER_TRY(expr)                   \
    do {                                 \
        int s__ = (expr);                \
        if (s__ != ASER_OK) return s__;  \
    } while (0)

static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

size_t aser_reconstruct_workspace(int64_t m, int64_t n, int r, const aser_svd_opts* o);

// Dense fp64 solver of the truncated SVD for small layers (spectrum.hip); see aser_error_reconstruct.
size_t aser_exact_workspace(int64_t m, int64_t n, int r);
int aser_exact_reconstruct(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt, const float* S, int64_t lds,
                           int r, float* L_A, float* L_B, float* sigma, double* err2_dev);
// True when aser_error_reconstruct takes the dense solver: a small layer with default options outside the fast
// mode, or a rank beyond the widest subspace block of the iteration (kAserMaxIterRank), whatever the options.
static const int kAserMaxIterRank = 128;
static const int kAserMaxRank = 256;          // one thread per wanted eigenvector in the dense solver's inverse iteration
static const int64_t kAserMaxDenseSide = 16384;
static inline bool aser_use_exact_solver(int precision, int64_t m, int64_t n, int r, const aser_svd_opts* o) {
    if (r > kAserMaxIterRank) return true;
    return precision != ASER_PRECISION_FAST && m * n <= ((int64_t)1 << 20) && !(o && (o->max_iter > 0 || o->block > 0));
}

// Makes ctx's device current (first compute call) and checks a launch.
int aser_prepare_device(aser_ctx* ctx);
int aser_check_launch(aser_ctx* ctx, const char* what);

// ---------------------------------------------------------------------------------------------
// C (op)= alpha * A^T B with both operands stored K-major ("TN" form):
//   A: K x M row-major (lda), B: K x N row-major (ldb), C: M x N row-major (ldc), all device.
// Input types: bf16 (one exact MFMA product, fp32 accumulate) or fp32 split on the fly into
// bf16 hi + lo (three MFMA products: hi*hi + hi*lo + lo*hi).
// GEMM_IN_F32X6: fp32 split into three bf16 terms, the six products down to 2^-24 (fp32-exact class);
// tiles up to 256 x 128.
enum GemmIn { GEMM_IN_BF16 = 0, GEMM_IN_F32X3 = 1, GEMM_IN_F32X6 = 2 };

// Input form of an fp32 contraction of a problem whose operands have at most `entries` entries: the
// three-product split (2^-16 per product) or the six-product one (2^-24).  In the automatic mode small
// problems take the exact form: it costs microseconds there, and small layers are where a residual can be
// a few 1e-5 of the matrix norm (int8 weights, a rank near half the width), which 2^-16 does not resolve.
static inline int aser_f32_form(const aser_ctx* ctx, int64_t entries) {
    if (ctx->precision == ASER_PRECISION_EXACT) return GEMM_IN_F32X6;
    if (ctx->precision == ASER_PRECISION_FAST) return GEMM_IN_F32X3;
    return entries <= ((int64_t)1 << 20) ? GEMM_IN_F32X6 : GEMM_IN_F32X3;
}
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

enum GemmEpi {
    GEMM_EPI_STORE = 0,    // C = alpha * acc            (needs k_parts == 1)
    GEMM_EPI_ATOMIC = 1,   // atomicAdd(C, alpha * acc)  (any k_parts)
    GEMM_EPI_RMW = 2,      // C += alpha * acc           (needs k_parts == 1, disjoint tiles)
    GEMM_EPI_RESID = 3     // *sumsq += ||C + alpha * acc||_F^2, C only read (needs k_parts == 1)
};
enum GemmTiles {
    GEMM_TILES_ALL = 0,    // every BM x BN tile of C
    GEMM_TILES_LOWER = 1,  // tiles meeting the lower triangle (needs M == N, BM == BN)
    GEMM_TILES_UPPER = 2   // tiles meeting the upper triangle
};
enum GemmKRange {
    GEMM_K_FULL = 0,
    GEMM_K_GE_COL = 1      // B[k][j] == 0 for k < j (B lower triangular): start at k = tile's first column
};

struct GemmArgs {
    const void* A; int64_t lda;
    const void* B; int64_t ldb;
    float* C; int64_t ldc;
    float* Ct; int64_t ldct;   // optional transposed copy of the result: Ct[j][i] = C[i][j] (STORE only)
    int64_t M, N, K;
    float alpha;
    int in_type, epi, tiles, krange;
    int k_parts;               // split of the K range over blockIdx.y
    int bm, bn;                // tile: 256x256, 128x256, 256x128 or 128x128
    int upper_only;            // ATOMIC only: skip entries with row > col (C is symmetric, its upper part is used)
    int pair_cols;             // TILES_ALL, k_parts == 1, 256 x 128 tiles: a workgroup takes tile columns j and tn - 1 - j of its tile row
                               // (equal work per workgroup when K shrinks linearly with the column, K_GE_COL)
    double* sumsq;             // RESID only: device scalar that receives the sum of squares (accumulates)
    const int* gate;           // plain schedules only (may be null): every workgroup returns at once when *gate == 0
};
int aser_gemm_tn(aser_ctx* ctx, const GemmArgs& g);

// Number of K parts for a split-K update with atomic accumulation, from a cost model fitted to kernel
// traces (microseconds; u = tile area in units of 128 x 128): one workgroup per CU, so the workgroups run
// in ceil(tiles * parts / 256) rounds; a round costs 4 us of prologue and flush plus 0.75 u per 32-deep K
// step; every workgroup adds 0.06 u of atomic traffic that the others wait behind.  More parts shorten
// the K loop but multiply the atomics, and one workgroup more than 256 doubles the rounds.
// A part keeps at least min_steps K steps.
// share > 1: that many layers are in flight on the device (aser_calibrate_layers).  What a launch costs the
// other layers is the compute-unit time it holds, workgroups x their duration / 256, and every other layer
// pays it; the cost then is the launch's own duration plus (share - 1) times that.
static inline int aser_split_k_parts(int64_t tiles, int64_t ksteps, int64_t min_steps, double u, int share = 1) {
    const int64_t max_parts = ksteps / min_steps > 0 ? ksteps / min_steps : 1;
    int best = 1;
    double best_cost = 0.0;
    for (int64_t p = 1; p <= max_parts && p <= 64; ++p) {
        const int64_t wgs = tiles * p, rounds = ceil_div64(wgs, 256), steps = ceil_div64(ksteps, p);
        const double per_wg = 0.75 * u * (double)steps + 4.0;
        double cost = (double)rounds * per_wg + 0.06 * u * (double)wgs;
        if (share > 1) cost += (double)(share - 1) * (double)wgs * per_wg / 256.0;
        if (p == 1 || cost < best_cost) { best_cost = cost; best = (int)p; }
    }
    return best;
}

// Gram update G(lower) += X^T X with the XCD-aware persistent schedule (bf16 or fp32 X).
int aser_syrk_gram(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                   float* G, int64_t ldg);

// ---------------------------------------------------------------------------------------------
// Bandwidth-bound kernels
int aser_fill_f32(aser_ctx* ctx, float* p, int64_t rows, int64_t cols, int64_t ld, float v);
int aser_fill_bytes(aser_ctx* ctx, void* p, size_t bytes);   // zero fill
int aser_col_abs_sum_x(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                       double* abs_sum, int64_t* count);
int aser_col_abs_sum_w(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw, double* wsum);
int aser_transpose_f32(aser_ctx* ctx, const float* A, int64_t rows, int64_t cols, int64_t lda, float* At, int64_t ldat);

// Small dense kernels (one workgroup, matrices in LDS)
// Upper Cholesky of the b x b block D (ld) in place: upper part <- R (D = R^T R), the part below the diagonal is neither read nor written;
// Rinv (b x b, ld = b) <- R^-1 (upper).  b <= 128.  On a non-positive pivot at column j,
// atomicMin(info, pivot_base + j + 1) and the factor is meaningless from that column on.  clear_d: D is overwritten with
// zeros instead of the factor (callers that only need R^-1 and reuse D as an accumulation target).
// Lmul / Cmul (both may be null): Cmul = Lmul R^-1 for an upper triangular b x b Lmul (ld = b).
// beta_out (device, two words, may be null): word 0 receives -(0.9 s^2 / 2)^2 as a float, s the smallest diagonal
// entry of R; word 1 receives, as an int, 1 when the largest diagonal entry of R exceeds 64 s and else 0.
// gate (device, may be null): the kernel returns at once when *gate == 0.
int aser_chol_block(aser_ctx* ctx, float* D, int64_t ld, int b, float* Rinv, int32_t* info, int32_t pivot_base,
                    bool clear_d = false, const float* Lmul = nullptr, float* Cmul = nullptr, float* beta_out = nullptr,
                    const int* gate = nullptr);
// Symmetric eigen-decomposition of the b x b matrix Mb (ld = b) by cyclic Jacobi: eigenvalues
// descending into lambda (b), eigenvectors as columns of V (b x b, ld = b).  b <= 128, b even.
// `gate` (device, may be null): the kernel returns at once when *gate == 0.
int aser_jacobi_eig(aser_ctx* ctx, const float* Mb, int b, float* lambda, float* V, const int* gate);
// Same result by tridiagonalisation + multisection + twisted factorisation (much faster).  Scratch: refl
// (b * 128 floats) and tri (384 floats).  *cluster_flag (device) is written: 1 when two eigenvalues are too
// close for that method, else 0; the caller then runs aser_jacobi_eig gated on the flag.  2 <= b <= 128.
int aser_tridiag_eig(aser_ctx* ctx, const float* Mb, int b, float* lambda, float* V, float* refl, float* tri,
                     int* cluster_flag);
// C (rows x c) = A (rows x k) * B (k x c), fp32 MFMA; k, c <= 128, k % 4 == 0, A 16-byte aligned with
// lda % 4 == 0.  C may not alias A.  The first clear_rows rows of A (k columns each; may exceed `rows`) are
// set to zero after they have been read.  transposed: the result is stored as C^T (c x rows, leading dimension ldc).
// C (rows x b) = (A1 + alpha A2 P) B1 (A2 null: C = A1 B1); tall blocks and b x b factors, all with leading
// dimension b <= 128 (b % 4 == 0), 16-byte aligned; alpha is read from device memory.  Afterwards the rows of A1
// and the first zrows rows of Zclr (may be null) are zero.
int aser_combine_f32(aser_ctx* ctx, float* A1, const float* B1, const float* A2, const float* P, const float* alpha_dev,
                     float* C, int64_t rows, int b, float* Zclr, int64_t zrows);
int aser_gemm_small_f32(aser_ctx* ctx, float* A, int64_t lda, const float* B, int64_t ldb,
                        float* C, int64_t ldc, int64_t rows, int k, int c, int64_t clear_rows = 0, bool transposed = false);
