// Error reconstruction via whitening SVD (Sec. 4.1, Eq. 6): rank-r truncated SVD of A = T S by
// blocked subspace iteration with Rayleigh-Ritz, and the LoRA-style factors
//     L_A = U_r Sigma_r,   L_B = V_r^T S^-1 = Sigma_r^-1 U_r^T T.
//
// Every large product is arranged in the K-major "A^T B" form of the MFMA kernel:
//     A   = (T^T)^T S            A^T from a transpose pass
//     Z   = A^T Q   (n x b)      K = m, operands A and Q
//     A Zt          (m x b)      K = n, operands A^T and Zt = A^T Q = Z R_z (Z itself is never formed)
//     Z^T Z, Q^T Q  (b x b)      Gram matrices of the Cholesky-QR orthogonalisation
//     C^T = T^T Q   (n x b)      for L_B
// The b x b work (Cholesky, inverse, symmetric eigen-solver) runs in one workgroup in LDS.
//
// The subspace iteration carries a momentum term (the heavy-ball acceleration of the power method,
// in block form): with X_k = Q_k C_k the un-normalised iterates, X_{k+1} = (A A^T) X_k - beta X_{k-1}.
// In terms of the orthonormal blocks, with any invertible R~ that makes Zt R~^-1 well conditioned and the
// Cholesky-QR step Y = Q_{k+1} R_q:
//     Y = (A Zt + beta' Q_{k-1} P_k) R~^-1,   Zt = A^T Q_k,   P_{k+1} = R~^-1 R_q^-1,   beta' = -beta,
// formed by one kernel from the two tall blocks and the two b x b factors (it also clears the two
// accumulation targets it has read); Z = Zt R~^-1 itself is never formed.  R~ is the Cholesky factor of
// Zt^T Zt (a second Cholesky-QR) in the first iterations, while the subspace still turns, and then only in
// every other iteration: between two refreshes the factor of the previous iteration serves (the iterate is
// the same in exact arithmetic, R~ only keeps the columns of A Zt R~^-1 from collapsing onto the leading
// directions, and Zt of consecutive iterations differ by the convergence error).  beta = (0.9 s^2 / 2)^2
// with s the smallest diagonal entry of R~: s^2 stays below the b-th eigenvalue of A A^T, which
// keeps every wanted direction (eigenvalue above 2 sqrt(beta)) in the amplified regime.  On the
// bulk of a quantisation-error spectrum this reaches in 10 iterations what the plain iteration
// needs about 16 for; the excess over the optimal whitened error halves with every iteration.
#include <limits.h>
#include <math.h>

#include "aser_internal.h"

namespace {

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// Leading columns of the start block: Q[i][c] = T[i][cols[c]] for c < k (row-major m x b block).
__global__ void lead_columns_kernel(const float* __restrict__ T, int64_t m, int64_t ldt, const int32_t* __restrict__ cols,
                                    int k, int64_t n, float* __restrict__ Q, int b) {
    const int64_t total = m * k;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = t / k;
        const int c = (int)(t % k);
        const int64_t col = cols[c];
        if (col >= 0 && col < n) Q[i * b + c] = T[i * ldt + col];
    }
}

// Start block: uniform values in [-1, 1) from a counter-based hash of (seed, index).
// Also resets the two status words of the solver (thread 0).
__global__ void random_block_kernel(float* Q, int64_t total, uint32_t seed, double* res2, int32_t* qr) {
    if (blockIdx.x == 0 && threadIdx.x == 0) { *res2 = 0.0; *qr = 0; }
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t h = mix32((uint32_t)i * 0x9E3779B9U + mix32(seed + (uint32_t)(i >> 32)));
        Q[i] = (float)(h >> 8) * (1.0f / 8388608.0f) - 1.0f;
    }
}

// From the Ritz pairs (lambda descending, Uhat b x b): sigma_i = sqrt(lambda_i),
// WA (b x r) = Uhat[:, :r] diag(sigma), WBt (b x r) = Uhat[:, :r] diag(1 / sigma).
__global__ void ritz_factors_kernel(const float* lambda, const float* Uhat, int b, int r, float* sigma, float* WA, float* WBt) {
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < b * r; t += gridDim.x * blockDim.x) {
        const int k = t / r, i = t % r;
        const float lam = lambda[i];
        const float sg = lam > 0.f ? sqrtf(lam) : 0.f;
        const float u = Uhat[k * b + i];
        WA[t] = u * sg;
        WBt[t] = sg > 0.f ? u / sg : 0.f;
        if (k == 0) sigma[i] = sg;
    }
}

struct Plan {
    int b, iters;
    uint32_t seed;
    size_t off_big0, off_big1, off_big2, off_tall, tall_bytes, off_small, total;
};

int default_block(int r) {
    int b = 2 * r;
    if (b > 128) b = 128;
    if (b < r) b = r;
    b = (b + 31) / 32 * 32;
    return b;
}

int make_plan(int64_t m, int64_t n, int r, const aser_svd_opts* o, Plan* p) {
    p->b = (o && o->block > 0) ? o->block : default_block(r);
    // default: 9 iterations, 12 for wide layers (the bulk of the spectrum gets denser with the size),
    // 30 when the block has fewer than r oversampling columns (r > 64: the wanted directions at the
    // edge of the bulk then converge at the rate of the gap to the next singular value alone)
    p->iters = (o && o->max_iter > 0) ? o->max_iter
             : (p->b < 2 * r ? 30 : (((m > n ? m : n) > 8192) ? 12 : 9));
    p->seed = (o && o->seed) ? o->seed : 1u;
    const int64_t mx = m > n ? m : n;
    size_t off = 0;
    p->off_big0 = off; off += align_up((size_t)m * n * 4, 256);        // T^T
    p->off_big1 = off; off += align_up((size_t)m * n * 4, 256);        // A
    p->off_big2 = off; off += align_up((size_t)m * n * 4, 256);        // A^T
    // five tall blocks (three on the Q side, two on the Z side) that change roles by pointer swap
    p->tall_bytes = align_up((size_t)mx * p->b * 4, 256);
    p->off_tall = off; off += 5 * p->tall_bytes;
    p->off_small = off; off += align_up((size_t)p->b * p->b * 4, 256) * 6 + 8192 + align_up((size_t)p->b * 128 * 4, 256) * 3;
    p->total = off;
    return ASER_OK;
}

}  // namespace

size_t aser_reconstruct_workspace(int64_t m, int64_t n, int r, const aser_svd_opts* o) {
    Plan p;
    make_plan(m, n, r, o, &p);
    size_t need = p.total;
    if (r > kAserMaxIterRank) return aser_exact_workspace(m, n, r) + 256;   // only the dense solver takes such a rank
    if (m * n <= ((int64_t)1 << 20)) {                     // small layers may take the dense solver
        const size_t ex = aser_exact_workspace(m, n, r) + 256;
        if (ex > need) need = ex;
    }
    return need;
}

namespace {

// Arguments of C += A^T B with K split over workgroups (fp32 atomics).
GemmArgs atomic_args(int share, int form, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                     int64_t M, int64_t N, int64_t K, int bm, int bn, bool upper_only = false) {
    GemmArgs g{};
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.Ct = nullptr; g.ldct = 0;
    g.M = M; g.N = N; g.K = K; g.alpha = 1.f;
    g.in_type = form; g.epi = GEMM_EPI_ATOMIC; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_FULL;
    g.bm = bm; g.bn = bn; g.upper_only = upper_only ? 1 : 0;
    // Split K by the cost model of aser_split_k_parts.  Every part pays a pipeline fill and an atomic
    // flush of its whole tile, so parts keep at least 8 K steps (4 when the output is tiny and the
    // call is pure latency).
    const int64_t tiles = ceil_div64(M, bm) * ceil_div64(N, bn);
    const int64_t ksteps = ceil_div64(K, 32);
    g.k_parts = aser_split_k_parts(tiles, ksteps, tiles <= 4 ? 4 : 8, (double)(bm * bn) / (128.0 * 128.0), share);
    return g;
}

// C += A^T B with K split over workgroups (fp32 atomics); `clear` zeroes C first.
int gemm_tn_atomic(aser_ctx* ctx, int form, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                   int64_t M, int64_t N, int64_t K, int bm, int bn, bool clear, bool upper_only = false) {
    if (clear) ASER_TRY(aser_fill_f32(ctx, C, M, N, ldc, 0.f));
    return aser_gemm_tn(ctx, atomic_args(ctx->share, form, A, lda, B, ldb, C, ldc, M, N, K, bm, bn, upper_only));
}

// The factorisation kernel reports a non-positive pivot with atomicMin(info, base + column + 1); the
// flag of this file starts at zero, so a negative base makes any failed pivot show as a negative flag.
constexpr int32_t kPivotBase = -1000;

// out (rows x b) = Y R^-1 with R^T R = Y^T Y (Cholesky-QR); R^-1 is left in Rinv.  Mb must be zero on
// entry and is zero again on return.  The first clear_rows rows of Y are cleared after they have
// been read (0: Y is left alone).  Lmul / Cmul: the factorisation kernel also leaves Cmul = Lmul R^-1
// (see aser_chol_block); both null: nothing.
int chol_qr(aser_ctx* ctx, int form, float* Y, float* out, int64_t rows, int64_t clear_rows, int b, float* Mb, float* Rinv,
            int32_t* info, const float* Lmul = nullptr, float* Cmul = nullptr) {
    ASER_TRY(gemm_tn_atomic(ctx, form, Y, b, Y, b, Mb, b, b, b, rows, 128, 128, false, /*upper_only=*/true));
    ASER_TRY(aser_chol_block(ctx, Mb, b, b, Rinv, info, kPivotBase, /*clear_d=*/true, Lmul, Cmul));
    return aser_gemm_small_f32(ctx, Y, b, Rinv, b, out, b, rows, b, b, clear_rows);
}

// The plan with the block width made legal for the shape: ASER_OK, or ASER_ERR_SHAPE with a text in *why.
int legal_plan(int64_t m, int64_t n, int r, const aser_svd_opts* opts, Plan* p, const char** why) {
    if (m <= 0 || n <= 0) { *why = "bad shape"; return ASER_ERR_SHAPE; }
    if (r <= 0 || r > m || r > n || r > 128) { *why = "need 0 < r <= min(m, n, 128)"; return ASER_ERR_SHAPE; }
    make_plan(m, n, r, opts, p);
    if (p->b < r || p->b > 128 || (p->b % 32) != 0 || p->b > m || p->b > n) {
        // a block wider than the matrix makes no sense; shrink to the largest legal width
        int b = p->b;
        if (opts && opts->block > 0) { *why = "block must be a multiple of 32 in [r, min(128, m, n)]"; return ASER_ERR_SHAPE; }
        const int64_t lim = (m < n ? m : n);
        while (b > lim) b -= 32;
        if (b < r) { *why = "no legal block width for this r and shape"; return ASER_ERR_SHAPE; }
        aser_svd_opts o2 = opts ? *opts : aser_svd_opts{0, 0, 0};
        o2.block = b;
        make_plan(m, n, r, &o2, p);
    }
    return ASER_OK;
}

}  // namespace

extern "C" int aser_svd_plan(int64_t m, int64_t n, int32_t r, const aser_svd_opts* opts, int32_t* block, int32_t* iters) {
    if (r > kAserMaxIterRank) {                            // the dense solver: no block, no iterations
        if (m <= 0 || n <= 0 || r > m || r > n || r > kAserMaxRank || (m < n ? m : n) > kAserMaxDenseSide) return ASER_ERR_SHAPE;
        if (block) *block = 0;
        if (iters) *iters = 0;
        return ASER_OK;
    }
    Plan p;
    const char* why = "";
    const int st = legal_plan(m, n, r, opts, &p, &why);
    if (st != ASER_OK) return st;
    if (block) *block = p.b;
    if (iters) *iters = p.iters;
    return ASER_OK;
}

extern "C" int aser_error_reconstruct_enqueue(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt,
                                              const float* S, int64_t lds, int32_t r, const int32_t* idx, int32_t f,
                                              const aser_svd_opts* opts, float* L_A, float* L_B, float* sigma) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (ctx->rec_pending) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "error_reconstruct_enqueue: the previous one has not been finished (aser_finish)");
    if (!T || !S || !L_A || !L_B || !sigma) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "error_reconstruct: null pointer");
    if (m <= 0 || n <= 0 || ldt < n || lds < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: bad shape");
    if (f < 0 || f > n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: f must be in [0, n]");
    if (f > 0 && !idx) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "error_reconstruct: idx is null with f > 0");
    const bool exact = aser_use_exact_solver(ctx->precision, m, n, r, opts);
    Plan p;
    if (exact) {                                         // the dense solver has no subspace block: any r up to min(m, n, 256)
        if (r <= 0 || r > m || r > n || r > kAserMaxRank)
            ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: need 0 < r <= min(m, n, %d)", kAserMaxRank);
        if (r > kAserMaxIterRank && (m < n ? m : n) > kAserMaxDenseSide)
            ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: r > %d takes the dense solver, which needs min(m, n) <= %lld",
                      kAserMaxIterRank, (long long)kAserMaxDenseSide);
        make_plan(m, n, r <= kAserMaxIterRank ? r : kAserMaxIterRank, opts, &p);
    } else {
        const char* why = "";
        const int st = legal_plan(m, n, r, opts, &p, &why);
        if (st != ASER_OK) ASER_FAIL(ctx, st, "error_reconstruct: %s", why);
    }
    if (((uintptr_t)T & 3) || ((uintptr_t)S & 3)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "error_reconstruct: misaligned pointer");
    if (!ctx->ws || (!exact && ctx->ws_bytes < p.total + kAserWsTail))
        ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "error_reconstruct: workspace too small (%zu needed)", p.total + kAserWsTail);
    ASER_TRY(aser_prepare_device(ctx));

    char* ws = (char*)ctx->ws;
    if (exact) {
        // Small layers: the dense fp64 solver (every eigenvalue of the Gram matrix of T S, eigenvectors of the
        // r largest).  Small layers are where a residual can be a few 1e-4 of ||T S||_F (int8 weights, a rank
        // near half the width): fp32 iterations resolve that to two digits at best, and what they return then
        // depends on the iteration count.  The work is microseconds to a few milliseconds at these sizes.
        const size_t ex = aser_exact_workspace(m, n, r);
        if (ctx->ws_bytes < ex + 256 + kAserWsTail)
            ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "error_reconstruct: workspace too small (%zu needed)", ex + 256 + kAserWsTail);
        ASER_TRY(aser_exact_reconstruct(ctx, T, m, n, ldt, S, lds, r, L_A, L_B, sigma, &aser_status_dev(ctx)->res2));
        ctx->rec_pending = true;
        ctx->rec_exact = true;
        ctx->rec_iters = 0;
        return aser_enqueue_status_copy(ctx);
    }
    const int b = p.b;
    const int form = aser_f32_form(ctx, m * n);          // three or six bf16 products per fp32 product
    float* big0 = (float*)(ws + p.off_big0);     // T^T (n x m)
    float* A = (float*)(ws + p.off_big1);        // m x n
    float* At = (float*)(ws + p.off_big2);       // A^T (n x m), written by the same product as A
    float* tall[5];
    for (int i = 0; i < 5; ++i) tall[i] = (float*)(ws + p.off_tall + i * p.tall_bytes);   // max(m, n) x b each
    char* sm = ws + p.off_small;
    const size_t bb = align_up((size_t)b * b * 4, 256);
    float* Mb = (float*)sm;
    float* Rz_inv = (float*)(sm + bb);
    float* Uhat = (float*)(sm + 2 * bb);
    float* Rq_inv = (float*)(sm + 3 * bb);
    float* Pm = (float*)(sm + 4 * bb);
    float* beta_dev = (float*)(sm + 5 * bb);               // the momentum coefficient beta' (one float) and, behind it,
    const int* gate_dev = (const int*)(beta_dev + 1);      // whether the next iteration has to renew R~ (see iterate)
    sm += 3 * bb;                                          // the scalars and the r-wide blocks follow the six matrices
    float* lambda = (float*)(sm + 3 * bb);                 // b floats
    double* normA2 = &aser_status_dev(ctx)->res2;          // both in the status block that the one copy at the end brings to the host
    int32_t* info = &aser_status_dev(ctx)->qr;
    int32_t* cluster = (int32_t*)(sm + 3 * bb + 3072);
    float* tri = (float*)(sm + 3 * bb + 4096);             // 384 floats
    const size_t b128 = align_up((size_t)b * 128 * 4, 256);
    float* WA = (float*)(sm + 3 * bb + 8192);
    float* WBt = (float*)(sm + 3 * bb + 8192 + b128);
    float* refl = (float*)(sm + 3 * bb + 8192 + 2 * b128);

    // A = T S through T^T (K-major operand); the product's epilogue also writes A^T
    ASER_TRY(aser_transpose_f32(ctx, T, m, n, ldt, big0, m));
    {
        GemmArgs g{};
        g.A = big0; g.lda = m; g.B = S; g.ldb = lds; g.C = A; g.ldc = n; g.Ct = At; g.ldct = m;
        g.M = m; g.N = n; g.K = n; g.alpha = 1.f;
        g.in_type = form; g.epi = GEMM_EPI_STORE; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_GE_COL;
        g.k_parts = 1;
        // S is lower triangular, so the K range of a tile shrinks with its column: pairing column j with
        // column tn - 1 - j gives every workgroup the same work
        g.pair_cols = (m > 1024 && n > 1024) ? 1 : 0;
        g.bm = g.pair_cols ? 256 : 128; g.bn = 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
    }
    // two clearing passes for everything that must start at zero: the scalars (lambda .. cluster share
    // 4 KB) and, contiguous in the workspace, the two accumulation targets and Mb
    ASER_TRY(aser_fill_bytes(ctx, lambda, 4096));
    ASER_TRY(aser_fill_bytes(ctx, tall[3], 2 * p.tall_bytes + bb));

    // start block and subspace iteration with momentum
    float *Qcur = tall[0], *Qold = tall[1], *Qacc = tall[2];   // Q_k, Q_{k-1} (or spare), accumulation target
    float *Zt = tall[3], *Qraw = tall[4];                      // accumulation targets of A^T Q and A Zt (kept zero)
    {
        const int64_t total = m * (int64_t)b;
        const int blocks = (int)(ceil_div64(total, 256) < 2048 ? ceil_div64(total, 256) : 2048);
        hipLaunchKernelGGL(random_block_kernel, dim3(blocks), dim3(256), 0, ctx->stream, Qacc, total, p.seed, normA2, info);
        ASER_TRY(aser_check_launch(ctx, "random_block"));
        if (f > 0) {
            // graded start: the unquantized outlier columns of T first (their span holds the largest left
            // singular directions of T S), the random columns behind them
            const int k = f < b ? f : b;
            const int64_t tot = m * (int64_t)k;
            const int blk = (int)(ceil_div64(tot, 256) < 1024 ? ceil_div64(tot, 256) : 1024);
            hipLaunchKernelGGL(lead_columns_kernel, dim3(blk), dim3(256), 0, ctx->stream, T, m, ldt, idx, k, n, Qacc, b);
            ASER_TRY(aser_check_launch(ctx, "lead_columns"));
        }
    }
    ASER_TRY(chol_qr(ctx, form, Qacc, Qcur, m, 0, b, Mb, Rq_inv, info));                 // Q_0
    const int bmA = 128, bnB = 128;
    int done = 0;                                        // subspace iterations so far
    auto iterate = [&](int count) -> int {
        for (int c = 0; c < count; ++c, ++done) {
            const bool it = done > 0;                    // momentum term present from the second iteration on
            // R~ from this iteration's Zt; in the odd iterations from the fourth on only if the last factor's
            // diagonal spans more than a factor of 64 (the factorisation kernel left that decision in gate_dev:
            // with a wide spread the columns of Zt R~^-1 for a stale R~ drift apart faster than the next
            // Cholesky-QR tolerates), otherwise the previous iteration's factor serves and both kernels return at once
            const int* gate = (done < 3 || (done & 1) == 0) ? nullptr : gate_dev;
            ASER_TRY(gemm_tn_atomic(ctx, form, A, n, Qcur, b, Zt, b, n, b, m, bmA, bnB, false));    // Zt = A^T Q_k
            {
                GemmArgs gz = atomic_args(ctx->share, form, Zt, b, Zt, b, Mb, b, b, b, n, 128, 128, /*upper_only=*/true);
                gz.gate = gate;
                ASER_TRY(aser_gemm_tn(ctx, gz));
                ASER_TRY(aser_chol_block(ctx, Mb, b, b, Rz_inv, info, kPivotBase, /*clear_d=*/true, nullptr, nullptr, beta_dev, gate));
            }
            ASER_TRY(gemm_tn_atomic(ctx, form, At, m, Zt, b, Qraw, b, m, b, n, bmA, bnB, false));   // A Zt
            // (A Zt + beta' Q_{k-1} P_k) R~^-1; Qraw and Zt are zero again afterwards
            ASER_TRY(aser_combine_f32(ctx, Qraw, Rz_inv, it ? Qold : nullptr, Pm, beta_dev, Qacc, m, b, Zt, n));
            // = Q_{k+1} R_q, into the old block; also P_{k+1} = R~^-1 R_q^-1
            ASER_TRY(chol_qr(ctx, form, Qacc, Qold, m, 0, b, Mb, Rq_inv, info, Rz_inv, Pm));
            { float* t = Qold; Qold = Qcur; Qcur = t; }
        }
        return ASER_OK;
    };
    // Rayleigh-Ritz on the current block, the factors, and the residual; leaves Zt, Qraw and Mb in use
    auto finish = [&]() -> int {
        ASER_TRY(chol_qr(ctx, form, Qcur, Qacc, m, 0, b, Mb, Rq_inv, info));                 // second pass: orthonormal to fp32
        float* Qp = Qacc;
        // Rayleigh-Ritz: Z = A^T Q, eigen-pairs of Z^T Z = Q^T A A^T Q
        ASER_TRY(gemm_tn_atomic(ctx, form, A, n, Qp, b, Zt, b, n, b, m, bmA, bnB, false));
        float* Zp = Zt;
        float* tp = Qraw;
        ASER_TRY(gemm_tn_atomic(ctx, form, Zp, b, Zp, b, Mb, b, b, b, n, 128, 128, false));
        ASER_TRY(aser_tridiag_eig(ctx, Mb, b, lambda, Uhat, refl, tri, cluster));
        ASER_TRY(aser_jacobi_eig(ctx, Mb, b, lambda, Uhat, cluster));      // only runs if eigenvalues cluster
        hipLaunchKernelGGL(ritz_factors_kernel, dim3(16), dim3(256), 0, ctx->stream, (const float*)lambda, (const float*)Uhat, b,
                           (int)r, sigma, WA, WBt);
        ASER_TRY(aser_check_launch(ctx, "ritz_factors"));
        // Whitened error of Eq. 8 as an explicit residual: ||A - U_r (U_r^T A)||_F, formed tile by tile in
        // the product's epilogue (A is read once and nothing is written).
        // U_r^T A = (Z Uhat_r)^T with Z = A^T Q; the subtraction form avoids the cancellation of
        // ||A||^2 - sum sigma_i^2 when the top singular values carry almost all of the norm.
        ASER_TRY(aser_gemm_small_f32(ctx, Zp, b, Uhat, b, L_B, n, n, b, r, 0, true));  // (V_r Sigma_r)^T (r x n), parked in L_B
        ASER_TRY(aser_gemm_small_f32(ctx, Qp, b, Uhat, b, tp, m, m, b, r, 0, true));   // U_r^T (r x m)
        {
            GemmArgs g{};
            g.A = tp; g.lda = m; g.B = L_B; g.ldb = n; g.C = A; g.ldc = n; g.Ct = nullptr; g.ldct = 0;
            g.M = m; g.N = n; g.K = r; g.alpha = -1.f; g.sumsq = normA2;
            g.in_type = form; g.epi = GEMM_EPI_RESID; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_FULL;
            g.k_parts = 1;
            g.bm = 128; g.bn = 128;                           // short K: many small workgroups hide the latency of reading A
            ASER_TRY(aser_gemm_tn(ctx, g));
        }
        // L_A = Q (Uhat_r Sigma_r)
        ASER_TRY(aser_gemm_small_f32(ctx, Qp, b, WA, r, L_A, r, m, b, r));
        // L_B^T = (T^T Q) (Uhat_r Sigma_r^-1)  ->  L_B
        ASER_TRY(gemm_tn_atomic(ctx, form, T, ldt, Qp, b, Zp, b, n, b, m, bmA, bnB, true));  // C^T = T^T Q (n x b)
        return aser_gemm_small_f32(ctx, Zp, b, WBt, r, L_B, n, n, b, r, 0, true);            // (n x r)^T = L_B
    };
    ASER_TRY(iterate(p.iters));
    ASER_TRY(finish());
    // Nothing above waits for the device.  The squared residual, the pivot flag of the orthogonalisation and
    // whatever earlier calls left pending travel to the host in one copy, which aser_finish waits for.
    ctx->rec_pending = true;
    ctx->rec_exact = false;
    ctx->rec_iters = done;
    return aser_enqueue_status_copy(ctx);
}

extern "C" int aser_finish(aser_ctx* ctx, double* err, int32_t* n_iter) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!ctx->rec_pending) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "finish: no aser_error_reconstruct_enqueue is pending on this context");
    ctx->rec_pending = false;
    AserPending pend;                                        // with the status words of calls that did not synchronise
    ASER_TRY(aser_wait_status(ctx, &pend));
    ASER_TRY(aser_report_pending(ctx, pend, "error_reconstruct"));
    const double h_res2 = pend.res2;
    if (ctx->rec_exact) {
        if (!(h_res2 >= 0.0) || h_res2 > 1e300)
            ASER_FAIL(ctx, ASER_ERR_NO_CONVERGE, "error_reconstruct: non-finite values in T or S");
    } else if (pend.qr < 0 || !(h_res2 >= 0.0) || h_res2 > 1e300) {
        ASER_FAIL(ctx, ASER_ERR_NO_CONVERGE,
                  "error_reconstruct: the Cholesky-QR orthogonalisation broke down (pivot %d of a block Gram matrix is not "
                  "positive): the singular values of the subspace span more than the products resolve",
                  pend.qr < 0 ? pend.qr - kPivotBase : 0);
    }
    if (err) *err = sqrt(h_res2 > 0.0 ? h_res2 : 0.0);
    if (n_iter) *n_iter = ctx->rec_iters;
    return ASER_OK;
}

extern "C" int aser_error_reconstruct(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt,
                                      const float* S, int64_t lds, int32_t r, const int32_t* idx, int32_t f,
                                      const aser_svd_opts* opts,
                                      float* L_A, float* L_B, float* sigma, double* err, int32_t* n_iter) {
    ASER_TRY(aser_error_reconstruct_enqueue(ctx, T, m, n, ldt, S, lds, r, idx, f, opts, L_A, L_B, sigma));
    return aser_finish(ctx, err, n_iter);
}
