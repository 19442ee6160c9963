// Error reconstruction via whitening SVD (Sec. 4.1, Eq. 6): rank-r truncated SVD of A = T S by
// blocked subspace iteration with Rayleigh-Ritz, and the LoRA-style factors
//     L_A = U_r Sigma_r,   L_B = V_r^T S^-1 = Sigma_r^-1 U_r^T T.
//
// Every large product is arranged in the K-major "A^T B" form of the MFMA kernel:
//     A   = (T^T)^T S            A^T from a transpose pass
//     Z   = A^T Q   (n x b)      K = m, operands A and Q
//     Q   = A Z     (m x b)      K = n, operands A^T and Z
//     Z^T Z, Q^T Q  (b x b)      Gram matrices of the Cholesky-QR orthogonalisation
//     C^T = T^T Q   (n x b)      for L_B
// The b x b work (Cholesky, inverse, symmetric eigen-solver) runs in one workgroup in LDS.
#include <math.h>

#include "aser_internal.h"

namespace {

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// Start block: uniform values in [-1, 1) from a counter-based hash of (seed, index).
__global__ void random_block_kernel(float* Q, int64_t total, uint32_t seed) {
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
    size_t off_big0, off_big1, off_Q, off_Z, off_tmp, off_small, total;
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
    p->iters = (o && o->max_iter > 0) ? o->max_iter : 12;
    p->seed = (o && o->seed) ? o->seed : 1u;
    const int64_t mx = m > n ? m : n;
    size_t off = 0;
    p->off_big0 = off; off += align_up((size_t)m * n * 4, 256);        // T^T, later A^T
    p->off_big1 = off; off += align_up((size_t)m * n * 4, 256);        // A
    // Q, Z and the scratch block change roles by pointer swap, so all three take the larger size
    p->off_Q = off; off += align_up((size_t)mx * p->b * 4, 256);
    p->off_Z = off; off += align_up((size_t)mx * p->b * 4, 256);
    p->off_tmp = off; off += align_up((size_t)mx * p->b * 4, 256);
    p->off_small = off; off += align_up((size_t)p->b * p->b * 4, 256) * 3 + 8192 + align_up((size_t)p->b * 128 * 4, 256) * 3;
    p->total = off;
    return ASER_OK;
}

}  // namespace

size_t aser_reconstruct_workspace(int64_t m, int64_t n, int r, const aser_svd_opts* o) {
    Plan p;
    make_plan(m, n, r, o, &p);
    return p.total;
}

namespace {

// C += A^T B with K split over workgroups (fp32 atomics); `clear` zeroes C first.
int gemm_tn_atomic(aser_ctx* ctx, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                   int64_t M, int64_t N, int64_t K, int bm, int bn, bool clear, bool upper_only = false) {
    if (clear) ASER_TRY(aser_fill_f32(ctx, C, M, N, ldc, 0.f));
    GemmArgs g{};
    g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.Ct = nullptr; g.ldct = 0;
    g.M = M; g.N = N; g.K = K; g.alpha = 1.f;
    g.in_type = GEMM_IN_F32X3; g.epi = GEMM_EPI_ATOMIC; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_FULL;
    g.bm = bm; g.bn = bn; g.upper_only = upper_only ? 1 : 0;
    // Split K so that about 256 workgroups run.  Every part pays a pipeline fill and an atomic
    // flush of its whole tile, so parts keep at least 8 K steps (4 when the output is tiny and the
    // call is pure latency).
    const int64_t tiles = ceil_div64(M, bm) * ceil_div64(N, bn);
    int64_t parts = ceil_div64(256, tiles);
    const int64_t ksteps = ceil_div64(K, 32);
    const int64_t min_steps = tiles <= 4 ? 4 : 8;
    const int64_t max_parts = ksteps / min_steps > 0 ? ksteps / min_steps : 1;
    if (parts > max_parts) parts = max_parts;
    g.k_parts = (int)(parts < 1 ? 1 : parts);
    return aser_gemm_tn(ctx, g);
}

// Y (rows x b) <- Y R^-1 with R^T R = Y^T Y (Cholesky-QR).  Mb must be zero on entry and is zero again
// on return.  The new Y is returned in *Y (swapped with *tmp); the old buffer, now *tmp, has been
// cleared: it is ready as the target of the next accumulating product.
int chol_qr(aser_ctx* ctx, float** Y, float** tmp, int64_t rows, int64_t clear_rows, int b, float* Mb, float* Rinv,
            int32_t* info) {
    ASER_TRY(gemm_tn_atomic(ctx, *Y, b, *Y, b, Mb, b, b, b, rows, 128, 128, false, /*upper_only=*/true));
    ASER_TRY(aser_chol_block(ctx, Mb, b, b, Rinv, info, 0, /*clear_d=*/true));
    ASER_TRY(aser_gemm_small_f32(ctx, *Y, b, Rinv, b, *tmp, b, rows, b, b, clear_rows));
    float* t = *Y; *Y = *tmp; *tmp = t;
    return ASER_OK;
}

}  // namespace

extern "C" int aser_error_reconstruct(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt,
                                      const float* S, int64_t lds, int32_t r, const aser_svd_opts* opts,
                                      float* L_A, float* L_B, float* sigma, double* err, int32_t* n_iter) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!T || !S || !L_A || !L_B || !sigma) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "error_reconstruct: null pointer");
    if (m <= 0 || n <= 0 || ldt < n || lds < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: bad shape");
    if (r <= 0 || r > m || r > n || r > 128) ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: need 0 < r <= min(m, n, 128)");
    Plan p;
    make_plan(m, n, r, opts, &p);
    if (p.b < r || p.b > 128 || (p.b % 32) != 0 || p.b > m || p.b > n) {
        // a block wider than the matrix makes no sense; shrink to the largest legal width
        int b = p.b;
        if (opts && opts->block > 0) ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: block must be a multiple of 32 in [r, min(128, m, n)]");
        const int64_t lim = (m < n ? m : n);
        while (b > lim) b -= 32;
        if (b < r) ASER_FAIL(ctx, ASER_ERR_SHAPE, "error_reconstruct: no legal block width for this r and shape");
        aser_svd_opts o2 = opts ? *opts : aser_svd_opts{0, 0, 0, 0};
        o2.block = b;
        make_plan(m, n, r, &o2, &p);
    }
    if (((uintptr_t)T & 3) || ((uintptr_t)S & 3)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "error_reconstruct: misaligned pointer");
    if (!ctx->ws || ctx->ws_bytes < p.total) ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "error_reconstruct: workspace too small (%zu needed)", p.total);
    ASER_TRY(aser_prepare_device(ctx));

    char* ws = (char*)ctx->ws;
    const int b = p.b;
    float* big0 = (float*)(ws + p.off_big0);     // T^T (n x m), later A^T (n x m)
    float* A = (float*)(ws + p.off_big1);        // m x n
    float* Q = (float*)(ws + p.off_Q);           // m x b
    float* Z = (float*)(ws + p.off_Z);           // n x b
    float* tmp = (float*)(ws + p.off_tmp);       // max(m, n) x b
    char* sm = ws + p.off_small;
    const size_t bb = align_up((size_t)b * b * 4, 256);
    float* Mb = (float*)sm;
    float* Rinv = (float*)(sm + bb);
    float* Uhat = (float*)(sm + 2 * bb);
    float* lambda = (float*)(sm + 3 * bb);                 // b floats
    double* normA2 = (double*)(sm + 3 * bb + 1024);
    int32_t* info = (int32_t*)(sm + 3 * bb + 2048);
    int32_t* cluster = (int32_t*)(sm + 3 * bb + 3072);
    float* tri = (float*)(sm + 3 * bb + 4096);             // 384 floats
    const size_t b128 = align_up((size_t)b * 128 * 4, 256);
    float* WA = (float*)(sm + 3 * bb + 8192);
    float* WBt = (float*)(sm + 3 * bb + 8192 + b128);
    float* refl = (float*)(sm + 3 * bb + 8192 + 2 * b128);

    // A = T S through T^T (K-major operand), A^T
    ASER_TRY(aser_transpose_f32(ctx, T, m, n, ldt, big0, m));
    {
        GemmArgs g{};
        g.A = big0; g.lda = m; g.B = S; g.ldb = lds; g.C = A; g.ldc = n; g.Ct = nullptr; g.ldct = 0;
        g.M = m; g.N = n; g.K = n; g.alpha = 1.f;
        g.in_type = GEMM_IN_F32X3; g.epi = GEMM_EPI_STORE; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_GE_COL;
        g.k_parts = 1;
        g.bm = (m > 1024) ? 256 : 128; g.bn = (n > 1024) ? 256 : 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
    }
    ASER_TRY(aser_fill_bytes(ctx, normA2, 8));
    ASER_TRY(aser_fill_bytes(ctx, info, 4));
    ASER_TRY(aser_transpose_f32(ctx, A, m, n, n, big0, m));
    float* At = big0;

    // start block and subspace iteration
    {
        const int64_t total = m * (int64_t)b;
        const int blocks = (int)(ceil_div64(total, 256) < 2048 ? ceil_div64(total, 256) : 2048);
        hipLaunchKernelGGL(random_block_kernel, dim3(blocks), dim3(256), 0, ctx->stream, Q, total, p.seed);
        ASER_TRY(aser_check_launch(ctx, "random_block"));
    }
    // Three tall buffers rotate: after every chol_qr `tp` is all zero, so the next product can
    // accumulate into it without a separate clearing pass.
    float* Qp = Q;
    float* Zp = Z;
    float* tp = tmp;
    const int64_t mx = m > n ? m : n;
    ASER_TRY(aser_fill_f32(ctx, Mb, b, b, b, 0.f));
    ASER_TRY(chol_qr(ctx, &Qp, &tp, m, mx, b, Mb, Rinv, info));
    const int bmA = 128, bnB = 128;
    for (int it = 0; it < p.iters; ++it) {
        ASER_TRY(gemm_tn_atomic(ctx, A, n, Qp, b, tp, b, n, b, m, bmA, bnB, false));    // Z = A^T Q
        { float* t = Zp; Zp = tp; tp = t; }
        ASER_TRY(chol_qr(ctx, &Zp, &tp, n, mx, b, Mb, Rinv, info));
        ASER_TRY(gemm_tn_atomic(ctx, At, m, Zp, b, tp, b, m, b, n, bmA, bnB, false));   // Q = A Z
        { float* t = Qp; Qp = tp; tp = t; }
        ASER_TRY(chol_qr(ctx, &Qp, &tp, m, mx, b, Mb, Rinv, info));
    }
    ASER_TRY(chol_qr(ctx, &Qp, &tp, m, mx, b, Mb, Rinv, info));                        // second pass: orthonormal to fp32
    // Rayleigh-Ritz: Z = A^T Q, eigen-pairs of Z^T Z = Q^T A A^T Q
    ASER_TRY(gemm_tn_atomic(ctx, A, n, Qp, b, tp, b, n, b, m, bmA, bnB, false));
    { float* t = Zp; Zp = tp; tp = t; }
    ASER_TRY(gemm_tn_atomic(ctx, Zp, b, Zp, b, Mb, b, b, b, n, 128, 128, false));
    ASER_TRY(aser_tridiag_eig(ctx, Mb, b, lambda, Uhat, refl, tri, cluster));
    ASER_TRY(aser_jacobi_eig(ctx, Mb, b, lambda, Uhat, cluster));      // only runs if eigenvalues cluster
    hipLaunchKernelGGL(ritz_factors_kernel, dim3(16), dim3(256), 0, ctx->stream, (const float*)lambda, (const float*)Uhat, b,
                       (int)r, sigma, WA, WBt);
    ASER_TRY(aser_check_launch(ctx, "ritz_factors"));
    // Whitened error of Eq. 8 as an explicit residual: A <- A - U_r (U_r^T A), then ||A||_F.
    // U_r^T A = (Z Uhat_r)^T with Z = A^T Q; the subtraction form avoids the cancellation of
    // ||A||^2 - sum sigma_i^2 when the top singular values carry almost all of the norm.
    ASER_TRY(aser_gemm_small_f32(ctx, Zp, b, Uhat, b, tp, r, n, b, r));            // V_r Sigma_r  (n x r)
    ASER_TRY(aser_transpose_f32(ctx, tp, n, r, r, L_B, n));                        // (r x n), parked in L_B
    ASER_TRY(aser_gemm_small_f32(ctx, Qp, b, Uhat, b, tp, r, m, b, r));            // U_r  (m x r)
    ASER_TRY(aser_transpose_f32(ctx, tp, m, r, r, Zp, m));                         // U_r^T (r x m)
    {
        GemmArgs g{};
        g.A = Zp; g.lda = m; g.B = L_B; g.ldb = n; g.C = A; g.ldc = n; g.Ct = nullptr; g.ldct = 0;
        g.M = m; g.N = n; g.K = r; g.alpha = -1.f;
        g.in_type = GEMM_IN_F32X3; g.epi = GEMM_EPI_RMW; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_FULL;
        g.k_parts = 1;
        g.bm = (m > 1024) ? 256 : 128; g.bn = (n > 1024) ? 256 : 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
    }
    ASER_TRY(aser_sumsq_f32(ctx, A, m, n, n, normA2));
    // L_A = Q (Uhat_r Sigma_r)
    ASER_TRY(aser_gemm_small_f32(ctx, Qp, b, WA, r, L_A, r, m, b, r));
    // L_B^T = (T^T Q) (Uhat_r Sigma_r^-1)  ->  L_B
    ASER_TRY(gemm_tn_atomic(ctx, T, ldt, Qp, b, Zp, b, n, b, m, bmA, bnB, true));  // C^T = T^T Q (n x b)
    ASER_TRY(aser_gemm_small_f32(ctx, Zp, b, WBt, r, tp, r, n, b, r));             // n x r
    ASER_TRY(aser_transpose_f32(ctx, tp, n, r, r, L_B, n));

    double h_res2 = 0.0;
    ASER_HIP(ctx, hipMemcpyAsync(&h_res2, normA2, 8, hipMemcpyDeviceToHost, ctx->stream));
    ASER_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (err) *err = sqrt(h_res2 > 0.0 ? h_res2 : 0.0);
    if (n_iter) *n_iter = p.iters;
    return ASER_OK;
}
