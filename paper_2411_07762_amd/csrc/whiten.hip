// Whitening factor of Eq. 5 / Algorithm 1: S = chol(M^-1 G M^-1), blocked, one block row at a time.
//
// The factorisation runs on the upper triangle (G' = R^T R, R = S^T) so that every contraction
// has the K-major "A^T B" form of the MFMA kernel.  For block row k (rows k .. k+b):
//   update           G'[k:k+b, k:] -= R[:k, k:k+b]^T R[:k, k:]   (A, B = the finished rows above; K = k)
//   diagonal block   R11 = chol(D), R11^-1                       (one workgroup, LDS)
//   row panel        R12 = (R11^-1)^T * G'[k, k+b:]              (A = R11^-1, B = the panel, in place)
// A final pass moves R to the lower triangle (S = R^T) and clears the strict upper triangle; writing
// R12^T from the panel kernel instead cost 4 us per panel in scattered 16-byte stores.
#include <limits.h>

#include "aser_internal.h"

namespace {

constexpr int kNb = 128;

// S[i][j] = S[j][i] = G[i][j] / (m_i m_j) for i >= j, plus the damping term on the diagonal.
__global__ __launch_bounds__(256) void whiten_prep_kernel(const float* G, int64_t ldg, int64_t n, const float* mdiag,
                                                          float* S, int64_t lds, const double* diag_sum, float damp) {
    __shared__ float tile[64][65];
    // blockIdx.x enumerates tile pairs (bi >= bj)
    const int64_t t = blockIdx.x;
    int64_t bi = (int64_t)((sqrt(8.0 * (double)t + 1.0) - 1.0) * 0.5);
    while (bi * (bi + 1) / 2 > t) --bi;
    while ((bi + 1) * (bi + 2) / 2 <= t) ++bi;
    const int64_t bj = t - bi * (bi + 1) / 2;
    const int64_t r0 = bi * 64, c0 = bj * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const float add = (damp > 0.f && diag_sum) ? (float)((double)damp * (*diag_sum) / (double)n) : 0.f;
    for (int i = ty; i < 64; i += 4) {
        const int64_t r = r0 + i, c = c0 + tx;
        float v = 0.f;
        if (r < n && c < n) {
            const float g = (r >= c) ? G[r * ldg + c] : G[c * ldg + r];
            const float mi = mdiag ? mdiag[r] : 1.f, mj = mdiag ? mdiag[c] : 1.f;
            v = g / (mi * mj);
            if (r == c) v += add;
        }
        tile[i][tx] = v;
    }
    __syncthreads();
    if (bi == bj) {                                      // only the upper triangle is worked on from here
        for (int i = ty; i < 64; i += 4) {
            const int64_t r = r0 + i, c = c0 + tx;
            if (r < n && c < n) S[r * lds + c] = tile[i][tx];
        }
    } else {
        for (int i = ty; i < 64; i += 4) {
            const int64_t r = c0 + i, c = r0 + tx;      // transposed tile
            if (r < n && c < n) S[r * lds + c] = tile[tx][i];
        }
    }
}

__global__ __launch_bounds__(256) void diag_scaled_sum_kernel(const float* G, int64_t ldg, int64_t n, const float* mdiag,
                                                              double* out) {
    __shared__ double red[4];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) {
        const double mi = mdiag ? (double)mdiag[i] : 1.0;
        acc += (double)G[i * ldg + i] / (mi * mi);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) *out = red[0] + red[1] + red[2] + red[3];
}

// The factor was built as R = S^T in the upper triangle.  One pass over pairs of 64 x 64 tiles moves it
// to the lower triangle (through LDS, both sides coalesced) and clears the strict upper triangle.
__global__ __launch_bounds__(256) void upper_to_lower_kernel(float* S, int64_t n, int64_t lds) {
    __shared__ float tile[64][65];
    const int64_t t = blockIdx.x;
    int64_t bi = (int64_t)((sqrt(8.0 * (double)t + 1.0) - 1.0) * 0.5);
    while (bi * (bi + 1) / 2 > t) --bi;
    while ((bi + 1) * (bi + 2) / 2 <= t) ++bi;
    const int64_t bj = t - bi * (bi + 1) / 2;          // bi >= bj: upper tile (bj, bi) -> lower tile (bi, bj)
    const int64_t u0 = bj * 64, v0 = bi * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int64_t r = u0 + i, c = v0 + tx;
        float v = 0.f;
        if (r < n && c < n) {
            v = S[r * lds + c];
            if (c > r) S[r * lds + c] = 0.f;
        }
        tile[i][tx] = v;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int64_t r = v0 + i, c = u0 + tx;          // lower entry (r, c) = upper entry (c, r)
        if (r < n && c < n && r > c) S[r * lds + c] = tile[tx][i];
    }
}

}  // namespace

extern "C" int aser_whiten(aser_ctx* ctx, const float* G, int64_t ldg, int64_t n, const float* mdiag, float damp,
                           float* S, int64_t lds, int32_t* info) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!G || !S) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "whiten: null pointer");
    if (n <= 0 || ldg < n || lds < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "whiten: bad shape");
    if (!(damp >= 0.f)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "whiten: damp must be >= 0");
    if (((uintptr_t)G & 3) || ((uintptr_t)S & 3)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "whiten: misaligned pointer");
    const size_t need = (size_t)kNb * kNb * 4 + 512 + kAserWsTail;
    if (!ctx->ws || ctx->ws_bytes < need) ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "whiten: workspace too small");
    ASER_TRY(aser_prepare_device(ctx));

    float* Rinv = (float*)ctx->ws;
    int32_t* info_dev = (int32_t*)((char*)ctx->ws + ctx->ws_bytes - kAserWsTail);
    double* diag_sum = (double*)((char*)ctx->ws + (size_t)kNb * kNb * 4 + 256);

    // A flag still pending from an earlier asynchronous call is kept (the factorisation lowers it with
    // atomicMin): that call's failed pivot is then still reported, by whichever call synchronises next.
    if (ctx->pending_info_dev != info_dev) ASER_TRY(aser_set_i32(ctx, info_dev, (int32_t)INT_MAX));
    if (damp > 0.f) {
        hipLaunchKernelGGL(diag_scaled_sum_kernel, dim3(1), dim3(256), 0, ctx->stream, G, ldg, n, mdiag, diag_sum);
        ASER_TRY(aser_check_launch(ctx, "diag_sum"));
    }
    const int64_t t64 = ceil_div64(n, 64);
    hipLaunchKernelGGL(whiten_prep_kernel, dim3((unsigned)(t64 * (t64 + 1) / 2)), dim3(256), 0, ctx->stream, G, ldg, n,
                       mdiag, S, lds, (const double*)diag_sum, damp);
    ASER_TRY(aser_check_launch(ctx, "whiten_prep"));

    // Up-looking blocked Cholesky on the upper triangle (R = S^T): block row j first receives the
    // contribution of all finished rows above it in one product with a long K (split over
    // workgroups, fp32 atomics), then its diagonal block is factored and the row is multiplied by
    // the inverse of that factor.  Every entry of the matrix is updated once, by one launch.
    // Wide matrices take the long-K update for two block rows at a time (256 x 256 tiles convert each
    // fp32 operand element once per 256 instead of 128 result columns or rows); the second block row of
    // a pair then still lacks the contribution of the first, a K = 128 update of its own.
    const bool pairs = n >= 12288;   // measured: 11008 columns are still faster one block row at a time
    const int form = aser_f32_form(ctx, n * n);   // three or six bf16 products per fp32 product
    const bool six = form == GEMM_IN_F32X6;
    auto update = [&](int64_t row0, int64_t rows, int64_t kfrom, int64_t klen, int bm, int bn) -> int {
        GemmArgs u{};
        u.A = S + kfrom * lds + row0; u.lda = lds; u.B = S + kfrom * lds + row0; u.ldb = lds;
        u.C = S + row0 * lds + row0; u.ldc = lds; u.Ct = nullptr; u.ldct = 0;
        u.M = rows; u.N = n - row0; u.K = klen; u.alpha = -1.f;
        u.in_type = form; u.epi = GEMM_EPI_ATOMIC; u.tiles = GEMM_TILES_ALL; u.krange = GEMM_K_FULL;
        if (six && bm == 256 && bn == 256) bn = 128;    // the six-product form has no 256 x 256 tile
        u.bm = bm; u.bn = bn; u.upper_only = 1;
        const int64_t tiles = ceil_div64(u.M, u.bm) * ceil_div64(u.N, u.bn), ksteps = ceil_div64(klen, 32);
        u.k_parts = aser_split_k_parts(tiles, ksteps, 4, (double)(bm * bn) / (128.0 * 128.0), ctx->share);
        return aser_gemm_tn(ctx, u);
    };
    for (int64_t k0 = 0; k0 < n; k0 += kNb) {
        const int b = (int)((n - k0 < kNb) ? n - k0 : kNb);
        float* D = S + k0 * lds + k0;
        if (pairs) {
            if (k0 % (2 * kNb) == 0) {
                if (k0 > 0) ASER_TRY(update(k0, (n - k0 < 2 * kNb) ? n - k0 : 2 * kNb, 0, k0, 256, 256));
            } else {
                ASER_TRY(update(k0, b, k0 - kNb, kNb, 128, 128));   // K = 128 only, as the row panel: many small tiles
            }
        } else if (k0 > 0) {
            ASER_TRY(update(k0, b, 0, k0, 128, (n - k0 >= 4096) ? 256 : 128));
        }
        ASER_TRY(aser_chol_block(ctx, D, lds, b, Rinv, info_dev, (int32_t)k0));
        const int64_t rem = n - k0 - b;
        if (rem <= 0) break;
        float* S12 = S + k0 * lds + (k0 + b);
        GemmArgs p{};
        p.A = Rinv; p.lda = b; p.B = S12; p.ldb = lds; p.C = S12; p.ldc = lds;
        p.Ct = nullptr; p.ldct = 0;
        p.M = b; p.N = rem; p.K = b; p.alpha = 1.f;
        p.in_type = form; p.epi = GEMM_EPI_STORE; p.tiles = GEMM_TILES_ALL; p.krange = GEMM_K_FULL;
        p.k_parts = 1; p.bm = 128; p.bn = 128;           // K = 128 only: twice the workgroups beat the wider tile (16.6 -> 12 us at c1)
        ASER_TRY(aser_gemm_tn(ctx, p));
    }
    hipLaunchKernelGGL(upper_to_lower_kernel, dim3((unsigned)(t64 * (t64 + 1) / 2)), dim3(256), 0, ctx->stream, S, n, lds);
    ASER_TRY(aser_check_launch(ctx, "upper_to_lower"));

    if (!info) {                                         // asynchronous: the flag is read by the next synchronising call
        ctx->pending_info_dev = info_dev;
        return ASER_OK;
    }
    ctx->pending_info_dev = info_dev;
    AserPending pend;
    ASER_TRY(aser_sync_status(ctx, &pend));
    *info = (pend.pivot == INT_MAX) ? 0 : pend.pivot;
    return aser_report_pending(ctx, pend, "whiten");
}
