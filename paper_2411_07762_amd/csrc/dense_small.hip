// Small dense factorisations that run in one workgroup with their matrices in LDS: the diagonal
// blocks of the blocked Cholesky (Eq. 5), the b x b Cholesky of the orthogonalisation, and the
// Jacobi eigen-solver of the Rayleigh-Ritz step of the truncated SVD (Eq. 6).  Plus a plain
// fp32 FMA product for "tall times small" updates.
#include "aser_internal.h"

namespace {

constexpr int kMaxB = 128;
constexpr int kLdsPitch = kMaxB + 1;

// ------------------------------------------------------------------------------------ Cholesky block
// D = R^T R on the upper part of a b x b block; R^-1 by column-wise back substitution.
__global__ __launch_bounds__(256) void chol_block_kernel(float* D, int64_t ld, int b, float* Rinv, int32_t* info,
                                                         int32_t pivot_base) {
    extern __shared__ float sm[];
    float* a = sm;                                   // b x pitch, upper part
    float* x = sm + kMaxB * kLdsPitch;               // inverse, b x pitch
    float* invd = x + kMaxB * kLdsPitch;             // 1 / R[j][j]
    const int tid = threadIdx.x;
    for (int t = tid; t < b * b; t += 256) {
        const int i = t / b, k = t % b;
        a[i * kLdsPitch + k] = (k >= i) ? D[i * ld + k] : 0.f;
        x[i * kLdsPitch + k] = 0.f;
    }
    __syncthreads();
    const int rows_per_pass = 256 / b > 0 ? 256 / b : 1;
    for (int j = 0; j < b; ++j) {
        float piv = a[j * kLdsPitch + j];
        if (!(piv > 0.f)) {
            if (tid == 0 && info) atomicMin(info, pivot_base + j + 1);
            piv = 1.f;
        }
        const float inv = 1.0f / sqrtf(piv);
        if (tid == 0) invd[j] = inv;
        const float inv2 = inv * inv;
        const int k = tid % b;
        for (int i = j + 1 + tid / b; i < b; i += rows_per_pass) {
            if (k >= i && tid < rows_per_pass * b)
                a[i * kLdsPitch + k] -= (a[j * kLdsPitch + i] * a[j * kLdsPitch + k]) * inv2;
        }
        __syncthreads();
    }
    // scale rows: R[j][k] = a[j][k] * invd[j]; a non-positive pivot was replaced by 1
    for (int t = tid; t < b * b; t += 256) {
        const int j = t / b, k = t % b;
        if (k >= j) {
            float v = a[j * kLdsPitch + k] * invd[j];
            if (k == j) v = 1.0f / invd[j];
            a[j * kLdsPitch + k] = v;
        }
    }
    __syncthreads();
    for (int t = tid; t < b * b; t += 256) {
        const int j = t / b, k = t % b;
        if (k >= j) {
            const float v = a[j * kLdsPitch + k];
            D[j * ld + k] = v;
            D[k * ld + j] = v;
        }
    }
    // inverse: thread k solves R x = e_k from the bottom (x[k] = 1 / R[k][k], zero below)
    if (tid < b) {
        const int k = tid;
        x[k * kLdsPitch + k] = invd[k];
    }
    __syncthreads();
    for (int p = b - 2; p >= 0; --p) {
        if (tid < b && tid > p) {
            const int k = tid;
            float s = 0.f;
            for (int q = p + 1; q <= k; ++q) s += a[p * kLdsPitch + q] * x[q * kLdsPitch + k];
            x[p * kLdsPitch + k] = -s * invd[p];
        }
        // no barrier: thread k only reads its own column of x
    }
    __syncthreads();
    for (int t = tid; t < b * b; t += 256) {
        const int i = t / b, k = t % b;
        Rinv[i * b + k] = (k >= i) ? x[i * kLdsPitch + k] : 0.f;
    }
}

// ------------------------------------------------------------------------------------ Jacobi
// Cyclic Jacobi with the round-robin pairing: b / 2 disjoint rotations per round, b - 1 rounds
// per sweep.  M and V live in LDS.
__global__ __launch_bounds__(1024) void jacobi_kernel(const float* Mb, int b, float* lambda, float* Vout, int max_sweeps) {
    extern __shared__ float sm[];
    float* M = sm;
    float* V = sm + kMaxB * kLdsPitch;
    float* cs = V + kMaxB * kLdsPitch;               // c[b/2], s[b/2]
    int* top = (int*)(cs + kMaxB);
    int* bot = top + kMaxB / 2;
    float* red = (float*)(bot + kMaxB / 2);          // 32 floats
    const int tid = threadIdx.x, nt = blockDim.x;
    const int half = b / 2;
    for (int t = tid; t < b * b; t += nt) {
        const int i = t / b, k = t % b;
        M[i * kLdsPitch + k] = 0.5f * (Mb[i * b + k] + Mb[k * b + i]);
        V[i * kLdsPitch + k] = (i == k) ? 1.f : 0.f;
    }
    if (tid < half) { top[tid] = 2 * tid; bot[tid] = 2 * tid + 1; }
    __syncthreads();

    for (int sweep = 0; sweep < max_sweeps; ++sweep) {
        // convergence: off-diagonal mass against the diagonal mass
        float off = 0.f, dia = 0.f;
        for (int t = tid; t < b * b; t += nt) {
            const int i = t / b, k = t % b;
            const float v = M[i * kLdsPitch + k];
            if (i == k) dia += v * v; else off += v * v;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) { off += __shfl_xor(off, o, 64); dia += __shfl_xor(dia, o, 64); }
        if ((tid & 63) == 0) { red[tid >> 6] = off; red[16 + (tid >> 6)] = dia; }
        __syncthreads();
        float offs = 0.f, dias = 0.f;
        for (int w = 0; w < nt / 64; ++w) { offs += red[w]; dias += red[16 + w]; }
        __syncthreads();
        if (offs <= 1e-13f * dias) break;

        for (int round = 0; round < b - 1; ++round) {
            if (tid < half) {
                const int p = top[tid], q = bot[tid];
                const float app = M[p * kLdsPitch + p], aqq = M[q * kLdsPitch + q], apq = M[p * kLdsPitch + q];
                float c = 1.f, s = 0.f;
                if (fabsf(apq) > 1e-30f && fabsf(apq) > 1e-9f * sqrtf(fabsf(app * aqq))) {
                    const float tau = (aqq - app) / (2.f * apq);
                    const float t = (tau >= 0.f ? 1.f : -1.f) / (fabsf(tau) + sqrtf(1.f + tau * tau));
                    c = 1.f / sqrtf(1.f + t * t);
                    s = t * c;
                }
                cs[tid] = c;
                cs[half + tid] = s;
            }
            __syncthreads();
            // rows: M <- J^T M
            for (int t = tid; t < half * b; t += nt) {
                const int pr = t / b, k = t % b;
                const int p = top[pr], q = bot[pr];
                const float c = cs[pr], s = cs[half + pr];
                const float mp = M[p * kLdsPitch + k], mq = M[q * kLdsPitch + k];
                M[p * kLdsPitch + k] = c * mp - s * mq;
                M[q * kLdsPitch + k] = s * mp + c * mq;
            }
            __syncthreads();
            // columns: M <- M J, V <- V J
            for (int t = tid; t < half * b; t += nt) {
                const int pr = t % half, k = t / half;
                const int p = top[pr], q = bot[pr];
                const float c = cs[pr], s = cs[half + pr];
                const float mp = M[k * kLdsPitch + p], mq = M[k * kLdsPitch + q];
                M[k * kLdsPitch + p] = c * mp - s * mq;
                M[k * kLdsPitch + q] = s * mp + c * mq;
                const float vp = V[k * kLdsPitch + p], vq = V[k * kLdsPitch + q];
                V[k * kLdsPitch + p] = c * vp - s * vq;
                V[k * kLdsPitch + q] = s * vp + c * vq;
            }
            __syncthreads();
            // rotate the pairing: top[0] fixed, the rest moves round the ring
            int nt_top = 0, nt_bot = 0;
            if (tid < half) {
                if (tid == 0) nt_top = top[0];
                else if (tid == 1) nt_top = bot[0];
                else nt_top = top[tid - 1];
                nt_bot = (tid == half - 1) ? top[half - 1] : bot[tid + 1];
            }
            __syncthreads();
            if (tid < half) { top[tid] = nt_top; bot[tid] = nt_bot; }
            __syncthreads();
        }
    }
    // eigenvalues = diagonal; sort descending (ties -> lower index first)
    __syncthreads();
    if (tid < b) {
        const float li = M[tid * kLdsPitch + tid];
        int rank = 0;
        for (int j = 0; j < b; ++j) {
            const float lj = M[j * kLdsPitch + j];
            if (lj > li || (lj == li && j < tid)) ++rank;
        }
        lambda[rank] = li;
        top[tid] = rank;     // pairing table is no longer needed (b <= 128 = 2 * half slots: use top+bot)
    }
    __syncthreads();
    for (int t = tid; t < b * b; t += nt) {
        const int k = t / b, i = t % b;
        Vout[k * b + top[i]] = V[k * kLdsPitch + i];
    }
}

// ------------------------------------------------------------------------------------ small fp32 product
// C (rows x c) = A (rows x k) * B (k x c).  16 rows per workgroup; B is staged through LDS in
// slices of 32 k-values.
__global__ __launch_bounds__(256) void gemm_small_kernel(const float* __restrict__ A, int64_t lda,
                                                         const float* __restrict__ B, int64_t ldb, float* __restrict__ C,
                                                         int64_t ldc, int64_t rows, int k, int c) {
    __shared__ float As[16][33];
    __shared__ float Bs[32][257];
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const int64_t r0 = (int64_t)blockIdx.x * 16;
    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = 0.f;
    for (int k0 = 0; k0 < k; k0 += 32) {
        for (int t = tid; t < 16 * 32; t += 256) {
            const int r = t >> 5, kk = t & 31;
            As[r][kk] = (r0 + r < rows && k0 + kk < k) ? A[(r0 + r) * lda + k0 + kk] : 0.f;
        }
        for (int t = tid; t < 32 * c; t += 256) {
            const int kk = t / c, cc = t % c;
            Bs[kk][cc] = (k0 + kk < k) ? B[(int64_t)(k0 + kk) * ldb + cc] : 0.f;
        }
        __syncthreads();
#pragma unroll 8
        for (int kk = 0; kk < 32; ++kk) {
            const float av = As[ty][kk];
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int cc = tx + 16 * j;
                if (cc < c) acc[j] = fmaf(av, Bs[kk][cc], acc[j]);
            }
        }
        __syncthreads();
    }
    if (r0 + ty < rows) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int cc = tx + 16 * j;
            if (cc < c) C[(r0 + ty) * ldc + cc] = acc[j];
        }
    }
}

}  // namespace

int aser_chol_block(aser_ctx* ctx, float* D, int64_t ld, int b, float* Rinv, int32_t* info, int32_t pivot_base) {
    if (b <= 0 || b > kMaxB) ASER_FAIL(ctx, ASER_ERR_SHAPE, "chol_block: block size out of range");
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(2 * kMaxB * kLdsPitch + kMaxB) * 4;
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)chol_block_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(chol_block_kernel, dim3(1), dim3(256), lds, ctx->stream, D, ld, b, Rinv, info, pivot_base);
    return aser_check_launch(ctx, "chol_block");
}

int aser_jacobi_eig(aser_ctx* ctx, const float* Mb, int b, float* lambda, float* V) {
    if (b <= 0 || b > kMaxB || (b & 1)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "jacobi: block size must be even and <= 128");
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(2 * kMaxB * kLdsPitch + kMaxB + kMaxB + 32) * 4;
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)jacobi_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(jacobi_kernel, dim3(1), dim3(1024), lds, ctx->stream, Mb, b, lambda, V, 30);
    return aser_check_launch(ctx, "jacobi");
}

int aser_gemm_small_f32(aser_ctx* ctx, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                        int64_t rows, int k, int c) {
    if (rows <= 0) return ASER_OK;
    if (k <= 0 || c <= 0 || c > 256) ASER_FAIL(ctx, ASER_ERR_SHAPE, "gemm_small: k > 0 and 0 < c <= 256 required");
    hipLaunchKernelGGL(gemm_small_kernel, dim3((unsigned)ceil_div64(rows, 16)), dim3(256), 0, ctx->stream, A, lda, B, ldb,
                       C, ldc, rows, k, c);
    return aser_check_launch(ctx, "gemm_small");
}
