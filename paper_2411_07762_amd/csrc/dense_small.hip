// The Jacobi eigen-solver (fallback of the Rayleigh-Ritz step of the truncated SVD, Eq. 6), one
// workgroup with its matrices in LDS, and a plain fp32 FMA product for "tall times small" updates.
#include "aser_internal.h"

namespace {

constexpr int kMaxB = 128;
constexpr int kLdsPitch = kMaxB + 1;

// ------------------------------------------------------------------------------------ Jacobi
// Cyclic Jacobi with the round-robin pairing: b / 2 disjoint rotations per round, b - 1 rounds
// per sweep.  M and V live in LDS.
__global__ __launch_bounds__(1024) void jacobi_kernel(const float* Mb, int b, float* lambda, float* Vout, int max_sweeps,
                                                      const int* gate) {
    if (gate && *gate == 0) return;                  // the fast solver already delivered the result
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
// C (rows x c) = A (rows x k) * B (k x c) in plain fp32 FMAs.  A workgroup owns 32 rows x 128
// columns; a thread owns 2 rows x 8 columns and reads its operands from LDS as float2 / float4.
__global__ __launch_bounds__(256) void gemm_small_kernel(const float* __restrict__ A, int64_t lda,
                                                         const float* __restrict__ B, int64_t ldb, float* __restrict__ C,
                                                         int64_t ldc, int64_t rows, int k, int c) {
    __shared__ __attribute__((aligned(16))) float As[32][34];     // [kk][row]
    __shared__ __attribute__((aligned(16))) float Bs[32][132];    // [kk][col]
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    const int64_t r0 = (int64_t)blockIdx.x * 32;
    const int c0 = blockIdx.y * 128;
    float acc[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < k; k0 += 32) {
        {
            const int r = tid >> 3, kq = (tid & 7) * 4;
            const int64_t gr = r0 + r;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int kk = kq + e;
                As[kk][r] = (gr < rows && k0 + kk < k) ? A[gr * lda + k0 + kk] : 0.f;
            }
        }
        {
            const int kk = tid >> 3, cq = (tid & 7) * 16;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int cc = c0 + cq + e;
                Bs[kk][cq + e] = (k0 + kk < k && cc < c) ? B[(int64_t)(k0 + kk) * ldb + cc] : 0.f;
            }
        }
        __syncthreads();
#pragma unroll 8
        for (int kk = 0; kk < 32; ++kk) {
            const float2 av = *(const float2*)&As[kk][2 * ty];
            const float4 b0 = *(const float4*)&Bs[kk][8 * tx];
            const float4 b1 = *(const float4*)&Bs[kk][8 * tx + 4];
            const float a2[2] = {av.x, av.y};
            const float b8[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(a2[i], b8[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int64_t gr = r0 + 2 * ty + i;
        if (gr >= rows) continue;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int cc = c0 + 8 * tx + j;
            if (cc < c) C[gr * ldc + cc] = acc[i][j];
        }
    }
}

}  // namespace

int aser_jacobi_eig(aser_ctx* ctx, const float* Mb, int b, float* lambda, float* V, const int* gate) {
    if (b <= 0 || b > kMaxB || (b & 1)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "jacobi: block size must be even and <= 128");
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(2 * kMaxB * kLdsPitch + kMaxB + kMaxB + 32) * 4;
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)jacobi_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(jacobi_kernel, dim3(1), dim3(1024), lds, ctx->stream, Mb, b, lambda, V, 30, gate);
    return aser_check_launch(ctx, "jacobi");
}

int aser_gemm_small_f32(aser_ctx* ctx, const float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                        int64_t rows, int k, int c) {
    if (rows <= 0) return ASER_OK;
    if (k <= 0 || c <= 0) ASER_FAIL(ctx, ASER_ERR_SHAPE, "gemm_small: k > 0 and c > 0 required");
    dim3 grid((unsigned)ceil_div64(rows, 32), (unsigned)((c + 127) / 128));
    hipLaunchKernelGGL(gemm_small_kernel, grid, dim3(256), 0, ctx->stream, A, lda, B, ldb, C, ldc, rows, k, c);
    return aser_check_launch(ctx, "gemm_small");
}
