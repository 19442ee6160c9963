// The Jacobi eigen-solver (fallback of the Rayleigh-Ritz step of the truncated SVD, Eq. 6), one
// workgroup with its matrices in LDS, and an fp32 MFMA product for "tall times small" updates.
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
// C (rows x c) = A (rows x k) * B (k x c) in fp32, k, c <= 128, on the fp32 MFMA instruction (16 x 16 x 4:
// true fp32 products and sums).  A workgroup owns 32 rows; its A rows and all of B go to LDS in one shot
// (every global load is issued before the first LDS store: one memory round trip); wavefront w owns
// the 16 x 64 piece (row tile w / 2, column tiles 4 (w % 2) ...), four accumulator tiles.  The first
// clear_rows rows of A (may exceed `rows`) are cleared once they have been read, which leaves A ready
// as the target of an accumulating product.
typedef float gs_f4v __attribute__((ext_vector_type(4)));
constexpr int kGsRows = 32;
constexpr int kGsPitch = 132;

// acc[j] += A-rows (16 rt ...) x B-columns (16 (ct0 + j) ...) over k: lane (t_i, t_q) feeds A(t_i, 4 s + t_q) and
// B(4 s + t_q, t_i); acc[j][e] is row 4 t_q + e, column t_i of tile j.
__device__ __forceinline__ void small_product(gs_f4v (&acc)[4], const float* As, const float* Bs, int k, int rt, int ct0,
                                              int t_i, int t_q) {
    const float* pa = As + (16 * rt + t_i) * kGsPitch + t_q;
    const float* pb = Bs + t_q * kGsPitch + 16 * ct0 + t_i;
    for (int s = 0; s < k / 4; ++s) {
        const float a = pa[4 * s];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, pb[4 * s * kGsPitch + 16 * j], acc[j], 0, 0, 0);
    }
}

__global__ __launch_bounds__(256) void gemm_small_kernel(float* __restrict__ A, int64_t lda, const float* __restrict__ B,
                                                         int64_t ldb, float* __restrict__ C, int64_t ldc, int64_t rows,
                                                         int k, int c, int64_t clear_rows, int vec_b, int transposed) {
    extern __shared__ __align__(16) float gs_sm[];
    float* As = gs_sm;                          // [32][132]
    float* Bs = gs_sm + kGsRows * kGsPitch;     // [128][132]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t_i = lane & 15, t_q = lane >> 4, rt = wave >> 1, ct0 = (wave & 1) * 4;
    const int64_t r0 = (int64_t)blockIdx.x * kGsRows;

    // A: 32 rows x 128 k = 1024 float4, four per thread (k is a multiple of 4 and rows are 16-byte aligned)
    float4 av[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int q = tid + 256 * u, r = q >> 5, k4 = (q & 31) * 4;
        av[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r0 + r < rows && k4 < k) av[u] = *(const float4*)(A + (r0 + r) * lda + k4);
    }
    // B: 128 x 128 = 4096 float4, sixteen per thread
    float4 bv[16];
    if (vec_b) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int q = tid + 256 * u, kk = q >> 5, c4 = (q & 31) * 4;
            bv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (kk < k && c4 < c) bv[u] = *(const float4*)(B + (int64_t)kk * ldb + c4);
        }
    } else {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int q = tid + 256 * u, kk = q >> 5, c4 = (q & 31) * 4;
            float t[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (kk < k && c4 + e < c) t[e] = B[(int64_t)kk * ldb + c4 + e];
            bv[u] = make_float4(t[0], t[1], t[2], t[3]);
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int q = tid + 256 * u, r = q >> 5, k4 = (q & 31) * 4;
        *(float4*)(As + r * kGsPitch + k4) = av[u];
        if (r0 + r < clear_rows && k4 < k) *(float4*)(A + (r0 + r) * lda + k4) = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int q = tid + 256 * u, kk = q >> 5, c4 = (q & 31) * 4;
        *(float4*)(Bs + kk * kGsPitch + c4) = bv[u];
    }
    __syncthreads();

    gs_f4v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = gs_f4v{0.f, 0.f, 0.f, 0.f};
    small_product(acc, As, Bs, k, rt, ct0, t_i, t_q);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int cc = 16 * (ct0 + j) + t_i;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t gr = r0 + 16 * rt + 4 * t_q + e;
            if (gr < rows && cc < c) {
                if (transposed) C[(int64_t)cc * ldc + gr] = acc[j][e];      // C^T (c x rows, ld = ldc)
                else C[gr * ldc + cc] = acc[j][e];
            }
        }
    }
}

// C (rows x b) = (A1 + alpha A2 P) B1 for two tall blocks and two b x b factors (A2 null: C = A1 B1), alpha read
// from device memory; b a multiple of 4 up to 128, all leading dimensions b.  After they have been read, the rows
// of A1 and the first zrows rows of Zclr (may be null) are cleared: both are accumulation targets of the products
// that follow.  Same staging and the same MFMA product as gemm_small_kernel: A2 P first, then the sum goes back to
// LDS (every lane writes the entries its accumulators hold) as the left operand of the second product.
__global__ __launch_bounds__(256) void combine_kernel(float* __restrict__ A1, const float* __restrict__ B1,
                                                      const float* __restrict__ A2, const float* __restrict__ P,
                                                      const float* __restrict__ alpha_dev,
                                                      float* __restrict__ C, int64_t rows, int b,
                                                      float* __restrict__ Zclr, int64_t zrows) {
    extern __shared__ __align__(16) float gs_sm[];
    float* As = gs_sm;                          // [32][132]
    float* Bs = gs_sm + kGsRows * kGsPitch;     // [128][132]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t_i = lane & 15, t_q = lane >> 4, rt = wave >> 1, ct0 = (wave & 1) * 4;
    const int64_t r0 = (int64_t)blockIdx.x * kGsRows;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    gs_f4v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = gs_f4v{0.f, 0.f, 0.f, 0.f};
    // this lane's entries of A1 (those its accumulators will hold in the sum), read before A1 is cleared
    float u1[4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int cc = 16 * (ct0 + j) + t_i;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t gr = r0 + 16 * rt + 4 * t_q + e;
            u1[j][e] = (gr < rows && cc < b) ? A1[gr * b + cc] : 0.f;
        }
    }
    const float alpha = A2 ? *alpha_dev : 0.f;
    for (int term = A2 ? 0 : 1; term < 2; ++term) {
        const float* A = term ? nullptr : A2;
        const float* B = term ? B1 : P;
        float4 av[4], bv[16];
        if (A) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = tid + 256 * u, r = q >> 5, k4 = (q & 31) * 4;
                av[u] = zero4;
                if (r0 + r < rows && k4 < b) av[u] = *(const float4*)(A + (r0 + r) * b + k4);
            }
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int q = tid + 256 * u, kk = q >> 5, c4 = (q & 31) * 4;
            bv[u] = zero4;
            if (kk < b && c4 < b) bv[u] = *(const float4*)(B + (int64_t)kk * b + c4);
        }
        __syncthreads();                                // the previous product's readers (and the readers of A1) are done
        if (A) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = tid + 256 * u, r = q >> 5, k4 = (q & 31) * 4;
                *(float4*)(As + r * kGsPitch + k4) = av[u];
            }
        } else {
            // left operand of the second product: A1 + alpha (A2 P), the entries this lane's accumulators hold
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    As[(16 * rt + 4 * t_q + e) * kGsPitch + 16 * (ct0 + j) + t_i] = fmaf(alpha, acc[j][e], u1[j][e]);
            // the two accumulation targets are clear again
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int q = tid + 256 * u, r = q >> 5, k4 = (q & 31) * 4;
                if (r0 + r < rows && k4 < b) *(float4*)(A1 + (r0 + r) * b + k4) = zero4;
                if (Zclr && r0 + r < zrows && k4 < b) *(float4*)(Zclr + (r0 + r) * b + k4) = zero4;
            }
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int q = tid + 256 * u, kk = q >> 5, c4 = (q & 31) * 4;
            *(float4*)(Bs + kk * kGsPitch + c4) = bv[u];
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = gs_f4v{0.f, 0.f, 0.f, 0.f};
        small_product(acc, As, Bs, b, rt, ct0, t_i, t_q);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int cc = 16 * (ct0 + j) + t_i;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t gr = r0 + 16 * rt + 4 * t_q + e;
            if (gr < rows && cc < b) C[gr * b + cc] = acc[j][e];
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

int aser_gemm_small_f32(aser_ctx* ctx, float* A, int64_t lda, const float* B, int64_t ldb, float* C, int64_t ldc,
                        int64_t rows, int k, int c, int64_t clear_rows, bool transposed) {
    if (rows <= 0) return ASER_OK;
    if (k <= 0 || c <= 0 || k > 128 || c > 128 || (k & 3)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "gemm_small: need 0 < k, c <= 128, k %% 4 == 0");
    if (((uintptr_t)A & 15) || (lda & 3)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_small: A must be 16-byte aligned with lda %% 4 == 0");
    const int vec_b = (((uintptr_t)B & 15) == 0 && (ldb & 3) == 0 && (c & 3) == 0) ? 1 : 0;
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(kGsRows + 128) * kGsPitch * sizeof(float);
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)gemm_small_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set[ctx->device] = true;
    }
    const int64_t cover = rows > clear_rows ? rows : clear_rows;
    hipLaunchKernelGGL(gemm_small_kernel, dim3((unsigned)ceil_div64(cover, kGsRows)), dim3(256), lds, ctx->stream, A, lda, B, ldb,
                       C, ldc, rows, k, c, clear_rows, vec_b, transposed ? 1 : 0);
    return aser_check_launch(ctx, "gemm_small");
}

int aser_combine_f32(aser_ctx* ctx, float* A1, const float* B1, const float* A2, const float* P, const float* alpha_dev,
                     float* C, int64_t rows, int b, float* Zclr, int64_t zrows) {
    if (rows <= 0) return ASER_OK;
    if (b <= 0 || b > 128 || (b & 3)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "combine: need 0 < b <= 128, b %% 4 == 0");
    if (((uintptr_t)A1 & 15) || ((uintptr_t)B1 & 15) || ((uintptr_t)A2 & 15) || ((uintptr_t)P & 15) || ((uintptr_t)C & 15) ||
        ((uintptr_t)Zclr & 15))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "combine: operands must be 16-byte aligned");
    if (A2 && (!P || !alpha_dev)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "combine: the second term needs its factor and its coefficient");
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(kGsRows + 128) * kGsPitch * sizeof(float);
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)combine_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set[ctx->device] = true;
    }
    const int64_t cover = (Zclr && zrows > rows) ? zrows : rows;
    hipLaunchKernelGGL(combine_kernel, dim3((unsigned)ceil_div64(cover, kGsRows)), dim3(256), lds, ctx->stream, A1, B1, A2, P,
                       alpha_dev, C, rows, b, Zclr, zrows);
    return aser_check_launch(ctx, "combine");
}
