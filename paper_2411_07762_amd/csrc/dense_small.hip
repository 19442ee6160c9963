// Small dense factorisations that run in one workgroup with their matrices in LDS: the diagonal
// blocks of the blocked Cholesky (Eq. 5), the b x b Cholesky of the orthogonalisation, and the
// Jacobi eigen-solver of the Rayleigh-Ritz step of the truncated SVD (Eq. 6).  Plus a plain
// fp32 FMA product for "tall times small" updates.
#include "aser_internal.h"

namespace {

constexpr int kMaxB = 128;
constexpr int kLdsPitch = kMaxB + 1;

// ------------------------------------------------------------------------------------ Cholesky block
// D = R^T R on the upper part of a b x b block (b <= 128) together with R^-1, in one sweep.
//
// The 128 x 128 matrix lives in registers: thread (bi, bj) of the 16 x 16 thread grid holds the
// 8 x 8 block (bi, bj), upper blocks only.  Step j eliminates with pivot a_jj:
//   rows i > j  (Cholesky, right-looking):   a[i][k] -= a[j][i] * a[j][k] / a_jj      for k > j
//   rows i < j  (Gauss-Jordan on R):         c[i][k] -= c[i][j] * a[j][k] / a_jj      for k > j
// where rows above j are kept in the scaled form c[i][k] = a[i][k] / a_ii.  Both updates are the
// same rank-1 update with the "cross" through (j, j): column j above the diagonal and row j to
// its right.  The owners of the cross publish it through LDS (double buffered, one barrier per
// step).  Row j of R is cross / sqrt(a_jj); column j of R^-1 is -c[i][j] / sqrt(a_jj) above the
// diagonal and 1 / sqrt(a_jj) on it.  Rows and columns beyond b are padded with the identity.
// Publishes the cross of step jn = 8 jbn + jln (jln is a compile-time constant at every call site):
// column jn above the diagonal from the blocks (bi <= jbn, jbn), row jn from the blocks (jbn, bj >= jbn).
template <int JLN>
__device__ __forceinline__ void publish_cross(float* cross, const float (&a)[8][8], int bi, int bj, int jbn) {
    if (bj == jbn) {
        if (bi < jbn) {
            float4* dst = (float4*)(cross + 8 * bi);
            dst[0] = make_float4(a[0][JLN], a[1][JLN], a[2][JLN], a[3][JLN]);
            dst[1] = make_float4(a[4][JLN], a[5][JLN], a[6][JLN], a[7][JLN]);
        } else if (bi == jbn) {
#pragma unroll
            for (int r = 0; r < JLN; ++r) cross[8 * bi + r] = a[r][JLN];
#pragma unroll
            for (int c = JLN; c < 8; ++c) cross[8 * bj + c] = a[JLN][c];
        }
    } else if (bi == jbn && bj > jbn) {
        float4* dst = (float4*)(cross + 8 * bj);
        dst[0] = make_float4(a[JLN][0], a[JLN][1], a[JLN][2], a[JLN][3]);
        dst[1] = make_float4(a[JLN][4], a[JLN][5], a[JLN][6], a[JLN][7]);
    }
}

template <int JL>
__device__ __forceinline__ void chol_step(float (&a)[8][8], float (*cross)[128], float* Rs, float* Xs, int jb, int tid,
                                          int bi, int bj, bool upper, int b, int32_t* info, int32_t pivot_base) {
    const int j = 8 * jb + JL;
    const float* cr = cross[j & 1];
    float piv = cr[j];
    if (!(piv > 0.f)) {
        if (tid == 0 && j < b && info) atomicMin(info, pivot_base + j + 1);
        piv = 1.f;
    }
    const float rs = __builtin_amdgcn_rsqf(piv);      // 1 ulp: as good as the fp32 data it scales
    const float pinv = rs * rs;
    if (tid < 128) {
        const int k = tid;
        const float cv = cr[k];
        const float rv = (k == j) ? piv * rs : cv * rs;
        if (k >= j) Rs[j * kLdsPitch + k] = rv;
        Xs[k * kLdsPitch + j] = (k > j) ? 0.f : ((k == j) ? rs : -cv * rs);
    }
    if (upper) {
        // One uniform 8 x 8 rank-1 update per thread; factors outside the active region (columns
        // <= j, the pivot row) are zeroed instead of branching on the block position.
        const float4 v0 = *(const float4*)(cr + 8 * bi), v1 = *(const float4*)(cr + 8 * bi + 4);
        const float4 w0 = *(const float4*)(cr + 8 * bj), w1 = *(const float4*)(cr + 8 * bj + 4);
        float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        float w[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
        const float wscale = (bj < jb) ? 0.f : pinv;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            w[c] *= wscale;
            if (c <= JL) w[c] = (bj == jb) ? 0.f : w[c];
        }
        const float vpiv = v[JL];
        v[JL] = (bi == jb) ? 0.f : vpiv;
#pragma unroll
        for (int r = 0; r < 8; ++r)
#pragma unroll
            for (int c = 0; c < 8; ++c) a[r][c] -= v[r] * w[c];
        if (bi == jb) {                               // pivot row: keep it in the scaled form a[j][k] / a_jj
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const bool on = (bj > jb) || (c > JL);
                a[JL][c] *= on ? pinv : 1.f;
            }
        }
        const int jbn = jb + (JL == 7 ? 1 : 0);
        if (8 * jb + JL + 1 < 128) publish_cross<(JL + 1) & 7>(cross[(j + 1) & 1], a, bi, bj, jbn);
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void chol_block_kernel(float* D, int64_t ld, int b, float* Rinv, int32_t* info,
                                                         int32_t pivot_base) {
    // Results are staged in LDS and written out once at the end.
    extern __shared__ float sm[];
    float* Rs = sm;                                   // R, row j at Rs[j * pitch + k]
    float* Xs = sm + kMaxB * kLdsPitch;               // R^-1, entry (i, j) at Xs[i * pitch + j]
    float (*cross)[128] = (float (*)[128])(Xs + kMaxB * kLdsPitch);
    const int tid = threadIdx.x, bi = tid >> 4, bj = tid & 15;
    const bool upper = bi <= bj;
    float a[8][8];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int i = 8 * bi + r, k = 8 * bj + c;
            float v = (i == k) ? 1.f : 0.f;
            if (upper && i < b && k < b && k >= i) v = D[(int64_t)i * ld + k];
            a[r][c] = v;
        }
    if (upper) publish_cross<0>(cross[0], a, bi, bj, 0);
    __syncthreads();
    const int nblk = (b + 7) / 8;
    for (int jb = 0; jb < nblk; ++jb) {
        chol_step<0>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
        chol_step<1>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
        chol_step<2>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
        chol_step<3>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
        chol_step<4>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
        chol_step<5>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
        chol_step<6>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
        chol_step<7>(a, cross, Rs, Xs, jb, tid, bi, bj, upper, b, info, pivot_base);
    }
    // write out: R above the diagonal, R^T below it, and R^-1
    for (int t = tid; t < b * b; t += 256) {
        const int i = t / b, k = t % b;
        D[(int64_t)i * ld + k] = (k >= i) ? Rs[i * kLdsPitch + k] : Rs[k * kLdsPitch + i];
        Rinv[t] = (k >= i) ? Xs[i * kLdsPitch + k] : 0.f;
    }
}

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

int aser_chol_block(aser_ctx* ctx, float* D, int64_t ld, int b, float* Rinv, int32_t* info, int32_t pivot_base) {
    if (b <= 0 || b > kMaxB) ASER_FAIL(ctx, ASER_ERR_SHAPE, "chol_block: block size out of range");
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(2 * kMaxB * kLdsPitch + 2 * 128) * 4;
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)chol_block_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(chol_block_kernel, dim3(1), dim3(256), lds, ctx->stream, D, ld, b, Rinv, info, pivot_base);
    return aser_check_launch(ctx, "chol_block");
}

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
