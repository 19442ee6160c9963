// Remaining layer-output error of the quantized, compensated layer under activation quantization:
//     || X W^T  -  X'_q W~^T ||_F      over a sample of tokens,
// with X' = X M^-1 the smoothed activations (Eq. 10), X'_q their per-token RTN image (Sec. 5.1) and
// W~ = deq(Q(W_s)) + L_A L_B the compensated weight (end of Sec. 4.2).  This is the quantity that the
// paper's error figure plots per layer (Sec. 5.3: ||W X - W_q X_q||_F for RTN, the same norm after
// reconstruction for the other methods), in this library's tokens x channels orientation.
//
// Both outputs are contractions over the channel dimension, which is the contiguous dimension of
// every operand here (X rows, W rows, code rows).  The MFMA kernel of this library wants operands that
// are contiguous along the OTHER dimension (K-major), so each operand goes through one transposing
// pass that also does its element-wise work: dequantisation of the weight codes, widening of bf16,
// the division by M, dequantisation of the activation codes.  Then
//     W~^T += L_B^T L_A^T          (K = r)
//     Y     = (X^T)^T W^T          (K = n), ||Y||_F^2
//     err^2 = ||Y - (X'_q^T)^T W~^T||_F^2   formed tile by tile in the product's epilogue.
// All products are fp32-class (three bf16 MFMA products per fp32 product).
#include <math.h>

#include "aser_internal.h"

namespace {

// Wc[j][o] = code[o][j] * scale[o]: codes m x n (int8, or int4 pairs with the even column in the low
// nibble), output n x m.  64 x 64 tiles through LDS, both sides coalesced.
__global__ __launch_bounds__(256) void dequant_transpose_kernel(const uint8_t* __restrict__ codes, int layout,
                                                                const float* __restrict__ scales, int64_t m, int64_t n,
                                                                float* __restrict__ Wc) {
    __shared__ float tile[64][65];
    const int64_t o0 = (int64_t)blockIdx.y * 64, j0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t pitch = (layout == ASER_CODES_INT8) ? n : n / 2;
    for (int i = ty; i < 64; i += 4) {
        const int64_t o = o0 + i, j = j0 + tx;
        float v = 0.f;
        if (o < m && j < n) {
            int q;
            if (layout == ASER_CODES_INT8) {
                q = (int)(int8_t)codes[o * pitch + j];
            } else {
                const uint8_t b = codes[o * pitch + (j >> 1)];
                const int nib = (j & 1) ? (b >> 4) : (b & 0xF);
                q = (nib ^ 8) - 8;                       // two's-complement nibble
            }
            v = (float)q * scales[o];
        }
        tile[i][tx] = v;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int64_t j = j0 + i, o = o0 + tx;
        if (j < n && o < m) Wc[j * m + o] = tile[tx][i];
    }
}

// out[i][t] = f(X[t][i]) as fp32, X: rows x n (bf16 or fp32), out: n x rows.
//   MODE 0: the value itself           MODE 1: X[t][i] / mdiag[i] (IEEE division; x / 1 = x)
//   MODE 2: codes[t][i] * scales[t]    (X unused)
template <bool BF16, int MODE>
__global__ __launch_bounds__(256) void x_transpose_kernel(const void* __restrict__ X, int64_t rows, int64_t n, int64_t ldx,
                                                          const float* __restrict__ mdiag, const int8_t* __restrict__ codes,
                                                          const float* __restrict__ scales, float* __restrict__ out) {
    __shared__ float tile[64][65];
    const int64_t t0 = (int64_t)blockIdx.y * 64, i0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int a = ty; a < 64; a += 4) {
        const int64_t t = t0 + a, i = i0 + tx;
        float v = 0.f;
        if (t < rows && i < n) {
            if (MODE == 2) {
                v = (float)codes[t * n + i] * scales[t];
            } else {
                v = BF16 ? __uint_as_float((uint32_t)((const uint16_t*)X)[t * ldx + i] << 16) : ((const float*)X)[t * ldx + i];
                if (MODE == 1 && mdiag) v = v / mdiag[i];
            }
        }
        tile[a][tx] = v;
    }
    __syncthreads();
    for (int a = ty; a < 64; a += 4) {
        const int64_t i = i0 + a, t = t0 + tx;
        if (i < n && t < rows) out[i * rows + t] = tile[tx][a];
    }
}

__global__ __launch_bounds__(256) void sumsq_f32_kernel(const float* __restrict__ p, int64_t total, double* __restrict__ out) {
    __shared__ double red[4];
    double acc = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const double v = (double)p[i];
        acc += v * v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(out, red[0] + red[1] + red[2] + red[3]);
}

struct EvalPlan {
    size_t off_wt, off_wc, off_xt, off_xq, off_y, off_lat, off_codes, off_scales, off_scal, total;
};

void eval_plan(int64_t m, int64_t n, int64_t rows, int r, EvalPlan* p) {
    size_t off = 0;
    p->off_wt = off; off += align_up((size_t)m * n * 4, 256);
    p->off_wc = off; off += align_up((size_t)m * n * 4, 256);
    p->off_xt = off; off += align_up((size_t)rows * n * 4, 256);
    p->off_xq = off; off += align_up((size_t)rows * n * 4, 256);
    p->off_y = off; off += align_up((size_t)rows * m * 4, 256);
    p->off_lat = off; off += align_up((size_t)(r > 0 ? r : 1) * m * 4, 256);
    p->off_codes = off; off += align_up((size_t)rows * n, 256);
    p->off_scales = off; off += align_up((size_t)rows * 4, 256);
    p->off_scal = off; off += 256;
    p->total = off;
}

}  // namespace

extern "C" size_t aser_output_error_workspace_bytes(int64_t m, int64_t n, int64_t rows, int32_t r) {
    if (m <= 0 || n <= 0 || rows <= 0 || r < 0) return 0;
    EvalPlan p;
    eval_plan(m, n, rows, r, &p);
    return p.total + kAserWsTail;
}

extern "C" int aser_layer_output_error(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                       const void* X, int x_dtype, int64_t rows, int64_t ldx, const float* mdiag,
                                       const void* codes, int32_t layout, const float* scales,
                                       const float* L_A, const float* L_B, int32_t r, int32_t act_bits,
                                       double* err, double* ref_norm) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!W || !X || !codes || !scales || !err) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "layer_output_error: null pointer");
    if (x_dtype != ASER_DTYPE_BF16 && x_dtype != ASER_DTYPE_F32) ASER_FAIL(ctx, ASER_ERR_DTYPE, "layer_output_error: dtype must be bf16 or f32");
    if (m <= 0 || n <= 0 || rows <= 0 || ldw < n || ldx < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "layer_output_error: bad shape");
    if (r < 0 || (r > 0 && (!L_A || !L_B))) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "layer_output_error: r > 0 needs L_A and L_B");
    if (layout != ASER_CODES_INT8 && layout != ASER_CODES_INT4_PACKED)
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "layer_output_error: unknown code layout");
    if (layout == ASER_CODES_INT4_PACKED && (n & 1)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "layer_output_error: packed int4 needs even n");
    if (act_bits != 0 && (act_bits < 2 || act_bits > 8)) ASER_FAIL(ctx, ASER_ERR_DTYPE, "layer_output_error: act_bits must be 0 or in [2, 8]");
    if (n > 32768) ASER_FAIL(ctx, ASER_ERR_SHAPE, "layer_output_error: n > 32768 is not supported");
    if (((uintptr_t)W & 3) || ((uintptr_t)scales & 3) || ((uintptr_t)X & (x_dtype == ASER_DTYPE_BF16 ? 1 : 3)))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "layer_output_error: misaligned pointer");
    EvalPlan pl;
    eval_plan(m, n, rows, r, &pl);
    if (!ctx->ws || ctx->ws_bytes < pl.total + kAserWsTail)
        ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "layer_output_error: workspace too small (%zu needed)", pl.total + kAserWsTail);
    ASER_TRY(aser_prepare_device(ctx));
    char* ws = (char*)ctx->ws;
    float* Wt = (float*)(ws + pl.off_wt);
    float* Wc = (float*)(ws + pl.off_wc);
    float* Xt = (float*)(ws + pl.off_xt);
    float* Xq = (float*)(ws + pl.off_xq);
    float* Y = (float*)(ws + pl.off_y);
    float* LAt = (float*)(ws + pl.off_lat);
    int8_t* acodes = (int8_t*)(ws + pl.off_codes);
    float* ascales = (float*)(ws + pl.off_scales);
    double* scal = (double*)(ws + pl.off_scal);           // [0] = ||Y||^2, [1] = err^2
    const bool bf16 = x_dtype == ASER_DTYPE_BF16;

    ASER_TRY(aser_fill_bytes(ctx, scal, 256));
    // weights: W^T and W~^T = deq(codes)^T + L_B^T L_A^T
    ASER_TRY(aser_transpose_f32(ctx, W, m, n, ldw, Wt, m));
    {
        dim3 grid((unsigned)ceil_div64(n, 64), (unsigned)ceil_div64(m, 64));
        hipLaunchKernelGGL(dequant_transpose_kernel, grid, dim3(256), 0, ctx->stream, (const uint8_t*)codes, (int)layout, scales,
                           m, n, Wc);
        ASER_TRY(aser_check_launch(ctx, "dequant_transpose"));
    }
    if (r > 0) {
        ASER_TRY(aser_transpose_f32(ctx, L_A, m, r, r, LAt, m));
        GemmArgs g{};
        g.A = L_B; g.lda = n; g.B = LAt; g.ldb = m; g.C = Wc; g.ldc = m;
        g.M = n; g.N = m; g.K = r; g.alpha = 1.f;
        g.in_type = GEMM_IN_F32X3; g.epi = GEMM_EPI_RMW; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_FULL;
        g.k_parts = 1; g.bm = 128; g.bn = 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
    }
    // activations: X^T and the (quantized, dequantized) smoothed activations transposed
    dim3 xgrid((unsigned)ceil_div64(n, 64), (unsigned)ceil_div64(rows, 64));
    if (bf16)
        hipLaunchKernelGGL((x_transpose_kernel<true, 0>), xgrid, dim3(256), 0, ctx->stream, X, rows, n, ldx, mdiag,
                           (const int8_t*)nullptr, (const float*)nullptr, Xt);
    else
        hipLaunchKernelGGL((x_transpose_kernel<false, 0>), xgrid, dim3(256), 0, ctx->stream, X, rows, n, ldx, mdiag,
                           (const int8_t*)nullptr, (const float*)nullptr, Xt);
    ASER_TRY(aser_check_launch(ctx, "x_transpose"));
    if (act_bits == 0) {
        if (bf16)
            hipLaunchKernelGGL((x_transpose_kernel<true, 1>), xgrid, dim3(256), 0, ctx->stream, X, rows, n, ldx, mdiag,
                               (const int8_t*)nullptr, (const float*)nullptr, Xq);
        else
            hipLaunchKernelGGL((x_transpose_kernel<false, 1>), xgrid, dim3(256), 0, ctx->stream, X, rows, n, ldx, mdiag,
                               (const int8_t*)nullptr, (const float*)nullptr, Xq);
    } else {
        ASER_TRY(aser_quantize_act_rtn(ctx, X, x_dtype, rows, n, ldx, mdiag, act_bits, acodes, ascales));
        hipLaunchKernelGGL((x_transpose_kernel<false, 2>), xgrid, dim3(256), 0, ctx->stream, (const void*)nullptr, rows, n, ldx,
                           mdiag, (const int8_t*)acodes, (const float*)ascales, Xq);
    }
    ASER_TRY(aser_check_launch(ctx, "x_transpose_q"));
    // Y = X W^T, its norm, and the residual against the compensated output
    {
        GemmArgs g{};
        g.A = Xt; g.lda = rows; g.B = Wt; g.ldb = m; g.C = Y; g.ldc = m;
        g.M = rows; g.N = m; g.K = n; g.alpha = 1.f;
        g.in_type = GEMM_IN_F32X3; g.epi = GEMM_EPI_STORE; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_FULL;
        g.k_parts = 1;
        g.bm = g.bn = (rows >= 2048 && m >= 2048) ? 256 : 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
    }
    {
        const int64_t total = rows * m;
        const int blocks = (int)(ceil_div64(total, 256 * 8) < 2048 ? ceil_div64(total, 256 * 8) : 2048);
        hipLaunchKernelGGL(sumsq_f32_kernel, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, ctx->stream, (const float*)Y, total, scal);
        ASER_TRY(aser_check_launch(ctx, "sumsq"));
    }
    {
        GemmArgs g{};
        g.A = Xq; g.lda = rows; g.B = Wc; g.ldb = m; g.C = Y; g.ldc = m;
        g.M = rows; g.N = m; g.K = n; g.alpha = -1.f; g.sumsq = scal + 1;
        g.in_type = GEMM_IN_F32X3; g.epi = GEMM_EPI_RESID; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_FULL;
        g.k_parts = 1; g.bm = 128; g.bn = 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
    }
    double h[2] = {0.0, 0.0};
    ASER_HIP(ctx, hipMemcpyAsync(h, scal, sizeof(h), hipMemcpyDeviceToHost, ctx->stream));
    ASER_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (!(h[0] >= 0.0) || !(h[1] >= 0.0)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "layer_output_error: non-finite values in the inputs");
    *err = sqrt(h[1]);
    if (ref_norm) *ref_norm = sqrt(h[0]);
    return ASER_OK;
}
