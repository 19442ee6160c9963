// Bandwidth-bound kernels of the ASER calibration path (gfx950): channel statistics for the
// smoothing step (Sec. 4.2), per-channel RTN with the target T = E_q + W_o (Eq. 12), the
// per-token activation quantizer (Sec. 5.1), and the layout helpers around the MFMA kernel.
// All of them stream their operands once with 16-byte accesses that are contiguous along the
// channel dimension; row reductions use wavefront shuffles.
#include "aser_internal.h"

namespace {

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// max over the workgroup (blockDim.x multiple of 64, at most 1024); red: >= 16 floats of LDS
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < nw; ++i) r = fmaxf(r, red[i]);
    __syncthreads();
    return r;
}

// ------------------------------------------------------------------------------------ fills
__global__ void fill_f32_kernel(float* p, int64_t rows, int64_t cols, int64_t ld, float v) {
    const int64_t total = rows * cols;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
        p[(i / cols) * ld + (i % cols)] = v;
}

__global__ void fill_zero_kernel(uint32_t* p, int64_t words) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

// ------------------------------------------------------------------------------------ column |.| sums
// Each thread owns one 16-byte column group and a strip of rows; fp64 partial sums go to
// abs_sum with one fp64 atomic per column and strip.
template <bool BF16>
__global__ __launch_bounds__(256) void col_abs_sum_kernel(const void* X, int64_t rows, int64_t n, int64_t ld,
                                                          int64_t rows_per_block, double* out, int64_t* count,
                                                          int64_t count_add) {
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int ESZ = BF16 ? 2 : 4;
    if (count && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
        atomicAdd((unsigned long long*)count, (unsigned long long)count_add);
    if (!out) return;
    const int64_t col = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
    if (col >= n) return;
    const int nc = (n - col >= VEC) ? VEC : (int)(n - col);
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < rows) ? r0 + rows_per_block : rows;
    const char* base = (const char*)X + col * ESZ;
    const bool vec_ok = nc == VEC && (((uintptr_t)base & 15) == 0) && (((ld * ESZ) & 15) == 0);
    double acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0;
    if (vec_ok) {
        int64_t r = r0;
        for (; r + 4 <= r1; r += 4) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *(const uint4*)(base + (r + u) * ld * ESZ);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    if (BF16) {
                        acc[2 * d] += (double)fabsf(bf16_lo(w[d]));
                        acc[2 * d + 1] += (double)fabsf(bf16_hi(w[d]));
                    } else {
                        acc[d] += (double)fabsf(__uint_as_float(w[d]));
                    }
                }
            }
        }
        for (; r < r1; ++r) {
            const uint4 v = *(const uint4*)(base + r * ld * ESZ);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (BF16) {
                    acc[2 * d] += (double)fabsf(bf16_lo(w[d]));
                    acc[2 * d + 1] += (double)fabsf(bf16_hi(w[d]));
                } else {
                    acc[d] += (double)fabsf(__uint_as_float(w[d]));
                }
            }
        }
    } else {
        for (int64_t r = r0; r < r1; ++r) {
            const char* q = base + r * ld * ESZ;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if (e < nc) {
                    const float x = BF16 ? __uint_as_float((uint32_t)(*(const uint16_t*)(q + 2 * e)) << 16)
                                         : *(const float*)(q + 4 * e);
                    acc[e] += (double)fabsf(x);
                }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        if (e < nc) atomicAdd(out + col + e, acc[e]);
}

// ------------------------------------------------------------------------------------ transpose
__global__ __launch_bounds__(256) void transpose_kernel(const float* A, int64_t rows, int64_t cols, int64_t lda,
                                                        float* At, int64_t ldat) {
    __shared__ float tile[64][65];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int64_t r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < rows && c < cols) ? A[r * lda + c] : 0.f;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int64_t c = c0 + i, r = r0 + tx;
        if (c < cols && r < rows) At[c * ldat + r] = tile[tx][i];
    }
}

// ------------------------------------------------------------------------------------ sum of squares
__global__ __launch_bounds__(256) void sumsq_kernel(const float* A, int64_t rows, int64_t cols, int64_t lda, double* out) {
    __shared__ double red[4];
    double acc = 0.0;
    const int64_t total = rows * cols;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const float v = A[(i / cols) * lda + (i % cols)];
        acc += (double)v * (double)v;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(out, red[0] + red[1] + red[2] + red[3]);
}

// ------------------------------------------------------------------------------------ weight RTN
// One workgroup per output row.  The row stays in registers between the absmax reduction and
// the quantization, so W is read from HBM once.  Integer decisions (scale, codes) are taken in
// IEEE fp32 with correctly rounded division and round-half-to-even.
template <int VPT>   // float4 per thread
__global__ __launch_bounds__(256) void rtn_kernel(const float* __restrict__ W, int64_t n, int64_t ldw,
                                                  const int32_t* __restrict__ idx, const float* __restrict__ mdiag, int f,
                                                  float qmax, int layout, uint8_t* __restrict__ codes, int64_t code_pitch,
                                                  float* __restrict__ scales, float* __restrict__ T, int64_t ldt) {
    extern __shared__ uint32_t smem_u32[];
    uint32_t* mask = smem_u32;                       // ceil(n / 32) words: 1 = outlier column
    float* red = (float*)(smem_u32 + ((n + 31) / 32));
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const int mask_words = (int)((n + 31) / 32);
    for (int i = tid; i < mask_words; i += 256) mask[i] = 0u;
    __syncthreads();
    for (int i = tid; i < f; i += 256) {
        const int c = idx[i];
        atomicOr(&mask[c >> 5], 1u << (c & 31));
    }
    __syncthreads();

    const float* wrow = W + row * ldw;
    const bool vec_ok = (((uintptr_t)wrow & 15) == 0) && ((n & 3) == 0);
    float4 v[VPT];
    uint32_t om[VPT];                                 // 4 outlier bits per float4
    float amax = 0.f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * 256 + tid) * 4;
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        om[u] = 0u;
        if (c < n) {
            if (vec_ok) {
                v[u] = *(const float4*)(wrow + c);
            } else {
                float t[4] = {0.f, 0.f, 0.f, 0.f};
                for (int e = 0; e < 4; ++e)
                    if (c + e < n) t[e] = wrow[c + e];
                v[u] = make_float4(t[0], t[1], t[2], t[3]);
            }
            // c is a multiple of 4, so the four bits sit in one mask word
            om[u] = (mask[c >> 5] >> (c & 31)) & 0xFu;
            const float a0 = (om[u] & 1u) ? 0.f : fabsf(v[u].x), a1 = (om[u] & 2u) ? 0.f : fabsf(v[u].y);
            const float a2 = (om[u] & 4u) ? 0.f : fabsf(v[u].z), a3 = (om[u] & 8u) ? 0.f : fabsf(v[u].w);
            amax = fmaxf(amax, fmaxf(fmaxf(a0, a1), fmaxf(a2, a3)));
        }
    }
    amax = block_max(amax, red);
    const float scale = (amax == 0.f) ? 1.f : amax / qmax;
    if (tid == 0) scales[row] = scale;

    uint8_t* crow = codes + row * code_pitch;
    float* trow = T ? T + row * ldt : nullptr;
    const bool t_vec = T && (((uintptr_t)trow & 15) == 0) && ((n & 3) == 0);
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * 256 + tid) * 4;
        if (c >= n) continue;
        const float w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
        float t[4];
        int q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if ((om[u] >> e) & 1u) {
                q[e] = 0;
                t[e] = (c + e < n) ? w[e] * mdiag[c + e] : 0.f;
            } else {
                float qf = rintf(w[e] / scale);
                qf = fminf(fmaxf(qf, -qmax), qmax);
                q[e] = (int)qf;
                t[e] = __fmaf_rn(-qf, scale, w[e]);
            }
        }
        if (layout == ASER_CODES_INT8) {
            if (vec_ok && (((uintptr_t)crow & 3) == 0)) {
                const uint32_t packed = (uint32_t)(q[0] & 0xFF) | ((uint32_t)(q[1] & 0xFF) << 8) |
                                        ((uint32_t)(q[2] & 0xFF) << 16) | ((uint32_t)(q[3] & 0xFF) << 24);
                *(uint32_t*)(crow + c) = packed;
            } else {
                for (int e = 0; e < 4; ++e)
                    if (c + e < n) crow[c + e] = (uint8_t)(q[e] & 0xFF);
            }
        } else {   // int4, n even: columns (c, c+1) -> byte c/2, low nibble = even column
            if (c + 1 < n) crow[c / 2] = (uint8_t)((q[0] & 0xF) | ((q[1] & 0xF) << 4));
            if (c + 3 < n) crow[c / 2 + 1] = (uint8_t)((q[2] & 0xF) | ((q[3] & 0xF) << 4));
        }
        if (trow) {
            if (t_vec) {
                *(float4*)(trow + c) = make_float4(t[0], t[1], t[2], t[3]);
            } else {
                for (int e = 0; e < 4; ++e)
                    if (c + e < n) trow[c + e] = t[e];
            }
        }
    }
}

// ------------------------------------------------------------------------------------ activation RTN
// One workgroup per token.  X' = X / m with an IEEE fp32 division, per-token absmax scale.
template <bool BF16, int VPT>   // 4-element groups per thread
__global__ __launch_bounds__(256) void act_rtn_kernel(const void* __restrict__ X, int64_t n, int64_t ldx,
                                                      const float* __restrict__ mdiag, float qmax,
                                                      int8_t* __restrict__ codes, float* __restrict__ scales) {
    __shared__ float red[16];
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    float4 v[VPT];
    float amax = 0.f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * 256 + tid) * 4;
        float t[4] = {0.f, 0.f, 0.f, 0.f};
        if (c < n) {
            for (int e = 0; e < 4; ++e) {
                if (c + e < n) {
                    float x;
                    if (BF16) x = __uint_as_float((uint32_t)(((const uint16_t*)X)[row * ldx + c + e]) << 16);
                    else x = ((const float*)X)[row * ldx + c + e];
                    t[e] = mdiag ? x / mdiag[c + e] : x;
                }
            }
        }
        v[u] = make_float4(t[0], t[1], t[2], t[3]);
        amax = fmaxf(amax, fmaxf(fmaxf(fabsf(t[0]), fabsf(t[1])), fmaxf(fabsf(t[2]), fabsf(t[3]))));
    }
    amax = block_max(amax, red);
    const float scale = (amax == 0.f) ? 1.f : amax / qmax;
    if (tid == 0) scales[row] = scale;
    int8_t* crow = codes + row * n;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * 256 + tid) * 4;
        if (c >= n) continue;
        const float t[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
        for (int e = 0; e < 4; ++e) {
            if (c + e < n) {
                float qf = rintf(t[e] / scale);
                qf = fminf(fmaxf(qf, -qmax), qmax);
                crow[c + e] = (int8_t)(int)qf;
            }
        }
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------- launchers
int aser_fill_f32(aser_ctx* ctx, float* p, int64_t rows, int64_t cols, int64_t ld, float v) {
    if (rows <= 0 || cols <= 0) return ASER_OK;
    const int64_t total = rows * cols;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_f32_kernel, dim3(blocks), dim3(256), 0, ctx->stream, p, rows, cols, ld, v);
    return aser_check_launch(ctx, "fill_f32");
}

int aser_fill_bytes(aser_ctx* ctx, void* p, size_t bytes) {
    if (bytes == 0) return ASER_OK;
    if (((uintptr_t)p & 3) || (bytes & 3)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "fill: unaligned");
    const int64_t words = (int64_t)(bytes / 4);
    const int blocks = (int)((words + 255) / 256 < 4096 ? (words + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, ctx->stream, (uint32_t*)p, words);
    return aser_check_launch(ctx, "fill_zero");
}

int aser_col_abs_sum_x(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                       double* abs_sum, int64_t* count) {
    const int vec = (x_dtype == ASER_DTYPE_BF16) ? 8 : 4;
    const int64_t groups = ceil_div64(n, vec);
    const int64_t gx = ceil_div64(groups, 256);
    int64_t rpb = 64;
    while (ceil_div64(rows, rpb) > 65535) rpb *= 2;
    const int64_t gy = ceil_div64(rows, rpb);
    dim3 grid((unsigned)gx, (unsigned)gy);
    if (x_dtype == ASER_DTYPE_BF16)
        hipLaunchKernelGGL(col_abs_sum_kernel<true>, grid, dim3(256), 0, ctx->stream, X, rows, n, ldx, rpb, abs_sum, count, rows);
    else
        hipLaunchKernelGGL(col_abs_sum_kernel<false>, grid, dim3(256), 0, ctx->stream, X, rows, n, ldx, rpb, abs_sum, count, rows);
    return aser_check_launch(ctx, "col_abs_sum_x");
}

int aser_col_abs_sum_w(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw, double* wsum) {
    const int64_t gx = ceil_div64(ceil_div64(n, 4), 256);
    int64_t rpb = 32;
    while (ceil_div64(m, rpb) > 65535) rpb *= 2;
    dim3 grid((unsigned)gx, (unsigned)ceil_div64(m, rpb));
    hipLaunchKernelGGL(col_abs_sum_kernel<false>, grid, dim3(256), 0, ctx->stream, (const void*)W, m, n, ldw, rpb, wsum,
                       (int64_t*)nullptr, (int64_t)0);
    return aser_check_launch(ctx, "col_abs_sum_w");
}

int aser_transpose_f32(aser_ctx* ctx, const float* A, int64_t rows, int64_t cols, int64_t lda, float* At, int64_t ldat) {
    dim3 grid((unsigned)ceil_div64(cols, 64), (unsigned)ceil_div64(rows, 64));
    hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, ctx->stream, A, rows, cols, lda, At, ldat);
    return aser_check_launch(ctx, "transpose");
}

int aser_sumsq_f32(aser_ctx* ctx, const float* A, int64_t rows, int64_t cols, int64_t lda, double* out) {
    const int64_t total = rows * cols;
    const int blocks = (int)((total + 4095) / 4096 < 2048 ? (total + 4095) / 4096 : 2048);
    hipLaunchKernelGGL(sumsq_kernel, dim3(blocks > 0 ? blocks : 1), dim3(256), 0, ctx->stream, A, rows, cols, lda, out);
    return aser_check_launch(ctx, "sumsq");
}

// ---------------------------------------------------------------------------------------- ABI: stage 3
extern "C" int aser_quantize_rtn(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                 const int32_t* idx, const float* mdiag, int32_t f, int32_t bits, int32_t layout,
                                 void* codes, float* scales, float* T, int64_t ldt) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!W || !codes || !scales) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: null pointer");
    if (m <= 0 || n <= 0 || ldw < n || (T && ldt < n)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: bad shape");
    if (f < 0 || f > n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: f out of range");
    if (f > 0 && (!idx || !mdiag)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: idx/mdiag needed when f > 0");
    if (bits != 4 && bits != 8) ASER_FAIL(ctx, ASER_ERR_DTYPE, "quantize_rtn: bits must be 4 or 8");
    if (layout != ASER_CODES_INT8 && layout != ASER_CODES_INT4_PACKED)
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: unknown code layout");
    if (layout == ASER_CODES_INT4_PACKED && (bits != 4 || (n & 1)))
        ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: packed int4 needs bits == 4 and even n");
    if (n > 32768) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: n > 32768 is not supported");
    if (((uintptr_t)W & 3) || ((uintptr_t)scales & 3) || (T && ((uintptr_t)T & 3)))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: misaligned pointer");
    ASER_TRY(aser_prepare_device(ctx));
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const int64_t pitch = (layout == ASER_CODES_INT8) ? n : n / 2;
    const size_t lds = (size_t)((n + 31) / 32) * 4 + 64;
    const int64_t groups = ceil_div64(n, 4);
    dim3 grid((unsigned)m);
#define ASER_RTN_LAUNCH(V)                                                                                     \
    hipLaunchKernelGGL(rtn_kernel<V>, grid, dim3(256), lds, ctx->stream, W, n, ldw, idx, mdiag, (int)f, qmax, \
                       (int)layout, (uint8_t*)codes, pitch, scales, T, ldt)
    if (groups <= 256 * 4) ASER_RTN_LAUNCH(4);
    else if (groups <= 256 * 8) ASER_RTN_LAUNCH(8);
    else if (groups <= 256 * 16) ASER_RTN_LAUNCH(16);
    else ASER_RTN_LAUNCH(32);
#undef ASER_RTN_LAUNCH
    return aser_check_launch(ctx, "rtn");
}

// ---------------------------------------------------------------------------------------- ABI: activation RTN
extern "C" int aser_quantize_act_rtn(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                                     const float* mdiag, int32_t bits, int8_t* codes, float* scales) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!X || !codes || !scales) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_act_rtn: null pointer");
    if (x_dtype != ASER_DTYPE_BF16 && x_dtype != ASER_DTYPE_F32) ASER_FAIL(ctx, ASER_ERR_DTYPE, "quantize_act_rtn: dtype");
    if (rows < 0 || n <= 0 || ldx < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_act_rtn: bad shape");
    if (bits < 2 || bits > 8) ASER_FAIL(ctx, ASER_ERR_DTYPE, "quantize_act_rtn: bits must be in [2, 8]");
    if (n > 32768) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_act_rtn: n > 32768 is not supported");
    if (rows == 0) return ASER_OK;
    ASER_TRY(aser_prepare_device(ctx));
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const int64_t groups = ceil_div64(n, 4);
    dim3 grid((unsigned)rows);
#define ASER_ACT_LAUNCH(B, V) \
    hipLaunchKernelGGL((act_rtn_kernel<B, V>), grid, dim3(256), 0, ctx->stream, X, n, ldx, mdiag, qmax, codes, scales)
    if (x_dtype == ASER_DTYPE_BF16) {
        if (groups <= 256 * 4) ASER_ACT_LAUNCH(true, 4);
        else if (groups <= 256 * 16) ASER_ACT_LAUNCH(true, 16);
        else ASER_ACT_LAUNCH(true, 32);
    } else {
        if (groups <= 256 * 4) ASER_ACT_LAUNCH(false, 4);
        else if (groups <= 256 * 16) ASER_ACT_LAUNCH(false, 16);
        else ASER_ACT_LAUNCH(false, 32);
    }
#undef ASER_ACT_LAUNCH
    return aser_check_launch(ctx, "act_rtn");
}
