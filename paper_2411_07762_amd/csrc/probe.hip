// Measurement aid, not part of the method: the rate a loop of nothing but MFMA instructions reaches on this
// device, one workgroup of four wavefronts per compute unit (the occupancy of the Gram kernel and of the
// inference kernel, whose 256 accumulator registers per lane allow no more) or four per compute unit.  The
// shader clock drops under this load, so the figure sits well below the product of unit count, nominal clock
// and operations per cycle; bench.py prints it next to the nominal peak.
#include "aser_internal.h"

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));

// operands from a counter hash: every lane and register differs, the bits toggle like those of real data
__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

template <bool INT8>
__global__ __launch_bounds__(256) void mfma_rate_kernel(float* out, int iters) {
    const uint32_t t = blockIdx.x * 256u + threadIdx.x;
    float s = 0.f;
    if (INT8) {
        v16i_t acc[16];
        v4i_t a[4], b[4];
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) { a[i][e] = (int)mix(t * 32u + i * 4u + e); b[i][e] = (int)mix(t * 32u + 16u + i * 4u + e); }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i * 4 + j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) s += (float)acc[i][e];
    } else {
        f32x16_t acc[16];
        bf16x8_t a[4], b[4];
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t wa[4], wb[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // two bf16 values of magnitude about one per word (exponent bits fixed, sign and mantissa hashed)
                wa[e] = (mix(t * 32u + i * 4u + e) & 0x807F807Fu) | 0x3F803F80u;
                wb[e] = (mix(t * 32u + 16u + i * 4u + e) & 0x807F807Fu) | 0x3F803F80u;
            }
            a[i] = __builtin_bit_cast(bf16x8_t, make_uint4(wa[0], wa[1], wa[2], wa[3]));
            b[i] = __builtin_bit_cast(bf16x8_t, make_uint4(wb[0], wb[1], wb[2], wb[3]));
        }
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i * 4 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i * 4 + j], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) s += acc[i][e];
    }
    out[t] = s;
}

}  // namespace

extern "C" int aser_mfma_rate_probe(aser_ctx* ctx, int32_t kind, int32_t workgroups_per_cu, int32_t iters, double* tops) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!tops) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "mfma_rate_probe: null pointer");
    if (kind != 0 && kind != 1) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "mfma_rate_probe: kind must be 0 (bf16) or 1 (int8)");
    if (workgroups_per_cu < 1 || workgroups_per_cu > 4 || iters < 1 || iters > 1000000)
        ASER_FAIL(ctx, ASER_ERR_SHAPE, "mfma_rate_probe: need 1 <= workgroups_per_cu <= 4 and 1 <= iters <= 1000000");
    const int64_t wgs = 256 * (int64_t)workgroups_per_cu;
    if (!ctx->ws || ctx->ws_bytes < (size_t)wgs * 256 * 4 + kAserWsTail)
        ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "mfma_rate_probe: workspace too small (%zu needed)", (size_t)wgs * 256 * 4 + kAserWsTail);
    ASER_TRY(aser_prepare_device(ctx));
    hipEvent_t e0, e1;
    ASER_HIP(ctx, hipEventCreate(&e0));
    ASER_HIP(ctx, hipEventCreate(&e1));
    float ms = 0.f;
    int st = ASER_OK;
    for (int rep = 0; rep < 2 && st == ASER_OK; ++rep) {         // the first launch warms up
        hipError_t e = hipEventRecord(e0, ctx->stream);
        if (kind == 1) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3((unsigned)wgs), dim3(256), 0, ctx->stream, (float*)ctx->ws, rep ? iters : 16);
        else hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3((unsigned)wgs), dim3(256), 0, ctx->stream, (float*)ctx->ws, rep ? iters : 16);
        st = aser_check_launch(ctx, "mfma_rate");
        if (e == hipSuccess) e = hipEventRecord(e1, ctx->stream);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e != hipSuccess && st == ASER_OK) { snprintf(ctx->err, sizeof(ctx->err), "mfma_rate_probe: %s", hipGetErrorString(e)); st = ASER_ERR_HIP; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != ASER_OK) return st;
    const double ops = (double)wgs * 4.0 * (double)iters * 16.0 * (kind == 1 ? 65536.0 : 32768.0);
    *tops = ops / ((double)ms * 1e-3) / 1e12;
    return ASER_OK;
}
