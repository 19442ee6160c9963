// Measurement aid, not part of the method: the rate a loop of nothing but MFMA instructions reaches on this
// device, one workgroup of four wavefronts per compute unit (the occupancy of the Gram kernel and of the
// inference kernel, whose 256 accumulator registers per lane allow no more) or four per compute unit.  The
// shader clock drops under this load, so the figure sits well below the product of unit count, nominal clock
// and operations per cycle; bench.py prints it next to the nominal peak.
// A second pair of kinds runs the same number of MFMA instructions with the operand traffic of a 256 x 256 tile
// with 64-byte K steps around them and nothing else (no epilogue, no tails): per step and workgroup 32 KB of
// LDS-direct loads from a 32 MB operand image laid out and shared between workgroups like the tiles of the
// inference kernel, 16 fragment reads of 16 bytes per lane and wavefront, one wait and one barrier.  What this
// loop loses against the first is the price of moving the operands on this device (stalls and, mostly, a lower
// shader clock: the chip runs into its power limit), whatever the kernel around them does.
#include "aser_internal.h"
#include <type_traits>

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

constexpr int kTrafficStage = 32768, kTrafficStages = 4;
constexpr int64_t kTrafficImage = 2ll * 16 * 256 * 4096;          // two operands, 16 tiles of 256 rows x 4096 bytes

__global__ void traffic_fill_kernel(uint32_t* p, int64_t words) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < words; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = (mix((uint32_t)i) & 0x807F807Fu) | 0x3F803F80u;     // pairs of bf16 values of magnitude about one; as int8 codes, mixed bytes
}

// One step = two half-steps of 16 MFMA (4 x 4 fragments), 8 fragment reads for the next half-step and 4
// LDS-direct loads each; the loads of step s land in ring slot (s + 3) % 4, which is read three steps later.
template <bool INT8>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void mfma_traffic_kernel(const char* src, float* out, int steps) {
    extern __shared__ __align__(16) char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int i = tid; i < kTrafficStage * kTrafficStages / 4; i += 256) ((uint32_t*)smem)[i] = (mix((uint32_t)i * 977u + blockIdx.x) & 0x807F807Fu) | 0x3F803F80u;
    __syncthreads();
    const int tile = (blockIdx.x & 7) * 32 + (blockIdx.x >> 3);    // the workgroups of an XCD share two row tiles of the first operand
    v4i_t ra[2][4], rb[2][4];
    int offa[4], offb[4];
    const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 128;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r0 = wm0 + 32 * i + (lane & 31), r1 = wn0 + 32 * i + (lane & 31);
        offa[i] = r0 * 64 + (((lane >> 5) ^ ((r0 >> 2) & 3)) << 4);
        offb[i] = 16384 + r1 * 64 + (((lane >> 5) ^ ((r1 >> 2) & 3)) << 4);
        ra[0][i] = *(const v4i_t*)(smem + offa[i]);
        rb[0][i] = *(const v4i_t*)(smem + offb[i]);
        ra[1][i] = ra[0][i];
        rb[1][i] = rb[0][i];
    }
    const uint32_t ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const int ca = (lane & 3) ^ ((lane >> 4) & 3);
    const char* gp[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const int tsel = (t >> 2) ? tile % 16 : tile / 16;
        gp[t] = src + (int64_t)(t >> 2) * (kTrafficImage / 2) + ((int64_t)tsel * 256 + 16 * (4 * wave + (t & 3)) + (lane >> 2)) * 4096 + 16 * ca;
    }
    typename std::conditional<INT8, v16i_t, f32x16_t>::type acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0;
    int koff = 0;
    auto half = [&](int s, auto htag) {
        constexpr int H = decltype(htag)::value;
        const char* st = smem + (s & 3) * kTrafficStage;
        const uint32_t dst = ring + ((s + 3) & 3) * kTrafficStage;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int i = q >> 2, j = q & 3;
            if constexpr (INT8) acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ra[H][i], rb[H][j], acc[q], 0, 0, 0);
            else acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, ra[H][i]), __builtin_bit_cast(bf16x8_t, rb[H][j]), acc[q], 0, 0, 0);
            if (q < 4) ra[H ^ 1][q] = *(const v4i_t*)(st + (offa[q] ^ (H ? 0 : 32)));
            if (q >= 4 && q < 8) rb[H ^ 1][q - 4] = *(const v4i_t*)(st + (offb[q - 4] ^ (H ? 0 : 32)));
            if ((q & 3) == 3) {
                const int tt = 4 * H + (q >> 2);
                const uint32_t d = dst + (tt < 4 ? (4 * wave + tt) * 1024 : 16384 + (4 * wave + tt - 4) * 1024);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(d), "v"(gp[tt] + koff) : "memory", "m0");
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    for (int s = 0; s < steps; ++s) {
        half(s, std::integral_constant<int, 0>{});
        __builtin_amdgcn_s_waitcnt(0x0F78);                        // vmcnt(8): the loads of step s - 1 have landed
        __syncthreads();
        half(s, std::integral_constant<int, 1>{});
        koff = (koff + 64) & 4095;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) sum += (float)acc[i][e];
    const v4i_t sink = ra[0][0] ^ ra[1][1] ^ rb[0][2] ^ rb[1][3];
    out[blockIdx.x * 256 + tid] = sum + (float)(sink.x ^ sink.y ^ sink.z ^ sink.w);
}

}  // namespace

extern "C" int aser_mfma_rate_probe(aser_ctx* ctx, int32_t kind, int32_t workgroups_per_cu, int32_t iters, double* tops) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!tops) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "mfma_rate_probe: null pointer");
    if (kind < 0 || kind > 3) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "mfma_rate_probe: kind must be 0 (bf16), 1 (int8), 2 or 3 (the same with operand traffic)");
    if (workgroups_per_cu < 1 || workgroups_per_cu > 4 || iters < 1 || iters > 1000000)
        ASER_FAIL(ctx, ASER_ERR_SHAPE, "mfma_rate_probe: need 1 <= workgroups_per_cu <= 4 and 1 <= iters <= 1000000");
    const bool traffic = kind >= 2;
    if (traffic && workgroups_per_cu != 1) ASER_FAIL(ctx, ASER_ERR_SHAPE, "mfma_rate_probe: kinds 2 and 3 run one workgroup per compute unit");
    const int64_t wgs = 256 * (int64_t)workgroups_per_cu;
    const size_t need = (size_t)wgs * 256 * 4 + (traffic ? (size_t)kTrafficImage : 0) + kAserWsTail;
    if (!ctx->ws || ctx->ws_bytes < need) ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "mfma_rate_probe: workspace too small (%zu needed)", need);
    ASER_TRY(aser_prepare_device(ctx));
    const char* image = (const char*)ctx->ws + (size_t)wgs * 256 * 4;   // 1 KiB multiples: 16-byte aligned like the workspace
    if (traffic) {
        constexpr int kLds = kTrafficStage * kTrafficStages;
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)mfma_traffic_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)mfma_traffic_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, kLds));
        hipLaunchKernelGGL(traffic_fill_kernel, dim3(2048), dim3(256), 0, ctx->stream, (uint32_t*)image, kTrafficImage / 4);
        ASER_TRY(aser_check_launch(ctx, "traffic_fill"));
    }
    hipEvent_t e0, e1;
    ASER_HIP(ctx, hipEventCreate(&e0));
    ASER_HIP(ctx, hipEventCreate(&e1));
    float ms = 0.f;
    int st = ASER_OK;
    for (int rep = 0; rep < 2 && st == ASER_OK; ++rep) {         // the first launch warms up
        hipError_t e = hipEventRecord(e0, ctx->stream);
        const int n_it = rep ? iters : 16;
        if (kind == 3) hipLaunchKernelGGL(mfma_traffic_kernel<true>, dim3(256), dim3(256), kTrafficStage * kTrafficStages, ctx->stream, image, (float*)ctx->ws, (n_it + 1) / 2);
        else if (kind == 2) hipLaunchKernelGGL(mfma_traffic_kernel<false>, dim3(256), dim3(256), kTrafficStage * kTrafficStages, ctx->stream, image, (float*)ctx->ws, (n_it + 1) / 2);
        else if (kind == 1) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3((unsigned)wgs), dim3(256), 0, ctx->stream, (float*)ctx->ws, rep ? iters : 16);
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
    // kinds 2 and 3 take a step (32 instructions per wavefront) per two rounds
    const double rounds = traffic ? 2.0 * (double)((iters + 1) / 2) : (double)iters;
    const double ops = (double)wgs * 4.0 * rounds * 16.0 * ((kind & 1) ? 65536.0 : 32768.0);
    *tops = ops / ((double)ms * 1e-3) / 1e12;
    return ASER_OK;
}
