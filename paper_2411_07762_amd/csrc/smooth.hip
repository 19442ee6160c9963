// Activation smoothing via outlier analysis (Sec. 4.2): channel scores Xbar * Wbar, the index set
// I_f of the f largest scores, the diagonal m of Eq. 11 and the outlier part W_o of W M.
// All statistics are fp64 so that the selected indices do not depend on summation order in
// any realistic case; ties go to the lower channel index.
#include "aser_internal.h"

namespace {

constexpr int kSelMaxN = 32768;

struct Cand {
    double s;
    int i;
};

// a beats b: larger score, or equal score and lower index
__device__ __forceinline__ bool beats(double sa, int ia, double sb, int ib) {
    return (sa > sb) || (sa == sb && ia < ib);
}

// The better of a lane's candidate and that of the lane a DPP pattern pairs it with.
template <int CTRL>
__device__ __forceinline__ void dpp_best(double& s, int& i) {
    const int lo = __double2loint(s), hi = __double2hiint(s);
    const int lo2 = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xF, 0xF, false);
    const int hi2 = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xF, 0xF, false);
    const int i2 = __builtin_amdgcn_update_dpp(i, i, CTRL, 0xF, 0xF, false);
    const double s2 = __hiloint2double(hi2, lo2);
    if (beats(s2, i2, s, i)) { s = s2; i = i2; }
}

// Best candidate of the wavefront, in every lane: four DPP steps inside each row of 16 lanes
// (lane ^ 1, lane ^ 2, rotations by 4 and 8), then the four row results through scalar registers.
__device__ __forceinline__ void wave_best(double& s, int& i) {
    dpp_best<0xB1>(s, i);      // quad_perm [1, 0, 3, 2]
    dpp_best<0x4E>(s, i);      // quad_perm [2, 3, 0, 1]
    dpp_best<0x124>(s, i);     // row_ror 4
    dpp_best<0x128>(s, i);     // row_ror 8
    const int lo = __double2loint(s), hi = __double2hiint(s);
    double bs = __hiloint2double(__builtin_amdgcn_readlane(hi, 0), __builtin_amdgcn_readlane(lo, 0));
    int bi = __builtin_amdgcn_readlane(i, 0);
#pragma unroll
    for (int r = 16; r < 64; r += 16) {
        const double rs = __hiloint2double(__builtin_amdgcn_readlane(hi, r), __builtin_amdgcn_readlane(lo, r));
        const int ri = __builtin_amdgcn_readlane(i, r);
        if (beats(rs, ri, bs, bi)) { bs = rs; bi = ri; }
    }
    s = bs;
    i = bi;
}

__global__ __launch_bounds__(256) void score_kernel(const double* abs_sum, const int64_t* count, const double* wsum,
                                                    int64_t m, int64_t n, double* score) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const double xbar = abs_sum[i] / (double)(*count);
    const double wbar = wsum[i] / (double)m;
    score[i] = xbar * wbar;
}

// One workgroup.  Every thread keeps its scores (channels tid, tid + 1024, ...) in registers with
// its current local best; each of the f rounds is a workgroup arg-max, after which only the
// winner's owner rescans its registers.  Then the smoothing diagonal of Eq. 11 is written.
template <int kSelThreads, int kSelPerThread>   // kSelThreads * kSelPerThread >= n
__global__ __launch_bounds__(kSelThreads) void select_kernel(const double* __restrict__ score,
                                                             const double* __restrict__ abs_sum,
                                                             const int64_t* __restrict__ count, int n, int f,
                                                             int32_t* __restrict__ idx, float* __restrict__ mdiag,
                                                             int32_t* __restrict__ no_candidate) {
    __shared__ double red_s[2][kSelThreads / 64];
    __shared__ int red_i[2][kSelThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    for (int i = tid; i < n; i += kSelThreads) mdiag[i] = 1.0f;

    double sc[kSelPerThread];
#pragma unroll
    for (int u = 0; u < kSelPerThread; ++u) {
        const int c = u * kSelThreads + tid;
        sc[u] = (c < n) ? score[c] : -1.0;          // scores are >= 0; -1 marks "absent / taken"
        if (!(sc[u] <= 1.7e308)) sc[u] = -1.0;      // NaN or +Inf (no tokens, or non-finite statistics): never a candidate
    }
    double best_s = -1.0;
    int best_i = 0x7FFFFFFF;
#pragma unroll
    for (int u = 0; u < kSelPerThread; ++u) {
        const int c = u * kSelThreads + tid;
        if (sc[u] >= 0.0 && beats(sc[u], c, best_s, best_i)) { best_s = sc[u]; best_i = c; }
    }

    for (int round = 0; round < f; ++round) {
        double s = best_s;
        int i = best_i;
        wave_best(s, i);
        // per-wave winners go to the buffer of this round's parity; every thread then finds the
        // overall winner itself, so one barrier per round is enough
        double* rs = red_s[round & 1];
        int* ri = red_i[round & 1];
        if (lane == 0) { rs[wave] = s; ri[wave] = i; }
        __syncthreads();
        double ws = rs[0];
        int wi = ri[0];
#pragma unroll
        for (int w = 1; w < kSelThreads / 64; ++w)
            if (beats(rs[w], ri[w], ws, wi)) { ws = rs[w]; wi = ri[w]; }
        // No candidate left (fewer than f channels with a finite score): the slot gets -1, which every
        // consumer of idx skips, and the flag makes the next synchronising call fail with a status.
        const bool none = wi < 0 || wi >= n;
        if (tid == 0) {
            idx[round] = none ? -1 : wi;
            if (none) *no_candidate = 1;
        }
        if (!none && (wi % kSelThreads) == tid) {    // owner: retire the winner, rescan
            best_s = -1.0;
            best_i = 0x7FFFFFFF;
#pragma unroll
            for (int u = 0; u < kSelPerThread; ++u) {
                const int c = u * kSelThreads + tid;
                if (c == wi) sc[u] = -1.0;
                if (sc[u] >= 0.0 && beats(sc[u], c, best_s, best_i)) { best_s = sc[u]; best_i = c; }
            }
        }
    }
    __syncthreads();
    if (f > 0) {
        // X_min over the selected channels (Eq. 11): one channel per thread (idx was written by thread 0
        // before the barrier above), then a workgroup minimum
        const double cnt = (double)(*count);
        double xmin = 1.0e300;
        for (int k = tid; k < f; k += kSelThreads) {
            const int c = idx[k];
            if (c < 0) continue;
            const double x = abs_sum[c] / cnt;
            xmin = x < xmin ? x : xmin;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double x2 = __shfl_xor(xmin, o, 64);
            xmin = x2 < xmin ? x2 : xmin;
        }
        if (lane == 0) red_s[0][wave] = xmin;
        __syncthreads();
        xmin = red_s[0][0];
#pragma unroll
        for (int w = 1; w < kSelThreads / 64; ++w) xmin = red_s[0][w] < xmin ? red_s[0][w] : xmin;
        for (int k = tid; k < f; k += kSelThreads) {
            const int c = idx[k];
            if (c >= 0) mdiag[c] = (float)((abs_sum[c] / cnt) / xmin);
        }
    }
}

__global__ __launch_bounds__(256) void gather_wo_kernel(const float* __restrict__ W, int64_t m, int64_t n, int64_t ldw,
                                                        const int32_t* __restrict__ idx, const float* __restrict__ mdiag,
                                                        int f, float* __restrict__ W_o) {
    const int64_t total = m * f;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x) {
        const int64_t o = t / f;
        const int k = (int)(t % f);
        const int c = idx[k];
        W_o[t] = (c >= 0 && c < n) ? W[o * ldw + c] * mdiag[c] : 0.f;
    }
}

}  // namespace

// The two fp64 arrays of n entries (column sums of |W|, scores) and the selection's status word, wherever
// they live: in the bound workspace (aser_smooth_outliers) or in this file's static array.
static int smooth_run(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw, const double* abs_sum,
                      const int64_t* count, int32_t f, int32_t* idx, float* mdiag, float* W_o, double* score,
                      double* wsum, double* sc_scratch, int32_t* sel_flag) {
    if (ctx->pending_sel_dev != sel_flag) ASER_TRY(aser_set_i32(ctx, sel_flag, 0));
    ctx->pending_sel_dev = sel_flag;
    double* sc = score ? score : sc_scratch;
    ASER_TRY(aser_fill_bytes(ctx, wsum, (size_t)n * 8));
    ASER_TRY(aser_col_abs_sum_w(ctx, W, m, n, ldw, wsum));
    hipLaunchKernelGGL(score_kernel, dim3((unsigned)ceil_div64(n, 256)), dim3(256), 0, ctx->stream, abs_sum, count,
                       (const double*)wsum, m, n, sc);
    ASER_TRY(aser_check_launch(ctx, "score"));
    // few threads for few channels: a round costs instructions per wavefront, and every wavefront
    // of the single workgroup repeats the same reduction
    if (n <= 4096)
        hipLaunchKernelGGL((select_kernel<256, 16>), dim3(1), dim3(256), 0, ctx->stream, (const double*)sc, abs_sum, count,
                           (int)n, (int)f, idx, mdiag, sel_flag);
    else if (n <= 16384)
        hipLaunchKernelGGL((select_kernel<512, 32>), dim3(1), dim3(512), 0, ctx->stream, (const double*)sc, abs_sum, count,
                           (int)n, (int)f, idx, mdiag, sel_flag);
    else
        hipLaunchKernelGGL((select_kernel<1024, 32>), dim3(1), dim3(1024), 0, ctx->stream, (const double*)sc, abs_sum, count,
                           (int)n, (int)f, idx, mdiag, sel_flag);
    ASER_TRY(aser_check_launch(ctx, "select"));
    if (W_o && f > 0) {
        const int64_t total = m * f;
        const int blocks = (int)(ceil_div64(total, 256) < 2048 ? ceil_div64(total, 256) : 2048);
        hipLaunchKernelGGL(gather_wo_kernel, dim3(blocks), dim3(256), 0, ctx->stream, W, m, n, ldw, (const int32_t*)idx,
                           (const float*)mdiag, (int)f, W_o);
        ASER_TRY(aser_check_launch(ctx, "gather_wo"));
    }
    return ASER_OK;
}

static int smooth_validate(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw, const double* abs_sum,
                           const int64_t* count, int32_t f, const int32_t* idx, const float* mdiag, const double* score) {
    if (!W || !abs_sum || !count || !mdiag) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "smooth_outliers: null pointer");
    if (m <= 0 || n <= 0 || ldw < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "smooth_outliers: bad shape");
    if (f < 0 || f > n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "smooth_outliers: f must be in [0, n]");
    if (f > 0 && !idx) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "smooth_outliers: idx is null");
    if (n > kSelMaxN) ASER_FAIL(ctx, ASER_ERR_SHAPE, "smooth_outliers: n > 32768 is not supported");
    if (((uintptr_t)abs_sum & 7) || ((uintptr_t)count & 7) || (score && ((uintptr_t)score & 7)))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "smooth_outliers: misaligned fp64/int64 pointer");
    return ASER_OK;
}

extern "C" int aser_smooth_outliers(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                    const double* abs_sum, const int64_t* count, int32_t f,
                                    int32_t* idx, float* mdiag, float* W_o, double* score) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    ASER_TRY(smooth_validate(ctx, W, m, n, ldw, abs_sum, count, f, idx, mdiag, score));
    const size_t need = align_up((size_t)n * 8, 256) * 2 + kAserWsTail;
    if (!ctx->ws || ctx->ws_bytes < need) ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "smooth_outliers: workspace too small");
    ASER_TRY(aser_prepare_device(ctx));
    // word 1 of the workspace tail: raised by the selection when it runs out of usable channels
    int32_t* sel_flag = (int32_t*)((char*)ctx->ws + ctx->ws_bytes - kAserWsTail) + 1;
    return smooth_run(ctx, W, m, n, ldw, abs_sum, count, f, idx, mdiag, W_o, score, (double*)ctx->ws,
                      (double*)((char*)ctx->ws + align_up((size_t)n * 8, 256)), sel_flag);
}

// ---------------------------------------------------------------------------------------------
// The same stage for callers that cannot allocate and therefore have no workspace to bind (code under
// HIP graph capture, serving loops, harnesses that forbid hipMalloc): the two fp64 arrays and the status
// word live in a static device array of fixed size instead.  Every device holds its own copy of the
// array at its own address, looked up once per device.
constexpr size_t kScratchColBytes = (size_t)kSelMaxN * 8;             // one fp64 per channel, n <= 32768
constexpr size_t kScratchBytes = 2 * kScratchColBytes + 256;          // |W| column sums, scores, status word
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

static void* g_scratch_ptr[16] = {nullptr};

extern "C" int aser_smooth_outliers_noalloc(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                            const double* abs_sum, const int64_t* count, int32_t f,
                                            int32_t* idx, float* mdiag, float* W_o, double* score) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    ASER_TRY(smooth_validate(ctx, W, m, n, ldw, abs_sum, count, f, idx, mdiag, score));
    if ((size_t)n * 8 > kScratchColBytes)
        ASER_FAIL(ctx, ASER_ERR_SHAPE, "smooth_outliers_noalloc: n = %lld exceeds the static scratch (%d channels)",
                  (long long)n, kSelMaxN);
    if (ctx->device < 0 || ctx->device >= 16)
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "smooth_outliers_noalloc: device index %d is outside [0, 16)", ctx->device);
    ASER_TRY(aser_prepare_device(ctx));
    if (!g_scratch_ptr[ctx->device]) {
        // the array's name is only a host-side handle: its device address comes from the runtime, with
        // the context's device current (aser_prepare_device has just made it so)
        void* p = nullptr;
        ASER_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) ASER_FAIL(ctx, ASER_ERR_HIP, "smooth_outliers_noalloc: no device address for the static scratch");
        g_scratch_ptr[ctx->device] = p;
    }
    char* base = (char*)g_scratch_ptr[ctx->device];
    // every call on this device shares the array and finds the last call's contents in it: the column
    // sums are cleared by smooth_run, the scores are overwritten, the status word is reset unless it is
    // still pending on this context
    return smooth_run(ctx, W, m, n, ldw, abs_sum, count, f, idx, mdiag, W_o, score, (double*)base,
                      (double*)(base + kScratchColBytes), (int32_t*)(base + 2 * kScratchColBytes));
}
