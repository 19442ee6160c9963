// Context management and stage 1 (Gram accumulation, Eq. 5) of the C ABI.
#include <limits.h>
#include <new>

#include "aser_internal.h"

extern "C" const char* aser_status_string(int status) {
    switch (status) {
        case ASER_OK: return "ok";
        case ASER_ERR_INVALID_ARG: return "invalid argument";
        case ASER_ERR_SHAPE: return "bad shape";
        case ASER_ERR_DTYPE: return "unsupported dtype or bit width";
        case ASER_ERR_NOT_SPD: return "matrix is not positive definite";
        case ASER_ERR_NO_CONVERGE: return "no convergence";
        case ASER_ERR_WORKSPACE: return "workspace missing or too small";
        case ASER_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

extern "C" int aser_create(aser_ctx** out, int device, void* hip_stream) {
    if (!out || device < 0) return ASER_ERR_INVALID_ARG;
    aser_ctx* c = new (std::nothrow) aser_ctx();
    if (!c) return ASER_ERR_INVALID_ARG;
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    c->ws = nullptr;
    c->ws_bytes = 0;
    c->device_ready = false;
    c->precision = ASER_PRECISION_AUTO;
    c->pending_info_dev = nullptr;
    c->pending_sel_dev = nullptr;
    c->host_status = nullptr;
    c->rec_pending = false;
    c->rec_exact = false;
    c->rec_iters = 0;
    c->share = 1;
    c->err[0] = 0;
    *out = c;
    return ASER_OK;
}

extern "C" int aser_destroy(aser_ctx* ctx) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (ctx->host_status) (void)hipHostFree(ctx->host_status);
    delete ctx;
    return ASER_OK;
}

extern "C" int aser_set_precision(aser_ctx* ctx, int precision) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (precision != ASER_PRECISION_AUTO && precision != ASER_PRECISION_FAST && precision != ASER_PRECISION_EXACT)
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "set_precision: unknown mode %d", precision);
    ctx->precision = precision;
    return ASER_OK;
}

extern "C" const char* aser_last_error(const aser_ctx* ctx) { return ctx ? ctx->err : "null context"; }

extern "C" int aser_set_workspace(aser_ctx* ctx, void* dev_ptr, size_t bytes) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (dev_ptr && ((uintptr_t)dev_ptr & 255)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "set_workspace: pointer must be 256-byte aligned");
    if (!dev_ptr && bytes) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "set_workspace: null pointer with non-zero size");
    if (ctx->rec_pending) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "set_workspace: an enqueued aser_error_reconstruct still uses the workspace (aser_finish first)");
    int pending_status = ASER_OK;
    if (ctx->pending_info_dev || ctx->pending_sel_dev) {
        // deferred status words live in the old workspace: fetch them before that memory goes away
        AserPending pend;
        ASER_TRY(aser_sync_status(ctx, &pend));
        pending_status = aser_report_pending(ctx, pend, "set_workspace");
    }
    ctx->ws = dev_ptr;
    ctx->ws_bytes = dev_ptr ? (bytes & ~(size_t)255) : 0;   // whole 256-byte units: the status words sit at the end
    return pending_status;
}

extern "C" size_t aser_workspace_bytes(int64_t m, int64_t n, int32_t r, const aser_svd_opts* opts) {
    if (m <= 0 || n <= 0) return 0;
    size_t need = align_up((size_t)n * 8, 256) * 2;             // smoothing: column sums of |W|, scores
    const size_t chol = (size_t)128 * 128 * 4 + 512;            // whitening: inverse of a diagonal block, damping sum
    if (chol > need) need = chol;
    if (r > 0) {
        const size_t rec = aser_reconstruct_workspace(m, n, r, opts);
        if (rec > need) need = rec;
    }
    return need + kAserWsTail;                                  // the whitening's pivot flag sits behind everything
}

int aser_prepare_device(aser_ctx* ctx) {
    if (!ctx->device_ready) {
        ASER_HIP(ctx, hipSetDevice(ctx->device));
        if (!ctx->host_status) ASER_HIP(ctx, hipHostMalloc(&ctx->host_status, 64, hipHostMallocDefault));
        ctx->device_ready = true;
    } else {
        int cur = -1;
        ASER_HIP(ctx, hipGetDevice(&cur));
        if (cur != ctx->device) ASER_HIP(ctx, hipSetDevice(ctx->device));
    }
    return ASER_OK;
}

int aser_enqueue_status_copy(aser_ctx* ctx) {
    if (!ctx->ws || ctx->ws_bytes < kAserWsTail) return ASER_OK;   // no workspace: nothing can be pending
    ASER_TRY(aser_prepare_device(ctx));
    ASER_HIP(ctx, hipMemcpyAsync(ctx->host_status, aser_status_dev(ctx), sizeof(AserStatusBlock), hipMemcpyDeviceToHost, ctx->stream));
    return ASER_OK;
}

int aser_wait_status(aser_ctx* ctx, AserPending* p) {
    p->pivot = INT_MAX;
    p->sel = 0;
    p->qr = 0;
    p->res2 = 0.0;
    ASER_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (!ctx->ws || ctx->ws_bytes < kAserWsTail || !ctx->host_status) return ASER_OK;
    const AserStatusBlock* h = (const AserStatusBlock*)ctx->host_status;
    if (ctx->pending_info_dev) p->pivot = h->pivot;
    if (ctx->pending_sel_dev) p->sel = h->sel;
    p->qr = h->qr;
    p->res2 = h->res2;
    return ASER_OK;
}

int aser_sync_status(aser_ctx* ctx, AserPending* p) {
    ASER_TRY(aser_enqueue_status_copy(ctx));
    return aser_wait_status(ctx, p);
}

int aser_report_pending(aser_ctx* ctx, const AserPending& p, const char* who) {
    ctx->pending_info_dev = nullptr;
    ctx->pending_sel_dev = nullptr;
    if (p.sel != 0)
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG,
                  "smooth_outliers: fewer than f channels have a finite score (no tokens accumulated, or NaN/Inf in the "
                  "statistics or in W); reported by %s", who);
    if (p.pivot != INT_MAX && p.pivot != 0)
        ASER_FAIL(ctx, ASER_ERR_NOT_SPD, "whiten: non-positive pivot at index %d (reported by %s)", p.pivot, who);
    return ASER_OK;
}

int aser_check_launch(aser_ctx* ctx, const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) ASER_FAIL(ctx, ASER_ERR_HIP, "launch of %s failed: %s", what, hipGetErrorString(e));
    return ASER_OK;
}

extern "C" int aser_gram_accumulate(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                                    float* G, int64_t ldg, double* abs_sum, int64_t* count) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!X || !G) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gram_accumulate: null pointer");
    if (x_dtype != ASER_DTYPE_BF16 && x_dtype != ASER_DTYPE_F32) ASER_FAIL(ctx, ASER_ERR_DTYPE, "gram_accumulate: dtype must be bf16 or f32");
    if (rows < 0 || n <= 0 || ldx < n || ldg < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "gram_accumulate: bad shape");
    const uintptr_t xa = (x_dtype == ASER_DTYPE_BF16) ? 1 : 3;
    if (((uintptr_t)X & xa) || ((uintptr_t)G & 3) || (abs_sum && ((uintptr_t)abs_sum & 7)) || (count && ((uintptr_t)count & 7)))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gram_accumulate: misaligned pointer");
    if (rows == 0) return ASER_OK;
    ASER_TRY(aser_prepare_device(ctx));
    if (abs_sum || count) ASER_TRY(aser_col_abs_sum_x(ctx, X, x_dtype, rows, n, ldx, abs_sum, count));
    return aser_syrk_gram(ctx, X, x_dtype, rows, n, ldx, G, ldg);
}
