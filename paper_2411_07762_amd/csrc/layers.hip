// Algorithm 1's loop over the layers of a model with several layers in flight.  A layer's calibration is a
// dependent chain of a few hundred launches, most of them small (the block-row steps of the Cholesky
// factorisation, the products and factorisations of the subspace iteration); layers do not depend on one
// another once their inputs are stored, so the chains of different layers run side by side on different
// streams.  The host enqueues a whole layer without waiting and waits for a context only when it needs it
// for the next layer.
#include <time.h>
#include <stdio.h>
#include <vector>

#include "aser_internal.h"

namespace {

// Keeps one wavefront busy for about `ticks` ticks of the constant-rate wall clock (100 MHz), and no longer than
// `max_rounds` rounds of the loop whatever that clock does.
__global__ void delay_kernel(long long ticks, int max_rounds, long long* sink) {
    const long long t0 = wall_clock64();
    long long t = t0;
    for (int i = 0; i < max_rounds && t - t0 < ticks; ++i) {
        __builtin_amdgcn_s_sleep(32);
        t = wall_clock64();
    }
    if (sink && threadIdx.x == 0) *sink = t - t0;
}

// Host wall-clock ms of `reps` delay kernels on a (and, if given, as many on b), both streams idle before and after.
int timed_delays(hipStream_t a, hipStream_t b, bool use_b, int reps, double* ms) {
    if (hipStreamSynchronize(a) != hipSuccess || (use_b && hipStreamSynchronize(b) != hipSuccess)) return ASER_ERR_HIP;
    timespec t0, t1;
    clock_gettime(CLOCK_MONOTONIC, &t0);
    for (int i = 0; i < reps; ++i) {
        hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, a, (long long)20000, 1 << 16, (long long*)nullptr);
        if (use_b) hipLaunchKernelGGL(delay_kernel, dim3(1), dim3(64), 0, b, (long long)20000, 1 << 16, (long long*)nullptr);
    }
    if (hipGetLastError() != hipSuccess) return ASER_ERR_HIP;
    if (hipStreamSynchronize(a) != hipSuccess || (use_b && hipStreamSynchronize(b) != hipSuccess)) return ASER_ERR_HIP;
    clock_gettime(CLOCK_MONOTONIC, &t1);
    *ms = (t1.tv_sec - t0.tv_sec) * 1e3 + (t1.tv_nsec - t0.tv_nsec) * 1e-6;
    return ASER_OK;
}

// Bytes of workspace behind the stage calls' own scratch that the layer's intermediates take when the
// descriptor leaves them to the context (null G with activations given, null T, null S).
size_t intermediates_bytes(const aser_layer_desc& L) {
    size_t extra = 0;
    const size_t nn = align_up((size_t)L.n * L.n * 4, 256), mn = align_up((size_t)L.m * L.n * 4, 256);
    if (L.X && !L.G) extra += nn + align_up((size_t)L.n * 8, 256) + 256;
    if (!L.T) extra += mn;
    if (!L.S) extra += nn;
    return extra;
}

// make_ready (may be null): receives a new event that is recorded on the layer's stream behind its Gram update, for
// the layers that share its statistics (created here, behind the first argument checks; the caller destroys it).
// wait_for (may be null): the layer's first launch waits for it (the statistics' owner runs on another stream).
int enqueue_layer(aser_ctx* ctx, const aser_layer_desc& in, hipEvent_t* make_ready, hipEvent_t wait_for) {
    aser_layer_desc L = in;
    if (L.m <= 0 || L.n <= 0) ASER_FAIL(ctx, ASER_ERR_SHAPE, "calibrate_layers: bad shape");
    if (!L.X && !L.G) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "calibrate_layers: neither activations nor finished statistics");
    hipEvent_t stats_ready = nullptr;
    if (make_ready) {
        if (!L.X || !L.G || !L.abs_sum || !L.count)
            ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "calibrate_layers: a layer whose statistics others share keeps G, abs_sum and count in buffers of its own");
        ASER_TRY(aser_prepare_device(ctx));
        ASER_HIP(ctx, hipEventCreateWithFlags(make_ready, hipEventDisableTiming));
        stats_ready = *make_ready;
    }
    if (wait_for) {
        ASER_TRY(aser_prepare_device(ctx));
        ASER_HIP(ctx, hipStreamWaitEvent(ctx->stream, wait_for, 0));
    }
    if (intermediates_bytes(L) > 0) {
        // intermediates that the caller does not want to keep live in the context's workspace, behind what
        // the stage calls use for this shape (the status block stays at the very end)
        size_t off = aser_workspace_bytes(L.m, L.n, L.r, L.opts) - kAserWsTail;
        if (!ctx->ws || ctx->ws_bytes < off + intermediates_bytes(L) + kAserWsTail)
            ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "calibrate_layers: workspace too small (%zu needed)",
                      off + intermediates_bytes(L) + kAserWsTail);
        auto take = [&](size_t bytes) { char* p = (char*)ctx->ws + off; off += align_up(bytes, 256); return p; };
        if (L.X && !L.G) {
            L.G = (float*)take((size_t)L.n * L.n * 4);
            L.ldg = L.n;
            L.abs_sum = (double*)take((size_t)L.n * 8);
            L.count = (int64_t*)take(256);
            L.clear_stats = 1;
        }
        if (!L.T) { L.T = (float*)take((size_t)L.m * L.n * 4); L.ldt = L.n; }
        if (!L.S) { L.S = (float*)take((size_t)L.n * L.n * 4); L.lds = L.n; }
    }
    if (L.X) {
        if (L.clear_stats) {
            if (!L.G || L.ldg < L.n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "calibrate_layers: bad Gram matrix");
            ASER_TRY(aser_prepare_device(ctx));
            if (L.ldg == L.n) ASER_TRY(aser_fill_bytes(ctx, L.G, (size_t)L.n * L.n * 4));
            else ASER_TRY(aser_fill_f32(ctx, L.G, L.n, L.n, L.ldg, 0.f));
            if (L.abs_sum) ASER_TRY(aser_fill_bytes(ctx, L.abs_sum, (size_t)L.n * 8));
            if (L.count) ASER_TRY(aser_fill_bytes(ctx, L.count, 8));
        }
        ASER_TRY(aser_gram_accumulate(ctx, L.X, L.x_dtype, L.rows, L.n, L.ldx, L.G, L.ldg, L.abs_sum, L.count));
    }
    if (stats_ready) ASER_HIP(ctx, hipEventRecord(stats_ready, ctx->stream));
    ASER_TRY(aser_smooth_outliers(ctx, L.W, L.m, L.n, L.ldw, L.abs_sum, L.count, L.f, L.idx, L.mdiag, nullptr, nullptr));
    ASER_TRY(aser_quantize_rtn(ctx, L.W, L.m, L.n, L.ldw, L.idx, L.mdiag, L.f, L.bits, L.layout, L.codes, L.scales, L.T, L.ldt));
    ASER_TRY(aser_whiten(ctx, L.G, L.ldg, L.n, L.mdiag, L.damp, L.S, L.lds, nullptr));
    return aser_error_reconstruct_enqueue(ctx, L.T, L.m, L.n, L.ldt, L.S, L.lds, L.r, L.idx, L.f, L.opts, L.L_A, L.L_B, L.sigma);
}

}  // namespace

extern "C" int aser_calibrate_layers(aser_ctx* const* ctxs, int32_t n_ctx, aser_layer_desc* layers, int32_t n_layers) {
    constexpr int kMaxCtx = 64;
    if (!ctxs || n_ctx < 1 || n_ctx > kMaxCtx || n_layers < 0 || (n_layers > 0 && !layers)) return ASER_ERR_INVALID_ARG;
    for (int c = 0; c < n_ctx; ++c)
        if (!ctxs[c] || ctxs[c]->rec_pending) return ASER_ERR_INVALID_ARG;
    int first_bad = ASER_OK;
    int running[kMaxCtx];                                      // the layer in flight on each context, or -1
    for (int c = 0; c < n_ctx; ++c) running[c] = -1;
    int share = n_ctx < n_layers ? n_ctx : n_layers;
    for (int c = 0; c < n_ctx; ++c) ctxs[c]->share = share > 0 ? share : 1;
    // layers whose statistics a later layer takes over (stats_from) record an event behind their Gram update
    std::vector<hipEvent_t> ready;
    std::vector<char> wanted, stats_ok;
    try {                                                      // no exception crosses the ABI
        ready.assign((size_t)n_layers, (hipEvent_t)nullptr);
        wanted.assign((size_t)n_layers, 0);
        stats_ok.assign((size_t)n_layers, 0);
    } catch (...) {
        for (int c = 0; c < n_ctx; ++c) ctxs[c]->share = 1;
        return ASER_ERR_INVALID_ARG;
    }
    for (int k = 0; k < n_layers; ++k) {
        const int32_t from = layers[k].stats_from;
        if (from >= 1 && from <= k) wanted[(size_t)from - 1] = 1;
    }
    auto finish = [&](int c) {
        if (running[c] < 0) return;
        aser_layer_desc& L = layers[running[c]];
        L.status = aser_finish(ctxs[c], &L.err, &L.n_iter);
        if (L.status != ASER_OK && first_bad == ASER_OK) first_bad = L.status;
        running[c] = -1;
    };
    for (int k = 0; k < n_layers; ++k) {
        // the next layer goes to a free context, else to the first one whose stream has drained
        int c = -1;
        for (int i = 0; i < n_ctx && c < 0; ++i)
            if (running[i] < 0) c = i;
        while (c < 0) {
            for (int i = 0; i < n_ctx && c < 0; ++i)
                if (hipStreamQuery(ctxs[i]->stream) != hipErrorNotReady) c = i;   // drained, or an error that aser_finish reports
            if (c < 0) {
                const timespec nap = {0, 20000};
                nanosleep(&nap, nullptr);
            }
        }
        finish(c);
        aser_layer_desc& L = layers[k];
        L.err = 0.0;
        L.n_iter = 0;
        aser_ctx* ctx = ctxs[c];
        aser_layer_desc use = L;
        hipEvent_t wait_for = nullptr;
        L.status = ASER_OK;
        if (L.stats_from != 0) {
            const int32_t j = L.stats_from - 1;
            if (j < 0 || j >= k) {
                snprintf(ctx->err, sizeof(ctx->err), "calibrate_layers: stats_from of layer %d must name an earlier layer (1-based)", k);
                L.status = ASER_ERR_INVALID_ARG;
            } else if (!stats_ok[(size_t)j]) {
                snprintf(ctx->err, sizeof(ctx->err), "calibrate_layers: layer %d shares the statistics of layer %d, which was not started", k, j);
                L.status = ASER_ERR_INVALID_ARG;
            } else {
                const aser_layer_desc& O = layers[j];               // same input: same channel count
                if (O.n != L.n) {
                    snprintf(ctx->err, sizeof(ctx->err), "calibrate_layers: layers %d and %d share statistics but differ in n", k, j);
                    L.status = ASER_ERR_SHAPE;
                }
                use.X = nullptr;
                use.G = O.G; use.ldg = O.ldg; use.abs_sum = O.abs_sum; use.count = O.count;
                wait_for = ready[(size_t)j];
            }
        }
        if (L.status == ASER_OK) {
            L.status = enqueue_layer(ctx, use, wanted[(size_t)k] ? &ready[(size_t)k] : nullptr, wait_for);
            // later layers may take the statistics over when all five stages of their owner were enqueued
            stats_ok[(size_t)k] = (char)(wanted[(size_t)k] && ready[(size_t)k] && (L.status == ASER_OK) ? 1 : 0);
        }
        if (ctx->rec_pending) running[c] = k;
        else if (L.status != ASER_OK && first_bad == ASER_OK) first_bad = L.status;
    }
    for (int c = 0; c < n_ctx; ++c) finish(c);
    for (int c = 0; c < n_ctx; ++c) ctxs[c]->share = 1;
    for (hipEvent_t e : ready)
        if (e) (void)hipEventDestroy(e);                       // every stream that waited for it has drained
    return first_bad;
}

extern "C" size_t aser_layer_workspace_bytes(const aser_layer_desc* layer) {
    if (!layer || layer->m <= 0 || layer->n <= 0) return 0;
    return aser_workspace_bytes(layer->m, layer->n, layer->r, layer->opts) + intermediates_bytes(*layer);
}

extern "C" int aser_pick_concurrent_streams(int32_t device, void* const* candidates, int32_t n_candidates, int32_t want,
                                            int32_t* chosen, int32_t* n_chosen) {
    if (device < 0 || !candidates || n_candidates < 1 || want < 1 || !chosen || !n_chosen) return ASER_ERR_INVALID_ARG;
    if (hipSetDevice(device) != hipSuccess) return ASER_ERR_HIP;
    *n_chosen = 0;
    double single = 0.0;
    {
        double warm;
        const int st = timed_delays((hipStream_t)candidates[0], nullptr, false, 2, &warm);
        if (st != ASER_OK) return st;
    }
    for (int c = 0; c < n_candidates && *n_chosen < want; ++c) {
        hipStream_t sc = (hipStream_t)candidates[c];
        int st = timed_delays(sc, nullptr, false, 3, &single);
        if (st != ASER_OK) return st;
        bool ok = true;
        for (int k = 0; k < *n_chosen && ok; ++k) {
            double pair = 0.0;
            st = timed_delays((hipStream_t)candidates[chosen[k]], sc, true, 3, &pair);
            if (st != ASER_OK) return st;
            ok = pair < 1.5 * single;                        // serialised streams take twice as long
        }
        if (ok) chosen[(*n_chosen)++] = c;
    }
    return ASER_OK;
}
