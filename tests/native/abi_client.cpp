// A caller of libaser.so that knows nothing of Python or PyTorch: plain HIP allocations and streams, the five
// stage calls of include/aser.h on one small seeded layer, then the same layer twice through
// aser_calibrate_layers on two contexts.  Checks on the host, in double precision, what follows from the
// definitions alone: deq(codes) + T = W M entry by entry (Eq. 12), the outlier set against the scores computed
// here, and that the two ways of driving the library agree.  Exit status 0 and "abi_client ok" on success.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <vector>

#include "aser.h"

#define HIP_OK(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) { printf("%s: %s\n", #call, hipGetErrorString(e_)); return 2; } \
    } while (0)
#define ASER_CALL(ctx, call)                                                              \
    do {                                                                                  \
        int s_ = (call);                                                                  \
        if (s_ != ASER_OK) { printf("%s: status %d (%s)\n", #call, s_, aser_last_error(ctx)); return 3; } \
    } while (0)

static uint32_t lcg(uint32_t* s) { *s = *s * 1664525u + 1013904223u; return *s; }
static float unif(uint32_t* s) { return (float)(lcg(s) >> 8) * (1.0f / 16777216.0f); }
static float gauss(uint32_t* s) {
    const float u1 = unif(s) + 1e-7f, u2 = unif(s);
    return sqrtf(-2.0f * logf(u1)) * cosf(6.2831853f * u2);
}

template <typename T>
static T* dev_alloc(size_t count) {
    void* p = nullptr;
    if (hipMalloc(&p, count * sizeof(T) + 256) != hipSuccess) { printf("hipMalloc failed\n"); exit(2); }
    return (T*)p;
}

struct Layer {
    float *G, *mdiag, *scales, *T, *S, *L_A, *L_B, *sigma;
    double* abs_sum;
    int64_t* count;
    int32_t* idx;
    int8_t* codes;
};

static Layer make_layer(int64_t m, int64_t n, int r, int f) {
    Layer L;
    L.G = dev_alloc<float>(n * n); L.mdiag = dev_alloc<float>(n); L.scales = dev_alloc<float>(m);
    L.T = dev_alloc<float>(m * n); L.S = dev_alloc<float>(n * n); L.L_A = dev_alloc<float>(m * r);
    L.L_B = dev_alloc<float>(r * n); L.sigma = dev_alloc<float>(r); L.abs_sum = dev_alloc<double>(n);
    L.count = dev_alloc<int64_t>(1); L.idx = dev_alloc<int32_t>(f); L.codes = dev_alloc<int8_t>(m * n);
    return L;
}

int main() {
    const int64_t m = 192, n = 320, N = 1500;
    const int r = 24, f = 6, bits = 4;
    uint32_t seed = 20241107u;
    std::vector<float> W(m * n), X(N * n);
    for (auto& w : W) w = 0.02f * gauss(&seed);
    for (auto& x : X) x = gauss(&seed);
    const int planted[3] = {5, 131, 300};
    for (int64_t t = 0; t < N; ++t)
        for (int p : planted) X[t * n + p] *= 30.0f;

    HIP_OK(hipSetDevice(0));
    float* dW = dev_alloc<float>(m * n);
    float* dX = dev_alloc<float>(N * n);
    HIP_OK(hipMemcpy(dW, W.data(), W.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dX, X.data(), X.size() * 4, hipMemcpyHostToDevice));

    // ---- the five stage calls on one context and stream
    hipStream_t s0;
    HIP_OK(hipStreamCreate(&s0));
    aser_ctx* ctx = nullptr;
    if (aser_create(&ctx, 0, s0) != ASER_OK) { printf("aser_create failed\n"); return 3; }
    const size_t ws_bytes = aser_workspace_bytes(m, n, r, nullptr);
    void* ws = dev_alloc<char>(ws_bytes + 256);
    ws = (void*)(((uintptr_t)ws + 255) & ~(uintptr_t)255);
    ASER_CALL(ctx, aser_set_workspace(ctx, ws, ws_bytes));
    Layer A = make_layer(m, n, r, f);
    HIP_OK(hipMemsetAsync(A.G, 0, n * n * 4, s0));
    HIP_OK(hipMemsetAsync(A.abs_sum, 0, n * 8, s0));
    HIP_OK(hipMemsetAsync(A.count, 0, 8, s0));
    ASER_CALL(ctx, aser_gram_accumulate(ctx, dX, ASER_DTYPE_F32, N, n, n, A.G, n, A.abs_sum, A.count));
    ASER_CALL(ctx, aser_smooth_outliers(ctx, dW, m, n, n, A.abs_sum, A.count, f, A.idx, A.mdiag, nullptr, nullptr));
    ASER_CALL(ctx, aser_quantize_rtn(ctx, dW, m, n, n, A.idx, A.mdiag, f, bits, ASER_CODES_INT8, A.codes, A.scales, A.T, n));
    int32_t info = -1;
    ASER_CALL(ctx, aser_whiten(ctx, A.G, n, n, A.mdiag, 0.f, A.S, n, &info));
    double err = -1.0;
    int32_t n_iter = -1;
    ASER_CALL(ctx, aser_error_reconstruct(ctx, A.T, m, n, n, A.S, n, r, A.idx, f, nullptr, A.L_A, A.L_B, A.sigma, &err, &n_iter));
    if (info != 0 || !(err > 0.0) || !isfinite(err)) { printf("bad info %d or error %g\n", info, err); return 4; }

    // ---- host checks of what the definitions fix
    std::vector<int32_t> idx(f);
    std::vector<float> mdiag(n), scales(m), T(m * n);
    std::vector<int8_t> codes(m * n);
    HIP_OK(hipMemcpy(idx.data(), A.idx, f * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(mdiag.data(), A.mdiag, n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(scales.data(), A.scales, m * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(T.data(), A.T, m * n * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(codes.data(), A.codes, m * n, hipMemcpyDeviceToHost));
    std::vector<double> score(n);
    for (int64_t i = 0; i < n; ++i) {
        double xs = 0.0, wsum = 0.0;
        for (int64_t t = 0; t < N; ++t) xs += fabs((double)X[t * n + i]);
        for (int64_t o = 0; o < m; ++o) wsum += fabs((double)W[o * n + i]);
        score[i] = (xs / N) * (wsum / m);
    }
    std::vector<int32_t> order(n);
    for (int64_t i = 0; i < n; ++i) order[i] = (int32_t)i;
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return score[a] > score[b]; });
    for (int k = 0; k < f; ++k)
        if (idx[k] != order[k]) { printf("outlier %d: library %d, host %d\n", k, idx[k], order[k]); return 5; }
    for (int p : planted)
        if (std::find(idx.begin(), idx.end(), p) == idx.end()) { printf("planted channel %d not selected\n", p); return 5; }
    double worst = 0.0;
    for (int64_t o = 0; o < m; ++o)
        for (int64_t j = 0; j < n; ++j) {
            const double wm = (double)W[o * n + j] * (double)mdiag[j];
            const double back = (double)codes[o * n + j] * (double)scales[o] + (double)T[o * n + j];
            worst = fmax(worst, fabs(back - wm) / (fabs(wm) + 1e-12));
            if (abs((int)codes[o * n + j]) > 7) { printf("code out of the int4 range\n"); return 6; }
        }
    if (worst > 1e-5) { printf("deq + T != W M: %g\n", worst); return 6; }

    // ---- the passes around a caller's own weight quantizer (here: keep three decimal binary digits below the row maximum)
    float* dWs = dev_alloc<float>(m * n);
    float* dWq = dev_alloc<float>(m * n);
    ASER_CALL(ctx, aser_smoothed_weight(ctx, dW, m, n, n, A.idx, f, dWs, n));
    std::vector<float> Ws(m * n), Wq(m * n), T2(m * n);
    HIP_OK(hipMemcpy(Ws.data(), dWs, m * n * 4, hipMemcpyDeviceToHost));
    for (int64_t o = 0; o < m; ++o)
        for (int64_t j = 0; j < n; ++j) {
            const bool out = std::find(idx.begin(), idx.end(), (int32_t)j) != idx.end();
            if (Ws[o * n + j] != (out ? 0.f : W[o * n + j])) { printf("W_s differs at %ld %ld\n", (long)o, (long)j); return 9; }
            Wq[o * n + j] = ldexpf(rintf(ldexpf(Ws[o * n + j], 8)), -8);
        }
    HIP_OK(hipMemcpy(dWq, Wq.data(), m * n * 4, hipMemcpyHostToDevice));
    ASER_CALL(ctx, aser_quant_target(ctx, dW, m, n, n, A.mdiag, dWq, n, dWq, n));     // in place
    HIP_OK(hipMemcpy(T2.data(), dWq, m * n * 4, hipMemcpyDeviceToHost));
    for (int64_t i = 0; i < m * n; ++i) {
        const double want = (double)W[i] * (double)mdiag[i % n] - (double)Wq[i];
        if (fabs((double)T2[i] - want) > 1.2e-7 * fabs(want)) { printf("T = W M - W_q differs at %ld\n", (long)i); return 9; }
    }

    // ---- the same layer twice through aser_calibrate_layers, two contexts
    hipStream_t s1, s2;
    HIP_OK(hipStreamCreate(&s1));
    HIP_OK(hipStreamCreate(&s2));
    aser_ctx* cs[2] = {nullptr, nullptr};
    aser_create(&cs[0], 0, s1);
    aser_create(&cs[1], 0, s2);
    Layer B[2] = {make_layer(m, n, r, f), make_layer(m, n, r, f)};
    aser_layer_desc d[2];
    for (int k = 0; k < 2; ++k) {
        aser_layer_desc z = {};
        z.X = dX; z.x_dtype = ASER_DTYPE_F32; z.rows = N; z.ldx = n;        // G, T, S left to the context's workspace
        z.W = dW; z.m = m; z.n = n; z.ldw = n; z.f = f; z.bits = bits; z.idx = B[k].idx; z.mdiag = B[k].mdiag;
        z.layout = ASER_CODES_INT8; z.r = r; z.codes = B[k].codes; z.scales = B[k].scales;
        z.L_A = B[k].L_A; z.L_B = B[k].L_B; z.sigma = B[k].sigma;
        d[k] = z;
    }
    const size_t ws2_bytes = aser_layer_workspace_bytes(&d[0]);
    for (int k = 0; k < 2; ++k) {
        void* w2 = dev_alloc<char>(ws2_bytes + 256);
        w2 = (void*)(((uintptr_t)w2 + 255) & ~(uintptr_t)255);
        ASER_CALL(cs[k], aser_set_workspace(cs[k], w2, ws2_bytes));
    }
    const int st = aser_calibrate_layers(cs, 2, d, 2);
    if (st != ASER_OK) { printf("aser_calibrate_layers: %d / %d %d\n", st, d[0].status, d[1].status); return 7; }
    for (int k = 0; k < 2; ++k) {
        std::vector<int8_t> c2(m * n);
        std::vector<int32_t> i2(f);
        HIP_OK(hipMemcpy(c2.data(), B[k].codes, m * n, hipMemcpyDeviceToHost));
        HIP_OK(hipMemcpy(i2.data(), B[k].idx, f * 4, hipMemcpyDeviceToHost));
        if (c2 != codes || i2 != idx) { printf("layer %d in flight: codes or outlier set differ\n", k); return 8; }
        if (fabs(d[k].err - err) > 1e-5 * err) { printf("layer %d in flight: error %.9g against %.9g\n", k, d[k].err, err); return 8; }
    }
    printf("abi_client ok: whitened error %.6g, %d iterations, deq + T = W M to %.1e\n", err, n_iter, worst);
    return 0;
}
