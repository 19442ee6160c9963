// Symmetric eigen-solver for the Rayleigh-Ritz step of the truncated SVD (Eq. 6): all eigenpairs
// of a b x b matrix (b <= 128), eigenvalues descending.  Two kernels:
//
//   tridiag_kernel   one workgroup of 256 threads, the matrix lives in registers (8 x 8 elements per
//                    thread, rows and columns dealt cyclically).
//                    Householder tridiagonalisation M = Q T Q^T in fp32: per reflector one
//                    mat-vec reduced along 16-lane DPP rows, one rank-2 update, two barriers.
//   ritz_pair_kernel one wavefront per eigenvalue, b wavefronts spread over the chip.  In fp64:
//                    65-section on Sturm counts (8 rounds), twisted factorisation of T - lambda I
//                    (forward and backward recurrences side by side in two lanes), eigenvector from
//                    the twist index; then back-transformation through the b - 2 reflectors in fp32.
//
// The tridiagonal problem is solved in fp64 because the spectrum it sees (squared singular values
// of a quantisation-error matrix) has a dense bulk whose spacing is close to fp32 resolution of
// the largest eigenvalue; in fp64 the vectors of distinct eigenvalues come out orthogonal to about
// 1e-16 / relative gap.  If two eigenvalues are closer than 1e-8 of the spectral radius a flag is
// raised instead and the caller runs the Jacobi solver, which does not care about clusters.
#include <type_traits>

#include "aser_internal.h"

namespace {

constexpr int kB = 128;

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// sum over each row of 16 lanes, result in every lane of the row
__device__ __forceinline__ float row16_sum(float v) {
    v += dpp_f<0xB1>(v);     // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);     // quad_perm [2,3,0,1]
    v += dpp_f<0x124>(v);    // row_ror 4
    v += dpp_f<0x128>(v);    // row_ror 8
    return v;
}

__device__ __forceinline__ float wave_sum(float v) {
    v = row16_sum(v);
    const int iv = __float_as_int(v);
    return (__int_as_float(__builtin_amdgcn_readlane(iv, 0)) + __int_as_float(__builtin_amdgcn_readlane(iv, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(iv, 32)) + __int_as_float(__builtin_amdgcn_readlane(iv, 48)));
}

// 256 threads in a 16 x 16 grid, thread (ti, tj) holds a[s][c] = A[ti + 16 s][tj + 16 c], s, c = 0..7.
// The 16 lanes of a DPP row share their matrix rows, so the mat-vec reduction never leaves the row,
// and the cyclic layout lets every thread skip the slots that lie wholly inside the finished part
// (the work shrinks with the trailing block).  Vectors live in LDS in the same cyclic order
// (element i at (i % 16) * 8 + i / 16) so that a thread reads its 8 values as two float4.
__device__ __forceinline__ int cyc(int i) { return (i & 15) * 8 + (i >> 4); }

__global__ __launch_bounds__(256) void tridiag_kernel(const float* __restrict__ Mb, int b, float* __restrict__ refl /* [k][128] */,
                                                      float* __restrict__ tri /* d | e | tau, 128 each */,
                                                      int* __restrict__ cluster_flag) {
    // Everything the loop produces stays in LDS until the end: a global store inside the loop
    // would have to drain before each barrier.
    extern __shared__ __align__(16) float sm[];
    float (*xc)[kB] = (float (*)[kB])sm;        // [2][kB] column k of the current matrix (cyclic order), double-buffered
    float* pb = sm + 2 * kB;                    // tau * A v (cyclic order)
    float* td = pb + kB;
    float* te = td + kB;
    float* tt = te + kB;
    float* rs = tt + kB;                        // [b - 2][kB] reflectors (natural order)
    const int tid = threadIdx.x, lane = tid & 63;
    const int ti = tid >> 4, tj = tid & 15;

    float a[8][8];
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            // unconditional loads from clamped indices: all 128 of a thread are in flight together
            const int r = ti + 16 * s, q = tj + 16 * c;
            const int rc = r < b ? r : b - 1, qc = q < b ? q : b - 1;
            const float lo = Mb[rc * b + qc], up = Mb[qc * b + rc];
            a[s][c] = (r < b && q < b) ? 0.5f * (lo + up) : 0.f;
        }
    if (tid == 0) *cluster_flag = 0;
    if (tid < kB) { td[tid] = 0.f; te[tid] = 0.f; tt[tid] = 0.f; }
    if (tj == 0) {
        *(float4*)(xc[0] + 8 * ti) = make_float4(a[0][0], a[1][0], a[2][0], a[3][0]);
        *(float4*)(xc[0] + 8 * ti + 4) = make_float4(a[4][0], a[5][0], a[6][0], a[7][0]);
    }
    __syncthreads();

    for (int k = 0; k + 2 < b; ++k) {
        const float* cur = xc[k & 1];
        // reflector k annihilates A[k+2.., k]; lane l looks at cyclic positions l and l + 64
        const int i0 = ((lane >> 3) & 15) + 16 * (lane & 7), i1 = i0 + 8;      // natural indices of those positions
        const float x0 = cur[lane], x1 = cur[lane + 64];
        const float alpha = cur[cyc(k + 1)];
        const float sigma = wave_sum(((i0 > k + 1) ? x0 * x0 : 0.f) + ((i1 > k + 1) ? x1 * x1 : 0.f));
        float beta = alpha, tk = 0.f, scal = 0.f;
        if (sigma > 1e-30f * alpha * alpha && sigma > 0.f) {
            beta = -copysignf(sqrtf(alpha * alpha + sigma), alpha);
            tk = (beta - alpha) / beta;
            scal = 1.0f / (alpha - beta);
        }
        auto vat = [&](int idx, float x) { return (idx <= k) ? 0.f : ((idx == k + 1) ? 1.f : x * scal); };
        const int smin = (k + 1) >> 4;              // slots below hold only indices <= k
        float vr[8], vc[8];
        {
            const float4 ra = *(const float4*)(cur + 8 * ti), rb = *(const float4*)(cur + 8 * ti + 4);
            const float4 ca = *(const float4*)(cur + 8 * tj), cb = *(const float4*)(cur + 8 * tj + 4);
            const float xr[8] = {ra.x, ra.y, ra.z, ra.w, rb.x, rb.y, rb.z, rb.w};
            const float xq[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
#pragma unroll
            for (int s = 0; s < 8; ++s) { vr[s] = vat(ti + 16 * s, xr[s]); vc[s] = vat(tj + 16 * s, xq[s]); }
        }
        // p = tau * A v on the trailing block
        float ps[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) ps[s] = 0.f;
        // one uniform branch per step picks the body compiled for this number of finished slots
        auto matvec = [&](auto first) {
            constexpr int S0 = decltype(first)::value;
#pragma unroll
            for (int s = S0; s < 8; ++s) {
#pragma unroll
                for (int c = S0; c < 8; ++c) ps[s] += a[s][c] * vc[c];
                ps[s] = row16_sum(ps[s]);
                ps[s] = (ti + 16 * s > k) ? tk * ps[s] : 0.f;
            }
        };
        switch (smin) {
            case 0: matvec(std::integral_constant<int, 0>{}); break;
            case 1: matvec(std::integral_constant<int, 1>{}); break;
            case 2: matvec(std::integral_constant<int, 2>{}); break;
            case 3: matvec(std::integral_constant<int, 3>{}); break;
            case 4: matvec(std::integral_constant<int, 4>{}); break;
            case 5: matvec(std::integral_constant<int, 5>{}); break;
            case 6: matvec(std::integral_constant<int, 6>{}); break;
            default: matvec(std::integral_constant<int, 7>{}); break;
        }
        if (tj == 0) {
            *(float4*)(pb + 8 * ti) = make_float4(ps[0], ps[1], ps[2], ps[3]);
            *(float4*)(pb + 8 * ti + 4) = make_float4(ps[4], ps[5], ps[6], ps[7]);
#pragma unroll
            for (int s = 0; s < 8; ++s) rs[k * kB + ti + 16 * s] = vr[s];
        }
        if (tid == 0) { te[k] = beta; tt[k] = tk; }
        if (ti == (k & 15) && tj == (k & 15)) {
            float dv = a[0][0];
#pragma unroll
            for (int s = 1; s < 8; ++s)
                if ((k >> 4) == s) dv = a[s][s];
            td[k] = dv;
        }
        __syncthreads();
        // A -= v w^T + w v^T with w = p - (tau/2)(p^T v) v
        const float kk = wave_sum(pb[lane] * vat(i0, x0) + pb[lane + 64] * vat(i1, x1));
        const float a2 = -0.5f * tk * kk;
        float wr[8], wc[8];
        {
            const float4 ra = *(const float4*)(pb + 8 * ti), rb = *(const float4*)(pb + 8 * ti + 4);
            const float4 ca = *(const float4*)(pb + 8 * tj), cb = *(const float4*)(pb + 8 * tj + 4);
            const float pr[8] = {ra.x, ra.y, ra.z, ra.w, rb.x, rb.y, rb.z, rb.w};
            const float pq[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
#pragma unroll
            for (int s = 0; s < 8; ++s) { wr[s] = pr[s] + a2 * vr[s]; wc[s] = pq[s] + a2 * vc[s]; }
        }
        auto update = [&](auto first) {
            constexpr int S0 = decltype(first)::value;
#pragma unroll
            for (int s = S0; s < 8; ++s)
#pragma unroll
                for (int c = S0; c < 8; ++c) a[s][c] -= vr[s] * wc[c] + wr[s] * vc[c];
        };
        switch (smin) {
            case 0: update(std::integral_constant<int, 0>{}); break;
            case 1: update(std::integral_constant<int, 1>{}); break;
            case 2: update(std::integral_constant<int, 2>{}); break;
            case 3: update(std::integral_constant<int, 3>{}); break;
            case 4: update(std::integral_constant<int, 4>{}); break;
            case 5: update(std::integral_constant<int, 5>{}); break;
            case 6: update(std::integral_constant<int, 6>{}); break;
            default: update(std::integral_constant<int, 7>{}); break;
        }
        // next column to the other buffer
        if (tj == ((k + 1) & 15)) {
            const int cs = (k + 1) >> 4;
            float y[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                y[s] = a[s][0];
#pragma unroll
                for (int c = 1; c < 8; ++c)
                    if (cs == c) y[s] = a[s][c];
            }
            float* nxt = xc[(k + 1) & 1];
            *(float4*)(nxt + 8 * ti) = make_float4(y[0], y[1], y[2], y[3]);
            *(float4*)(nxt + 8 * ti + 4) = make_float4(y[4], y[5], y[6], y[7]);
        }
        __syncthreads();
    }
    // the last 2 x 2 block
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int r = ti + 16 * s, q = tj + 16 * c;
            if (r == q && (r == b - 1 || r == b - 2)) td[r] = a[s][c];
            if (r == b - 1 && q == b - 2) te[b - 2] = a[s][c];
        }
    __syncthreads();
    for (int t = tid; t < (b - 2) * kB; t += 256) refl[t] = rs[t];
    for (int t = tid; t < 3 * kB; t += 256) tri[t] = td[t];
}

__device__ __forceinline__ double fast_rcp(double q) {
    double r = __builtin_amdgcn_rcp(q);
    r = fma(fma(-q, r, 1.0), r, r);
    r = fma(fma(-q, r, 1.0), r, r);
    return r;
}

__device__ __forceinline__ double wave_max_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    return v;
}
__device__ __forceinline__ double wave_min_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmin(v, __shfl_xor(v, o, 64));
    return v;
}

// number of eigenvalues of the tridiagonal (d, e^2) below x
__device__ __forceinline__ int sturm_count(const double* d, const double* e2, int b, double x, double tiny) {
    double q = d[0] - x;
    if (fabs(q) < tiny) q = -tiny;
    int cnt = q < 0.0;
    for (int i = 1; i < b; ++i) {
        q = fma(-e2[i - 1], fast_rcp(q), d[i] - x);
        if (fabs(q) < tiny) q = -tiny;
        cnt += q < 0.0;
    }
    return cnt;
}

// One wavefront: eigenvalue number blockIdx.x (ascending) of the tridiagonal and its eigenvector,
// mapped back through the reflectors.  Writes lambda[b - 1 - m] and column b - 1 - m of Vout.
__global__ __launch_bounds__(64) void ritz_pair_kernel(const float* __restrict__ tri, const float* __restrict__ refl, int b,
                                                       float* __restrict__ lambda, float* __restrict__ Vout,
                                                       int* __restrict__ cluster_flag) {
    __shared__ double dd[kB], e2[kB], Dp[kB], Dm[kB], zz[kB];
    __shared__ float ef[kB], tau[kB];
    extern __shared__ __align__(16) float rl[];     // [b - 2][kB] reflectors, read once up front
    const int lane = threadIdx.x;
    const int m = blockIdx.x;
    // the reflectors, 16 float4 per lane in flight at a time
    for (int t0 = 0; t0 < (b - 2) * (kB / 4); t0 += 64 * 16) {
        float4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int t = t0 + u * 64 + lane;
            v[u] = (t < (b - 2) * (kB / 4)) ? ((const float4*)refl)[t] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int t = t0 + u * 64 + lane;
            if (t < (b - 2) * (kB / 4)) ((float4*)rl)[t] = v[u];
        }
    }

    double glo = 1e300, ghi = -1e300;
    for (int i = lane; i < kB; i += 64) {
        const float di = (i < b) ? tri[i] : 0.f;
        const float ei = (i + 1 < b) ? tri[kB + i] : 0.f;
        const float el = (i > 0 && i < b) ? tri[kB + i - 1] : 0.f;
        dd[i] = (double)di;
        e2[i] = (double)ei * (double)ei;
        ef[i] = ei;
        tau[i] = (i + 2 < b) ? tri[2 * kB + i] : 0.f;
        if (i < b) {
            const double rad = fabs((double)ei) + fabs((double)el);
            glo = fmin(glo, (double)di - rad);
            ghi = fmax(ghi, (double)di + rad);
        }
    }
    glo = wave_min_d(glo);
    ghi = wave_max_d(ghi);
    const double radius = fmax(fabs(glo), fabs(ghi));
    const double tiny = fmax(radius * 1e-60, 1e-290);
    __syncthreads();

    // ---- eigenvalue: 64 interior points per round
    double lo = glo - 1e-12 * radius - tiny, hi = ghi + 1e-12 * radius + tiny;
    for (int round = 0; round < 8; ++round) {
        const double x = lo + (hi - lo) * ((double)(lane + 1) * (1.0 / 65.0));
        const int cnt = sturm_count(dd, e2, b, x, tiny);
        const double clo = wave_max_d((cnt <= m) ? x : lo);
        const double chi = wave_min_d((cnt > m) ? x : hi);
        lo = clo;
        hi = chi;
    }
    const double lam = 0.5 * (lo + hi);
    int bad = 0;
    if (m + 1 < b) bad = sturm_count(dd, e2, b, lam + 1e-8 * radius, tiny) > m + 1;

    // ---- twisted factorisation: lane 0 runs D+ downwards, lane 1 runs D- upwards
    {
        const int dir = lane & 1;
        double q = 0.0;
        for (int t = 0; t < b; ++t) {
            const int i = dir ? (b - 1 - t) : t;
            const double dx = dd[i] - lam;
            q = (t == 0) ? dx : fma(-e2[dir ? i : i - 1], fast_rcp(q), dx);
            if (fabs(q) < tiny) q = tiny;
            if (lane < 2) (dir ? Dm : Dp)[i] = q;
        }
    }
    __syncthreads();
    int twist;
    {
        double best = 1e300;
        int bi = 0;
        for (int i = lane; i < b; i += 64) {
            const double g = fabs(Dp[i] + Dm[i] - (dd[i] - lam));
            if (g < best) { best = g; bi = i; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double ob = __shfl_xor(best, o, 64);
            const int oi = __shfl_xor(bi, o, 64);
            if (ob < best || (ob == best && oi < bi)) { best = ob; bi = oi; }
        }
        twist = bi;
    }
    // z_twist = 1; z_i = -(e_i / D+_i) z_{i+1} above it, z_i = -(e_{i-1} / D-_i) z_{i-1} below it
    for (int i = lane; i < b; i += 64) {
        double rat = 1.0;
        if (i < twist) rat = -(double)ef[i] * fast_rcp(Dp[i]);
        if (i > twist) rat = -(double)ef[i - 1] * fast_rcp(Dm[i]);
        zz[i] = rat;
    }
    __syncthreads();
    {
        const int dir = lane & 1;
        const int steps = max(twist, b - 1 - twist);
        double z = 1.0;
        for (int t = 1; t <= steps; ++t) {
            const int i = dir ? twist + t : twist - t;
            if (i >= 0 && i < b && lane < 2) {
                z *= zz[i];
                zz[i] = z;
            }
        }
    }
    __syncthreads();
    float y0, y1;
    {
        const double z0 = (lane < b) ? zz[lane] : 0.0, z1 = (lane + 64 < b) ? zz[lane + 64] : 0.0;
        double nrm = z0 * z0 + z1 * z1;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) nrm += __shfl_xor(nrm, o, 64);
        if (!(nrm < 1e300)) bad = 1;
        const double inv = 1.0 / sqrt(nrm);
        y0 = (float)(z0 * inv);
        y1 = (float)(z1 * inv);
    }
    if (bad && lane == 0) *cluster_flag = 1;

    // ---- back-transformation y <- H_0 H_1 ... H_{b-3} y
    if (b >= 3) {
        float v0 = rl[(b - 3) * kB + lane], v1 = rl[(b - 3) * kB + lane + 64];
        for (int k = b - 3; k >= 0; --k) {
            const int kn = k > 0 ? k - 1 : 0;
            const float n0 = rl[kn * kB + lane], n1 = rl[kn * kB + lane + 64];
            const float s = tau[k] * wave_sum(v0 * y0 + v1 * y1);
            y0 -= s * v0;
            y1 -= s * v1;
            v0 = n0;
            v1 = n1;
        }
    }
    const int c = b - 1 - m;
    if (lane == 0) lambda[c] = (float)lam;
    if (lane < b) Vout[lane * b + c] = y0;
    if (lane + 64 < b) Vout[(lane + 64) * b + c] = y1;
}

}  // namespace

int aser_tridiag_eig(aser_ctx* ctx, const float* Mb, int b, float* lambda, float* V, float* refl, float* tri, int* cluster_flag) {
    if (b < 2 || b > kB) ASER_FAIL(ctx, ASER_ERR_SHAPE, "sym_eig: block size must be in [2, 128]");
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(6 + (kB - 2)) * kB * sizeof(float);
    const size_t lds_r = (size_t)(kB - 2) * kB * sizeof(float);
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)tridiag_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)ritz_pair_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_r));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(tridiag_kernel, dim3(1), dim3(256), lds, ctx->stream, Mb, b, refl, tri, cluster_flag);
    hipLaunchKernelGGL(ritz_pair_kernel, dim3(b), dim3(64), lds_r, ctx->stream, (const float*)tri, (const float*)refl, b, lambda, V,
                       cluster_flag);
    return aser_check_launch(ctx, "tridiag_eig");
}
