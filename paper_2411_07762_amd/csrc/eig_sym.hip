// Symmetric eigen-solver for the Rayleigh-Ritz step of the truncated SVD (Eq. 6): all eigenpairs
// of a b x b matrix (b <= 128), eigenvalues descending.  Two kernels:
//
//   tridiag_kernel   one workgroup, the matrix lives in registers (2 x 8 elements per thread).
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

// Thread t holds rows 2 (t >> 4) + {0, 1} and columns 8 (t & 15) + {0..7}: the 16 lanes of a DPP
// row share their two matrix rows, so the mat-vec reduction never leaves the row.
__global__ __launch_bounds__(1024) void tridiag_kernel(const float* __restrict__ Mb, int b, float* __restrict__ refl /* [k][128] */,
                                                       float* __restrict__ tri /* d | e | tau, 128 each */,
                                                       int* __restrict__ cluster_flag) {
    // Everything the loop produces stays in LDS until the end: a global store inside the loop
    // would have to drain before each barrier.
    extern __shared__ __align__(16) float sm[];
    float (*xc)[kB] = (float (*)[kB])sm;        // [2][kB] column k of the current matrix, double-buffered
    float* pb = sm + 2 * kB;
    float* td = pb + kB;
    float* te = td + kB;
    float* tt = te + kB;
    float* rs = tt + kB;                        // [b - 2][kB] reflectors
    const int tid = threadIdx.x, lane = tid & 63;
    const int r0 = 2 * (tid >> 4), c0 = 8 * (tid & 15);

    float a[2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = r0 + i, c = c0 + j;
            a[i][j] = (r < b && c < b) ? 0.5f * (Mb[r * b + c] + Mb[c * b + r]) : 0.f;
        }
    if (tid == 0) *cluster_flag = 0;
    if (tid < kB) { td[tid] = 0.f; te[tid] = 0.f; tt[tid] = 0.f; }
    if (c0 == 0) { xc[0][r0] = a[0][0]; xc[0][r0 + 1] = a[1][0]; }
    __syncthreads();

    for (int k = 0; k + 2 < b; ++k) {
        const float* cur = xc[k & 1];
        // reflector k annihilates A[k+2.., k]
        const float x0 = cur[lane], x1 = cur[lane + 64];
        const float alpha = cur[k + 1];
        const float sigma = wave_sum(((lane > k + 1) ? x0 * x0 : 0.f) + ((lane + 64 > k + 1) ? x1 * x1 : 0.f));
        float beta = alpha, tk = 0.f, scal = 0.f;
        if (sigma > 1e-30f * alpha * alpha && sigma > 0.f) {
            beta = -copysignf(sqrtf(alpha * alpha + sigma), alpha);
            tk = (beta - alpha) / beta;
            scal = 1.0f / (alpha - beta);
        }
        auto vat = [&](int idx, float x) { return (idx <= k) ? 0.f : ((idx == k + 1) ? 1.f : x * scal); };
        float vr[2], vc[8];
        {
            const float2 xr = *(const float2*)(cur + r0);
            const float4 xa = *(const float4*)(cur + c0), xb = *(const float4*)(cur + c0 + 4);
            vr[0] = vat(r0, xr.x); vr[1] = vat(r0 + 1, xr.y);
            vc[0] = vat(c0 + 0, xa.x); vc[1] = vat(c0 + 1, xa.y); vc[2] = vat(c0 + 2, xa.z); vc[3] = vat(c0 + 3, xa.w);
            vc[4] = vat(c0 + 4, xb.x); vc[5] = vat(c0 + 5, xb.y); vc[6] = vat(c0 + 6, xb.z); vc[7] = vat(c0 + 7, xb.w);
        }
        // p = tau * A v on the trailing block (rows <= k are dead)
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) { s0 += a[0][j] * vc[j]; s1 += a[1][j] * vc[j]; }
        s0 = row16_sum(s0);
        s1 = row16_sum(s1);
        if (c0 == 0) {
            pb[r0] = (r0 > k) ? tk * s0 : 0.f;
            pb[r0 + 1] = (r0 + 1 > k) ? tk * s1 : 0.f;
        }
        if (tid < 64) {
            rs[k * kB + lane] = vat(lane, x0);
            rs[k * kB + lane + 64] = vat(lane + 64, x1);
        }
        if (tid == 0) { te[k] = beta; tt[k] = tk; }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (r0 + i == k && c0 + j == k) td[k] = a[i][j];
        __syncthreads();
        // A -= v w^T + w v^T with w = p - (tau/2)(p^T v) v
        const float kk = wave_sum(pb[lane] * vat(lane, x0) + pb[lane + 64] * vat(lane + 64, x1));
        const float a2 = -0.5f * tk * kk;
        float wr[2], wc[8];
        {
            const float2 pr = *(const float2*)(pb + r0);
            const float4 pa = *(const float4*)(pb + c0), pc = *(const float4*)(pb + c0 + 4);
            wr[0] = pr.x + a2 * vr[0]; wr[1] = pr.y + a2 * vr[1];
            wc[0] = pa.x + a2 * vc[0]; wc[1] = pa.y + a2 * vc[1]; wc[2] = pa.z + a2 * vc[2]; wc[3] = pa.w + a2 * vc[3];
            wc[4] = pc.x + a2 * vc[4]; wc[5] = pc.y + a2 * vc[5]; wc[6] = pc.z + a2 * vc[6]; wc[7] = pc.w + a2 * vc[7];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) a[i][j] -= vr[i] * wc[j] + wr[i] * vc[j];
        // next column to the other buffer
        if (c0 == ((k + 1) & ~7)) {
            const int jj = (k + 1) & 7;
            float y0 = a[0][0], y1 = a[1][0];
#pragma unroll
            for (int j = 1; j < 8; ++j)
                if (jj == j) { y0 = a[0][j]; y1 = a[1][j]; }
            float* nxt = xc[(k + 1) & 1];
            nxt[r0] = y0;
            nxt[r0 + 1] = y1;
        }
        __syncthreads();
    }
    // the last 2 x 2 block
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = r0 + i, c = c0 + j;
            if (r == c && (r == b - 1 || r == b - 2)) td[r] = a[i][j];
            if (r == b - 1 && c == b - 2) te[b - 2] = a[i][j];
        }
    __syncthreads();
    for (int t = tid; t < (b - 2) * kB; t += 1024) refl[t] = rs[t];
    if (tid < 3 * kB) tri[tid] = td[tid];
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
    for (int t = lane; t < (b - 2) * (kB / 4); t += 64) ((float4*)rl)[t] = ((const float4*)refl)[t];

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
    hipLaunchKernelGGL(tridiag_kernel, dim3(1), dim3(1024), lds, ctx->stream, Mb, b, refl, tri, cluster_flag);
    hipLaunchKernelGGL(ritz_pair_kernel, dim3(b), dim3(64), lds_r, ctx->stream, (const float*)tri, (const float*)refl, b, lambda, V,
                       cluster_flag);
    return aser_check_launch(ctx, "tridiag_eig");
}
