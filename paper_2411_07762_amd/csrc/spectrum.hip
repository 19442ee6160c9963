// The whole singular spectrum of the whitened error T S (Eq. 6), and what the paper derives from it:
// the rank chosen by the threshold alpha on the cumulative sum of singular values (Eq. 9) and the
// effective rank, the exponential of the entropy of the normalised singular values (Eq. 3, Eq. 4).
//
// A truncated solver does not produce the sum over ALL singular values that Eq. 9 divides by, so this
// path computes every one of them, in fp64 behind the product T S:
//   B = Z Z^T  (k x k, k = min(m, n), Z = T S or its transpose)   fp64 accumulation of exact fp32 products
//   B -> tridiagonal (d, e) by Householder reflections            two launches per column, see below
//   eigenvalues of (d, e) by bisection on Sturm counts            one thread per eigenvalue
//   sigma_i = sqrt(lambda_i), descending.
// The singular values of T S and of (T S)^T agree, so B is formed on the shorter side.
//
// Tridiagonalisation.  Step j turns column j into (d_j, e_j, 0, ...) with H = I - tau v v^T and needs
// p = tau B22 v and the rank-2 update B22 -= v w^T + w v^T with w = p - (tau / 2)(v^T p) v.  Both are
// passes over the trailing matrix, and they are fused across steps: the pass of step j applies the
// update of step j and, on the values it has just written, forms B22' v' for the NEXT reflector v'
// (which only needs row j + 1 of the updated matrix, computed ahead by a one-workgroup kernel).  So a
// step is one small kernel plus one pass that reads and writes the trailing matrix once: 16 (k - j)^2
// bytes, 16 k^3 / 3 in total; the path is bound by HBM (or by the last-level cache when B fits).
// B is kept as a full symmetric matrix so that every pass walks rows with unit stride.
#include <math.h>

#include "aser_internal.h"

namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------------
// B += P^T P for P: K x k fp32 (row-major, ldp), B: k x k fp64 (ld = k), lower-triangle tiles of
// 64 x 64 written to both (i, j) and (j, i).  256 threads as 16 x 16, a 4 x 4 block of B each.
// K is split over blockIdx.y; partial tiles are added with fp64 atomics (B is cleared first).
template <typename TIN>
__global__ __launch_bounds__(256) void gram_f64_kernel(const TIN* __restrict__ P, int64_t K, int64_t k, int64_t ldp,
                                                       double* __restrict__ B, int k_parts) {
    typedef TIN tin4_t __attribute__((ext_vector_type(4)));
    __shared__ __align__(32) TIN sa[16][64];
    __shared__ __align__(32) TIN sb[16][64];
    const int64_t t = blockIdx.x;
    int64_t bi = (int64_t)((sqrt(8.0 * (double)t + 1.0) - 1.0) * 0.5);
    while (bi * (bi + 1) / 2 > t) --bi;
    while ((bi + 1) * (bi + 2) / 2 <= t) ++bi;
    const int64_t bj = t - bi * (bi + 1) / 2;
    const int64_t I0 = bi * 64, J0 = bj * 64;
    const int64_t per = (((K + 15) / 16 + k_parts - 1) / k_parts) * 16;
    const int64_t k0 = (int64_t)blockIdx.y * per;
    const int64_t k1 = (k0 + per < K) ? k0 + per : K;
    if (k0 >= k1) return;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int lr = tid >> 4, lc = (tid & 15) * 4;          // this thread's 4 floats of a 16 x 64 slab
    const bool vec_ok = (((uintptr_t)P & (4 * sizeof(TIN) - 1)) == 0) && ((ldp & 3) == 0);
    double acc[4][4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[u][v] = 0.0;
    for (int64_t kk = k0; kk < k1; kk += 16) {
        const int64_t row = kk + lr;
        tin4_t a = {0, 0, 0, 0}, b = {0, 0, 0, 0};
        if (row < k1) {
            const TIN* pr = P + row * ldp;
            if (vec_ok && I0 + lc + 4 <= k) a = *(const tin4_t*)(pr + I0 + lc);
            else
                for (int e = 0; e < 4; ++e)
                    if (I0 + lc + e < k) a[e] = pr[I0 + lc + e];
            if (vec_ok && J0 + lc + 4 <= k) b = *(const tin4_t*)(pr + J0 + lc);
            else
                for (int e = 0; e < 4; ++e)
                    if (J0 + lc + e < k) b[e] = pr[J0 + lc + e];
        }
        __syncthreads();                                  // the previous slab has been consumed
        *(tin4_t*)&sa[lr][lc] = a;
        *(tin4_t*)&sb[lr][lc] = b;
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            const tin4_t av = *(const tin4_t*)&sa[s][ty * 4];
            const tin4_t bv = *(const tin4_t*)&sb[s][tx * 4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[u][v] = fma((double)av[u], (double)bv[v], acc[u][v]);
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int64_t i = I0 + ty * 4 + u, j = J0 + tx * 4 + v;
            if (i >= k || j >= k) continue;
            if (bi == bj && j > i) continue;              // diagonal tile: the lower half is mirrored below
            unsafeAtomicAdd(B + i * k + j, acc[u][v]);
            if (i != j) unsafeAtomicAdd(B + j * k + i, acc[u][v]);
        }
}

__device__ __forceinline__ double block_sum(double v, double* red) {   // blockDim.x multiple of 64, <= 1024
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();                                      // red may still be read from an earlier call
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    double r = 0.0;
    for (int i = 0; i < nw; ++i) r += red[i];
    return r;
}

// One workgroup between two passes.  With j >= 0: finishes step j (w from the pass's p = B22 v), then
// looks one row ahead: row j + 1 of the updated matrix gives d_{j+1} and the next reflector.  j = -1
// starts the chain from row 0 of B.  Vectors are indexed by absolute row; v_cur / v_next alternate.
//   tau[0]: tau of step j (read), tau[1]: tau of step j + 1 (written)
__global__ __launch_bounds__(1024) void tridiag_head_kernel(int64_t j, int64_t k, const double* __restrict__ B,
                                                            const double* __restrict__ v_cur, double* __restrict__ v_next,
                                                            double* __restrict__ w, const double* __restrict__ p,
                                                            double* __restrict__ d, double* __restrict__ e,
                                                            const double* __restrict__ tau_cur, double* __restrict__ tau_next,
                                                            double* __restrict__ vstore, double* __restrict__ taustore) {
    __shared__ double red[16];
    const int tid = threadIdx.x;
    const int64_t row = j + 1;
    double v_row = 0.0, w_row = 0.0;
    if (j >= 0) {
        const double tau = *tau_cur;
        double dot = 0.0;
        for (int64_t i = row + tid; i < k; i += 1024) dot += v_cur[i] * p[i];
        dot = block_sum(dot, red);
        const double kk = 0.5 * tau * tau * dot;
        for (int64_t i = row + tid; i < k; i += 1024) w[i] = tau * p[i] - kk * v_cur[i];
        __syncthreads();
        v_row = v_cur[row];
        w_row = w[row];
    }
    // row `row` of the updated matrix, from the diagonal on
    const double* brow = B + row * k;
    auto c_at = [&](int64_t i) -> double {
        double c = brow[i];
        if (j >= 0) c -= v_row * w[i] + w_row * v_cur[i];
        return c;
    };
    if (tid == 0) d[row] = c_at(row);
    if (row + 2 < k) {                                    // at least two entries below the diagonal: a reflector
        double n2 = 0.0;
        for (int64_t i = row + 1 + tid; i < k; i += 1024) {
            const double c = c_at(i);
            v_next[i] = c;
            n2 += c * c;
        }
        n2 = block_sum(n2, red);
        __syncthreads();
        if (tid == 0) {
            const double x0 = v_next[row + 1];
            const double alpha = (x0 > 0.0) ? -sqrt(n2) : sqrt(n2);
            const double v0 = x0 - alpha;
            const double vn2 = n2 - x0 * x0 + v0 * v0;
            v_next[row + 1] = v0;
            const double tnew = vn2 > 0.0 ? 2.0 / vn2 : 0.0;
            *tau_next = tnew;
            e[row] = alpha;
            if (taustore) taustore[row] = tnew;
        }
        if (vstore) {                                     // keep the reflector for the back-transformation of eigenvectors
            __syncthreads();
            for (int64_t i = row + 1 + tid; i < k; i += 1024) vstore[row * k + i] = v_next[i];
        }
    } else if (row + 2 == k) {                            // the last 2 x 2 block: no reflector
        if (tid == 0) {
            e[row] = c_at(row + 1);
            double dl = B[(k - 1) * k + (k - 1)];
            if (j >= 0) dl -= 2.0 * v_cur[k - 1] * w[k - 1];
            d[k - 1] = dl;
        }
    }
}

// Pass of step j over rows and columns >= c0 = j + 2: B -= v w^T + w v^T (skipped when !update), then
// p_i = sum_l B_il vn_l on the new values.  A workgroup owns 8 rows; a thread walks columns with unit
// stride across the workgroup and keeps its share of the 8 dot products in registers.
__global__ __launch_bounds__(256) void tridiag_pass_kernel(int64_t c0, int64_t k, double* __restrict__ B,
                                                           const double* __restrict__ v, const double* __restrict__ w,
                                                           const double* __restrict__ vn, double* __restrict__ p,
                                                           int update) {
    __shared__ double red[4][8];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t r0 = c0 + (int64_t)blockIdx.x * 8;
    double vi[8], wi[8], acc[8];
    double* rowp[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int64_t i = (r0 + r < k) ? r0 + r : k - 1;  // rows past the end repeat the last row; their results are dropped
        vi[r] = update ? v[i] : 0.0;
        wi[r] = update ? w[i] : 0.0;
        rowp[r] = B + i * k;
        acc[r] = 0.0;
    }
    const int nrows = (int)((k - r0 < 8) ? k - r0 : 8);
    for (int64_t l = c0 + tid; l < k; l += 256) {
        const double vl = update ? v[l] : 0.0, wl = update ? w[l] : 0.0, vnl = vn[l];
        double b[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) b[r] = rowp[r][l];
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if (update) {
                b[r] -= vi[r] * wl + wi[r] * vl;
                if (r < nrows) rowp[r][l] = b[r];
            }
            acc[r] = fma(b[r], vnl, acc[r]);
        }
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) acc[r] += __shfl_xor(acc[r], o, 64);
        if (lane == 0) red[wave][r] = acc[r];
    }
    __syncthreads();
    if (tid < nrows) p[r0 + tid] = red[0][tid] + red[1][tid] + red[2][tid] + red[3][tid];
}

// Eigenvalue number i (ascending) of the symmetric tridiagonal matrix (d, e) by bisection: the Sturm
// count of x (number of eigenvalues below x) is the number of negative terms of the sequence
// q_0 = d_0 - x, q_l = d_l - x - e_{l-1}^2 / q_{l-1}.  One thread per eigenvalue; the lanes of a
// wavefront read the same (d_l, e_l) at the same time.  sigma[k - 1 - i] = sqrt(max(lambda_i, 0)).
__global__ __launch_bounds__(64) void tridiag_bisect_kernel(int64_t k, const double* __restrict__ d,
                                                            const double* __restrict__ e, double* __restrict__ sigma,
                                                            double* __restrict__ lam_desc) {
    const int64_t i = (int64_t)blockIdx.x * 64 + threadIdx.x;
    // Gershgorin interval and the smallest pivot magnitude (every lane computes the same values)
    double lo = 1e300, hi = -1e300, emax2 = 0.0;
    for (int64_t l = 0; l < k; ++l) {
        const double el = (l + 1 < k) ? fabs(e[l]) : 0.0, ep = (l > 0) ? fabs(e[l - 1]) : 0.0;
        lo = fmin(lo, d[l] - el - ep);
        hi = fmax(hi, d[l] + el + ep);
        emax2 = fmax(emax2, el * el);
    }
    const double span = fmax(hi - lo, 1e-300);
    lo -= 1e-12 * span;
    hi += 1e-12 * span;
    const double pivmin = fmax(emax2 * 2.2e-308 * 4.0, 1e-300);
    if (i >= k) return;
    double a = lo, b = hi;
    for (int it = 0; it < 60; ++it) {
        const double x = 0.5 * (a + b);
        double q = d[0] - x;
        if (fabs(q) < pivmin) q = -pivmin;
        int64_t cnt = q < 0.0 ? 1 : 0;
        for (int64_t l = 1; l < k; ++l) {
            const double el = e[l - 1];
            q = d[l] - x - el * el / q;
            if (fabs(q) < pivmin) q = -pivmin;
            cnt += q < 0.0 ? 1 : 0;
        }
        if (cnt <= i) a = x; else b = x;
    }
    const double lam = 0.5 * (a + b);
    sigma[k - 1 - i] = lam > 0.0 ? sqrt(lam) : 0.0;
    if (lam_desc) lam_desc[k - 1 - i] = lam;
}

// The same eigenvalue by multisection, one wavefront per eigenvalue: the 64 lanes take the Sturm counts of 64
// points that cut the current interval into 65 parts, and the interval shrinks to the part where the count
// passes i: 11 rounds for the 60 halvings of the bisection, on k wavefronts instead of k / 64 (k = 4096: the
// sequential recurrence of 60 x k dependent divisions per thread was 25 ms on 64 compute units).
__global__ __launch_bounds__(64) void tridiag_multisect_kernel(int64_t k, const double* __restrict__ d,
                                                               const double* __restrict__ e, double* __restrict__ sigma,
                                                               double* __restrict__ lam_desc) {
    const int64_t i = blockIdx.x;
    const int lane = threadIdx.x;
    double lo = 1e300, hi = -1e300, emax2 = 0.0;
    for (int64_t l = 0; l < k; ++l) {
        const double el = (l + 1 < k) ? fabs(e[l]) : 0.0, ep = (l > 0) ? fabs(e[l - 1]) : 0.0;
        lo = fmin(lo, d[l] - el - ep);
        hi = fmax(hi, d[l] + el + ep);
        emax2 = fmax(emax2, el * el);
    }
    const double span = fmax(hi - lo, 1e-300);
    lo -= 1e-12 * span;
    hi += 1e-12 * span;
    const double pivmin = fmax(emax2 * 2.2e-308 * 4.0, 1e-300);
    double a = lo, b = hi;
    for (int it = 0; it < 11; ++it) {
        const double step = (b - a) * (1.0 / 65.0);
        const double x = a + step * (double)(lane + 1);
        double q = d[0] - x;
        if (fabs(q) < pivmin) q = -pivmin;
        int64_t cnt = q < 0.0 ? 1 : 0;
        for (int64_t l = 1; l < k; ++l) {
            const double el = e[l - 1];
            q = d[l] - x - el * el / q;
            if (fabs(q) < pivmin) q = -pivmin;
            cnt += q < 0.0 ? 1 : 0;
        }
        // the count grows with x: the points with cnt <= i are the first p of them
        const int p = __popcll(__builtin_amdgcn_ballot_w64(cnt <= i));
        const double xa = __shfl(x, p > 0 ? p - 1 : 0, 64), xb = __shfl(x, p < 64 ? p : 63, 64);
        const double na = p > 0 ? xa : a, nb = p < 64 ? xb : b;
        a = na;
        b = nb;
    }
    if (lane == 0) {
        const double lam = 0.5 * (a + b);
        sigma[k - 1 - i] = lam > 0.0 ? sqrt(lam) : 0.0;
        if (lam_desc) lam_desc[k - 1 - i] = lam;
    }
}

// Every eigenvalue of the tridiagonal matrix: bisection with a thread each for small matrices, multisection with a
// wavefront each from 1024 on.
int tridiag_eigenvalues(aser_ctx* ctx, int64_t k, const double* d, const double* e, double* sigma, double* lam_desc) {
    if (k >= 1024)
        hipLaunchKernelGGL(tridiag_multisect_kernel, dim3((unsigned)k), dim3(64), 0, ctx->stream, k, d, e, sigma, lam_desc);
    else
        hipLaunchKernelGGL(tridiag_bisect_kernel, dim3((unsigned)ceil_div64(k, 64)), dim3(64), 0, ctx->stream, k, d, e, sigma, lam_desc);
    return aser_check_launch(ctx, "tridiag_eigenvalues");
}

// Eq. 9 on a descending spectrum: running sums in index order; r = number of leading indices whose
// cumulative share stays below alpha, at least 1.  out: r, then sum, share(r), share(r + 1) as doubles.
__global__ void select_rank_kernel(const double* __restrict__ sigma, int64_t k, double alpha, int32_t* __restrict__ r_out,
                                   double* __restrict__ stats) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double total = 0.0;
    for (int64_t i = 0; i < k; ++i) total += sigma[i];
    double cum = 0.0, at_r = 0.0, next = 0.0;
    int64_t r = 0;
    bool open = true;
    for (int64_t i = 0; i < k && open; ++i) {
        cum += sigma[i];
        if (cum / total < alpha) { r = i + 1; at_r = cum / total; }
        else { next = cum / total; open = false; }
    }
    if (open) next = 1.0;
    if (r < 1) {                                          // the threshold lies below the first share: rank one
        r = 1;
        at_r = sigma[0] / total;
        next = (k > 1) ? (sigma[0] + sigma[1]) / total : 1.0;
    }
    *r_out = (int32_t)r;
    stats[0] = total;
    stats[1] = at_r;
    stats[2] = next;
}

// Eq. 3 and Eq. 4: exp(-sum p ln p), p = sigma / sum(sigma) + eps.  One workgroup.
__global__ __launch_bounds__(1024) void effective_rank_kernel(const double* __restrict__ sigma, int64_t k, double eps,
                                                              double* __restrict__ out) {
    __shared__ double red[16];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < k; i += 1024) s += sigma[i];
    const double total = block_sum(s, red);
    double h = 0.0;
    for (int64_t i = threadIdx.x; i < k; i += 1024) {
        const double p = sigma[i] / total + eps;
        if (p > 0.0) h -= p * log(p);
    }
    h = block_sum(h, red);
    if (threadIdx.x == 0) *out = exp(h);
}

// B (k x k fp64, full symmetric) = P^T P, cleared first; K split so that the grid fills the device.
template <typename TIN>
int gram_f64(aser_ctx* ctx, const TIN* P, int64_t K, int64_t k, int64_t ldp, double* B) {
    ASER_TRY(aser_fill_bytes(ctx, B, (size_t)k * k * 8));
    const int64_t t64 = ceil_div64(k, 64), tiles = t64 * (t64 + 1) / 2, ksteps = ceil_div64(K, 16);
    int64_t parts = ceil_div64(2048, tiles);
    if (parts > ksteps / 8) parts = ksteps / 8;
    if (parts < 1) parts = 1;
    if (parts > 64) parts = 64;
    hipLaunchKernelGGL(gram_f64_kernel<TIN>, dim3((unsigned)tiles, (unsigned)parts), dim3(256), 0, ctx->stream, P, K, k, ldp, B,
                       (int)parts);
    return aser_check_launch(ctx, "gram_f64");
}

// Householder chain on B (overwritten): head(-1), pass(-1), then head(j), pass(j) for j = 0 .. k - 3.
// vec: eight zeroed arrays of k doubles (v twice, w, p, d, e, tau, spare); d = vec[4], e = vec[5] on return.
// vstore (k x k) / taustore (k), both zeroed by the caller, receive the reflectors when not null.
int tridiagonalize(aser_ctx* ctx, double* B, int64_t k, double* const* vec, double* vstore, double* taustore) {
    double *v0 = vec[0], *v1 = vec[1], *w = vec[2], *p = vec[3], *d = vec[4], *e = vec[5], *tau = vec[6];
    double *vc = v0, *vn = v1;
    hipLaunchKernelGGL(tridiag_head_kernel, dim3(1), dim3(1024), 0, ctx->stream, (int64_t)-1, k, (const double*)B,
                       (const double*)vc, vn, w, (const double*)p, d, e, (const double*)tau, tau + 1, vstore, taustore);
    ASER_TRY(aser_check_launch(ctx, "tridiag_head"));
    int tsel = 1;                                          // tau[tsel] holds the tau of the reflector in vn
    for (int64_t j = -1; j + 3 < k; ++j) {
        // pass of step j: update with (vc, w) when j >= 0, then p = B22 vn
        const int64_t c0 = j + 2;
        hipLaunchKernelGGL(tridiag_pass_kernel, dim3((unsigned)ceil_div64(k - c0, 8)), dim3(256), 0, ctx->stream, c0, k, B,
                           (const double*)vc, (const double*)w, (const double*)vn, p, j >= 0 ? 1 : 0);
        ASER_TRY(aser_check_launch(ctx, "tridiag_pass"));
        { double* t = vc; vc = vn; vn = t; }
        hipLaunchKernelGGL(tridiag_head_kernel, dim3(1), dim3(1024), 0, ctx->stream, j + 1, k, (const double*)B,
                           (const double*)vc, vn, w, (const double*)p, d, e, (const double*)(tau + tsel), tau + (tsel ^ 1),
                           vstore, taustore);
        ASER_TRY(aser_check_launch(ctx, "tridiag_head"));
        tsel ^= 1;
    }
    return ASER_OK;
}

// ---------------------------------------------------------------------------------------------
// Dense fp64 solver for small layers: the rank-r truncated SVD of A = T S from the complete
// eigen-decomposition of the Gram matrix of its shorter side.  Eigenvalues as above (every one, so the
// whitened error is the square root of their tail sum); eigenvectors of the r largest by inverse
// iteration on the tridiagonal matrix, made orthonormal among themselves, and carried back through the
// stored reflectors.  No iteration count, no start block: what the iterative path approximates.

// out[i][j] = sum_{l >= j} T[i][l] S[l][j] in fp64 (S lower triangular); TRANSPOSED: stored as out[j][i].
template <bool TRANSPOSED>
__global__ __launch_bounds__(256) void ts_f64_kernel(const float* __restrict__ T, int64_t m, int64_t n, int64_t ldt,
                                                     const float* __restrict__ S, int64_t lds, double* __restrict__ out) {
    const int64_t j = (int64_t)blockIdx.x * 64 + (threadIdx.x & 63);
    const int64_t i = (int64_t)blockIdx.y * 4 + (threadIdx.x >> 6);
    if (i >= m || j >= n) return;
    const float* trow = T + i * ldt;
    double acc = 0.0;
    for (int64_t l = j; l < n; ++l) acc = fma((double)trow[l], (double)S[l * lds + j], acc);
    if (TRANSPOSED) out[j * m + i] = acc; else out[i * n + j] = acc;
}

__device__ __forceinline__ uint32_t hash32(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
    return x;
}

// One step of inverse iteration on the symmetric tridiagonal matrix (d, e): x <- (T - shift I)^-1 x by Gaussian
// elimination with row interchanges (a zero pivot becomes `tiny`), then scaled to unit maximum.  dd, du, du2: k
// doubles each of scratch.
__device__ __forceinline__ void invit_solve_one(int64_t k, const double* __restrict__ d, const double* __restrict__ e,
                                                double shift, double tiny, double* x, double* dd, double* du, double* du2) {
    double a = d[0] - shift, b = (k > 1) ? e[0] : 0.0;       // current row: diagonal and super-diagonal
    for (int64_t i = 0; i + 1 < k; ++i) {
        const double sub = e[i], dn = d[i + 1] - shift, en = (i + 2 < k) ? e[i + 1] : 0.0;
        if (fabs(a) >= fabs(sub)) {
            if (fabs(a) < tiny) a = tiny;
            const double mult = sub / a;
            dd[i] = a; du[i] = b; du2[i] = 0.0;
            x[i + 1] -= mult * x[i];
            a = dn - mult * b;
            b = en;
        } else {
            const double mult = a / sub;
            dd[i] = sub; du[i] = dn; du2[i] = en;
            const double xi = x[i];
            x[i] = x[i + 1];
            x[i + 1] = xi - mult * x[i];
            a = b - mult * dn;
            b = -mult * en;
        }
    }
    if (fabs(a) < tiny) a = tiny;
    dd[k - 1] = a;
    x[k - 1] /= dd[k - 1];
    if (k > 1) x[k - 2] = (x[k - 2] - du[k - 2] * x[k - 1]) / dd[k - 2];
    for (int64_t i = k - 3; i >= 0; --i) x[i] = (x[i] - du[i] * x[i + 1] - du2[i] * x[i + 2]) / dd[i];
    double mx = 0.0;
    for (int64_t i = 0; i < k; ++i) mx = fmax(mx, fabs(x[i]));
    const double sc = mx > 0.0 ? 1.0 / mx : 1.0;
    for (int64_t i = 0; i < k; ++i) x[i] *= sc;
}

__device__ __forceinline__ double tridiag_norm(int64_t k, const double* __restrict__ d, const double* __restrict__ e) {
    double tnorm = 0.0;
    for (int64_t l = 0; l < k; ++l) tnorm = fmax(tnorm, fabs(d[l]) + (l + 1 < k ? fabs(e[l]) : 0.0) + (l > 0 ? fabs(e[l - 1]) : 0.0));
    return tnorm;
}

__device__ __forceinline__ double invit_start_value(int64_t t) {
    return (double)(hash32((uint32_t)t * 0x9E3779B9U + 12345u) >> 8) * (1.0 / 8388608.0) - 1.0;
}

// Eigenvectors of the symmetric tridiagonal matrix (d, e) for the r largest eigenvalues lam[0 .. r),
// as rows of X (r x k).  One workgroup (small problems).  Three rounds of: thread c solves (T - lam_c I) y = x_c,
// then the vectors are orthonormalised in order (classical Gram-Schmidt, twice).  scr: r x 3 k doubles.
__global__ __launch_bounds__(256) void tridiag_invit_kernel(int64_t k, int r, const double* __restrict__ d,
                                                            const double* __restrict__ e, const double* __restrict__ lam,
                                                            double* __restrict__ X, double* __restrict__ scr) {
    __shared__ double dots[256];                      // r <= 256
    __shared__ double red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double tiny = fmax(tridiag_norm(k, d, e) * 2.3e-16, 1e-300);
    for (int64_t t = tid; t < (int64_t)r * k; t += 256) X[t] = invit_start_value(t);
    __syncthreads();
    for (int round = 0; round < 3; ++round) {
        if (tid < r) {
            const int c = tid;
            double* dd = scr + (int64_t)c * 3 * k;
            invit_solve_one(k, d, e, lam[c], tiny, X + (int64_t)c * k, dd, dd + k, dd + 2 * k);
        }
        __syncthreads();
        for (int c = 0; c < r; ++c) {
            double* x = X + (int64_t)c * k;
            for (int pass = 0; pass < 2; ++pass) {
                for (int j = wave; j < c; j += 4) {
                    const double* y = X + (int64_t)j * k;
                    double s = 0.0;
                    for (int64_t i = lane; i < k; i += 64) s += y[i] * x[i];
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
                    if (lane == 0) dots[j] = s;
                }
                __syncthreads();
                for (int64_t i = tid; i < k; i += 256) {
                    double v = x[i];
                    for (int j = 0; j < c; ++j) v -= dots[j] * X[(int64_t)j * k + i];
                    x[i] = v;
                }
                __syncthreads();
            }
            double s = 0.0;
            for (int64_t i = tid; i < k; i += 256) s += x[i] * x[i];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
            if (lane == 0) red[wave] = s;
            __syncthreads();
            const double nrm = sqrt(red[0] + red[1] + red[2] + red[3]);
            const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
            for (int64_t i = tid; i < k; i += 256) x[i] *= inv;
            __syncthreads();
        }
    }
}

// The same computation for large problems, one launch per step, because the orthonormalisation is r^2 k work that
// one workgroup takes most of a second for at k = 4096, r = 200: the start vectors, the r solves (one thread each),
// and per vector c and pass the dots against the vectors before it (one workgroup per earlier vector), the
// update (workgroups over the k entries) and, after the second pass, the normalisation (one workgroup).
__global__ void invit_start_kernel(int64_t total, double* __restrict__ X) {
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (int64_t)gridDim.x * blockDim.x)
        X[t] = invit_start_value(t);
}

__global__ __launch_bounds__(64) void invit_solve_kernel(int64_t k, int r, const double* __restrict__ d,
                                                         const double* __restrict__ e, const double* __restrict__ lam,
                                                         double* __restrict__ X, double* __restrict__ scr) {
    const int c = blockIdx.x * 64 + threadIdx.x;
    if (c >= r) return;
    const double tiny = fmax(tridiag_norm(k, d, e) * 2.3e-16, 1e-300);
    double* dd = scr + (int64_t)c * 3 * k;
    invit_solve_one(k, d, e, lam[c], tiny, X + (int64_t)c * k, dd, dd + k, dd + 2 * k);
}

__global__ __launch_bounds__(256) void invit_dots_kernel(int64_t k, int c, const double* __restrict__ X, double* __restrict__ dots) {
    __shared__ double red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, j = blockIdx.x;
    const double* y = X + (int64_t)j * k;
    const double* x = X + (int64_t)c * k;
    double s = 0.0;
    for (int64_t i = tid; i < k; i += 256) s += y[i] * x[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    if (tid == 0) dots[j] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void invit_update_kernel(int64_t k, int c, double* __restrict__ X, const double* __restrict__ dots) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= k) return;
    double v = X[(int64_t)c * k + i];
    for (int j = 0; j < c; ++j) v -= dots[j] * X[(int64_t)j * k + i];
    X[(int64_t)c * k + i] = v;
}

__global__ __launch_bounds__(256) void invit_normalize_kernel(int64_t k, int c, double* __restrict__ X) {
    __shared__ double red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double* x = X + (int64_t)c * k;
    double s = 0.0;
    for (int64_t i = tid; i < k; i += 256) s += x[i] * x[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    const double nrm = sqrt(red[0] + red[1] + red[2] + red[3]);
    const double inv = nrm > 0.0 ? 1.0 / nrm : 0.0;
    for (int64_t i = tid; i < k; i += 256) x[i] *= inv;
}

// x <- H_0 H_1 ... H_{k-3} x for every row x of X (one workgroup per row): eigenvectors of the tridiagonal
// matrix become eigenvectors of the Gram matrix.  H_j = I - tau_j v_j v_j^T, v_j in row j of vstore.
__global__ __launch_bounds__(256) void backtransform_kernel(int64_t k, const double* __restrict__ vstore,
                                                            const double* __restrict__ taustore, double* __restrict__ X) {
    __shared__ double red[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double* x = X + (int64_t)blockIdx.x * k;
    for (int64_t j = k - 3; j >= 0; --j) {
        const double* v = vstore + j * k;
        double s = 0.0;
        for (int64_t i = j + 1 + tid; i < k; i += 256) s += v[i] * x[i];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        __syncthreads();
        if (lane == 0) red[wave] = s;
        __syncthreads();
        const double f = taustore[j] * (red[0] + red[1] + red[2] + red[3]);
        for (int64_t i = j + 1 + tid; i < k; i += 256) x[i] -= f * v[i];
        __syncthreads();
    }
}

// Factors from the eigenvectors (rows of X, r x k) and eigenvalues lam (descending) of the Gram matrix.
//   k == m (left singular vectors u_c = X[c]):   L_A[i][c] = u_c[i] sigma_c,        L_B[c][j] = sum_i u_c[i] T[i][j] / sigma_c
//   k == n (right singular vectors v_c = X[c]):  L_A[i][c] = sum_j A[i][j] v_c[j],  L_B[c][j] = sum_i L_A[i][c] T[i][j] / sigma_c^2
// LA64: m x r fp64 scratch.  Two launches: phase 0 writes L_A (and LA64), phase 1 writes L_B, sigma and the error.
__global__ __launch_bounds__(256) void exact_factors_kernel(int phase, int left, int64_t m, int64_t n, int64_t k, int r,
                                                            const double* __restrict__ X, const double* __restrict__ lam,
                                                            const double* __restrict__ A64, const float* __restrict__ A32,
                                                            const float* __restrict__ T,
                                                            int64_t ldt, double* __restrict__ LA64, float* __restrict__ L_A,
                                                            float* __restrict__ L_B, float* __restrict__ sigma,
                                                            double* __restrict__ err2) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (phase == 0) {
        if (t >= m * r) return;
        const int64_t i = t / r;
        const int c = (int)(t % r);
        double v;
        if (left) {
            const double sg = lam[c] > 0.0 ? sqrt(lam[c]) : 0.0;
            v = X[(int64_t)c * k + i] * sg;
        } else {
            v = 0.0;
            if (A32) {
                for (int64_t j = 0; j < n; ++j) v = fma((double)A32[i * n + j], X[(int64_t)c * k + j], v);
            } else {
                for (int64_t j = 0; j < n; ++j) v = fma(A64[i * n + j], X[(int64_t)c * k + j], v);
            }
        }
        LA64[t] = v;
        L_A[t] = (float)v;
        return;
    }
    if (t == 0) {
        double tail = 0.0;
        for (int64_t i = k - 1; i >= r; --i) tail += lam[i] > 0.0 ? lam[i] : 0.0;    // smallest first
        *err2 = tail;
    }
    if (t < r) sigma[t] = lam[t] > 0.0 ? (float)sqrt(lam[t]) : 0.f;
    if (t >= (int64_t)r * n) return;
    const int c = (int)(t / n);
    const int64_t j = t % n;
    double acc = 0.0;
    for (int64_t i = 0; i < m; ++i) acc = fma(LA64[i * r + c], (double)T[i * ldt + j], acc);
    L_B[t] = lam[c] > 0.0 ? (float)(acc / lam[c]) : 0.f;     // L_A^T T / sigma^2 in both cases (L_A = u sigma)
}

struct ExactPlan {
    int64_t k;
    bool big;           // a layer beyond the small ones the solver was made for: T S from the MFMA kernel, multi-launch inverse iteration
    size_t off_a, off_b, off_vs, off_vec, off_x, off_scr, off_la, off_tt, off_dots, total;
};

void exact_plan(int64_t m, int64_t n, int r, ExactPlan* p) {
    p->k = m < n ? m : n;
    const size_t kk = align_up((size_t)p->k * p->k * 8, 256), vb = align_up((size_t)p->k * 8, 256);
    size_t off = 0;
    p->off_a = off; off += align_up((size_t)m * n * 8, 256);        // A (m x n) or A^T (n x m), fp64
    p->off_b = off; off += kk;                                      // Gram matrix, then scratch of the chain
    p->off_vs = off; off += kk;                                     // reflectors
    p->off_vec = off; off += 10 * vb;                               // eight chain vectors, tau store, eigenvalues
    p->off_x = off; off += align_up((size_t)r * p->k * 8, 256);
    p->off_scr = off; off += align_up((size_t)r * 3 * p->k * 8, 256);
    p->off_la = off; off += align_up((size_t)m * r * 8, 256);
    p->off_dots = off; off += 2048;                                 // up to 256 dot products
    p->big = m * n > ((int64_t)1 << 20);
    p->off_tt = off; off += p->big ? align_up((size_t)m * n * 4, 256) : 0;    // T^T for the fp32 product (A and A^T share off_a)
    p->total = off;
}

struct SpecPlan {
    int64_t k;
    size_t off_tt, off_a, off_at, off_b, off_vec, total;
};

void spectrum_plan(int64_t m, int64_t n, bool with_s, SpecPlan* p) {
    p->k = m < n ? m : n;
    size_t off = 0;
    const size_t mat = align_up((size_t)m * n * 4, 256);
    p->off_tt = off; off += (with_s || m <= n) ? mat : 0;          // T^T
    p->off_a = off; off += with_s ? mat : 0;                       // A = T S
    p->off_at = off; off += with_s ? mat : 0;                      // A^T
    p->off_b = off; off += align_up((size_t)p->k * p->k * 8, 256);
    p->off_vec = off; off += 8 * align_up((size_t)p->k * 8, 256);  // v (two), w, p, d, e, tau, scratch
    p->total = off;
}

}  // namespace

size_t aser_exact_workspace(int64_t m, int64_t n, int r) {
    ExactPlan p;
    exact_plan(m, n, r, &p);
    return p.total;
}

// The dense fp64 solver on the bound workspace: L_A, L_B, sigma and, in *err2_dev (device), the squared
// whitened error.  Asynchronous.  The caller has checked shapes and the workspace size.
int aser_exact_reconstruct(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt, const float* S, int64_t lds,
                           int r, float* L_A, float* L_B, float* sigma, double* err2_dev) {
    ExactPlan pl;
    exact_plan(m, n, r, &pl);
    char* ws = (char*)ctx->ws;
    const int64_t k = pl.k;
    const bool left = m <= n;
    double* A64 = (double*)(ws + pl.off_a);
    double* B = (double*)(ws + pl.off_b);
    double* vstore = (double*)(ws + pl.off_vs);
    const size_t vb = align_up((size_t)k * 8, 256);
    double* vec[8];
    for (int i = 0; i < 8; ++i) vec[i] = (double*)(ws + pl.off_vec + i * vb);
    double* taustore = (double*)(ws + pl.off_vec + 8 * vb);
    double* lam = (double*)(ws + pl.off_vec + 9 * vb);
    double* X = (double*)(ws + pl.off_x);
    double* scr = (double*)(ws + pl.off_scr);
    double* LA64 = (double*)(ws + pl.off_la);
    const float* A32 = nullptr;                            // m x n, row-major: the fp32 product of large layers
    if (pl.big) {
        // Large layers (a rank beyond the subspace iteration's): T S from the MFMA kernel (about 2^-16 relative per
        // product, as in the iteration and in aser_singular_values), its Gram matrix in fp64 from the widened entries
        float* Tt = (float*)(ws + pl.off_tt);
        float* A = (float*)(ws + pl.off_a);
        float* At = A + (size_t)m * n;
        ASER_TRY(aser_transpose_f32(ctx, T, m, n, ldt, Tt, m));
        GemmArgs g{};
        g.A = Tt; g.lda = m; g.B = S; g.ldb = lds; g.C = A; g.ldc = n; g.Ct = At; g.ldct = m;
        g.M = m; g.N = n; g.K = n; g.alpha = 1.f;
        g.in_type = aser_f32_form(ctx, m * n); g.epi = GEMM_EPI_STORE; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_GE_COL;
        g.k_parts = 1;
        g.pair_cols = (m > 1024 && n > 1024) ? 1 : 0;
        g.bm = g.pair_cols ? 256 : 128; g.bn = 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
        A32 = A;
        if (left) ASER_TRY(gram_f64<float>(ctx, At, n, k, m, B));
        else ASER_TRY(gram_f64<float>(ctx, A, m, k, n, B));
    } else {
        // A = T S in fp64; for m <= n stored transposed (n x m), which is the K-major operand of A A^T
        dim3 grid((unsigned)ceil_div64(n, 64), (unsigned)ceil_div64(m, 4));
        if (left) hipLaunchKernelGGL(ts_f64_kernel<true>, grid, dim3(256), 0, ctx->stream, T, m, n, ldt, S, lds, A64);
        else hipLaunchKernelGGL(ts_f64_kernel<false>, grid, dim3(256), 0, ctx->stream, T, m, n, ldt, S, lds, A64);
        ASER_TRY(aser_check_launch(ctx, "ts_f64"));
        ASER_TRY(gram_f64<double>(ctx, A64, left ? n : m, k, k, B));
    }
    ASER_TRY(aser_fill_bytes(ctx, vstore, (size_t)k * k * 8));
    ASER_TRY(aser_fill_bytes(ctx, vec[0], 10 * vb));
    ASER_TRY(tridiagonalize(ctx, B, k, vec, vstore, taustore));
    double* sig64 = vec[7];
    ASER_TRY(tridiag_eigenvalues(ctx, k, vec[4], vec[5], sig64, lam));
    if (pl.big) {
        const double* dd = vec[4];
        const double* ee = vec[5];
        double* dots = (double*)(ws + pl.off_dots);
        const int64_t total = (int64_t)r * k;
        hipLaunchKernelGGL(invit_start_kernel, dim3((unsigned)(ceil_div64(total, 256) < 1024 ? ceil_div64(total, 256) : 1024)), dim3(256),
                           0, ctx->stream, total, X);
        for (int round = 0; round < 3; ++round) {
            hipLaunchKernelGGL(invit_solve_kernel, dim3((unsigned)ceil_div64(r, 64)), dim3(64), 0, ctx->stream, k, r, dd, ee,
                               (const double*)lam, X, scr);
            for (int c = 0; c < r; ++c) {
                for (int pass = 0; pass < 2 && c > 0; ++pass) {
                    hipLaunchKernelGGL(invit_dots_kernel, dim3((unsigned)c), dim3(256), 0, ctx->stream, k, c, (const double*)X, dots);
                    hipLaunchKernelGGL(invit_update_kernel, dim3((unsigned)ceil_div64(k, 256)), dim3(256), 0, ctx->stream, k, c, X,
                                       (const double*)dots);
                }
                hipLaunchKernelGGL(invit_normalize_kernel, dim3(1), dim3(256), 0, ctx->stream, k, c, X);
            }
            ASER_TRY(aser_check_launch(ctx, "tridiag_invit (multi-launch)"));
        }
    } else {
        hipLaunchKernelGGL(tridiag_invit_kernel, dim3(1), dim3(256), 0, ctx->stream, k, r, (const double*)vec[4], (const double*)vec[5],
                           (const double*)lam, X, scr);
        ASER_TRY(aser_check_launch(ctx, "tridiag_invit"));
    }
    hipLaunchKernelGGL(backtransform_kernel, dim3((unsigned)r), dim3(256), 0, ctx->stream, k, (const double*)vstore,
                       (const double*)taustore, X);
    ASER_TRY(aser_check_launch(ctx, "backtransform"));
    for (int phase = 0; phase < 2; ++phase) {
        const int64_t total = phase == 0 ? m * (int64_t)r : (int64_t)r * n;
        hipLaunchKernelGGL(exact_factors_kernel, dim3((unsigned)ceil_div64(total, 256)), dim3(256), 0, ctx->stream, phase, left ? 1 : 0,
                           m, n, k, r, (const double*)X, (const double*)lam, (const double*)A64, A32, T, ldt, LA64, L_A, L_B, sigma,
                           err2_dev);
        ASER_TRY(aser_check_launch(ctx, "exact_factors"));
    }
    return ASER_OK;
}

extern "C" size_t aser_spectrum_workspace_bytes(int64_t m, int64_t n, int32_t with_s) {
    if (m <= 0 || n <= 0) return 0;
    SpecPlan p;
    spectrum_plan(m, n, with_s != 0, &p);
    return p.total + kAserWsTail;
}

extern "C" int aser_singular_values(aser_ctx* ctx, const float* T, int64_t m, int64_t n, int64_t ldt,
                                    const float* S, int64_t lds, double* sigma) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!T || !sigma) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "singular_values: null pointer");
    if (m <= 0 || n <= 0 || ldt < n || (S && lds < n)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "singular_values: bad shape");
    if (((uintptr_t)T & 3) || (S && ((uintptr_t)S & 3)) || ((uintptr_t)sigma & 7))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "singular_values: misaligned pointer");
    SpecPlan pl;
    spectrum_plan(m, n, S != nullptr, &pl);
    if (pl.k > 16384) ASER_FAIL(ctx, ASER_ERR_SHAPE, "singular_values: min(m, n) > 16384 is not supported");
    if (!ctx->ws || ctx->ws_bytes < pl.total + kAserWsTail)
        ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "singular_values: workspace too small (%zu needed)", pl.total + kAserWsTail);
    ASER_TRY(aser_prepare_device(ctx));
    char* ws = (char*)ctx->ws;
    float* Tt = (float*)(ws + pl.off_tt);
    float* A = (float*)(ws + pl.off_a);
    float* At = (float*)(ws + pl.off_at);
    double* B = (double*)(ws + pl.off_b);
    const size_t vb = align_up((size_t)pl.k * 8, 256);
    double* vec[8];
    for (int i = 0; i < 8; ++i) vec[i] = (double*)(ws + pl.off_vec + i * vb);
    double *d = vec[4], *e = vec[5];
    const int64_t k = pl.k;

    // the K-major operand of the Gram matrix on the shorter side: Z^T for m <= n, Z for m > n
    const float* P;
    int64_t ldp, K;
    if (S) {
        ASER_TRY(aser_transpose_f32(ctx, T, m, n, ldt, Tt, m));
        GemmArgs g{};
        g.A = Tt; g.lda = m; g.B = S; g.ldb = lds; g.C = A; g.ldc = n; g.Ct = At; g.ldct = m;
        g.M = m; g.N = n; g.K = n; g.alpha = 1.f;
        g.in_type = aser_f32_form(ctx, m * n); g.epi = GEMM_EPI_STORE; g.tiles = GEMM_TILES_ALL; g.krange = GEMM_K_GE_COL;
        g.k_parts = 1;
        g.pair_cols = (m > 1024 && n > 1024) ? 1 : 0;
        g.bm = g.pair_cols ? 256 : 128; g.bn = 128;
        ASER_TRY(aser_gemm_tn(ctx, g));
        if (m <= n) { P = At; ldp = m; K = n; } else { P = A; ldp = n; K = m; }
    } else if (m <= n) {
        ASER_TRY(aser_transpose_f32(ctx, T, m, n, ldt, Tt, m));
        P = Tt; ldp = m; K = n;
    } else {
        P = T; ldp = ldt; K = m;
    }
    ASER_TRY(gram_f64(ctx, P, K, k, ldp, B));
    ASER_TRY(aser_fill_bytes(ctx, vec[0], 8 * vb));
    ASER_TRY(tridiagonalize(ctx, B, k, vec, nullptr, nullptr));
    return tridiag_eigenvalues(ctx, k, d, e, sigma, nullptr);
}

extern "C" int aser_select_rank(aser_ctx* ctx, const double* sigma, int64_t k, double alpha, int32_t* r, double* stats) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!sigma || !r) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "select_rank: null pointer");
    if (k <= 0) ASER_FAIL(ctx, ASER_ERR_SHAPE, "select_rank: k must be positive");
    if (!(alpha > 0.0 && alpha < 1.0)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "select_rank: alpha must lie in (0, 1)");
    if ((uintptr_t)sigma & 7) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "select_rank: misaligned pointer");
    if (!ctx->ws || ctx->ws_bytes < kAserWsTail) ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "select_rank: workspace too small");
    ASER_TRY(aser_prepare_device(ctx));
    // results go to the workspace tail, behind the two status words (bytes 64 .. 127)
    char* slot = (char*)ctx->ws + ctx->ws_bytes - kAserWsTail + 64;
    int32_t* r_dev = (int32_t*)slot;
    double* st_dev = (double*)(slot + 8);
    hipLaunchKernelGGL(select_rank_kernel, dim3(1), dim3(64), 0, ctx->stream, sigma, k, alpha, r_dev, st_dev);
    ASER_TRY(aser_check_launch(ctx, "select_rank"));
    int32_t h_r = 0;
    double h_st[3] = {0.0, 0.0, 0.0};
    ASER_HIP(ctx, hipMemcpyAsync(&h_r, r_dev, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream));
    ASER_HIP(ctx, hipMemcpyAsync(h_st, st_dev, sizeof(h_st), hipMemcpyDeviceToHost, ctx->stream));
    ASER_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (!(h_st[0] > 0.0)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "select_rank: the singular values do not have a positive sum");
    *r = h_r;
    if (stats) { stats[0] = h_st[0]; stats[1] = h_st[1]; stats[2] = h_st[2]; }
    return ASER_OK;
}

extern "C" int aser_effective_rank(aser_ctx* ctx, const double* sigma, int64_t k, double eps, double* erank) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!sigma || !erank) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "effective_rank: null pointer");
    if (k <= 0) ASER_FAIL(ctx, ASER_ERR_SHAPE, "effective_rank: k must be positive");
    if (!(eps >= 0.0)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "effective_rank: eps must be >= 0");
    if ((uintptr_t)sigma & 7) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "effective_rank: misaligned pointer");
    if (!ctx->ws || ctx->ws_bytes < kAserWsTail) ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "effective_rank: workspace too small");
    ASER_TRY(aser_prepare_device(ctx));
    double* out_dev = (double*)((char*)ctx->ws + ctx->ws_bytes - kAserWsTail + 128);   // bytes 128 .. 135 of the tail
    hipLaunchKernelGGL(effective_rank_kernel, dim3(1), dim3(1024), 0, ctx->stream, sigma, k, eps, out_dev);
    ASER_TRY(aser_check_launch(ctx, "effective_rank"));
    double h = 0.0;
    ASER_HIP(ctx, hipMemcpyAsync(&h, out_dev, sizeof(double), hipMemcpyDeviceToHost, ctx->stream));
    ASER_HIP(ctx, hipStreamSynchronize(ctx->stream));
    *erank = h;
    return ASER_OK;
}
