// Cholesky factor and its inverse for one diagonal block (b <= 128) of the blocked Cholesky of
// the whitening step (Eq. 5) and of the Cholesky-QR steps of the truncated SVD (Eq. 6).
//
// One workgroup of 16 wavefronts, the block in LDS, blocked again into 32-wide sub-blocks k = 0..3.
// All arithmetic is fp32: the products run on the fp32 MFMA instructions.
//
//   1. one wavefront factors the 32 x 32 diagonal sub-block A_kk with the sub-block and an identity
//      next to it held in two 32 x 32 MFMA accumulators.  Pivot j: reciprocal square root of the
//      diagonal entry, row j scaled (that is row j of R_kk and, in the second accumulator, row j of
//      L_kk^-1 with R_kk = L_kk^T), then one rank-1 MFMA update per accumulator (the next row is
//      updated by plain FMAs on a copy, so the pivot chain does not wait for the MFMAs).  An accumulator
//      register holds row j in one half of the lanes and row j +- 4 in the other; the MFMA's second
//      k-slot takes a zero multiplier for that half, so no lane exchange is needed.
//   2. everyone, 16 x 16 MFMA tiles: row panel R[k, right] = L_kk^-1 A[k, right] and, for the
//      inverse, Y = R[above, k] X_kk with X_kk = R_kk^-1.
//   3. everyone: trailing update A[right, right] -= R[k, right]^T R[k, right] over the upper
//      triangle of tiles, and the new block column of the inverse X[above, k] = -X[above, above] Y.
//
// A non-positive pivot at column j is reported as atomicMin(info, pivot_base + j + 1); its row is
// left unscaled (the factor is meaningless from there on).  Rows and columns beyond b are padded with the identity.
#include "aser_internal.h"

namespace {

typedef float f16v __attribute__((ext_vector_type(16)));
typedef float f4v __attribute__((ext_vector_type(4)));

constexpr int kN = 128;       // largest block
constexpr int kP = 133;       // odd LDS pitch: a wavefront reads along a row or a column without bank conflicts
constexpr int kPY = 33;
constexpr int kSub = 32;
constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ float lane_bcast(float v, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// acc(16 x 16) += sum over nk4 * 4 values of k of  sa * Aop(i, k) * Bop(k, c).  pa points at
// Aop(lane & 15, lane >> 4), pb at Bop(lane >> 4, lane & 15); sak / sbk are the strides along k.
__device__ __forceinline__ f4v mma16(f4v acc, const float* pa, int sak, const float* pb, int sbk, int nk4, float sa) {
#pragma unroll 4
    for (int s = 0; s < nk4; ++s) {
        const float a = pa[s * 4 * sak] * sa, bv = pb[s * 4 * sbk];
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a, bv, acc, 0, 0, 0);
    }
    return acc;
}

// Trailing update of one 16 x 16 tile behind the sub-block at offset o: A[i][c] -= sum_k P[k][i] P[k][c]
// with the row panel P in rows o .. o + 31, tile (ti <= tc) counted from column o + 32.
__device__ __forceinline__ void trailing_tile(float* As, int o, int ti, int tc, int t_i, int t_q) {
    const float* prow = As + o * kP + o + kSub;
    float* out = As + (o + kSub + 16 * ti + 4 * t_q) * kP + o + kSub + 16 * tc + t_i;
    f4v c;
#pragma unroll
    for (int e = 0; e < 4; ++e) c[e] = out[e * kP];
    c = mma16(c, prow + t_q * kP + 16 * ti + t_i, kP, prow + t_q * kP + 16 * tc + t_i, kP, 8, -1.f);
#pragma unroll
    for (int e = 0; e < 4; ++e) out[e * kP] = c[e];
}

__global__ __launch_bounds__(kThreads) void chol_block_kernel(float* D, int64_t ld, int b, float* Rinv, int32_t* info,
                                                              int32_t pivot_base, int clear_d, const float* Lmul,
                                                              float* Cmul, float* beta_out, const int* gate) {
    extern __shared__ __align__(16) float sm[];
    if (gate && *gate == 0) return;
    float* As = sm;                      // working matrix, upper triangle -> R
    float* Xs = As + kN * kP;            // R^-1 (upper), zero elsewhere
    float* Ys = Xs + kN * kP;            // 96 x 32 scratch, then 64 words that take masked-off stores
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nsub = (b + kSub - 1) / kSub;
    const int nb = nsub * kSub;          // padded with the identity up to here
    // 16 x 16 tile roles of this lane
    const int t_i = lane & 15, t_q = lane >> 4;

    // all global loads of a thread are issued before the first LDS store; 16-byte loads when the block allows it
    const bool vec = (((uintptr_t)D | (uintptr_t)Rinv) & 15) == 0 && (ld & 3) == 0 && (b & 3) == 0;
    if (vec) {
        constexpr int kPer = kN * kN / 4 / kThreads;
        float4 v[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int t = tid + u * kThreads, i = t >> 5, k = (t & 31) * 4;
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (k + 3 >= i && k < b && i < b) v[u] = *(const float4*)(D + (int64_t)i * ld + k);
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int t = tid + u * kThreads, i = t >> 5, k = (t & 31) * 4;
            const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool in = k + q >= i && k + q < b && i < b;
                As[i * kP + k + q] = in ? e[q] : ((k + q == i) ? 1.f : 0.f);
                Xs[i * kP + k + q] = 0.f;
            }
        }
    } else {
        constexpr int kPer = kN * kN / kThreads;
        float v[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int t = tid + u * kThreads, i = t >> 7, k = t & 127;
            v[u] = (k == i) ? 1.f : 0.f;
            if (k >= i && k < b && i < b) v[u] = D[(int64_t)i * ld + k];
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int t = tid + u * kThreads, i = t >> 7, k = t & 127;
            As[i * kP + k] = v[u];
            Xs[i * kP + k] = 0.f;
        }
    }
    __syncthreads();

    // Round kb factors diagonal sub-block kb (one wavefront), forms its row panel and the Y block, and
    // updates what lies behind it.  The pivot chain is the long part and keeps a single wavefront busy,
    // so it runs beside the bulk of the previous round's updates: once the three 16 x 16 tiles of the
    // next diagonal sub-block are updated, wavefront 0 starts on it while the other fifteen finish the
    // rest of the trailing update and the new block column of the inverse.
    for (int kb = 0; kb <= nsub; ++kb) {
        const int o = kb * kSub;
        const int ncb = nsub - 1 - kb;             // 32-column blocks to the right

        // ---- 1. diagonal sub-block: accumulator register e of lane l holds row 8 (e / 4) + 4 (l / 32) + e % 4, column l % 32
        if (wave == 0 && kb < nsub) {
            const int h = lane >> 5, col = lane & 31;
            f16v a1, a2;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = 8 * (e / 4) + 4 * h + e % 4;
                a1[e] = As[(o + row) * kP + o + col];
                a2[e] = (row == col) ? 1.f : 0.f;
            }
            int bad = kSub;
            // LDS targets of this lane's row / column stores; the half of the lanes that holds another
            // row in the same register writes to a scratch word instead (no exec-mask changes in the chain)
            float* const dummy = Ys + 96 * kPY + lane;
            // One row of look-ahead keeps the MFMA latency out of the pivot chain: update j leaves row
            // j + 1 to two plain FMAs on a copy taken from the accumulators before the MFMAs of step j
            // are issued (their multiplier for that row is zero), so pivot j + 1 depends on pivot j
            // through a handful of VALU operations only, and the MFMAs run behind.
            float x1 = a1[0], x2 = a2[0];             // row j of both accumulators, all updates applied
#pragma unroll
            for (int j = 0; j < kSub; ++j) {
                const int hj = (j / 4) & 1;
                const int en = 4 * ((j + 1) / 8) + (j + 1) % 4;                    // register of row j + 1
                float y1 = 0.f, y2 = 0.f;
                if (j + 1 < kSub) {                                               // updates < j applied
                    // explicit early copies: read lazily, these elements would keep the old accumulator
                    // tuples alive and every VALU access to them would wait for the MFMA in flight
                    asm volatile("v_mov_b32 %0, %1" : "=v"(y1) : "v"(a1[en]));
                    asm volatile("v_mov_b32 %0, %1" : "=v"(y2) : "v"(a2[en]));
                }
                const float piv = lane_bcast(x1, 32 * hj + j);
                const bool ok = piv > 0.f;
                bad = ok ? bad : (bad < j ? bad : j);
                const float rs = __builtin_amdgcn_rsqf(ok ? piv : 1.f);   // 1 ulp: as good as the fp32 data it scales
                // Instruction order matters (one wave, in-order issue): the wave stalls at an MFMA
                // until the pipe accepts it, so the scalar work of the chain is placed behind the first
                // MFMA of the step and the work on the second accumulator behind the second.
                const float rv = x1 * rs;
                const float mult = (h == hj && col != j + 1) ? -rv : 0.f;
                if (j + 2 < kSub) a1 = __builtin_amdgcn_mfma_f32_32x32x2f32(mult, rv, a1, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                float m = 0.f;
                if (j + 1 < kSub) {
                    m = lane_bcast(rv, 32 * hj + j + 1);                           // r_j[j + 1]
                    // row j + 1 sits in the other half of the lanes when j + 1 starts a new group of four
                    const float rvn = (j % 4 == 3) ? __shfl_xor(rv, 32, 64) : rv;
                    x1 = fmaf(-m, rvn, y1);
                }
                *((h == hj) ? As + (o + j) * kP + o + col : dummy) = rv;   // row j of R_kk (left of the diagonal: dead)
                const float lv = x2 * rs;
                __builtin_amdgcn_sched_barrier(0);
                if (j + 2 < kSub) a2 = __builtin_amdgcn_mfma_f32_32x32x2f32(mult, lv, a2, 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (j + 1 < kSub) {
                    const float lvn = (j % 4 == 3) ? __shfl_xor(lv, 32, 64) : lv;
                    x2 = fmaf(-m, lvn, y2);
                }
                *((h == hj) ? Xs + (o + col) * kP + o + j : dummy) = lv;   // X_kk = (L_kk^-1)^T
            }
            if (bad < kSub && lane == 0 && o + bad < b && info) atomicMin(info, pivot_base + o + bad + 1);
        }
        if (kb > 0 && (wave > 0 || kb == nsub)) {
            // ---- rest of round kb - 1: new block column of the inverse (long jobs first), then the trailing
            // update without the tiles of diagonal sub-block kb (done before the last barrier)
            const int op = o - kSub;
            const int w0 = (kb < nsub) ? 1 : 0;
            const int nx = (op / 16) * 2;
            const int nt = 2 * (ncb + 1), ntri = nt * (nt + 1) / 2;
            for (int job = wave - w0; job < nx + ntri; job += kWaves - w0) {
                if (job < nx) {
                    // X[i][op + c] = -sum_{t >= i} X[i][t] Y[t][c]
                    const int it = job >> 1, cj = job & 1;
                    const float* pa = Xs + (16 * it + t_i) * kP + 16 * it + t_q;
                    const float* pb = Ys + (16 * it + t_q) * kPY + 16 * cj + t_i;
                    f4v x = {0.f, 0.f, 0.f, 0.f};
                    x = mma16(x, pa, 1, pb, kPY, (op - 16 * it) / 4, -1.f);
#pragma unroll
                    for (int e = 0; e < 4; ++e) Xs[(16 * it + 4 * t_q + e) * kP + op + 16 * cj + t_i] = x[e];
                } else {
                    // A[i][c] -= sum_k P[k][i] P[k][c] on tile (ti <= tc): rows ar and nt-1-ar of the
                    // triangle together hold nt + 1 tiles
                    const int idx = job - nx;
                    const int ar = idx / (nt + 1), cc = idx - ar * (nt + 1);
                    int ti, tc;
                    if (cc < nt - ar) { ti = ar; tc = ar + cc; }
                    else { ti = nt - 1 - ar; tc = ti + (cc - (nt - ar)); }
                    if (tc < 2) continue;                            // diagonal sub-block kb: already updated
                    trailing_tile(As, op, ti, tc, t_i, t_q);
                }
            }
        }
        __syncthreads();
        if (kb == nsub) break;

        // ---- 2. panel (one job per 16-column tile, both row halves) and Y (one job per 16 x 16 tile)
        {
            const int npan = 2 * ncb, ny = (o / 16) * 2;
            for (int job = wave; job < npan + ny; job += kWaves) {
                if (job < npan) {
                    // P[i][c] = sum_{k <= i} Linv[i][k] A[o + k][c],  Linv[i][k] = Xs[o + k][o + i]
                    float* colbase = As + o * kP + o + kSub + 16 * job;
                    const float* pb = colbase + t_q * kP + t_i;
                    const float* pa = Xs + (o + t_q) * kP + o + t_i;
                    f4v p0 = {0.f, 0.f, 0.f, 0.f}, p1 = {0.f, 0.f, 0.f, 0.f};
                    p0 = mma16(p0, pa, kP, pb, kP, 4, 1.f);            // rows 0..15: k < 16
                    p1 = mma16(p1, pa + 16, kP, pb, kP, 8, 1.f);       // rows 16..31: k < 32
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        colbase[(4 * t_q + e) * kP + t_i] = p0[e];
                        colbase[(16 + 4 * t_q + e) * kP + t_i] = p1[e];
                    }
                } else {
                    // Y[i][c] = sum_{k <= c} R[i][o + k] X_kk[k][c]
                    const int jy = job - npan, it = jy >> 1, cj = jy & 1;
                    const float* pa = As + (16 * it + t_i) * kP + o + t_q;
                    const float* pb = Xs + (o + t_q) * kP + o + 16 * cj + t_i;
                    f4v y = {0.f, 0.f, 0.f, 0.f};
                    y = mma16(y, pa, 1, pb, kP, cj ? 8 : 4, 1.f);
#pragma unroll
                    for (int e = 0; e < 4; ++e) Ys[(16 * it + 4 * t_q + e) * kPY + 16 * cj + t_i] = y[e];
                }
            }
        }
        __syncthreads();

        // ---- 3. the three tiles of the next diagonal sub-block
        if (ncb > 0) {
            if (wave < 3) trailing_tile(As, o, wave == 2 ? 1 : 0, wave == 0 ? 0 : 1, t_i, t_q);
            __syncthreads();
        }
    }

    // write out: R on and above the diagonal (or zeros over the whole input when clear_d; the part below the
    // diagonal is otherwise left as it is), and R^-1
    if (vec) {
        for (int t = tid; t < b * (kN / 4); t += kThreads) {
            const int i = t >> 5, k = (t & 31) * 4;
            if (k >= b) continue;
            float r[4], x[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                r[q] = (clear_d || k + q < i) ? 0.f : As[i * kP + k + q];
                x[q] = (k + q >= i) ? Xs[i * kP + k + q] : 0.f;
            }
            float* drow = D + (int64_t)i * ld + k;
            if (clear_d || k >= i) *(float4*)drow = make_float4(r[0], r[1], r[2], r[3]);
            else if (k + 3 >= i) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (k + q >= i) drow[q] = r[q];
            }
            *(float4*)(Rinv + i * b + k) = make_float4(x[0], x[1], x[2], x[3]);
        }
    } else {
        for (int t = tid; t < b * kN; t += kThreads) {
            const int i = t >> 7, k = t & 127;
            if (k < b) {
                if (clear_d || k >= i) D[(int64_t)i * ld + k] = clear_d ? 0.f : As[i * kP + k];
                Rinv[i * b + k] = (k >= i) ? Xs[i * kP + k] : 0.f;
            }
        }
    }
    if (!Lmul && !beta_out) return;
    // ---- optional: the momentum coefficient of the subspace iteration, -(0.9 s^2 / 2)^2 with s the smallest
    // diagonal entry of R, and whether the diagonal of R spans more than a factor of 64
    if (beta_out) {
        float smin = 3.0e38f, smax = 0.f;
        if (tid < b) smin = smax = 1.0f / fabsf(Xs[tid * kP + tid]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            smin = fminf(smin, __shfl_xor(smin, o, 64));
            smax = fmaxf(smax, __shfl_xor(smax, o, 64));
        }
        if (lane == 0 && wave < 2) { Ys[wave] = smin; Ys[2 + wave] = smax; }
        __syncthreads();
        if (tid == 0) {
            const float s = fminf(Ys[0], Ys[1]), hbeta = 0.45f * s * s;
            beta_out[0] = -hbeta * hbeta;
            ((int*)beta_out)[1] = (fmaxf(Ys[2], Ys[3]) > 64.f * s) ? 1 : 0;
        }
    }
    if (!Lmul) return;

    // ---- optional: Cmul = Lmul R^-1 for an upper triangular b x b Lmul (ld = b), with R^-1 still in LDS
    __syncthreads();                                      // everyone has read R out of As
    {
        constexpr int kPer = kN * kN / kThreads;
        float v[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int t = tid + u * kThreads, i = t >> 7, k = t & 127;
            v[u] = (k >= i && k < b) ? Lmul[i * b + k] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int t = tid + u * kThreads, i = t >> 7, k = t & 127;
            As[i * kP + k] = v[u];
        }
    }
    const float alpha = 1.f;
    __syncthreads();
    // 36 upper tiles of 16 x 16, longest k range first: tile (ti, tj) needs k in [16 ti, 16 tj + 16)
    for (int job = wave; job < 36; job += kWaves) {
        int d = 7, first = 0;
        while (job >= first + (8 - d)) { first += 8 - d; --d; }
        const int ti = job - first, tj = ti + d;
        f4v acc = {0.f, 0.f, 0.f, 0.f};
        acc = mma16(acc, As + (16 * ti + t_i) * kP + 16 * ti + t_q, 1, Xs + (16 * ti + t_q) * kP + 16 * tj + t_i, kP, 4 * (d + 1), alpha);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = 16 * ti + 4 * t_q + e, j = 16 * tj + t_i;
            if (i < b && j < b) Cmul[i * b + j] = acc[e];
        }
    }
    for (int t = tid; t < b * b; t += kThreads) {
        const int i = t / b, j = t % b;
        if ((i >> 4) > (j >> 4)) Cmul[t] = 0.f;
    }
}

}  // namespace

int aser_chol_block(aser_ctx* ctx, float* D, int64_t ld, int b, float* Rinv, int32_t* info, int32_t pivot_base, bool clear_d,
                    const float* Lmul, float* Cmul, float* beta_out, const int* gate) {
    if (b <= 0 || b > kN) ASER_FAIL(ctx, ASER_ERR_SHAPE, "chol_block: block size out of range");
    static bool attr_set[16] = {false};
    const size_t lds = (size_t)(2 * kN * kP + 96 * kPY + 64) * sizeof(float);
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)chol_block_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(chol_block_kernel, dim3(1), dim3(kThreads), lds, ctx->stream, D, ld, b, Rinv, info, pivot_base,
                       clear_d ? 1 : 0, Lmul, Cmul, beta_out, gate);
    return aser_check_launch(ctx, "chol_block");
}
