// Bandwidth-bound kernels of the ASER calibration path (gfx950): channel statistics for the
// smoothing step (Sec. 4.2), per-channel RTN with the target T = E_q + W_o (Eq. 12), the
// per-token activation quantizer (Sec. 5.1), and the layout helpers around the MFMA kernel.
// All of them stream their operands once with 16-byte accesses that are contiguous along the
// channel dimension; row reductions use wavefront shuffles.
#include "aser_internal.h"

namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// max over the workgroup (blockDim.x multiple of 64, at most 1024); red: >= 16 floats of LDS
__device__ __forceinline__ float block_max(float v, float* red) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < nw; ++i) r = fmaxf(r, red[i]);
    __syncthreads();
    return r;
}

// ------------------------------------------------------------------------------------ fills
__global__ void fill_f32_kernel(float* p, int64_t rows, int64_t cols, int64_t ld, float v) {
    const int64_t total = rows * cols;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x)
        p[(i / cols) * ld + (i % cols)] = v;
}

__global__ void set_i32_kernel(int32_t* p, int32_t v) { *p = v; }

__global__ void fill_zero_kernel(uint32_t* p, int64_t words) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < words; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0u;
}

__global__ void fill_zero16_kernel(uint4* p, int64_t quads) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < quads; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// ------------------------------------------------------------------------------------ column |.| sums
// A workgroup is 64 column groups (16 bytes each) x 4 row lanes over a strip of rows.  Each thread
// sums its rows in fp64; the four row lanes are combined through LDS and one fp64 atomic per
// column and strip goes to abs_sum.  The strips are long (about one workgroup per compute unit):
// the atomics on the few thousand shared addresses, not the reads, set the time of short strips
// (32768 x 4096 bf16: 85 us with 256-row strips, 49 us with 1024-row strips, 43 us without atomics).
template <bool BF16>
__global__ __launch_bounds__(256) void col_abs_sum_kernel(const void* X, int64_t rows, int64_t n, int64_t ld,
                                                          int64_t rows_per_block, double* out, int64_t* count,
                                                          int64_t count_add) {
    constexpr int VEC = BF16 ? 8 : 4;
    constexpr int ESZ = BF16 ? 2 : 4;
    __shared__ double part[3][64][VEC];
    if (count && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
        atomicAdd((unsigned long long*)count, (unsigned long long)count_add);
    if (!out) return;
    const int cgl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int64_t col = ((int64_t)blockIdx.x * 64 + cgl) * VEC;
    const int nc = (col >= n) ? 0 : ((n - col >= VEC) ? VEC : (int)(n - col));
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < rows) ? r0 + rows_per_block : rows;
    const char* base = (const char*)X + col * ESZ;
    const bool vec_ok = nc == VEC && (((uintptr_t)base & 15) == 0) && (((ld * ESZ) & 15) == 0);
    double acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.0;
    if (vec_ok) {
        int64_t r = r0 + rl;
        for (; r + 28 < r1; r += 32) {
            uint4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *(const uint4*)(base + (r + 4 * u) * ld * ESZ);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    if (BF16) {
                        acc[2 * d] += (double)fabsf(bf16_lo(w[d]));
                        acc[2 * d + 1] += (double)fabsf(bf16_hi(w[d]));
                    } else {
                        acc[d] += (double)fabsf(__uint_as_float(w[d]));
                    }
                }
            }
        }
        for (; r < r1; r += 4) {
            const uint4 v = *(const uint4*)(base + r * ld * ESZ);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                if (BF16) {
                    acc[2 * d] += (double)fabsf(bf16_lo(w[d]));
                    acc[2 * d + 1] += (double)fabsf(bf16_hi(w[d]));
                } else {
                    acc[d] += (double)fabsf(__uint_as_float(w[d]));
                }
            }
        }
    } else if (nc > 0) {
        for (int64_t r = r0 + rl; r < r1; r += 4) {
            const char* q = base + r * ld * ESZ;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                if (e < nc) {
                    const float x = BF16 ? __uint_as_float((uint32_t)(*(const uint16_t*)(q + 2 * e)) << 16)
                                         : *(const float*)(q + 4 * e);
                    acc[e] += (double)fabsf(x);
                }
            }
        }
    }
    if (rl > 0) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) part[rl - 1][cgl][e] = acc[e];
    }
    __syncthreads();
    if (rl == 0) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const double t = acc[e] + part[0][cgl][e] + part[1][cgl][e] + part[2][cgl][e];
            if (e < nc) atomicAdd(out + col + e, t);
        }
    }
}

// ------------------------------------------------------------------------------------ transpose
__global__ __launch_bounds__(256) void transpose_kernel(const float* A, int64_t rows, int64_t cols, int64_t lda,
                                                        float* At, int64_t ldat) {
    __shared__ float tile[64][65];
    const int64_t r0 = (int64_t)blockIdx.y * 64, c0 = (int64_t)blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int i = ty; i < 64; i += 4) {
        const int64_t r = r0 + i, c = c0 + tx;
        tile[i][tx] = (r < rows && c < cols) ? A[r * lda + c] : 0.f;
    }
    __syncthreads();
    for (int i = ty; i < 64; i += 4) {
        const int64_t c = c0 + i, r = r0 + tx;
        if (c < cols && r < rows) At[c * ldat + r] = tile[tx][i];
    }
}

// rint(x / scale) with the result of the IEEE division, at the cost of a multiplication: the
// quotient is first formed with the hardware reciprocal (relative error below 2e-7, so absolute
// error below 3e-5 for |x / scale| <= 128); only when that value lies within 1e-4 of a rounding
// boundary k + 1/2 can the two roundings differ, and then the correctly rounded division decides.
__device__ __forceinline__ float rint_div(float x, float scale, float rscale) {
    float q = x * rscale;
    const float aq = fabsf(q);
    const bool near = !(aq < 200.f) || fabsf(aq - floorf(aq) - 0.5f) < 1e-4f;   // also: reciprocal of a denormal scale
    // a wave-uniform branch, so that the division is really skipped and not just masked
    if (__builtin_amdgcn_ballot_w64(near) != 0) q = near ? x / scale : q;
    return rintf(q);
}

// ------------------------------------------------------------------------------------ weight RTN
// One workgroup per output row (256 to 1024 threads, two or four groups each, so that wide rows
// still run at full occupancy).  A thread owns groups of 8 consecutive columns; the row stays in
// registers between the absmax reduction and the quantization, so W is read from HBM once.  The
// global loads are issued before the outlier-column bitmask is built in LDS, so that its two
// barriers overlap the load latency.  Integer decisions (scale, codes) are taken in IEEE fp32 with
// correctly rounded division and round-half-to-even.
template <int VPT, int NT>   // 8-column groups per thread, threads per row
__global__ __launch_bounds__(NT) void rtn_kernel(const float* __restrict__ W, int64_t n, int64_t ldw,
                                                  const int32_t* __restrict__ idx, const float* __restrict__ mdiag, int f,
                                                  float qmax, int layout, uint8_t* __restrict__ codes, int64_t code_pitch,
                                                  float* __restrict__ scales, float* __restrict__ T, int64_t ldt) {
    extern __shared__ uint32_t smem_u32[];
    uint32_t* mask = smem_u32;                       // ceil(n / 32) words: 1 = outlier column
    float* red = (float*)(smem_u32 + ((n + 31) / 32));
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const float* wrow = W + row * ldw;
    const bool vec_ok = (((uintptr_t)wrow & 15) == 0) && ((n & 7) == 0);
    float v[VPT][8];
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * NT + tid) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[u][e] = 0.f;
        if (c < n) {
            if (vec_ok) {
                const f32x4_t x0 = *(const f32x4_t*)(wrow + c);
                const f32x4_t x1 = *(const f32x4_t*)(wrow + c + 4);
                v[u][0] = x0.x; v[u][1] = x0.y; v[u][2] = x0.z; v[u][3] = x0.w;
                v[u][4] = x1.x; v[u][5] = x1.y; v[u][6] = x1.z; v[u][7] = x1.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (c + e < n) v[u][e] = wrow[c + e];
            }
        }
    }
    const int mask_words = (int)((n + 31) / 32);
    for (int i = tid; i < mask_words; i += NT) mask[i] = 0u;
    __syncthreads();
    for (int i = tid; i < f; i += NT) {
        const int c = idx[i];
        if (c >= 0 && c < n) atomicOr(&mask[c >> 5], 1u << (c & 31));   // entries outside [0, n) are ignored
    }
    __syncthreads();

    uint32_t om[VPT];                                 // 8 outlier bits per group
    float amax = 0.f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * NT + tid) * 8;
        om[u] = 0u;
        if (c < n) {
            om[u] = (mask[c >> 5] >> (c & 31)) & 0xFFu;   // c is a multiple of 8: one mask word
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, ((om[u] >> e) & 1u) ? 0.f : fabsf(v[u][e]));
        }
    }
    amax = block_max(amax, red);
    const float scale = (amax == 0.f) ? 1.f : amax / qmax;
    // the reciprocal of a denormal scale is not finite: such a row takes true divisions throughout
    const bool plain = __builtin_amdgcn_readfirstlane(scale > 1e-30f ? 1 : 0) != 0;
    const float rscale = plain ? __builtin_amdgcn_rcpf(scale) : 0.f;
    if (tid == 0) scales[row] = scale;

    uint8_t* crow = codes + row * code_pitch;
    float* trow = T ? T + row * ldt : nullptr;
    const bool t_vec = T && (((uintptr_t)trow & 15) == 0) && ((n & 7) == 0);
    const bool c_vec = vec_ok && (((uintptr_t)crow & 7) == 0);
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * NT + tid) * 8;
        if (c >= n) continue;
        float t[8];
        int q[8];
        if (plain && __builtin_amdgcn_ballot_w64(om[u] != 0u) == 0) {
            // no outlier column in this wavefront's groups: rint(w / scale) from the reciprocal multiply
            // (error below 4e-5), one test per group for a quotient within 1e-4 of a rounding boundary
            // k + 1/2, where the correctly rounded division decides
            float r[8], dist[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float tq = v[u][e] * rscale;
                r[e] = rintf(tq);
                dist[e] = fabsf(tq - r[e]);
            }
            const float far = fmaxf(fmaxf(fmaxf(dist[0], dist[1]), fmaxf(dist[2], dist[3])),
                                    fmaxf(fmaxf(dist[4], dist[5]), fmaxf(dist[6], dist[7])));
            if (__builtin_amdgcn_ballot_w64(far > 0.4999f) != 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    if (dist[e] > 0.4999f) r[e] = rintf(v[u][e] / scale);
                    asm volatile("" : "+v"(r[e]));        // keeps the division behind its branch
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                q[e] = (int)r[e];
                t[e] = __fmaf_rn(-r[e], scale, v[u][e]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if ((om[u] >> e) & 1u) {
                    q[e] = 0;
                    t[e] = (c + e < n) ? v[u][e] * mdiag[c + e] : 0.f;
                } else {
                    float qf = plain ? rint_div(v[u][e], scale, rscale) : rintf(v[u][e] / scale);
                    qf = fminf(fmaxf(qf, -qmax), qmax);
                    q[e] = (int)qf;
                    t[e] = __fmaf_rn(-qf, scale, v[u][e]);
                }
            }
        }
        if (layout == ASER_CODES_INT8) {
            if (c_vec) {
                uint2 pk;
                pk.x = (uint32_t)(q[0] & 0xFF) | ((uint32_t)(q[1] & 0xFF) << 8) | ((uint32_t)(q[2] & 0xFF) << 16) |
                       ((uint32_t)(q[3] & 0xFF) << 24);
                pk.y = (uint32_t)(q[4] & 0xFF) | ((uint32_t)(q[5] & 0xFF) << 8) | ((uint32_t)(q[6] & 0xFF) << 16) |
                       ((uint32_t)(q[7] & 0xFF) << 24);
                const u32x2_t pkv = {pk.x, pk.y};
                __builtin_nontemporal_store(pkv, (u32x2_t*)(crow + c));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (c + e < n) crow[c + e] = (uint8_t)(q[e] & 0xFF);
            }
        } else {   // int4, n even: columns (c, c+1) -> byte c/2, low nibble = even column
            if (c_vec) {
                uint32_t pk = 0u;
#pragma unroll
                for (int e = 0; e < 8; ++e) pk |= (uint32_t)(q[e] & 0xF) << (4 * e);
                __builtin_nontemporal_store(pk, (uint32_t*)(crow + c / 2));
            } else {
#pragma unroll
                for (int e = 0; e < 8; e += 2)
                    if (c + e + 1 < n) crow[(c + e) / 2] = (uint8_t)((q[e] & 0xF) | ((q[e + 1] & 0xF) << 4));
            }
        }
        if (trow) {
            if (t_vec) {
                const f32x4_t t0 = {t[0], t[1], t[2], t[3]}, t1 = {t[4], t[5], t[6], t[7]};
                __builtin_nontemporal_store(t0, (f32x4_t*)(trow + c));
                __builtin_nontemporal_store(t1, (f32x4_t*)(trow + c + 4));
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (c + e < n) trow[c + e] = t[e];
            }
        }
    }
}

// ------------------------------------------------------------------------------------ other weight quantizers
// The two element-wise passes around a caller's own weight quantizer (Sec. 4.1, closing remark).  A workgroup takes
// 1024 columns of 8 rows, a thread four consecutive columns of each row (16-byte accesses where base and leading
// dimensions allow).  TARGET: out = W * m - Wq in one fused multiply-add.  Otherwise out = W with the outlier
// columns cleared; their bitmask for this workgroup's columns is built in LDS first.
template <bool TARGET>
__global__ __launch_bounds__(256) void base_quantizer_kernel(const float* __restrict__ W, int64_t m, int64_t n, int64_t ldw,
                                                             const int32_t* __restrict__ idx, int f,
                                                             const float* __restrict__ mdiag, const float* Wq, int64_t ldq,
                                                             float* out, int64_t ldo, int vec) {
    __shared__ uint32_t mask[32];
    const int tid = threadIdx.x;
    const int64_t c0 = (int64_t)blockIdx.x * 1024, c = c0 + 4 * tid, r0 = (int64_t)blockIdx.y * 8;
    float mm[4] = {1.f, 1.f, 1.f, 1.f};
    uint32_t drop = 0u;                                  // bit e: column c + e is an outlier column
    if (TARGET) {
        if (mdiag) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c + e < n) mm[e] = mdiag[c + e];
        }
    } else {
        if (tid < 32) mask[tid] = 0u;
        __syncthreads();
        for (int i = tid; i < f; i += 256) {
            const int64_t k = (int64_t)idx[i] - c0;
            if (idx[i] >= 0 && idx[i] < n && k >= 0 && k < 1024) atomicOr(&mask[k >> 5], 1u << (k & 31));
        }
        __syncthreads();
        drop = (mask[tid >> 3] >> (4 * (tid & 7))) & 0xFu;
    }
    if (c >= n) return;
    const bool full = vec && c + 4 <= n;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int64_t r = r0 + i;
        if (r >= m) break;
        float w[4] = {0.f, 0.f, 0.f, 0.f}, q[4] = {0.f, 0.f, 0.f, 0.f}, o[4];
        if (full) {
            const f32x4_t x = __builtin_nontemporal_load((const f32x4_t*)(W + r * ldw + c));
            w[0] = x.x; w[1] = x.y; w[2] = x.z; w[3] = x.w;
            if (TARGET) {
                const f32x4_t y = __builtin_nontemporal_load((const f32x4_t*)(Wq + r * ldq + c));
                q[0] = y.x; q[1] = y.y; q[2] = y.z; q[3] = y.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c + e < n) {
                    w[e] = W[r * ldw + c + e];
                    if (TARGET) q[e] = Wq[r * ldq + c + e];
                }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = TARGET ? __fmaf_rn(w[e], mm[e], -q[e]) : (((drop >> e) & 1u) ? 0.f : w[e]);
        if (full) {
            const f32x4_t z = {o[0], o[1], o[2], o[3]};
            __builtin_nontemporal_store(z, (f32x4_t*)(out + r * ldo + c));
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c + e < n) out[r * ldo + c + e] = o[e];
        }
    }
}

// ------------------------------------------------------------------------------------ activation RTN
// One workgroup per token (256 to 1024 threads).  X' = X / m with an IEEE fp32 division, per-token
// absmax scale.  A thread owns groups of 8 consecutive channels: one 16-byte load of bf16 (two of
// fp32), one 8-byte store of codes; the token stays in registers between the absmax reduction
// and the rounding.
template <bool BF16, int VPT, int NT>
__global__ __launch_bounds__(NT) void act_rtn_kernel(const void* __restrict__ X, int64_t n, int64_t ldx,
                                                     const float* __restrict__ mdiag, float qmax,
                                                     int8_t* __restrict__ codes, float* __restrict__ scales) {
    __shared__ float red[16];
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const char* xrow = (const char*)X + row * ldx * (BF16 ? 2 : 4);
    const bool vec_ok = (((uintptr_t)xrow & 15) == 0) && ((n & 7) == 0);
    const bool m_vec = mdiag && (((uintptr_t)mdiag & 15) == 0);
    float v[VPT][8];
    float amax = 0.f;
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * NT + tid) * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[u][e] = 0.f;
        if (c >= n) continue;
        if (vec_ok) {
            if (BF16) {
                const u32x4_t w = __builtin_nontemporal_load((const u32x4_t*)(xrow + c * 2));
                const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    v[u][2 * e] = __uint_as_float(ww[e] << 16);
                    v[u][2 * e + 1] = __uint_as_float(ww[e] & 0xFFFF0000u);
                }
            } else {
                const f32x4_t x0 = __builtin_nontemporal_load((const f32x4_t*)(xrow + c * 4));
                const f32x4_t x1 = __builtin_nontemporal_load((const f32x4_t*)(xrow + c * 4 + 16));
                v[u][0] = x0.x; v[u][1] = x0.y; v[u][2] = x0.z; v[u][3] = x0.w;
                v[u][4] = x1.x; v[u][5] = x1.y; v[u][6] = x1.z; v[u][7] = x1.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (c + e < n)
                    v[u][e] = BF16 ? __uint_as_float((uint32_t)(((const uint16_t*)xrow)[c + e]) << 16) : ((const float*)xrow)[c + e];
        }
        if (mdiag) {
            float mm[8];
            if (m_vec && c + 8 <= n) {
                const float4 m0 = *(const float4*)(mdiag + c), m1 = *(const float4*)(mdiag + c + 4);
                mm[0] = m0.x; mm[1] = m0.y; mm[2] = m0.z; mm[3] = m0.w; mm[4] = m1.x; mm[5] = m1.y; mm[6] = m1.z; mm[7] = m1.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) mm[e] = (c + e < n) ? mdiag[c + e] : 1.f;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const bool scaled = mm[e] != 1.f;                                        // x / 1 = x exactly
                if (__builtin_amdgcn_ballot_w64(scaled) != 0) v[u][e] = scaled ? v[u][e] / mm[e] : v[u][e];
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(v[u][e]));
    }
    amax = block_max(amax, red);
    const float scale = (amax == 0.f) ? 1.f : amax / qmax;
    // the reciprocal of a denormal scale is not finite: such a token takes true divisions throughout
    const bool plain = __builtin_amdgcn_readfirstlane(scale > 1e-30f ? 1 : 0) != 0;
    const float rscale = plain ? __builtin_amdgcn_rcpf(scale) : 0.f;
    if (tid == 0) scales[row] = scale;
    int8_t* crow = codes + row * n;
    const bool c_vec = (((uintptr_t)crow & 7) == 0) && ((n & 7) == 0);
#pragma unroll
    for (int u = 0; u < VPT; ++u) {
        const int64_t c = ((int64_t)u * NT + tid) * 8;
        if (c >= n) continue;
        // rint(x / scale) from the reciprocal multiply (error below 4e-5 for |quotient| <= 128); one test
        // per group for a quotient within 1e-4 of a rounding boundary k + 1/2, where the division decides
        float r[8], dist[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float tq = v[u][e] * rscale;
            r[e] = rintf(tq);
            dist[e] = fabsf(tq - r[e]);
        }
        const float far = fmaxf(fmaxf(fmaxf(dist[0], dist[1]), fmaxf(dist[2], dist[3])),
                                fmaxf(fmaxf(dist[4], dist[5]), fmaxf(dist[6], dist[7])));
        if (!plain || __builtin_amdgcn_ballot_w64(far > 0.4999f) != 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if (!plain || dist[e] > 0.4999f) r[e] = rintf(v[u][e] / scale);
                asm volatile("" : "+v"(r[e]));                // keeps the division behind its branch
            }
        }
        int q[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) q[e] = (int)r[e];
        if (c_vec) {
            const u32x2_t pk = {__builtin_amdgcn_perm((uint32_t)q[1], (uint32_t)q[0], 0x0c0c0400u) |
                                    __builtin_amdgcn_perm((uint32_t)q[3], (uint32_t)q[2], 0x04000c0cu),
                                __builtin_amdgcn_perm((uint32_t)q[5], (uint32_t)q[4], 0x0c0c0400u) |
                                    __builtin_amdgcn_perm((uint32_t)q[7], (uint32_t)q[6], 0x04000c0cu)};
            __builtin_nontemporal_store(pk, (u32x2_t*)(crow + c));
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (c + e < n) crow[c + e] = (int8_t)q[e];
        }
    }
}

// Tokens of at most 4096 channels (16-byte aligned rows, n % 16 == 0): one wavefront per token, 4 groups
// of 16 channels per lane (32 bytes of bf16 in, 16 bytes of codes out), all loads of a token in
// flight at once, absmax by lane shuffles: no LDS and no barrier.  The arithmetic, not the memory
// system, bounds this kernel, so everything that depends on M alone is done once per wavefront,
// which then walks several tokens: its 64 entries of M stay in registers, and a 64-bit scalar mask
// says in which of the 64 register slots any lane holds a scaled channel at all; the IEEE division
// x / m runs only in those slots (x / 1 = x exactly, so the other lanes of such a slot are not
// touched by it), behind scalar branches.  The next token's loads are issued before the current
// token is reduced.
template <bool BF16>
__device__ __forceinline__ void act_load_token(const char* xrow, int64_t n, int lane, u32x4_t (&raw)[BF16 ? 8 : 16]) {
    constexpr int PER = BF16 ? 2 : 4;                    // 16-byte loads per group of 16 channels
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t c = ((int64_t)u * 64 + lane) * 16;
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            raw[u * PER + q] = u32x4_t{0u, 0u, 0u, 0u};
            if (c < n) raw[u * PER + q] = *(const u32x4_t*)(xrow + c * (BF16 ? 2 : 4) + 16 * q);
        }
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void act_rtn_wave_kernel(const void* __restrict__ X, int64_t rows, int64_t n, int64_t ldx,
                                                           const float* __restrict__ mdiag, float qmax,
                                                           int8_t* __restrict__ codes, float* __restrict__ scales,
                                                           int tokens_per_wave) {
    const int lane = threadIdx.x & 63;
    const int64_t row0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * tokens_per_wave;
    if (row0 >= rows) return;
    const int64_t row1 = (row0 + tokens_per_wave < rows) ? row0 + tokens_per_wave : rows;
    const int64_t row_bytes = ldx * (BF16 ? 2 : 4);

    // The lane's 64 entries of M go to LDS ([slot][lane]; the four wavefronts of a workgroup hold the
    // same channels, so each writes the same values): the division slots read them back, and the
    // registers stay free for a third and fourth wavefront per SIMD.
    __shared__ float m_lds[64 * 64];
    uint64_t slots = 0;                                  // bit 16 u + e: some lane's channel of that slot has m != 1
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t c = ((int64_t)u * 64 + lane) * 16;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float4 m4 = make_float4(1.f, 1.f, 1.f, 1.f);
            if (mdiag && c < n) m4 = *(const float4*)(mdiag + c + 4 * q);
            const float mm[4] = {m4.x, m4.y, m4.z, m4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                m_lds[(16 * u + 4 * q + e) * 64 + lane] = mm[e];
                if (__builtin_amdgcn_ballot_w64(mm[e] != 1.f) != 0) slots |= 1ull << (16 * u + 4 * q + e);
            }
        }
    }
    // no barrier: a wavefront reads only what it wrote itself (the other wavefronts write the same values)

    u32x4_t raw[BF16 ? 8 : 16];
    act_load_token<BF16>((const char*)X + row0 * row_bytes, n, lane, raw);
    for (int64_t row = row0; row < row1; ++row) {
        float v[4][16];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (BF16) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t w = raw[2 * u + (e >> 2)][e & 3];
                    v[u][2 * e] = __uint_as_float(w << 16);
                    v[u][2 * e + 1] = __uint_as_float(w & 0xFFFF0000u);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) v[u][e] = __uint_as_float(raw[4 * u + (e >> 2)][e & 3]);
            }
        }
        if (row + 1 < row1) act_load_token<BF16>((const char*)X + (row + 1) * row_bytes, n, lane, raw);
        float amax = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                if ((slots >> (16 * u + e)) & 1) {
                    v[u][e] = v[u][e] / m_lds[(16 * u + e) * 64 + lane];
                    asm volatile("" : "+v"(v[u][e]));     // keeps the division behind its branch
                }
                amax = fmaxf(amax, fabsf(v[u][e]));
            }
        }
        amax = wave_max(amax);
        const float scale = (amax == 0.f) ? 1.f : amax / qmax;
        // the reciprocal of a denormal scale is not finite: then every quotient is a true division
        const bool plain = __builtin_amdgcn_readfirstlane(scale > 1e-30f ? 1 : 0) != 0;
        const float rscale = plain ? __builtin_amdgcn_rcpf(scale) : 0.f;
        if (lane == 0) scales[row] = scale;
        int8_t* crow = codes + row * n;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t c = ((int64_t)u * 64 + lane) * 16;
            u32x4_t pkv;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                // rint(x / scale) from a reciprocal multiply (error below 4e-5 for |quotient| <= 128); only
                // within 1e-4 of a rounding boundary k + 1/2 does the correctly rounded division decide.
                // One test per four channels: the largest distance to the nearest integer among them.
                float t[4], r[4], dist[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    t[e] = v[u][4 * d + e] * rscale;
                    r[e] = rintf(t[e]);
                    dist[e] = fabsf(t[e] - r[e]);
                }
                const float far = fmaxf(fmaxf(dist[0], dist[1]), fmaxf(dist[2], dist[3]));
                if (!plain || __builtin_amdgcn_ballot_w64(far > 0.4999f) != 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (!plain || dist[e] > 0.4999f) r[e] = rintf(v[u][4 * d + e] / scale);
                        asm volatile("" : "+v"(r[e]));
                    }
                }
                int qi[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) qi[e] = (int)r[e];
                pkv[d] = __builtin_amdgcn_perm((uint32_t)qi[1], (uint32_t)qi[0], 0x0c0c0400u) |
                         __builtin_amdgcn_perm((uint32_t)qi[3], (uint32_t)qi[2], 0x04000c0cu);
            }
            if (c < n) __builtin_nontemporal_store(pkv, (u32x4_t*)(crow + c));
        }
    }
}

}  // namespace

// ---------------------------------------------------------------------------------------- launchers
int aser_fill_f32(aser_ctx* ctx, float* p, int64_t rows, int64_t cols, int64_t ld, float v) {
    if (rows <= 0 || cols <= 0) return ASER_OK;
    const int64_t total = rows * cols;
    const int blocks = (int)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_f32_kernel, dim3(blocks), dim3(256), 0, ctx->stream, p, rows, cols, ld, v);
    return aser_check_launch(ctx, "fill_f32");
}

int aser_set_i32(aser_ctx* ctx, int32_t* p, int32_t v) {
    hipLaunchKernelGGL(set_i32_kernel, dim3(1), dim3(1), 0, ctx->stream, p, v);
    return aser_check_launch(ctx, "set_i32");
}

int aser_fill_bytes(aser_ctx* ctx, void* p, size_t bytes) {
    if (bytes == 0) return ASER_OK;
    if (((uintptr_t)p & 3) || (bytes & 3)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "fill: unaligned");
    if ((((uintptr_t)p | bytes) & 15) == 0 && bytes >= (1u << 16)) {          // large aligned ranges: 16-byte stores
        const int64_t quads = (int64_t)(bytes / 16);
        const int blocks16 = (int)((quads + 255) / 256 < 8192 ? (quads + 255) / 256 : 8192);
        hipLaunchKernelGGL(fill_zero16_kernel, dim3(blocks16), dim3(256), 0, ctx->stream, (uint4*)p, quads);
        return aser_check_launch(ctx, "fill_zero");
    }
    const int64_t words = (int64_t)(bytes / 4);
    const int blocks = (int)((words + 255) / 256 < 4096 ? (words + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, ctx->stream, (uint32_t*)p, words);
    return aser_check_launch(ctx, "fill_zero");
}

// Rows per strip of the column-sum kernels: the largest power of two that still leaves about one
// workgroup per compute unit, between 256 and 8192 (and few enough strips for the grid's y range).
static int64_t strip_rows(int64_t rows, int64_t col_groups) {
    int64_t rpb = 256;
    while (rpb < 8192 && rpb * 2 * 256 <= rows * col_groups) rpb *= 2;
    while (ceil_div64(rows, rpb) > 65535) rpb *= 2;
    return rpb;
}

int aser_col_abs_sum_x(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                       double* abs_sum, int64_t* count) {
    const int vec = (x_dtype == ASER_DTYPE_BF16) ? 8 : 4;
    const int64_t gx = ceil_div64(ceil_div64(n, vec), 64);
    const int64_t rpb = strip_rows(rows, gx);
    const int64_t gy = ceil_div64(rows, rpb);
    dim3 grid((unsigned)gx, (unsigned)gy);
    if (x_dtype == ASER_DTYPE_BF16)
        hipLaunchKernelGGL(col_abs_sum_kernel<true>, grid, dim3(256), 0, ctx->stream, X, rows, n, ldx, rpb, abs_sum, count, rows);
    else
        hipLaunchKernelGGL(col_abs_sum_kernel<false>, grid, dim3(256), 0, ctx->stream, X, rows, n, ldx, rpb, abs_sum, count, rows);
    return aser_check_launch(ctx, "col_abs_sum_x");
}

int aser_col_abs_sum_w(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw, double* wsum) {
    const int64_t gx = ceil_div64(ceil_div64(n, 4), 64);
    const int64_t rpb = strip_rows(m, gx);
    dim3 grid((unsigned)gx, (unsigned)ceil_div64(m, rpb));
    hipLaunchKernelGGL(col_abs_sum_kernel<false>, grid, dim3(256), 0, ctx->stream, (const void*)W, m, n, ldw, rpb, wsum,
                       (int64_t*)nullptr, (int64_t)0);
    return aser_check_launch(ctx, "col_abs_sum_w");
}

int aser_transpose_f32(aser_ctx* ctx, const float* A, int64_t rows, int64_t cols, int64_t lda, float* At, int64_t ldat) {
    dim3 grid((unsigned)ceil_div64(cols, 64), (unsigned)ceil_div64(rows, 64));
    hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, ctx->stream, A, rows, cols, lda, At, ldat);
    return aser_check_launch(ctx, "transpose");
}

// ---------------------------------------------------------------------------------------- ABI: stage 3
extern "C" int aser_quantize_rtn(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                 const int32_t* idx, const float* mdiag, int32_t f, int32_t bits, int32_t layout,
                                 void* codes, float* scales, float* T, int64_t ldt) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!W || !codes || !scales) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: null pointer");
    if (m <= 0 || n <= 0 || ldw < n || (T && ldt < n)) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: bad shape");
    if (f < 0 || f > n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: f out of range");
    if (f > 0 && (!idx || !mdiag)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: idx/mdiag needed when f > 0");
    if (bits != 4 && bits != 8) ASER_FAIL(ctx, ASER_ERR_DTYPE, "quantize_rtn: bits must be 4 or 8");
    if (layout != ASER_CODES_INT8 && layout != ASER_CODES_INT4_PACKED)
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: unknown code layout");
    if (layout == ASER_CODES_INT4_PACKED && (bits != 4 || (n & 1)))
        ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: packed int4 needs bits == 4 and even n");
    if (n > 32768) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_rtn: n > 32768 is not supported");
    if (((uintptr_t)W & 3) || ((uintptr_t)scales & 3) || (T && ((uintptr_t)T & 3)))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_rtn: misaligned pointer");
    ASER_TRY(aser_prepare_device(ctx));
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const int64_t pitch = (layout == ASER_CODES_INT8) ? n : n / 2;
    const size_t lds = (size_t)((n + 31) / 32) * 4 + 64;
    const int64_t groups = ceil_div64(n, 8);
    dim3 grid((unsigned)m);
#define ASER_RTN_LAUNCH(V, NT)                                                                                      \
    hipLaunchKernelGGL((rtn_kernel<V, NT>), grid, dim3(NT), lds, ctx->stream, W, n, ldw, idx, mdiag, (int)f, qmax, \
                       (int)layout, (uint8_t*)codes, pitch, scales, T, ldt)
    if (groups <= 256 * 2) ASER_RTN_LAUNCH(2, 256);
    else if (groups <= 512 * 2) ASER_RTN_LAUNCH(2, 512);
    else if (groups <= 768 * 2) ASER_RTN_LAUNCH(2, 768);       // 11008 columns: 1376 groups on 1536 slots instead of 2048
    else if (groups <= 1024 * 2) ASER_RTN_LAUNCH(2, 1024);
    else if (groups <= 1024 * 3) ASER_RTN_LAUNCH(3, 1024);     // 20480 columns: 2560 groups on 3072 slots instead of 4096
    else ASER_RTN_LAUNCH(4, 1024);
#undef ASER_RTN_LAUNCH
    return aser_check_launch(ctx, "rtn");
}

// ---------------------------------------------------------------------------------------- ABI: stage 3 around another quantizer
namespace {
int base_quantizer_launch(aser_ctx* ctx, bool target, const float* W, int64_t m, int64_t n, int64_t ldw, const int32_t* idx,
                          int32_t f, const float* mdiag, const float* Wq, int64_t ldq, float* out, int64_t ldo) {
    ASER_TRY(aser_prepare_device(ctx));
    const bool vec = (((uintptr_t)W | (uintptr_t)out | (uintptr_t)Wq) & 15) == 0 && ((ldw | ldo | ldq) & 3) == 0;
    for (int64_t r0 = 0; r0 < m; r0 += 8 * 65535) {             // the grid's second dimension holds 65535 row blocks
        const int64_t rows = m - r0 < 8 * 65535 ? m - r0 : 8 * 65535;
        dim3 grid((unsigned)ceil_div64(n, 1024), (unsigned)ceil_div64(rows, 8));
        const float* q = Wq ? Wq + r0 * ldq : nullptr;
        if (target)
            hipLaunchKernelGGL(base_quantizer_kernel<true>, grid, dim3(256), 0, ctx->stream, W + r0 * ldw, rows, n, ldw, idx, (int)f,
                               mdiag, q, ldq, out + r0 * ldo, ldo, vec ? 1 : 0);
        else
            hipLaunchKernelGGL(base_quantizer_kernel<false>, grid, dim3(256), 0, ctx->stream, W + r0 * ldw, rows, n, ldw, idx, (int)f,
                               mdiag, q, ldq, out + r0 * ldo, ldo, vec ? 1 : 0);
    }
    return aser_check_launch(ctx, target ? "quant_target" : "smoothed_weight");
}
}  // namespace

extern "C" int aser_smoothed_weight(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw,
                                    const int32_t* idx, int32_t f, float* Ws, int64_t ldws) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!W || !Ws) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "smoothed_weight: null pointer");
    if (m <= 0 || n <= 0 || ldw < n || ldws < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "smoothed_weight: bad shape");
    if (f < 0 || f > n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "smoothed_weight: f out of range");
    if (f > 0 && !idx) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "smoothed_weight: idx needed when f > 0");
    if (((uintptr_t)W & 3) || ((uintptr_t)Ws & 3)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "smoothed_weight: misaligned pointer");
    return base_quantizer_launch(ctx, false, W, m, n, ldw, idx, f, nullptr, nullptr, 0, Ws, ldws);
}

extern "C" int aser_quant_target(aser_ctx* ctx, const float* W, int64_t m, int64_t n, int64_t ldw, const float* mdiag,
                                 const float* Wq, int64_t ldq, float* T, int64_t ldt) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!W || !Wq || !T) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quant_target: null pointer");
    if (m <= 0 || n <= 0 || ldw < n || ldq < n || ldt < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quant_target: bad shape");
    if (T == Wq && ldt != ldq) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quant_target: in place needs ldt == ldq");
    if (((uintptr_t)W & 3) || ((uintptr_t)Wq & 3) || ((uintptr_t)T & 3) || (mdiag && ((uintptr_t)mdiag & 3)))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quant_target: misaligned pointer");
    return base_quantizer_launch(ctx, true, W, m, n, ldw, nullptr, 0, mdiag, Wq, ldq, T, ldt);
}

// ---------------------------------------------------------------------------------------- ABI: activation RTN
extern "C" int aser_quantize_act_rtn(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                                     const float* mdiag, int32_t bits, int8_t* codes, float* scales) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!X || !codes || !scales) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "quantize_act_rtn: null pointer");
    if (x_dtype != ASER_DTYPE_BF16 && x_dtype != ASER_DTYPE_F32) ASER_FAIL(ctx, ASER_ERR_DTYPE, "quantize_act_rtn: dtype");
    if (rows < 0 || n <= 0 || ldx < n) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_act_rtn: bad shape");
    if (bits < 2 || bits > 8) ASER_FAIL(ctx, ASER_ERR_DTYPE, "quantize_act_rtn: bits must be in [2, 8]");
    if (n > 32768) ASER_FAIL(ctx, ASER_ERR_SHAPE, "quantize_act_rtn: n > 32768 is not supported");
    if (rows == 0) return ASER_OK;
    ASER_TRY(aser_prepare_device(ctx));
    const float qmax = (float)((1 << (bits - 1)) - 1);
    const int64_t groups = ceil_div64(n, 8);
    dim3 grid((unsigned)rows);
#define ASER_ACT_LAUNCH(B, V, NT) \
    hipLaunchKernelGGL((act_rtn_kernel<B, V, NT>), grid, dim3(NT), 0, ctx->stream, X, n, ldx, mdiag, qmax, codes, scales)
    // at most four groups per thread (more cost registers and occupancy), then the fewest threads that cover the token
#define ASER_ACT_PICK(B)                                          \
    do {                                                          \
        if (groups <= 256 * 2) ASER_ACT_LAUNCH(B, 2, 256);        \
        else if (groups <= 256 * 3) ASER_ACT_LAUNCH(B, 3, 256);   \
        else if (groups <= 256 * 4) ASER_ACT_LAUNCH(B, 4, 256);   \
        else if (groups <= 512 * 3) ASER_ACT_LAUNCH(B, 3, 512);   \
        else if (groups <= 512 * 4) ASER_ACT_LAUNCH(B, 4, 512);   \
        else if (groups <= 1024 * 3) ASER_ACT_LAUNCH(B, 3, 1024); \
        else ASER_ACT_LAUNCH(B, 4, 1024);                         \
    } while (0)
    const int esz = (x_dtype == ASER_DTYPE_BF16) ? 2 : 4;
    const bool wave_ok = n <= 4096 && (n & 15) == 0 && ((uintptr_t)X & 15) == 0 && ((ldx * esz) & 15) == 0 &&
                         ((uintptr_t)codes & 15) == 0 && (!mdiag || ((uintptr_t)mdiag & 15) == 0);
    if (wave_ok) {
        // several tokens per wavefront once there are enough tokens for four workgroups per compute unit
        int tpw = (int)(rows / 4096);
        tpw = tpw < 1 ? 1 : (tpw > 4 ? 4 : tpw);                 // 2 to 8 measure alike, 16 is slower
        dim3 wgrid((unsigned)ceil_div64(rows, 4 * (int64_t)tpw));
        if (x_dtype == ASER_DTYPE_BF16)
            hipLaunchKernelGGL(act_rtn_wave_kernel<true>, wgrid, dim3(256), 0, ctx->stream, X, rows, n, ldx, mdiag, qmax, codes, scales, tpw);
        else
            hipLaunchKernelGGL(act_rtn_wave_kernel<false>, wgrid, dim3(256), 0, ctx->stream, X, rows, n, ldx, mdiag, qmax, codes, scales, tpw);
        return aser_check_launch(ctx, "act_rtn");
    }
    if (x_dtype == ASER_DTYPE_BF16) ASER_ACT_PICK(true);
    else ASER_ACT_PICK(false);
#undef ASER_ACT_PICK
#undef ASER_ACT_LAUNCH
    return aser_check_launch(ctx, "act_rtn");
}
