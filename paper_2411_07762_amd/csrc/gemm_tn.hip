// MFMA contraction kernel of the ASER calibration path for gfx950 (CDNA4).
//
// One kernel form serves every dense contraction of the path:  C (op)= alpha * A^T B  with
// both operands stored K-major (A: K x M, B: K x N, row-major).  The Gram matrix of Eq. 5
// (G = X^T X with X tokens x channels) has exactly this form, and the Cholesky panels and
// trailing updates, the whitened error T S, the subspace-iteration products and the small
// Gram matrices of the orthogonalisation are arranged by their callers to have it too.
//
// Data path.  Each workgroup (256 threads = 4 waves in a 2 x 2 grid) owns a BM x BN tile of C.
// Per K step a thread fetches an 8(k) x 8(bf16) or 8(k) x 4(fp32) block of each operand with
// 16-byte loads that are contiguous along the channel dimension, turns it in registers into
// k-contiguous 8 x bf16 chunks (a byte-permute transpose for bf16; for fp32 the hi/lo split
// packs pairs along k directly), and stores the chunks to LDS in the order the MFMA operands
// are read: chunk (k-block, row) at [kb][swizzle(row)].  v_mfma_f32_32x32x16_bf16 reads one
// chunk per lane (row = lane % 32, k-block = lane / 32).  Global loads for step s+1 are issued
// before the MFMAs of step s and written to the other LDS buffer after them: one barrier per
// step.  fp32 operands are split as x = hi + lo (bf16 each) and contribute hi*hi + hi*lo +
// lo*hi, accumulated in fp32.
#include "aser_internal.h"

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

namespace {

constexpr int kThreads = 256;

template <int IN> struct InTraits;
template <> struct InTraits<GEMM_IN_BF16> { static constexpr int BK = 64, NP = 1, VEC = 8; };
template <> struct InTraits<GEMM_IN_F32X3> { static constexpr int BK = 32, NP = 2, VEC = 4; };

// LDS position (in 16-byte chunks) of row `mn` inside one k-block.  The XOR pattern makes both
// the transposing stores (8 consecutive rows per lane) and the MFMA operand reads (32
// consecutive rows per half wave) hit distinct bank groups.
__device__ __forceinline__ int swz(int mn) { return (mn ^ ((mn >> 3) & 7)) ^ (((mn >> 6) & 1) << 3); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2_t v = {a, b};
    bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

// Per-thread fetch state of one operand tile (BMN rows of the tile, BK k-values per step).
template <int IN, int BMN>
struct Fetch {
    static constexpr int BK = InTraits<IN>::BK;
    static constexpr int VEC = InTraits<IN>::VEC;       // elements per 16-byte load
    static constexpr int GROUPS = BMN / VEC;            // 16-byte column groups across the tile
    static constexpr int ESZ = (IN == GEMM_IN_BF16) ? 2 : 4;

    const char* p;      // address of (k row of this thread's first load, first column)
    int64_t ld_bytes;
    int64_t k;          // k index of this thread's first row in the current step
    int cg, kb;         // column group and k-block handled by this thread
    int ncols;          // valid columns at this thread's group (0..VEC)
    bool active, vec_ok;
    uint4 r[8];

    __device__ __forceinline__ void init(const void* base, int64_t ld, int64_t mn0, int64_t MN, int64_t k0, int tid) {
        active = tid < GROUPS * (BK / 8);
        cg = tid % GROUPS;
        kb = tid / GROUPS;
        int64_t col = mn0 + (int64_t)cg * VEC;
        int64_t rem = MN - col;
        ncols = rem >= VEC ? VEC : (rem > 0 ? (int)rem : 0);
        k = k0 + kb * 8;
        ld_bytes = ld * ESZ;
        p = (const char*)base + k * ld_bytes + col * ESZ;
        vec_ok = (((uintptr_t)p & 15) == 0) && ((ld_bytes & 15) == 0) && ncols == VEC;
        if (ncols == 0) active = false;
    }

    __device__ __forceinline__ void load(int64_t kEnd) {
#pragma unroll
        for (int j = 0; j < 8; ++j) r[j] = make_uint4(0u, 0u, 0u, 0u);
        if (!active) return;
        if (vec_ok) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (k + j < kEnd) r[j] = *(const uint4*)(p + j * ld_bytes);
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (k + j < kEnd) {
                    const char* q = p + j * ld_bytes;
                    if (IN == GEMM_IN_BF16) {
                        uint32_t w[4] = {0u, 0u, 0u, 0u};
                        for (int e = 0; e < ncols; ++e)
                            w[e >> 1] |= (uint32_t)(*(const uint16_t*)(q + 2 * e)) << (16 * (e & 1));
                        r[j] = make_uint4(w[0], w[1], w[2], w[3]);
                    } else {
                        uint32_t w[4] = {0u, 0u, 0u, 0u};
                        for (int e = 0; e < ncols; ++e) w[e] = *(const uint32_t*)(q + 4 * e);
                        r[j] = make_uint4(w[0], w[1], w[2], w[3]);
                    }
                }
            }
        }
    }

    __device__ __forceinline__ void advance() {
        p += (int64_t)BK * ld_bytes;
        k += BK;
    }

    // Writes this thread's block as k-contiguous chunks into the operand's LDS area.
    __device__ __forceinline__ void store(uint4* lds) const {
        if (!active) return;
        constexpr int KB = BK / 8;
        if (IN == GEMM_IN_BF16) {
            const uint32_t* w = (const uint32_t*)r;       // w[4*j + d]: row j, channel pair d
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int d = c >> 1;
                const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
                uint4 o;
                o.x = __builtin_amdgcn_perm(w[4 * 1 + d], w[4 * 0 + d], sel);
                o.y = __builtin_amdgcn_perm(w[4 * 3 + d], w[4 * 2 + d], sel);
                o.z = __builtin_amdgcn_perm(w[4 * 5 + d], w[4 * 4 + d], sel);
                o.w = __builtin_amdgcn_perm(w[4 * 7 + d], w[4 * 6 + d], sel);
                lds[kb * BMN + swz(cg * 8 + c)] = o;
            }
        } else {
            const float* x = (const float*)r;             // x[4*j + c]: row j, column c
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint32_t hi[4], lo[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float a = x[4 * (2 * q) + c], b = x[4 * (2 * q + 1) + c];
                    const uint32_t h = pack_bf16x2(a, b);
                    const float ah = __uint_as_float(h << 16), bh = __uint_as_float(h & 0xFFFF0000u);
                    hi[q] = h;
                    lo[q] = pack_bf16x2(a - ah, b - bh);
                }
                const int pos = kb * BMN + swz(cg * 4 + c);
                lds[pos] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                lds[KB * BMN + pos] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
            }
        }
    }
};

template <int IN, int BM, int BN>
struct TileCfg {
    static constexpr int BK = InTraits<IN>::BK;
    static constexpr int NP = InTraits<IN>::NP;
    static constexpr int KB = BK / 8;
    static constexpr int A_CHUNKS = NP * KB * BM;
    static constexpr int B_CHUNKS = NP * KB * BN;
    static constexpr int STAGE_CHUNKS = A_CHUNKS + B_CHUNKS;
    static constexpr size_t LDS_BYTES = (size_t)2 * STAGE_CHUNKS * 16;
    static constexpr int TM = BM / 64, TN = BN / 64;     // 32 x 32 MFMA blocks per wave
};

// One tile of C over the K range [kBeg, kEnd).
template <int IN, int BM, int BN>
__device__ __forceinline__ void tile_body(const GemmArgs& g, int64_t I0, int64_t J0, int64_t kBeg, int64_t kEnd,
                                          uint4* smem) {
    using Cfg = TileCfg<IN, BM, BN>;
    constexpr int BK = Cfg::BK, NP = Cfg::NP, KB = Cfg::KB, TM = Cfg::TM, TN = Cfg::TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

    Fetch<IN, BM> fa;
    Fetch<IN, BN> fb;
    fa.init(g.A, g.lda, I0, g.M, kBeg, tid);
    fb.init(g.B, g.ldb, J0, g.N, kBeg, tid);

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int64_t steps = (kEnd - kBeg + BK - 1) / BK;
    if (steps > 0) {
        fa.load(kEnd);
        fb.load(kEnd);
        fa.store(smem);
        fb.store(smem + Cfg::A_CHUNKS);
        fa.advance();
        fb.advance();
    }
    __syncthreads();
    for (int64_t s = 0; s < steps; ++s) {
        const uint4* sa = smem + (s & 1) * Cfg::STAGE_CHUNKS;
        const uint4* sb = sa + Cfg::A_CHUNKS;
        const bool more = s + 1 < steps;
        if (more) {
            fa.load(kEnd);
            fb.load(kEnd);
        }
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int kb = 2 * kk + (lane >> 5);
            bf16x8_t a[NP][TM], b[NP][TN];
#pragma unroll
            for (int p = 0; p < NP; ++p) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[p][i] = __builtin_bit_cast(bf16x8_t, sa[(p * KB + kb) * BM + swz(wm0 + 32 * i + (lane & 31))]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[p][j] = __builtin_bit_cast(bf16x8_t, sb[(p * KB + kb) * BN + swz(wn0 + 32 * j + (lane & 31))]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if (NP == 2) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[1][i], b[0][j], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[1][j], acc[i][j], 0, 0, 0);
                    }
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[0][i], b[0][j], acc[i][j], 0, 0, 0);
                }
        }
        if (more) {
            uint4* da = smem + ((s + 1) & 1) * Cfg::STAGE_CHUNKS;
            fa.store(da);
            fb.store(da + Cfg::A_CHUNKS);
            fa.advance();
            fb.advance();
        }
        __syncthreads();
    }

    // Epilogue.  acc[i][j][e] is C(row, col) with row = 32 i + 8 (e / 4) + 4 (lane / 32) + e % 4,
    // col = 32 j + lane % 32 inside the wave's sub-tile.  The read-modify-write form loads a whole
    // 32 x 32 block before it stores, so that the loads overlap instead of forming a chain.
    const float alpha = g.alpha;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = J0 + wn0 + 32 * j + (lane & 31);
            const int64_t rbase = I0 + wm0 + 32 * i + 4 * (lane >> 5);
            if (col >= g.N) continue;
            float* cbase = g.C + rbase * g.ldc + col;
            if (g.epi == GEMM_EPI_RMW) {
                float old[16];
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    old[e] = (rbase + dr < g.M) ? cbase[(int64_t)dr * g.ldc] : 0.f;
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    if (rbase + dr < g.M) cbase[(int64_t)dr * g.ldc] = old[e] + alpha * acc[i][j][e];
                }
            } else if (g.epi == GEMM_EPI_ATOMIC) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    if (rbase + dr < g.M) unsafeAtomicAdd(cbase + (int64_t)dr * g.ldc, alpha * acc[i][j][e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    if (rbase + dr < g.M) cbase[(int64_t)dr * g.ldc] = alpha * acc[i][j][e];
                }
                if (g.Ct) {
                    // transposed copy: the 4 consecutive rows of one accumulator group are contiguous in Ct
                    float* tbase = g.Ct + col * g.ldct + rbase;
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int dr = 8 * q;
                        if (rbase + dr + 3 < g.M && ((((uintptr_t)(tbase + dr)) & 15) == 0)) {
                            *(float4*)(tbase + dr) = make_float4(alpha * acc[i][j][4 * q], alpha * acc[i][j][4 * q + 1],
                                                                 alpha * acc[i][j][4 * q + 2], alpha * acc[i][j][4 * q + 3]);
                        } else {
#pragma unroll
                            for (int u = 0; u < 4; ++u)
                                if (rbase + dr + u < g.M) tbase[dr + u] = alpha * acc[i][j][4 * q + u];
                        }
                    }
                }
            }
        }
}

// Tile and K-part of a workgroup for the plain schedules.
template <int IN, int BM, int BN>
__global__ __launch_bounds__(kThreads) void gemm_tn_kernel(GemmArgs g) {
    extern __shared__ uint4 smem[];
    constexpr int BK = InTraits<IN>::BK;
    const int64_t tm = (g.M + BM - 1) / BM, tn = (g.N + BN - 1) / BN;
    int64_t ti, tj;
    const int64_t t = blockIdx.x;
    if (g.tiles == GEMM_TILES_ALL) {
        ti = t / tn;
        tj = t % tn;
    } else {
        // t enumerates pairs (p, q) with p >= q: p (p + 1) / 2 + q
        int64_t p = (int64_t)((sqrt(8.0 * (double)t + 1.0) - 1.0) * 0.5);
        while (p * (p + 1) / 2 > t) --p;
        while ((p + 1) * (p + 2) / 2 <= t) ++p;
        const int64_t q = t - p * (p + 1) / 2;
        if (g.tiles == GEMM_TILES_LOWER) { ti = p; tj = q; } else { ti = q; tj = p; }
    }
    (void)tm;
    const int64_t I0 = ti * BM, J0 = tj * BN;
    int64_t k0 = 0;
    if (g.krange == GEMM_K_GE_COL) k0 = (J0 / BK) * BK;
    const int64_t ksteps = (g.K - k0 + BK - 1) / BK;
    const int64_t per = (ksteps + g.k_parts - 1) / g.k_parts;
    const int64_t kBeg = k0 + (int64_t)blockIdx.y * per * BK;
    int64_t kEnd = kBeg + per * BK;
    if (kEnd > g.K) kEnd = g.K;
    if (kBeg >= kEnd && g.epi != GEMM_EPI_STORE) return;
    tile_body<IN, BM, BN>(g, I0, J0, kBeg, kEnd, smem);
}

template <int IN, int BM, int BN>
int launch_plain(aser_ctx* ctx, const GemmArgs& g) {
    using Cfg = TileCfg<IN, BM, BN>;
    static bool attr_set[16] = {false};
    auto kern = gemm_tn_kernel<IN, BM, BN>;
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::LDS_BYTES));
        attr_set[ctx->device] = true;
    }
    const int64_t tm = ceil_div64(g.M, BM), tn = ceil_div64(g.N, BN);
    int64_t tiles = (g.tiles == GEMM_TILES_ALL) ? tm * tn : tm * (tm + 1) / 2;
    dim3 grid((unsigned)tiles, (unsigned)g.k_parts, 1);
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), Cfg::LDS_BYTES, ctx->stream, g);
    return aser_check_launch(ctx, "gemm_tn");
}

template <int IN>
int dispatch_tile(aser_ctx* ctx, const GemmArgs& g) {
    if (g.bm == 256 && g.bn == 256) return launch_plain<IN, 256, 256>(ctx, g);
    if (g.bm == 128 && g.bn == 256) return launch_plain<IN, 128, 256>(ctx, g);
    if (g.bm == 256 && g.bn == 128) return launch_plain<IN, 256, 128>(ctx, g);
    if (g.bm == 128 && g.bn == 128) return launch_plain<IN, 128, 128>(ctx, g);
    ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: unsupported tile %dx%d", g.bm, g.bn);
}

}  // namespace

int aser_gemm_tn(aser_ctx* ctx, const GemmArgs& g) {
    if (g.M <= 0 || g.N <= 0 || g.K < 0) ASER_FAIL(ctx, ASER_ERR_SHAPE, "gemm_tn: bad sizes");
    if (g.k_parts < 1 || (g.k_parts > 1 && g.epi != GEMM_EPI_ATOMIC))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: split K needs the atomic epilogue");
    if (g.tiles != GEMM_TILES_ALL && (g.M != g.N || g.bm != g.bn))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: triangular tiling needs a square problem and tile");
    if (g.Ct && g.epi != GEMM_EPI_STORE) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: Ct needs the store epilogue");
    if (g.in_type == GEMM_IN_BF16) return dispatch_tile<GEMM_IN_BF16>(ctx, g);
    if (g.in_type == GEMM_IN_F32X3) return dispatch_tile<GEMM_IN_F32X3>(ctx, g);
    ASER_FAIL(ctx, ASER_ERR_DTYPE, "gemm_tn: unknown input type");
}

// Gram update: lower-triangle tiles of G += X^T X.  K (= tokens) is split so that the grid
// fills the 256 compute units a few times over; partial tiles are added with fp32 atomics.
int aser_syrk_gram(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                   float* G, int64_t ldg) {
    GemmArgs g{};
    g.A = X; g.lda = ldx; g.B = X; g.ldb = ldx;
    g.C = G; g.ldc = ldg; g.Ct = nullptr; g.ldct = 0;
    g.M = n; g.N = n; g.K = rows; g.alpha = 1.f;
    g.in_type = (x_dtype == ASER_DTYPE_BF16) ? GEMM_IN_BF16 : GEMM_IN_F32X3;
    g.epi = GEMM_EPI_ATOMIC; g.tiles = GEMM_TILES_LOWER; g.krange = GEMM_K_FULL;
    g.bm = g.bn = (n <= 1024) ? 128 : 256;
    const int64_t t = ceil_div64(n, g.bm), tiles = t * (t + 1) / 2;
    const int bk = (g.in_type == GEMM_IN_BF16) ? 64 : 32;
    const int64_t ksteps = ceil_div64(rows, bk);
    int64_t parts = ceil_div64(1024, tiles);              // aim at >= 4 workgroups per CU
    const int64_t max_parts = ksteps / 16 > 0 ? ksteps / 16 : 1;   // keep >= 16 steps per part
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    g.k_parts = (int)parts;
    return aser_gemm_tn(ctx, g);
}
