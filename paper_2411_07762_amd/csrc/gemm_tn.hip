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
// chunk per lane (row = lane % 32, k-block = lane / 32).  Global loads run one step (256 x 256
// tile) or two steps (smaller tiles, two register sets) ahead of the MFMAs; LDS is double
// buffered with one barrier per step.  fp32 operands are split as x = hi + lo (bf16 each) and
// contribute hi*hi + hi*lo + lo*hi, accumulated in fp32.
#include <type_traits>

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
template <> struct InTraits<GEMM_IN_F32X6> { static constexpr int BK = 32, NP = 3, VEC = 4; };

// LDS position (in 16-byte chunks) of row `mn` inside one k-block.  The XOR pattern makes both
// the transposing stores (8 consecutive rows per lane) and the MFMA operand reads (32
// consecutive rows per half wave) hit distinct bank groups.
__device__ __forceinline__ int swz(int mn) { return (mn ^ ((mn >> 3) & 7)) ^ (((mn >> 6) & 1) << 3); }

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2_t v = {a, b};
    bf16x2_t h = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

// Eight 16-byte rows of one operand block in flight between global memory and LDS.
struct Staged {
    uint4 r[8];
};

// Per-thread fetch state of one operand tile (BMN rows of the tile, BK k-values per step).
// FAST: the operand is 16-byte aligned with leading dimension and extent multiples of the vector
// width, so every column group is whole; loads are branch-free (rows past the K range are read
// from the last valid row and zeroed, column groups past the extent are read from group 0 and
// simply never stored to C).  Otherwise a guarded element-wise path is used.
template <int IN, int BMN, bool FAST>
struct Fetch {
    static constexpr int BK = InTraits<IN>::BK;
    static constexpr int VEC = InTraits<IN>::VEC;       // elements per 16-byte load
    static constexpr int GROUPS = BMN / VEC;            // 16-byte column groups across the tile
    static constexpr int ESZ = (IN == GEMM_IN_BF16) ? 2 : 4;

    const char* p;      // address of (k row of this thread's first load in the next step, first column)
    const char* plast;  // same column group in the last valid k row (FAST)
    int64_t ld_bytes;
    int64_t k;          // k index of this thread's first row in the next step to be loaded
    int cg, kb;         // column group and k-block handled by this thread
    int ncols;          // valid columns at this thread's group (0..VEC)
    bool active, vec_ok;

    __device__ __forceinline__ void init(const void* base, int64_t ld, int64_t mn0, int64_t MN, int64_t k0,
                                         int64_t kEnd, int tid) {
        active = tid < GROUPS * (BK / 8);
        cg = tid % GROUPS;
        kb = tid / GROUPS;
        int64_t col = mn0 + (int64_t)cg * VEC;
        int64_t rem = MN - col;
        ncols = rem >= VEC ? VEC : (rem > 0 ? (int)rem : 0);
        k = k0 + kb * 8;
        ld_bytes = ld * ESZ;
        if (FAST) {
            if (ncols != VEC) col = 0;
            p = (const char*)base + k * ld_bytes + col * ESZ;
            plast = (const char*)base + (kEnd - 1) * ld_bytes + col * ESZ;
            vec_ok = true;
            return;
        }
        p = (const char*)base + k * ld_bytes + col * ESZ;
        plast = p;
        vec_ok = (((uintptr_t)p & 15) == 0) && ((ld_bytes & 15) == 0) && ncols == VEC;
        if (ncols == 0) active = false;
    }

    // Issues the loads of the next step into `st` and moves on by one step.
    __device__ __forceinline__ void load(Staged& st, int64_t kEnd) {
        load_rows(st, kEnd);
        p += (int64_t)BK * ld_bytes;
        k += BK;
    }

    __device__ __forceinline__ void load_rows(Staged& st, int64_t kEnd) {
        uint4* r = st.r;
        if (FAST) {
            if (!active) return;
            if (k + 8 <= kEnd) {
#pragma unroll
                for (int j = 0; j < 8; ++j) r[j] = *(const uint4*)(p + j * ld_bytes);
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const bool ok = k + j < kEnd;
                    const uint4 v = *(const uint4*)(ok ? p + j * ld_bytes : plast);
                    r[j] = ok ? v : make_uint4(0u, 0u, 0u, 0u);
                }
            }
            return;
        }
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

    // Writes a staged block as k-contiguous chunks into the operand's LDS area.
    __device__ __forceinline__ void store(const Staged& st, uint4* lds) const {
        if (!active) return;
        constexpr int KB = BK / 8;
        if (IN == GEMM_IN_BF16) {
            const uint32_t* w = (const uint32_t*)st.r;    // w[4*j + d]: row j, channel pair d
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
            const float* x = (const float*)st.r;          // x[4*j + c]: row j, column c
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint32_t hi[4], lo[4], lo2[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float a = x[4 * (2 * q) + c], b = x[4 * (2 * q + 1) + c];
                    const uint32_t h = pack_bf16x2(a, b);
                    const float ah = __uint_as_float(h << 16), bh = __uint_as_float(h & 0xFFFF0000u);
                    hi[q] = h;
                    const float ar = a - ah, br = b - bh;           // exact: the remainder has at most 16 significant bits
                    lo[q] = pack_bf16x2(ar, br);
                    if (IN == GEMM_IN_F32X6) {
                        const float am = __uint_as_float(lo[q] << 16), bm = __uint_as_float(lo[q] & 0xFFFF0000u);
                        lo2[q] = pack_bf16x2(ar - am, br - bm);     // third term: x = hi + mid + lo to 24 bits
                    }
                }
                const int pos = kb * BMN + swz(cg * 4 + c);
                lds[pos] = make_uint4(hi[0], hi[1], hi[2], hi[3]);
                lds[KB * BMN + pos] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                if (IN == GEMM_IN_F32X6) lds[2 * KB * BMN + pos] = make_uint4(lo2[0], lo2[1], lo2[2], lo2[3]);
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

// Scheduling hint: R groups of (one LDS read, then a share of MF MFMAs).
template <int R, int MF, int T>
struct SchedPattern {
    static __device__ __forceinline__ void emit() {
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, (MF * (T + 1)) / R - (MF * T) / R, 0);
        SchedPattern<R, MF, T + 1>::emit();
    }
};
template <int R, int MF>
struct SchedPattern<R, MF, R> {
    static __device__ __forceinline__ void emit() {}
};

// All MFMAs of one K step from LDS stage (sa, sb).  Operand fragments are double buffered: the
// LDS reads of k-slice kk + 1 are in flight while the MFMAs of slice kk execute (one wave per
// SIMD: nothing else hides the LDS latency), and the scheduling hints spread them evenly.
template <int IN, int BM, int BN>
__device__ __forceinline__ void mfma_step(f32x16_t (&acc)[BM / 64][BN / 64], const uint4* sa, const uint4* sb,
                                          const int (&offa)[BM / 64], const int (&offb)[BN / 64]) {
    using Cfg = TileCfg<IN, BM, BN>;
    constexpr int NP = Cfg::NP, KB = Cfg::KB, TM = Cfg::TM, TN = Cfg::TN, KK = Cfg::BK / 16;
    constexpr int R = NP * (TM + TN);                   // LDS reads per k-slice
    constexpr int MF = TM * TN * (NP == 3 ? 6 : (NP == 2 ? 3 : 1));     // MFMAs per k-slice
    bf16x8_t a[2][NP][TM], b[2][NP][TN];
#pragma unroll
    for (int p = 0; p < NP; ++p) {
#pragma unroll
        for (int i = 0; i < TM; ++i) a[0][p][i] = __builtin_bit_cast(bf16x8_t, sa[(p * KB) * BM + offa[i]]);
#pragma unroll
        for (int j = 0; j < TN; ++j) b[0][p][j] = __builtin_bit_cast(bf16x8_t, sb[(p * KB) * BN + offb[j]]);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, R, 0);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int cur = kk & 1, nxt = cur ^ 1;
        if (kk + 1 < KK) {
#pragma unroll
            for (int p = 0; p < NP; ++p) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
                    a[nxt][p][i] = __builtin_bit_cast(bf16x8_t, sa[(p * KB + 2 * (kk + 1)) * BM + offa[i]]);
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    b[nxt][p][j] = __builtin_bit_cast(bf16x8_t, sb[(p * KB + 2 * (kk + 1)) * BN + offb[j]]);
            }
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                if (NP == 3) {
                    // x = hi + mid + lo: all products down to 2^-24 of hi * hi, smallest first
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][NP - 1][i], b[cur][0][j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][0][i], b[cur][NP - 1][j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][1][i], b[cur][1][j], acc[i][j], 0, 0, 0);
                }
                if (NP >= 2) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][1][i], b[cur][0][j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][0][i], b[cur][1][j], acc[i][j], 0, 0, 0);
                }
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][0][i], b[cur][0][j], acc[i][j], 0, 0, 0);
            }
        if (kk + 1 < KK) SchedPattern<R, MF, 0>::emit();
        else __builtin_amdgcn_sched_group_barrier(0x008, MF, 0);
    }
}

// One tile of C over the K range [kBeg, kEnd).
//
// Pipeline: while step s is multiplied out of LDS stage s % 2, the operand blocks of step s + 1
// (loaded two steps earlier) are transposed/split into stage (s + 1) % 2 and the global loads of
// step s + 3 are issued into the register set that just became free.  Two register sets per
// operand keep two steps of global loads in flight, which covers an HBM round trip.
template <int IN, int BM, int BN, bool FAST>
__device__ __forceinline__ void tile_body(const GemmArgs& g, int64_t I0, int64_t J0, int64_t kBeg, int64_t kEnd,
                                          uint4* smem) {
    using Cfg = TileCfg<IN, BM, BN>;
    constexpr int BK = Cfg::BK, TM = Cfg::TM, TN = Cfg::TN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave >> 1) * (BM / 2), wn0 = (wave & 1) * (BN / 2);

    Fetch<IN, BM, FAST> fa;
    Fetch<IN, BN, FAST> fb;
    fa.init(g.A, g.lda, I0, g.M, kBeg, kEnd, tid);
    fb.init(g.B, g.ldb, J0, g.N, kBeg, kEnd, tid);

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // LDS chunk offsets of this lane's MFMA operands inside one k-block pair
    int offa[TM], offb[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) offa[i] = (lane >> 5) * BM + swz(wm0 + 32 * i + (lane & 31));
#pragma unroll
    for (int j = 0; j < TN; ++j) offb[j] = (lane >> 5) * BN + swz(wn0 + 32 * j + (lane & 31));

    const int64_t steps = (kEnd - kBeg + BK - 1) / BK;
    // Register sets for global loads in flight: the 256 x 256 tile has room for one step only, the
    // smaller tiles keep two steps in flight (four were measured and change nothing: their calls are
    // bound by the operand stream, 6 TB/s summed over the workgroups, not by its latency).
    constexpr int NSETS = (BM == 256 && BN == 256) ? 1 : 2;
    constexpr bool TWO_SETS = NSETS > 1;
    if (TWO_SETS) {
        Staged ra[NSETS], rb[NSETS];                    // set u holds steps u + 1, u + 1 + NSETS, ...
        if (steps > 0) {
            fa.load(ra[0], kEnd);
            fb.load(rb[0], kEnd);
            fa.store(ra[0], smem);
            fb.store(rb[0], smem + Cfg::A_CHUNKS);
#pragma unroll
            for (int u = 0; u < NSETS; ++u)
                if (steps > u + 1) { fa.load(ra[u], kEnd); fb.load(rb[u], kEnd); }
        }
        __syncthreads();
        for (int64_t s0 = 0; s0 < steps; s0 += NSETS) {
#pragma unroll
            for (int u = 0; u < NSETS; ++u) {
                const int64_t s = s0 + u;
                if (s < steps) {
                    // NSETS is even, so the LDS stage of step s is u & 1
                    const uint4* sa = smem + (u & 1) * Cfg::STAGE_CHUNKS;
                    uint4* da = smem + ((u + 1) & 1) * Cfg::STAGE_CHUNKS;
                    mfma_step<IN, BM, BN>(acc, sa, sa + Cfg::A_CHUNKS, offa, offb);
                    if (s + 1 < steps) {
                        fa.store(ra[u], da);
                        fb.store(rb[u], da + Cfg::A_CHUNKS);
                        if (s + 1 + NSETS < steps) { fa.load(ra[u], kEnd); fb.load(rb[u], kEnd); }
                    }
                    __syncthreads();
                }
            }
        }
    } else {
        Staged a0, b0;
        if (steps > 0) {
            fa.load(a0, kEnd);
            fb.load(b0, kEnd);
            fa.store(a0, smem);
            fb.store(b0, smem + Cfg::A_CHUNKS);
            if (steps > 1) { fa.load(a0, kEnd); fb.load(b0, kEnd); }
        }
        __syncthreads();
        for (int64_t s = 0; s < steps; ++s) {
            const uint4* sa = smem + (s & 1) * Cfg::STAGE_CHUNKS;
            uint4* da = smem + ((s + 1) & 1) * Cfg::STAGE_CHUNKS;
            mfma_step<IN, BM, BN>(acc, sa, sa + Cfg::A_CHUNKS, offa, offb);
            if (s + 1 < steps) {
                fa.store(a0, da);
                fb.store(b0, da + Cfg::A_CHUNKS);
                if (s + 2 < steps) { fa.load(a0, kEnd); fb.load(b0, kEnd); }
            }
            __syncthreads();
        }
    }

    // Epilogue.  acc[i][j][e] is C(row, col) with row = 32 i + 8 (e / 4) + 4 (lane / 32) + e % 4,
    // col = 32 j + lane % 32 inside the wave's sub-tile.
    const float alpha = g.alpha;
    if (BM == 128 && BN == 128 && g.epi == GEMM_EPI_RESID) {   // (the large tiles have no registers to spare for it)
        // squared Frobenius norm of C + alpha acc, nothing stored: the loads of one row of 32 x 32
        // blocks are in flight together, squares are summed in fp64, one atomic per wavefront
        double sum = 0.0;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t rbase = I0 + wm0 + 32 * i + 4 * (lane >> 5);
            float old[TN][16];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = J0 + wn0 + 32 * j + (lane & 31);
                const float* cbase = g.C + rbase * g.ldc + col;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    const bool in = col < g.N && rbase + dr < g.M;
                    old[j][e] = in ? cbase[(int64_t)dr * g.ldc] : 0.f;
                    if (!in) acc[i][j][e] = 0.f;
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                float part = 0.f;                          // 16 squares of comparable size in fp32, then fp64
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float d = old[j][e] + alpha * acc[i][j][e];
                    part = fmaf(d, d, part);
                }
                sum += (double)part;
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        if (lane == 0) atomicAdd(g.sumsq, sum);
        return;
    }
    if (g.epi == GEMM_EPI_RMW) {
        // read-modify-write: one row of 32 x 32 blocks (up to 64 values per lane) is loaded before
        // anything is stored, so that the loads overlap instead of forming a chain
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t rbase = I0 + wm0 + 32 * i + 4 * (lane >> 5);
            float old[TN][16];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = J0 + wn0 + 32 * j + (lane & 31);
                const float* cbase = g.C + rbase * g.ldc + col;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    old[j][e] = (col < g.N && rbase + dr < g.M) ? cbase[(int64_t)dr * g.ldc] : 0.f;
                }
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t col = J0 + wn0 + 32 * j + (lane & 31);
                float* cbase = g.C + rbase * g.ldc + col;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    if (col < g.N && rbase + dr < g.M) cbase[(int64_t)dr * g.ldc] = old[j][e] + alpha * acc[i][j][e];
                }
            }
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t col = J0 + wn0 + 32 * j + (lane & 31);
            const int64_t rbase = I0 + wm0 + 32 * i + 4 * (lane >> 5);
            if (col >= g.N) continue;
            float* cbase = g.C + rbase * g.ldc + col;
            if (g.epi == GEMM_EPI_ATOMIC) {
                // upper_only: entries left of the diagonal are never read by the caller; leaving them
                // out halves the atomic traffic of the small symmetric products
                const int64_t rmax = g.upper_only ? (col + 1 < g.M ? col + 1 : g.M) : g.M;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    if (rbase + dr < rmax) unsafeAtomicAdd(cbase + (int64_t)dr * g.ldc, alpha * acc[i][j][e]);
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
template <int IN, int BM, int BN, bool FAST>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_tn_kernel(GemmArgs g) {
    extern __shared__ uint4 smem[];
    constexpr int BK = InTraits<IN>::BK;
    if (g.gate && *g.gate == 0) return;
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
    tile_body<IN, BM, BN, FAST>(g, I0, J0, kBeg, kEnd, smem);
}

// 256 x 128 tiles, tile columns j and tn - 1 - j of one tile row per workgroup, one after the other:
// equal work per workgroup when the K range shrinks linearly with the column (B lower triangular).
template <int IN, bool FAST>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_tn_pair_kernel(GemmArgs g) {
    extern __shared__ uint4 smem[];
    constexpr int BK = InTraits<IN>::BK, BM = 256, BN = 128;
    const int64_t tn = (g.N + BN - 1) / BN, half = (tn + 1) / 2;
    const int64_t ti = blockIdx.x / half, j0 = blockIdx.x % half;
#pragma nounroll
    for (int rep = 0; rep < 2; ++rep) {
        const int64_t tj = rep ? tn - 1 - j0 : j0;
        if (rep && tj == j0) break;
        const int64_t J0 = tj * BN;
        const int64_t k0 = (g.krange == GEMM_K_GE_COL) ? (J0 / BK) * BK : 0;
        if (rep) __syncthreads();                        // the first tile's readers are done with the LDS stages
        tile_body<IN, BM, BN, FAST>(g, ti * BM, J0, k0, g.K, smem);
    }
}

// True when both operands allow the branch-free 16-byte fetch path.
template <int IN>
bool operands_fast(const GemmArgs& g) {
    constexpr int VEC = InTraits<IN>::VEC;
    return (((uintptr_t)g.A & 15) == 0) && (((uintptr_t)g.B & 15) == 0) && (g.lda % VEC == 0) && (g.ldb % VEC == 0) &&
           (g.M % VEC == 0) && (g.N % VEC == 0) && g.K > 0;
}

template <int IN, int BM, int BN, bool FAST>
int launch_plain(aser_ctx* ctx, const GemmArgs& g) {
    using Cfg = TileCfg<IN, BM, BN>;
    static bool attr_set[16] = {false};
    auto kern = gemm_tn_kernel<IN, BM, BN, FAST>;
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

template <int IN, bool FAST>
int launch_pair(aser_ctx* ctx, const GemmArgs& g) {
    using Cfg = TileCfg<IN, 256, 128>;
    static bool attr_set[16] = {false};
    auto kern = gemm_tn_pair_kernel<IN, FAST>;
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::LDS_BYTES));
        attr_set[ctx->device] = true;
    }
    const int64_t tm = ceil_div64(g.M, 256), tn = ceil_div64(g.N, 128);
    hipLaunchKernelGGL(kern, dim3((unsigned)(tm * ((tn + 1) / 2))), dim3(kThreads), Cfg::LDS_BYTES, ctx->stream, g);
    return aser_check_launch(ctx, "gemm_tn_pair");
}

template <int IN, bool FAST>
int dispatch_tile2(aser_ctx* ctx, const GemmArgs& g) {
    if (g.pair_cols) return launch_pair<IN, FAST>(ctx, g);
    if (g.bm == 256 && g.bn == 256) {
        if constexpr (IN == GEMM_IN_F32X6) {
            ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: the six-product form has no 256 x 256 tile (LDS)");
        } else {
            return launch_plain<IN, 256, 256, FAST>(ctx, g);
        }
    }
    if (g.bm == 128 && g.bn == 256) return launch_plain<IN, 128, 256, FAST>(ctx, g);
    if (g.bm == 256 && g.bn == 128) return launch_plain<IN, 256, 128, FAST>(ctx, g);
    if (g.bm == 128 && g.bn == 128) return launch_plain<IN, 128, 128, FAST>(ctx, g);
    ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: unsupported tile %dx%d", g.bm, g.bn);
}

template <int IN>
int dispatch_tile(aser_ctx* ctx, const GemmArgs& g) {
    if (operands_fast<IN>(g)) return dispatch_tile2<IN, true>(ctx, g);
    return dispatch_tile2<IN, false>(ctx, g);
}

// ---------------------------------------------------------------------------------------------
// Gram update with an XCD-aware persistent schedule.
//
// One workgroup per compute unit (256 of them; the tile's LDS footprint allows no more).  Work-
// groups are dealt to the 8 XCDs round-robin, so workgroup w runs on XCD w % 8 as slot w / 8.
// The token range is cut into C chunks (C = 1, 2, 4 or 8, chosen on the host); 8 / C XCDs share
// a chunk and split the lower-triangle tiles among them, each XCD taking 32 consecutive tiles of
// the tile order per round.  The tile order (strips of 8 tile columns, row-major inside a strip)
// makes 32 consecutive tiles a 4 x 8 patch that needs only 12 distinct 256-channel slabs of X
// per K step, and the 32 workgroups of an XCD sweep their chunk in lock step, so a slab is
// fetched from HBM about once per XCD and served to the other workgroups from that XCD's L2.
// Tiles left over after the full rounds are split along K so that every workgroup stays busy.
// Partial tiles are added to G with fp32 atomics (C chunks contribute to every tile).
__device__ __forceinline__ void tri_strip_tile(int64_t t, int nt, int* p_out, int* q_out) {
    for (int q0 = 0; q0 < nt; q0 += 8) {
        for (int p = q0; p < nt; ++p) {
            const int cnt = (p - q0 + 1 < 8) ? (p - q0 + 1) : 8;
            if (t < cnt) { *p_out = p; *q_out = q0 + (int)t; return; }
            t -= cnt;
        }
    }
    *p_out = 0; *q_out = 0;
}

template <int IN, int BM, bool FAST>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void gram_persistent_kernel(GemmArgs g) {
    extern __shared__ uint4 smem[];
    constexpr int BK = InTraits<IN>::BK;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int slots = gridDim.x >> 3;                                 // workgroups per XCD
    const int C = g.k_parts;                                          // K chunks: 1, 2, 4 or 8
    const int gsz = 8 / C;                                            // XCDs that share one K chunk
    const int chunk = xcd / gsz, xi = xcd % gsz;
    const int64_t W = (int64_t)gsz * slots;                           // workgroups per K chunk
    const int64_t widx = (int64_t)xi * slots + slot;                  // an XCD takes `slots` consecutive tiles
    const int nt = (int)((g.N + BM - 1) / BM);
    const int64_t T = (int64_t)nt * (nt + 1) / 2;
    const int64_t ksteps = (g.K + BK - 1) / BK;
    const int64_t per = (ksteps + C - 1) / C;
    const int64_t kx0 = (int64_t)chunk * per * BK;
    int64_t kx1 = kx0 + per * BK;
    if (kx1 > g.K) kx1 = g.K;
    if (kx0 >= kx1) return;
    const int64_t full = T / W, rem = T % W;
    const int64_t split = rem > 0 ? W / rem : 1;                      // K split of the left-over tiles
    const int64_t rounds = full + ((rem > 0 && widx < rem * split) ? 1 : 0);
    for (int64_t round = 0; round < rounds; ++round) {
        int64_t t = round * W + widx, k0 = kx0, k1 = kx1;
        if (round == full) {                                          // left-over tile, one K part of it
            t = full * W + widx % rem;
            const int64_t xsteps = (kx1 - kx0 + BK - 1) / BK;
            const int64_t pp = (xsteps + split - 1) / split;
            k0 = kx0 + (widx / rem) * pp * BK;
            k1 = k0 + pp * BK;
            if (k1 > kx1) k1 = kx1;
            if (k0 >= k1) break;
        }
        int p, q;
        tri_strip_tile(t, nt, &p, &q);
        tile_body<IN, BM, BM, FAST>(g, (int64_t)p * BM, (int64_t)q * BM, k0, k1, smem);
    }
}

template <int IN, bool FAST>
int launch_gram_persistent2(aser_ctx* ctx, const GemmArgs& g) {
    using Cfg = TileCfg<IN, 256, 256>;
    static bool attr_set[16] = {false};
    auto kern = gram_persistent_kernel<IN, 256, FAST>;
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)Cfg::LDS_BYTES));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(kern, dim3(256), dim3(kThreads), Cfg::LDS_BYTES, ctx->stream, g);
    return aser_check_launch(ctx, "gram_persistent");
}

// ---------------------------------------------------------------------------------------------
// Gram tiles for bf16 X without a register stage (the main path of the Gram update).
//
// X is tokens x channels, so a slab of 32 tokens x 256 channels is 32 rows of 512 contiguous
// bytes.  global_load_lds_dwordx4 copies it straight into LDS: a wavefront instruction moves
// 64 x 16 bytes to 1 KB of consecutive LDS (two slab rows), and each lane chooses which 16-byte
// chunk of the row it fetches, which is how the layout gets its XOR swizzle: chunk c of slab row
// k sits at chunk slot c ^ 4 (k & 3).  The MFMA operands (8 consecutive tokens of one channel
// per lane) come out of that token-major layout through ds_read_b64_tr_b16: 16 lanes read a
// 4 token x 16 channel block (4 lanes per row, 8 bytes each) and each lane receives the 4 tokens
// of its channel; with the swizzle the 4 rows of a block lie 64 bytes apart in the bank map, which is
// what this read needs to run without bank conflicts (the conflict counter reads zero; with rows 32
// bytes apart every read took twice as long).  So
// there is no transpose in registers, no LDS store instruction and no staging VGPRs; a ring of
// four 32 KB stages keeps three steps of loads in flight.  Rows past the token range and
// channels past n are fetched from a block of zeros.
__device__ uint4 g_zero_chunk[4];

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

constexpr int kDmaBK = 32;
constexpr int kDmaStages = 4;
constexpr int kDmaSlabBytes = kDmaBK * 512;
constexpr int kDmaStageBytes = 2 * kDmaSlabBytes;
constexpr size_t kDmaLdsBytes = (size_t)kDmaStages * kDmaStageBytes;

__device__ __forceinline__ bf16x8_t lds_tr_frag(const char* p, int off_lo, int off_hi) {
    typedef s16x4_t __attribute__((address_space(3))) * lds_s4p;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(p + off_lo));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4p)(p + off_hi));
    const s16x8_t v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, v);
}

// One 256 x 256 tile of G over tokens [kBeg, kEnd): G[I0.., J0..] += X[:, I0..]^T X[:, J0..].
//
// Step s multiplies stage s % 4 in two 16-token slices of 16 MFMAs each.  One wave per SIMD means
// nothing but instruction order hides latencies, so the order is pinned by hand: the operand reads
// of slice 1 are interleaved with the MFMAs of slice 0; the wait for the next stage, the barrier,
// the loads of stage s + 3 and the operand reads of the next step's slice 0 are interleaved with
// the MFMAs of slice 1.
__device__ __forceinline__ void gram_tile_dma(const GemmArgs& g, int64_t I0, int64_t J0, int64_t kBeg, int64_t kEnd,
                                              char* smem) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 128;

    // ---- fetch roles: this wave issues instructions 4 wave .. 4 wave + 3 of each slab; instruction i
    // covers slab rows 2 i and 2 i + 1, lane l is chunk slot l % 32 of row 2 i + l / 32
    const int drow = lane >> 5, slot = lane & 31;
    const char* zero = (const char*)g_zero_chunk;
    const int64_t ld_bytes = g.lda * 2;
    const int row0 = 8 * wave + drow;                    // slab row of this lane in its wave's first instruction
    const char* gp[2][4];                                // next source address per (operand, instruction)
    int64_t gstep[2][2];                                 // its advance per step (0 for chunks past n: they stay on the zeros)
    int64_t tok_next = kBeg + row0;                      // token of gp[.][0]
#pragma unroll
    for (int par = 0; par < 2; ++par) {
        const int chunk = slot ^ (4 * ((2 * par + drow) & 3));
        const int64_t ca = I0 + 8 * chunk, cb = J0 + 8 * chunk;
        gstep[0][par] = (ca < g.M) ? kDmaBK * ld_bytes : 0;
        gstep[1][par] = (cb < g.N) ? kDmaBK * ld_bytes : 0;
#pragma unroll
        for (int t = par; t < 4; t += 2) {
            gp[0][t] = (ca < g.M) ? (const char*)g.A + ca * 2 + (tok_next + 2 * t) * ld_bytes : zero;
            gp[1][t] = (cb < g.N) ? (const char*)g.B + cb * 2 + (tok_next + 2 * t) * ld_bytes : zero;
        }
    }
    // LDS byte address of the ring (what M0 must hold for the LDS-direct loads)
    const uint32_t ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + wave * 4096;
    // One load of stage `step` (op, t fixed at compile time by the callers' unrolling).  Written as
    // inline assembly on purpose: the compiler makes every LDS read wait for all LDS-direct loads it
    // knows of (it cannot tell the ring stages apart), which would undo the prefetch.  The stages are
    // kept apart by the explicit vmcnt waits and barriers below instead.
    auto issue_one = [&](int64_t step, int op, int t, bool tail) {
        const char* src = gp[op][t];
        if (tail && tok_next + 2 * t >= kEnd) src = zero;
        const uint32_t dst = ring + (uint32_t)(step & (kDmaStages - 1)) * kDmaStageBytes + op * kDmaSlabBytes + t * 1024;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst), "v"(src) : "memory", "m0");
        gp[op][t] += gstep[op][t & 1];
    };
    auto issue_all = [&](int64_t step) {
        const bool tail = kBeg + (step + 1) * kDmaBK > kEnd;
#pragma unroll
        for (int op = 0; op < 2; ++op)
#pragma unroll
            for (int t = 0; t < 4; ++t) issue_one(step, op, t, tail);
        tok_next += kDmaBK;
    };

    // ---- operand read offsets inside a stage (bytes), first of the four (k16 slice, half) reads
    int offa[4], offb[4];
    {
        const int krow = 8 * (lane >> 5) + ((lane & 15) >> 2);
        const int xr = 4 * ((lane & 15) >> 2);
        const int msub = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ma = wm0 + 32 * i + msub, mb = wn0 + 32 * i + msub;
            offa[i] = krow * 512 + (((ma >> 3) ^ xr) * 16) + (ma & 7) * 2;
            offb[i] = kDmaSlabBytes + krow * 512 + (((mb >> 3) ^ xr) * 16) + (mb & 7) * 2;
        }
    }

    f32x16_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int64_t nsteps = (kEnd - kBeg + kDmaBK - 1) / kDmaBK;
    __syncthreads();                                     // the previous tile's readers are done with the ring
    for (int64_t s = 0; s < kDmaStages - 1 && s < nsteps; ++s) issue_all(s);
    if (nsteps >= 3) __builtin_amdgcn_s_waitcnt(0x4F70);             // vmcnt(16): stage 0 landed
    else if (nsteps == 2) __builtin_amdgcn_s_waitcnt(0x0F78);        // vmcnt(8)
    else __builtin_amdgcn_s_waitcnt(0x0F70);                         // vmcnt(0)
    __syncthreads();
    bf16x8_t a0[4], b0[4], a1[4], b1[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a0[i] = lds_tr_frag(smem + offa[i], 0, 4 * 512);
        b0[i] = lds_tr_frag(smem + offb[i], 0, 4 * 512);
    }
    // STEADY steps have a successor, a stage to fetch and no ragged rows in it: no branch in the body.
    auto step = [&](int64_t s, auto steady_tag) {
        constexpr bool STEADY = decltype(steady_tag)::value;
        const char* st = smem + (int)(s & (kDmaStages - 1)) * kDmaStageBytes;
        const char* sn = smem + (int)((s + 1) & (kDmaStages - 1)) * kDmaStageBytes;
        const bool more = STEADY || s + 1 < nsteps;
        const bool fetch = STEADY || s + kDmaStages - 1 < nsteps;
        const bool tail = !STEADY && fetch && (kBeg + (s + kDmaStages) * kDmaBK > kEnd);
        // slice 0: 16 MFMAs, one operand fragment of slice 1 read after every second one
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[i], b0[j], acc[i][j], 0, 0, 0);
                if (j == 1) a1[i] = lds_tr_frag(st + offa[i], 16 * 512, 20 * 512);
                if (j == 3) b1[i] = lds_tr_frag(st + offb[i], 16 * 512, 20 * 512);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // slice 1: row 0 of MFMAs covers the wait and the barrier, rows 1 and 2 the eight loads of
        // stage s + 3, rows 2 and 3 the reads of the next step's slice 0
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[i], b1[j], acc[i][j], 0, 0, 0);
                if (i == 0 && j == 1 && more) {
                    // stage s + 1 has landed when at most the loads of stage s + 2 are in flight
                    if (STEADY || s + 2 < nsteps) __builtin_amdgcn_s_waitcnt(0x0F78);    // vmcnt(8)
                    else __builtin_amdgcn_s_waitcnt(0x0F70);                             // vmcnt(0)
                    __syncthreads();                      // everyone's share landed; stage s - 1 is free
                }
                if (fetch && i == 1) { issue_one(s + kDmaStages - 1, 0, j, tail); }
                if (fetch && i == 2 && j < 2) { issue_one(s + kDmaStages - 1, 1, 2 * j, tail); issue_one(s + kDmaStages - 1, 1, 2 * j + 1, tail); }
                if (more && i == 2 && j >= 2) {
                    a0[2 * (j - 2)] = lds_tr_frag(sn + offa[2 * (j - 2)], 0, 4 * 512);
                    a0[2 * (j - 2) + 1] = lds_tr_frag(sn + offa[2 * (j - 2) + 1], 0, 4 * 512);
                }
                if (more && i == 3) b0[j] = lds_tr_frag(sn + offb[j], 0, 4 * 512);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        if (fetch) tok_next += kDmaBK;
    };
    const int64_t full_steps = (kEnd - kBeg) / kDmaBK;               // stages without ragged rows
    int64_t s = 0;
    for (; s + kDmaStages - 1 < full_steps; ++s) step(s, std::true_type{});
    for (; s < nsteps; ++s) step(s, std::false_type{});

    // acc[i][j][e] is G(row, col) with row = 32 i + 8 (e / 4) + 4 (lane / 32) + e % 4, col = 32 j + lane % 32
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = J0 + wn0 + 32 * j + (lane & 31);
            const int64_t rbase = I0 + wm0 + 32 * i + 4 * (lane >> 5);
            if (col >= g.N) continue;
            float* cbase = g.C + rbase * g.ldc + col;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int dr = 8 * (e >> 2) + (e & 3);
                if (rbase + dr < g.M) unsafeAtomicAdd(cbase + (int64_t)dr * g.ldc, g.alpha * acc[i][j][e]);
            }
        }
}

// The persistent XCD-aware schedule of gram_persistent_kernel with the LDS-direct tile body.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void gram_dma_kernel(GemmArgs g) {
    extern __shared__ uint4 smem[];
    constexpr int BK = kDmaBK, BM = 256;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int slots = gridDim.x >> 3;
    const int C = g.k_parts;
    const int gsz = 8 / C;
    const int chunk = xcd / gsz, xi = xcd % gsz;
    const int64_t W = (int64_t)gsz * slots;
    const int64_t widx = (int64_t)xi * slots + slot;
    const int nt = (int)((g.N + BM - 1) / BM);
    const int64_t T = (int64_t)nt * (nt + 1) / 2;
    const int64_t ksteps = (g.K + BK - 1) / BK;
    const int64_t per = (ksteps + C - 1) / C;
    const int64_t kx0 = (int64_t)chunk * per * BK;
    int64_t kx1 = kx0 + per * BK;
    if (kx1 > g.K) kx1 = g.K;
    if (kx0 >= kx1) return;
    const int64_t full = T / W, rem = T % W;
    const int64_t split = rem > 0 ? W / rem : 1;
    const int64_t rounds = full + ((rem > 0 && widx < rem * split) ? 1 : 0);
    for (int64_t round = 0; round < rounds; ++round) {
        int64_t t = round * W + widx, k0 = kx0, k1 = kx1;
        if (round == full) {
            t = full * W + widx % rem;
            const int64_t xsteps = (kx1 - kx0 + BK - 1) / BK;
            const int64_t pp = (xsteps + split - 1) / split;
            k0 = kx0 + (widx / rem) * pp * BK;
            k1 = k0 + pp * BK;
            if (k1 > kx1) k1 = kx1;
            if (k0 >= k1) break;
        }
        int p, q;
        tri_strip_tile(t, nt, &p, &q);
        gram_tile_dma(g, (int64_t)p * BM, (int64_t)q * BM, k0, k1, (char*)smem);
    }
}

int launch_gram_dma(aser_ctx* ctx, const GemmArgs& g) {
    static bool attr_set[16] = {false};
    if (ctx->device >= 0 && ctx->device < 16 && !attr_set[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)gram_dma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kDmaLdsBytes));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL(gram_dma_kernel, dim3(256), dim3(kThreads), kDmaLdsBytes, ctx->stream, g);
    return aser_check_launch(ctx, "gram_dma");
}

template <int IN>
int launch_gram_persistent(aser_ctx* ctx, const GemmArgs& g) {
    if (operands_fast<IN>(g)) return launch_gram_persistent2<IN, true>(ctx, g);
    return launch_gram_persistent2<IN, false>(ctx, g);
}

}  // namespace

int aser_gemm_tn(aser_ctx* ctx, const GemmArgs& g) {
    if (g.M <= 0 || g.N <= 0 || g.K < 0) ASER_FAIL(ctx, ASER_ERR_SHAPE, "gemm_tn: bad sizes");
    if (g.k_parts < 1 || (g.k_parts > 1 && g.epi != GEMM_EPI_ATOMIC))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: split K needs the atomic epilogue");
    if (g.tiles != GEMM_TILES_ALL && (g.M != g.N || g.bm != g.bn))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: triangular tiling needs a square problem and tile");
    if (g.Ct && g.epi != GEMM_EPI_STORE) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: Ct needs the store epilogue");
    if (g.pair_cols && (g.tiles != GEMM_TILES_ALL || g.k_parts != 1 || g.bm != 256 || g.bn != 128))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: paired tile columns need all tiles, k_parts == 1 and 256 x 128 tiles");
    if (g.epi == GEMM_EPI_RESID && (!g.sumsq || g.k_parts != 1 || g.bm != 128 || g.bn != 128))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "gemm_tn: the residual epilogue needs sumsq, k_parts == 1 and 128 x 128 tiles");
    if (g.in_type == GEMM_IN_BF16) return dispatch_tile<GEMM_IN_BF16>(ctx, g);
    if (g.in_type == GEMM_IN_F32X3) return dispatch_tile<GEMM_IN_F32X3>(ctx, g);
    if (g.in_type == GEMM_IN_F32X6) return dispatch_tile<GEMM_IN_F32X6>(ctx, g);
    ASER_FAIL(ctx, ASER_ERR_DTYPE, "gemm_tn: unknown input type");
}

// Gram update: lower-triangle tiles of G += X^T X.  Large problems use the persistent schedule
// above; small ones split K over a plain grid.  Partial tiles are added with fp32 atomics.
int aser_syrk_gram(aser_ctx* ctx, const void* X, int x_dtype, int64_t rows, int64_t n, int64_t ldx,
                   float* G, int64_t ldg) {
    GemmArgs g{};
    g.A = X; g.lda = ldx; g.B = X; g.ldb = ldx;
    g.C = G; g.ldc = ldg; g.Ct = nullptr; g.ldct = 0;
    g.M = n; g.N = n; g.K = rows; g.alpha = 1.f;
    g.in_type = (x_dtype == ASER_DTYPE_BF16) ? GEMM_IN_BF16 : aser_f32_form(ctx, n * n);
    g.epi = GEMM_EPI_ATOMIC; g.tiles = GEMM_TILES_LOWER; g.krange = GEMM_K_FULL;
    const bool six = g.in_type == GEMM_IN_F32X6;         // no 256 x 256 tile: the plain grid with 128 x 128 tiles
    const int bk = (g.in_type == GEMM_IN_BF16) ? 64 : 32;
    const int64_t ksteps = ceil_div64(rows, bk);
    const int64_t t256 = ceil_div64(n, 256);
    const int64_t T256 = t256 * (t256 + 1) / 2;
    if (T256 >= 32 && ksteps >= 8 * 16 && !six) {
        // Number of K chunks: fewest steps on the busiest workgroup, each tile visit charged with
        // the cost of flushing a tile through atomics (about a dozen K steps).
        int best_c = 8;
        int64_t best_cost = -1;
        for (int c = 1; c <= 8; c *= 2) {
            const int64_t W = 256 / c, full = T256 / W, rem = T256 % W;
            const int64_t steps_c = ceil_div64(ksteps, c);
            const int64_t split = rem ? W / rem : 1;
            const int64_t cost = full * (steps_c + 12) + (rem ? ceil_div64(steps_c, split) + 12 : 0);
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_c = c; }
        }
        g.bm = g.bn = 256; g.k_parts = best_c;
        if (g.in_type == GEMM_IN_BF16 && operands_fast<GEMM_IN_BF16>(g)) return launch_gram_dma(ctx, g);
        return (g.in_type == GEMM_IN_BF16) ? launch_gram_persistent<GEMM_IN_BF16>(ctx, g)
                                           : launch_gram_persistent<GEMM_IN_F32X3>(ctx, g);
    }
    g.bm = g.bn = (n <= 1024 || six) ? 128 : 256;
    const int64_t t = ceil_div64(n, g.bm), tiles = t * (t + 1) / 2;
    int64_t parts = ceil_div64(1024, tiles);              // aim at >= 4 workgroups per CU
    const int64_t max_parts = ksteps / 16 > 0 ? ksteps / 16 : 1;   // keep >= 16 steps per part
    if (parts > max_parts) parts = max_parts;
    if (parts < 1) parts = 1;
    g.k_parts = (int)parts;
    return aser_gemm_tn(ctx, g);
}
