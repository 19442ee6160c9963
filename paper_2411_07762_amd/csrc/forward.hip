// The compensated layer at inference (end of Sec. 4.2: W_q X + L_A L_B X; overhead analysis of
// Sec. 5.3: s d^2 -> s d^2 + 2 s r d operations), in this library's tokens x channels orientation:
//     Y[t][o] = s_t c_o sum_i xq[t][i] wq[o][i]  +  sum_k P[t][k] L_A[o][k],
//     P[t][k] = s_t sum_i xq[t][i] L_B[k][i]
// with xq, s_t the per-token activation codes and scales (aser_quantize_act_rtn of X M^-1), wq, c_o
// the per-channel weight codes and scales (aser_quantize_rtn), both branches reading the same
// quantized activations.
//
// Every operand is contiguous along the contraction dimension (a token's channels, an output's
// channels, a row of L_B, a row of L_A), which is how MFMA operands want them: a lane holds 16
// consecutive int8 (v_mfma_i32_32x32x32_i8) or 8 consecutive bf16 (v_mfma_f32_32x32x16_bf16) of its
// row.  No transposes anywhere.
//
// Main kernel: a workgroup (4 waves, 2 x 2) owns 128 tokens x 256 outputs; per step 64 channels of
// both operands go through registers into LDS (16-byte chunks, XOR-swizzled so that the 16-byte operand
// reads of 32 consecutive rows hit distinct banks), double buffered, one barrier per step.  int4 codes
// are widened while staged: the low nibbles of a dword become the bytes (w << 4) & 0xF0F0F0F0 and the
// high nibbles w & 0xF0F0F0F0, i.e. 16 q as a signed byte, no borrow between bytes; the factor 16 goes
// into the scale.  That puts the even channels of a group of 32 into one 16-byte chunk and the odd ones
// into the next, so the activation bytes are put into the same order with two byte permutes per 8.
// The int32 sums are exact.  Epilogue: scale, then the rank-r branch as r / 16 further bf16 MFMA steps
// on the same accumulators (P from the small kernel below, L_A pre-split into bf16 planes), then store.
//
// Rank-r branch precision: L_A, L_B and P are fp32; a bf16 MFMA sees hi = bf16(x) and, in the split
// mode, also lo = bf16(x - hi) (three products hi hi + hi lo + lo hi per fp32 product; the activation
// codes are exact in bf16, so P needs two).  The plain mode uses hi alone, as an inference kernel that
// keeps the factors in 16-bit would.
#include <type_traits>

#include "aser_internal.h"

namespace {

typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef int v16i_t __attribute__((ext_vector_type(16)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int kFwdTM = 128, kFwdTN = 256, kFwdBK = 64;

__device__ __forceinline__ uint32_t bf16_hi_pair(float a, float b) {       // truncation-free: callers pass bf16-exact values or accept RNE below
    return (__float_as_uint(a) >> 16) | (__float_as_uint(b) & 0xFFFF0000u);
}
__device__ __forceinline__ uint32_t bf16_rne(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Both factors as bf16 planes in one launch: hi = bf16(x), lo = bf16(x - hi).  L_A (m x r) goes to [m][r_pad]
// with zero columns r .. r_pad, L_B (r x n) to [r_pad][n] with zero rows r .. r_pad.
__global__ __launch_bounds__(256) void split_factors_kernel(const float* __restrict__ L_A, const float* __restrict__ L_B, int64_t m,
                                                            int64_t n, int64_t r, int64_t r_pad, uint16_t* __restrict__ la_hi,
                                                            uint16_t* __restrict__ la_lo, uint16_t* __restrict__ lb_hi,
                                                            uint16_t* __restrict__ lb_lo) {
    const int64_t ta = m * r_pad, total = ta + r_pad * n;
    for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
        float x;
        uint16_t *hi, *lo;
        if (t < ta) {
            const int64_t i = t / r_pad, j = t % r_pad;
            x = j < r ? L_A[i * r + j] : 0.f;
            hi = la_hi + t; lo = la_lo + t;
        } else {
            const int64_t u = t - ta, k = u / n;
            x = k < r ? L_B[u] : 0.f;
            hi = lb_hi + u; lo = lb_lo + u;
        }
        const uint32_t h = bf16_rne(x);
        *hi = (uint16_t)h;
        *lo = (uint16_t)bf16_rne(x - __uint_as_float(h << 16));
    }
}

// byte offset of 16-byte chunk c (0..3) of row r inside a [rows][64 bytes] LDS tile
__device__ __forceinline__ int chunk_off(int r, int c) { return r * 64 + ((c ^ ((r >> 2) & 3)) << 4); }

// Stages 64 channels of `nrows` (128 or 256) code rows: thread t handles row t / 2 (+ 128 per repeat),
// half t % 2 = channels [32 half, 32 half + 32) of the step.
//   PLAIN  : int8 codes, 32 bytes copied as two chunks
//   PERMUTE: int8 codes reordered to (even channels, odd channels) per group of 32
//   NIBBLES: packed int4 codes (16 bytes) widened to 16 q bytes, even channels first
enum StageKind { STAGE_PLAIN = 0, STAGE_PERMUTE = 1, STAGE_NIBBLES = 2 };

template <int KIND, int REPS>
struct CodeStage {
    uint4 r[REPS][2];
    const char* p[REPS];
    bool ok[REPS];

    __device__ __forceinline__ void init(const void* base, int64_t row0, int64_t nrows_total, int64_t pitch_bytes, int tid) {
        const int half = tid & 1;
#pragma unroll
        for (int u = 0; u < REPS; ++u) {
            const int64_t row = row0 + (tid >> 1) + 128 * u;
            ok[u] = row < nrows_total;
            p[u] = (const char*)base + (ok[u] ? row : 0) * pitch_bytes + (KIND == STAGE_NIBBLES ? 16 : 32) * half;
        }
    }
    // loads channels [k0 + 32 half, +32) of the thread's rows; k0 + 64 may exceed n (n % 32 == 0)
    __device__ __forceinline__ void load(int64_t k0, int64_t n, int tid) {
        const bool in = k0 + 32 * (tid & 1) < n;
#pragma unroll
        for (int u = 0; u < REPS; ++u) {
            r[u][0] = make_uint4(0u, 0u, 0u, 0u);
            r[u][1] = make_uint4(0u, 0u, 0u, 0u);
            if (ok[u] && in) {
                if (KIND == STAGE_NIBBLES) {
                    r[u][0] = *(const uint4*)(p[u] + k0 / 2);
                } else {
                    r[u][0] = *(const uint4*)(p[u] + k0);
                    r[u][1] = *(const uint4*)(p[u] + k0 + 16);
                }
            }
        }
    }
    __device__ __forceinline__ void store(char* tile, int tid) const {
        const int half = tid & 1;
#pragma unroll
        for (int u = 0; u < REPS; ++u) {
            const int row = (tid >> 1) + 128 * u;
            uint4 c0, c1;
            if (KIND == STAGE_PLAIN) {
                c0 = r[u][0];
                c1 = r[u][1];
            } else if (KIND == STAGE_PERMUTE) {
                const uint4 a = r[u][0], b = r[u][1];
                c0 = make_uint4(__builtin_amdgcn_perm(a.y, a.x, 0x06040200u), __builtin_amdgcn_perm(a.w, a.z, 0x06040200u),
                                __builtin_amdgcn_perm(b.y, b.x, 0x06040200u), __builtin_amdgcn_perm(b.w, b.z, 0x06040200u));
                c1 = make_uint4(__builtin_amdgcn_perm(a.y, a.x, 0x07050301u), __builtin_amdgcn_perm(a.w, a.z, 0x07050301u),
                                __builtin_amdgcn_perm(b.y, b.x, 0x07050301u), __builtin_amdgcn_perm(b.w, b.z, 0x07050301u));
            } else {
                const uint4 w = r[u][0];
                c0 = make_uint4((w.x << 4) & 0xF0F0F0F0u, (w.y << 4) & 0xF0F0F0F0u, (w.z << 4) & 0xF0F0F0F0u, (w.w << 4) & 0xF0F0F0F0u);
                c1 = make_uint4(w.x & 0xF0F0F0F0u, w.y & 0xF0F0F0F0u, w.z & 0xF0F0F0F0u, w.w & 0xF0F0F0F0u);
            }
            *(uint4*)(tile + chunk_off(row, 2 * half)) = c0;
            *(uint4*)(tile + chunk_off(row, 2 * half + 1)) = c1;
        }
    }
};

struct FwdArgs {
    const int8_t* xq; const float* xs; int64_t rows, n;
    const void* wq; const float* ws; int64_t m;
    const uint16_t* p_hi; const uint16_t* p_lo;   // P = s_t (x_q L_B^T) as bf16 planes, rows x r_pad (p_hi null: no rank-r branch)
    const uint16_t* la_hi; const uint16_t* la_lo; int r_pad;   // m x r_pad bf16 planes
    float* Y; int64_t ldy;
};

template <bool W4, bool SPLIT>
__global__ __launch_bounds__(256) void cf_main_kernel(FwdArgs g) {
    extern __shared__ __align__(16) char smem[];
    constexpr int A_BYTES = kFwdTM * 64, B_BYTES = kFwdTN * 64, STAGE = A_BYTES + B_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t T0 = (int64_t)blockIdx.y * kFwdTM, O0 = (int64_t)blockIdx.x * kFwdTN;

    CodeStage<W4 ? STAGE_PERMUTE : STAGE_PLAIN, 1> sa;
    CodeStage<W4 ? STAGE_NIBBLES : STAGE_PLAIN, 2> sb;
    sa.init(g.xq, T0, g.rows, g.n, tid);
    sb.init(g.wq, O0, g.m, W4 ? g.n / 2 : g.n, tid);

    v16i_t acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    // operand read offsets: row of the lane inside the tile, chunk = 2 slice + lane / 32
    int offa[2][2], offb[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const int c = 2 * s + (lane >> 5);
#pragma unroll
        for (int i = 0; i < 2; ++i) offa[s][i] = chunk_off(wm * 64 + 32 * i + (lane & 31), c);
#pragma unroll
        for (int j = 0; j < 4; ++j) offb[s][j] = A_BYTES + chunk_off(wn * 128 + 32 * j + (lane & 31), c);
    }

    const int64_t steps = (g.n + kFwdBK - 1) / kFwdBK;
    sa.load(0, g.n, tid);
    sb.load(0, g.n, tid);
    sa.store(smem, tid);
    sb.store(smem + A_BYTES, tid);
    __syncthreads();
    for (int64_t s = 0; s < steps; ++s) {
        const char* cur = smem + (s & 1) * STAGE;
        char* nxt = smem + ((s + 1) & 1) * STAGE;
        const bool more = s + 1 < steps;
        if (more) {
            sa.load((s + 1) * kFwdBK, g.n, tid);
            sb.load((s + 1) * kFwdBK, g.n, tid);
        }
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            v4i_t a[2], b[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) a[i] = *(const v4i_t*)(cur + offa[sl][i]);
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = *(const v4i_t*)(cur + offb[sl][j]);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            sa.store(nxt, tid);
            sb.store(nxt + A_BYTES, tid);
        }
        __syncthreads();
    }

    // epilogue: acc[i][j][e] is (token, output) = (32 i + 8 (e / 4) + 4 (lane / 32) + e % 4, 32 j + lane % 32) of the wave's sub-tile
    const float wfix = W4 ? (1.0f / 16.0f) : 1.0f;
    f32x16_t y[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t col = O0 + wn * 128 + 32 * j + (lane & 31);
        const float cw = (col < g.m) ? g.ws[col] * wfix : 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t row = T0 + wm * 64 + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const float sx = (row < g.rows) ? g.xs[row] : 0.f;
                y[i][j][e] = (float)acc[i][j][e] * (sx * cw);
            }
    }
    if (g.p_hi) {
        for (int kk = 0; kk < g.r_pad; kk += 16) {
            const int kq = kk + 8 * (lane >> 5);
            bf16x8_t ph[2], pl[2], lh[4], ll[4];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int64_t row = T0 + wm * 64 + 32 * i + (lane & 31);
                uint4 vh = make_uint4(0u, 0u, 0u, 0u), vl = make_uint4(0u, 0u, 0u, 0u);
                if (row < g.rows) {
                    vh = *(const uint4*)(g.p_hi + row * g.r_pad + kq);
                    if (SPLIT) vl = *(const uint4*)(g.p_lo + row * g.r_pad + kq);
                }
                ph[i] = __builtin_bit_cast(bf16x8_t, vh);
                pl[i] = __builtin_bit_cast(bf16x8_t, vl);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t col = O0 + wn * 128 + 32 * j + (lane & 31);
                uint4 vh = make_uint4(0u, 0u, 0u, 0u), vl = make_uint4(0u, 0u, 0u, 0u);
                if (col < g.m) {
                    vh = *(const uint4*)(g.la_hi + col * g.r_pad + kq);
                    if (SPLIT) vl = *(const uint4*)(g.la_lo + col * g.r_pad + kq);
                }
                lh[j] = __builtin_bit_cast(bf16x8_t, vh);
                ll[j] = __builtin_bit_cast(bf16x8_t, vl);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (SPLIT) {
                        y[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl[i], lh[j], y[i][j], 0, 0, 0);
                        y[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph[i], ll[j], y[i][j], 0, 0, 0);
                    }
                    y[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph[i], lh[j], y[i][j], 0, 0, 0);
                }
        }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = O0 + wn * 128 + 32 * j + (lane & 31);
            if (col >= g.m) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t row = T0 + wm * 64 + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                if (row < g.rows) g.Y[row * g.ldy + col] = y[i][j][e];
            }
        }
}

// ---------------------------------------------------------------------------------------------
// The same product for layers of at least 256 tokens x 256 outputs, without a register stage: a workgroup
// (4 waves, 2 x 2, one per SIMD) owns 256 tokens x 256 outputs, all 256 accumulator registers of a wave hold
// its 128 x 128 part.  Per step 64 channels: global_load_lds_dwordx4 copies 16-byte chunks of the code rows
// straight into LDS (a wavefront instruction fills 1 KB of consecutive LDS; every lane picks the chunk it
// fetches, which gives the XOR swizzle of chunk_off), a ring of four stages keeps three steps of loads in
// flight, one barrier per step.  int8 rows are 64 bytes per step and feed the MFMA through one 16-byte read
// per operand; packed int4 rows are 32 bytes per step and a lane reads 16 of them once per step: lane group
// g = lane / 32 takes channels [32 g, 32 g + 32) of the step, the first 16 in the first MFMA slice and the other
// 16 in the second (so the activation operand of slice sl is 16-byte chunk 2 g + sl of its row), widens each
// half in registers to (even channels, odd channels) x 2 as 16 q bytes, and the activation operand gets the
// same channel order from four byte permutes.  The loads are inline assembly for the reason given at the Gram
// kernel: the compiler would make every LDS read wait for all LDS-direct loads in flight.
// Workgroup b runs on XCD b % 8; the tiles are numbered so that an XCD works on consecutive (token tile,
// output tile) pairs: its 32 workgroups share two token tiles and one sweep over the weight codes per step.
__device__ uint4 g_fwd_zero[4];

constexpr int kDmaTM = 256, kDmaTN = 256, kDmaStages = 4;

template <bool W4, bool SPLIT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void cf_dma_kernel(FwdArgs g, int tiles_n, int64_t tiles_total) {
    extern __shared__ __align__(16) char smem[];
    constexpr int A_BYTES = kDmaTM * 64, B_ROW = W4 ? 32 : 64, B_BYTES = kDmaTN * B_ROW, STAGE = A_BYTES + B_BYTES;
    constexpr int NLB = W4 ? 2 : 4;                       // LDS-direct loads of the weight slab per wave and stage (4 for the activations)
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm0 = (wave >> 1) * 128, wn0 = (wave & 1) * 128;
    const int64_t per_xcd = (tiles_total + 7) / 8;
    const int64_t tile = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (tile >= tiles_total) return;
    const int64_t T0 = (tile / tiles_n) * kDmaTM, O0 = (tile % tiles_n) * kDmaTN;

    // ---- fetch roles.  Activations: instruction t of this wave is slab rows 16 (4 wave + t) + lane / 4, chunk
    // slot lane % 4.  Weights (int8) alike; packed int4: rows 32 (2 wave + t) + lane / 2, slot lane % 2.
    const char* zero = (const char*)g_fwd_zero;
    const char* gp[2][4];
    int64_t gstep[2][4];
    bool tail_ok[2];                                      // the lane's chunk exists in a last step of 32 channels
    {
        const int ca = (lane & 3) ^ ((lane >> 4) & 3);
        tail_ok[0] = ca < 2;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int64_t row = T0 + 16 * (4 * wave + t) + (lane >> 2);
            const bool ok = row < g.rows;
            gp[0][t] = ok ? (const char*)g.xq + row * g.n + 16 * ca : zero;
            gstep[0][t] = ok ? 64 : 0;
        }
        if (W4) {
            const int cb = (lane & 1) ^ ((lane >> 4) & 1);
            tail_ok[1] = cb < 1;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t row = O0 + 32 * (2 * wave + (t & 1)) + (lane >> 1);
                const bool ok = row < g.m && t < 2;
                gp[1][t] = ok ? (const char*)g.wq + row * (g.n / 2) + 16 * cb : zero;
                gstep[1][t] = ok ? 32 : 0;
            }
        } else {
            tail_ok[1] = ca < 2;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int64_t row = O0 + 16 * (4 * wave + t) + (lane >> 2);
                const bool ok = row < g.m;
                gp[1][t] = ok ? (const char*)g.wq + row * g.n + 16 * ca : zero;
                gstep[1][t] = ok ? 64 : 0;
            }
        }
    }
    const uint32_t ring = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    auto issue_one = [&](int64_t step, int op, int t, bool tail) {
        const char* src = gp[op][t];
        if (tail && !tail_ok[op]) src = zero;
        const uint32_t dst = ring + (uint32_t)(step & (kDmaStages - 1)) * STAGE +
                             (op ? A_BYTES + (NLB * wave + t) * 1024 : (4 * wave + t) * 1024);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst), "v"(src) : "memory", "m0");
        gp[op][t] += gstep[op][t];
    };
    const int64_t nsteps = (g.n + 63) / 64;
    auto issue_all = [&](int64_t step) {
        const bool tail = 64 * (step + 1) > g.n;
#pragma unroll
        for (int t = 0; t < 4; ++t) issue_one(step, 0, t, tail);
#pragma unroll
        for (int t = 0; t < NLB; ++t) issue_one(step, 1, t, tail);
    };

    // ---- operand read offsets inside a stage for the first 32-channel slice; the second slice is the
    // neighbouring chunk pair of the activations: offset ^ 32 (int4 weights: the neighbouring chunk, offset ^ 16;
    // the weight fragment of both slices comes with one read)
    int offa[4], offb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        offa[i] = chunk_off(wm0 + 32 * i + (lane & 31), W4 ? 2 * (lane >> 5) : lane >> 5);
        const int brow = wn0 + 32 * i + (lane & 31);
        offb[i] = A_BYTES + (W4 ? brow * 32 + (((lane >> 5) ^ ((brow >> 3) & 1)) << 4) : chunk_off(brow, lane >> 5));
    }
    constexpr int kXorA = W4 ? 16 : 32, kXorB = 32;
    struct RawB { uint32_t x, y, z, w; };
    auto read_a = [&](const char* st, int sl, int i) { return *(const v4i_t*)(st + (offa[i] ^ (sl ? kXorA : 0))); };
    auto read_b = [&](const char* st, int sl, int i) { return *(const v4i_t*)(st + (W4 ? offb[i] : (offb[i] ^ (sl ? kXorB : 0)))); };
    // channel order of the widened int4 operand: (0 2 4 6)(1 3 5 7)(8 10 12 14)(9 11 13 15) of the lane's 16
    auto conv_a = [&](v4i_t a) {
        if (!W4) return a;
        return v4i_t{(int)__builtin_amdgcn_perm((uint32_t)a.y, (uint32_t)a.x, 0x06040200u), (int)__builtin_amdgcn_perm((uint32_t)a.y, (uint32_t)a.x, 0x07050301u),
                     (int)__builtin_amdgcn_perm((uint32_t)a.w, (uint32_t)a.z, 0x06040200u), (int)__builtin_amdgcn_perm((uint32_t)a.w, (uint32_t)a.z, 0x07050301u)};
    };
    auto conv_b = [&](v4i_t b, int sl) {
        if (!W4) return b;
        const uint32_t w0 = (uint32_t)(sl ? b.z : b.x), w1 = (uint32_t)(sl ? b.w : b.y);
        return v4i_t{(int)((w0 << 4) & 0xF0F0F0F0u), (int)(w0 & 0xF0F0F0F0u), (int)((w1 << 4) & 0xF0F0F0F0u), (int)(w1 & 0xF0F0F0F0u)};
    };

    v16i_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;

    // vmcnt values: one stage of this wave's loads is 4 + NLB instructions
    auto wait_loads = [&](int stages_in_flight) {
        if (W4) {
            if (stages_in_flight == 2) __builtin_amdgcn_s_waitcnt(0x0F7C);          // vmcnt(12)
            else if (stages_in_flight == 1) __builtin_amdgcn_s_waitcnt(0x0F76);     // vmcnt(6)
            else __builtin_amdgcn_s_waitcnt(0x0F70);
        } else {
            if (stages_in_flight == 2) __builtin_amdgcn_s_waitcnt(0x4F70);          // vmcnt(16)
            else if (stages_in_flight == 1) __builtin_amdgcn_s_waitcnt(0x0F78);     // vmcnt(8)
            else __builtin_amdgcn_s_waitcnt(0x0F70);
        }
    };
    for (int64_t s = 0; s < kDmaStages - 1 && s < nsteps; ++s) issue_all(s);
    wait_loads(nsteps >= 3 ? 2 : (nsteps == 2 ? 1 : 0));                            // stage 0 landed
    __syncthreads();
    v4i_t a0[4], b0[4], a1[4], b1[4], braw[4];            // braw: a step's packed int4 fragments (both slices in one read)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        a0[i] = conv_a(read_a(smem, 0, i));
        braw[i] = read_b(smem, 0, i);
        b0[i] = conv_b(braw[i], 0);
    }
    auto step = [&](int64_t s, auto steady_tag) {
        constexpr bool STEADY = decltype(steady_tag)::value;
        const char* st = smem + (int)(s & (kDmaStages - 1)) * STAGE;
        const char* sn = smem + (int)((s + 1) & (kDmaStages - 1)) * STAGE;
        const bool more = STEADY || s + 1 < nsteps;
        const bool fetch = STEADY || s + kDmaStages - 1 < nsteps;
        const bool tail = !STEADY && fetch && 64 * (s + kDmaStages) > g.n;
        // slice 0: the raw operands of slice 1 are read under rows 0 and 1 and put in order under rows 2 and 3
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[i], b0[j], acc[i][j], 0, 0, 0);
                if (i == 0) a1[j] = read_a(st, 1, j);
                if (!W4 && i == 1) b1[j] = read_b(st, 1, j);
                if (i == 2) a1[j] = conv_a(a1[j]);
                if (W4 && i == 3) b1[j] = conv_b(braw[j], 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // slice 1: row 0 covers the wait and the barrier and the reads of the next step's slice 0, row 1 the
        // rest of those reads and the loads of stage s + 3, rows 2 and 3 the reordering of what was read
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[i], b1[j], acc[i][j], 0, 0, 0);
                if (i == 0 && j == 1 && more) {
                    // stage s + 1 has landed when at most the loads of stage s + 2 are in flight
                    wait_loads((STEADY || s + 2 < nsteps) ? 1 : 0);
                    __syncthreads();                      // everyone's share landed; stage s - 1 is free
                }
                if (more && i == 0 && j >= 2) { a0[2 * (j - 2)] = read_a(sn, 0, 2 * (j - 2)); a0[2 * (j - 2) + 1] = read_a(sn, 0, 2 * (j - 2) + 1); }
                if (more && i == 1 && j < 2) {
                    if (W4) { braw[2 * j] = read_b(sn, 0, 2 * j); braw[2 * j + 1] = read_b(sn, 0, 2 * j + 1); }
                    else { b0[2 * j] = read_b(sn, 0, 2 * j); b0[2 * j + 1] = read_b(sn, 0, 2 * j + 1); }
                }
                if (fetch && i == 1 && j >= 2) { issue_one(s + kDmaStages - 1, 0, 2 * (j - 2), tail); issue_one(s + kDmaStages - 1, 0, 2 * (j - 2) + 1, tail); }
                if (fetch && i == 2 && j < 2) {
                    if (W4) issue_one(s + kDmaStages - 1, 1, j, tail);
                    else { issue_one(s + kDmaStages - 1, 1, 2 * j, tail); issue_one(s + kDmaStages - 1, 1, 2 * j + 1, tail); }
                }
                if (more && i == 2 && j >= 2) { a0[2 * (j - 2)] = conv_a(a0[2 * (j - 2)]); a0[2 * (j - 2) + 1] = conv_a(a0[2 * (j - 2) + 1]); }
                if (W4 && more && i == 3) b0[j] = conv_b(braw[j], 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    const int64_t full_steps = g.n / 64;
    int64_t s = 0;
    for (; s + kDmaStages - 1 < full_steps; ++s) step(s, std::true_type{});
    for (; s < nsteps; ++s) step(s, std::false_type{});

    // ---- epilogue.  acc[i][j][e] is (token, output) = (32 i + 8 (e / 4) + 4 (lane / 32) + e % 4, 32 j + lane % 32)
    // of the wave's part.  The scaled values take the place of the integer sums (the same registers); the tile's
    // token scales and output scales go through LDS (free after the barrier: every wave is out of the loop).
    const float wfix = W4 ? (1.0f / 16.0f) : 1.0f;
    __syncthreads();
    float* sxl = (float*)smem;
    float* swl = sxl + kDmaTM;
    sxl[tid] = (T0 + tid < g.rows) ? g.xs[T0 + tid] : 0.f;
    swl[tid] = (O0 + tid < g.m) ? g.ws[O0 + tid] * wfix : 0.f;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float sx[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) sx[e] = sxl[wm0 + 32 * i + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float cw = swl[wn0 + 32 * j + (lane & 31)];
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = __float_as_int((float)acc[i][j][e] * (sx[e] * cw));
        }
    }
    if (g.p_hi) {
#pragma nounroll
        for (int kk = 0; kk < g.r_pad; kk += 16) {
            const int kq = kk + 8 * (lane >> 5);
            bf16x8_t ph[4], pl[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t row = T0 + wm0 + 32 * i + (lane & 31);
                uint4 vh = make_uint4(0u, 0u, 0u, 0u), vl = make_uint4(0u, 0u, 0u, 0u);
                if (row < g.rows) {
                    vh = *(const uint4*)(g.p_hi + row * g.r_pad + kq);
                    if (SPLIT) vl = *(const uint4*)(g.p_lo + row * g.r_pad + kq);
                }
                ph[i] = __builtin_bit_cast(bf16x8_t, vh);
                pl[i] = __builtin_bit_cast(bf16x8_t, vl);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t col = O0 + wn0 + 32 * j + (lane & 31);
                uint4 vh = make_uint4(0u, 0u, 0u, 0u), vl = make_uint4(0u, 0u, 0u, 0u);
                if (col < g.m) {
                    vh = *(const uint4*)(g.la_hi + col * g.r_pad + kq);
                    if (SPLIT) vl = *(const uint4*)(g.la_lo + col * g.r_pad + kq);
                }
                const bf16x8_t lh = __builtin_bit_cast(bf16x8_t, vh), ll = __builtin_bit_cast(bf16x8_t, vl);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    f32x16_t y = __builtin_bit_cast(f32x16_t, acc[i][j]);
                    if (SPLIT) {
                        y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pl[i], lh, y, 0, 0, 0);
                        y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph[i], ll, y, 0, 0, 0);
                    }
                    y = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ph[i], lh, y, 0, 0, 0);
                    acc[i][j] = __builtin_bit_cast(v16i_t, y);
                }
            }
        }
    }
    // a tile that lies inside the output takes the store loop without the per-element tests
    const bool inner = T0 + kDmaTM <= g.rows && O0 + kDmaTN <= g.m;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t row0 = T0 + wm0 + 32 * i + 4 * (lane >> 5);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t col = O0 + wn0 + 32 * j + (lane & 31);
            float* yb = g.Y + row0 * g.ldy + col;
            if (inner) {
#pragma unroll
                for (int e = 0; e < 16; ++e) yb[(int64_t)(8 * (e >> 2) + (e & 3)) * g.ldy] = __int_as_float(acc[i][j][e]);
            } else if (col < g.m) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int dr = 8 * (e >> 2) + (e & 3);
                    if (row0 + dr < g.rows) yb[(int64_t)dr * g.ldy] = __int_as_float(acc[i][j][e]);
                }
            }
        }
    }
}

// P[t][k] = s_t sum_i xq[t][i] L_B[k][i] for 128 tokens per workgroup and all r_pad columns (RB blocks of
// 32).  L_B comes as bf16 planes [r_pad][n] (hi, lo).  Per step 64 channels: the code tile as in the main
// kernel (no reordering), the L_B tiles as 16-byte chunks of 8 bf16 with an XOR swizzle; codes become bf16
// exactly (|q| <= 128) on their way into the MFMA.  The launch is one workgroup per compute unit for 32768
// tokens, and a step is a chain of waits (tile stores, barrier, fragment reads, conversion, MFMA), so the
// workgroup has eight wavefronts, two per SIMD: wavefront w takes tokens 32 (w % 4) .. + 32 and the 16-channel
// slices 2 (w / 4), 2 (w / 4) + 1 of every step; the two halves of the sum meet in LDS at the end.  The loads
// of step s + 3 are issued in step s (three register stages, the step loop unrolled by three so that they are
// named at compile time), the LDS tiles are double buffered, one barrier per step.
constexpr int kDownThreads = 512;

template <int RB, bool SPLIT>
__global__ __launch_bounds__(kDownThreads) void cf_down_kernel(const int8_t* __restrict__ xq, const float* __restrict__ xs, int64_t rows,
                                                               int64_t n, const uint16_t* __restrict__ lb_hi,
                                                               const uint16_t* __restrict__ lb_lo, uint16_t* __restrict__ p_hi,
                                                               uint16_t* __restrict__ p_lo, int64_t ldp) {
    extern __shared__ __align__(16) char smem[];
    constexpr int RP = 32 * RB;                              // r_pad
    constexpr int A_BYTES = 128 * 64, B_BYTES = RP * 128;    // 64 bf16 per row
    constexpr int BUF = A_BYTES + 2 * B_BYTES;
    constexpr int BCHUNKS = RP * 8;                          // 16-byte chunks of a B plane per step
    constexpr int BCH = (BCHUNKS + kDownThreads - 1) / kDownThreads;
    constexpr int kAhead = 3;
    static_assert(2 * BUF >= 4 * RB * 16 * 64 * 4 + 128 * 4, "the partial sums of wavefronts 4 .. 7 and the token scales must fit the tile buffers");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tb = wave & 3, sh = wave >> 2;
    const int64_t T0 = (int64_t)blockIdx.x * 128;
    // staging role: 16-byte chunk tid % 4 of code row tid / 4
    const int srow = tid >> 2, sc = tid & 3;
    const bool srow_ok = T0 + srow < rows;
    const char* ap = (const char*)xq + (srow_ok ? T0 + srow : 0) * n + 16 * sc;
    const uint32_t amask = srow_ok ? 0xFFFFFFFFu : 0u;       // rows past the end read row 0 and drop it
    f32x16_t acc[RB];
#pragma unroll
    for (int j = 0; j < RB; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    uint4 ar[kAhead], bh[kAhead][BCH], bl[kAhead][BCH];
    // STEADY: all 64 channels of the step exist; the loads are unconditional (clamped addresses, the value
    // dropped afterwards), so that the loop body is straight-line code and the compiler's counting of the
    // loads in flight stays exact
    auto fetch = [&](auto utag, int64_t s, auto steady_tag) {
        constexpr int U = decltype(utag)::value;
        constexpr bool STEADY = decltype(steady_tag)::value;
        const int64_t k0 = s * 64;
        if (STEADY) {
            const uint4 v = *(const uint4*)(ap + k0);
            ar[U] = make_uint4(v.x & amask, v.y & amask, v.z & amask, v.w & amask);
        } else {
            ar[U] = make_uint4(0u, 0u, 0u, 0u);
            if (srow_ok && k0 + 16 * sc < n) ar[U] = *(const uint4*)(ap + k0);      // n % 32 == 0: a chunk of 16 is whole or absent
        }
#pragma unroll
        for (int u = 0; u < BCH; ++u) {
            const int q = tid + kDownThreads * u, c = q & 7;
            const int row = (q >> 3) < RP ? (q >> 3) : RP - 1;
            const int64_t k = k0 + 8 * c;
            if (STEADY) {
                bh[U][u] = *(const uint4*)(lb_hi + (int64_t)row * n + k);
                if (SPLIT) bl[U][u] = *(const uint4*)(lb_lo + (int64_t)row * n + k);
            } else {
                bh[U][u] = make_uint4(0u, 0u, 0u, 0u);
                bl[U][u] = make_uint4(0u, 0u, 0u, 0u);
                if (k < n) {
                    bh[U][u] = *(const uint4*)(lb_hi + (int64_t)row * n + k);
                    if (SPLIT) bl[U][u] = *(const uint4*)(lb_lo + (int64_t)row * n + k);
                }
            }
        }
    };
    const int64_t steps = (n + 63) / 64;
    const int64_t full_steps = n / 64;
    fetch(std::integral_constant<int, 0>{}, 0, std::false_type{});
    if (steps > 1) fetch(std::integral_constant<int, 1>{}, 1, std::false_type{});
    if (steps > 2) fetch(std::integral_constant<int, 2>{}, 2, std::false_type{});
    auto step = [&](auto utag, int64_t s, auto steady_tag) {
        constexpr int U = decltype(utag)::value;
        constexpr bool STEADY = decltype(steady_tag)::value;
        // buffer s % 2 was last read in step s - 2; every wavefront has left that step's reads behind it when
        // the first one passes the barrier of step s - 1
        char* sA = smem + (int)(s & 1) * BUF;
        char* sBh = sA + A_BYTES;
        char* sBl = sBh + B_BYTES;
        *(uint4*)(sA + chunk_off(srow, sc)) = ar[U];
#pragma unroll
        for (int u = 0; u < BCH; ++u) {
            const int q = tid + kDownThreads * u, row = q >> 3, c = q & 7;
            const int off = row * 128 + ((c ^ ((row >> 1) & 7)) << 4);
            if (q < BCHUNKS) {
                *(uint4*)(sBh + off) = bh[U][u];
                if (SPLIT) *(uint4*)(sBl + off) = bl[U][u];
            }
        }
        if (STEADY) fetch(utag, s + kAhead, std::true_type{});
        else if (s + kAhead < steps) fetch(utag, s + kAhead, std::false_type{});
        __syncthreads();
        const int arow = tb * 32 + (lane & 31);
#pragma unroll
        for (int ss = 0; ss < 2; ++ss) {                     // 16 channels per slice; this lane's 8: bytes [16 sl + 8 g, +8) of its row
            const int sl = 2 * sh + ss;
            const int g8 = lane >> 5;
            const uint2 raw = *(const uint2*)(sA + chunk_off(arow, sl) + 8 * g8);
            const uint32_t w2[2] = {raw.x ^ 0x80808080u, raw.y ^ 0x80808080u};      // q + 128 as unsigned bytes
            uint32_t pk[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t w = w2[q >> 1];
                const int b0 = 2 * (q & 1);
                const float f0 = (float)((w >> (8 * b0)) & 0xFFu) - 128.0f;
                const float f1 = (float)((w >> (8 * b0 + 8)) & 0xFFu) - 128.0f;
                pk[q] = bf16_hi_pair(f0, f1);
            }
            const bf16x8_t a = __builtin_bit_cast(bf16x8_t, make_uint4(pk[0], pk[1], pk[2], pk[3]));
            const int c = 2 * sl + g8;
#pragma unroll
            for (int j = 0; j < RB; ++j) {
                const int brow = 32 * j + (lane & 31);
                const int off = brow * 128 + ((c ^ ((brow >> 1) & 7)) << 4);
                const bf16x8_t bhv = *(const bf16x8_t*)(sBh + off);
                if (SPLIT) {
                    const bf16x8_t blv = *(const bf16x8_t*)(sBl + off);
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, blv, acc[j], 0, 0, 0);
                }
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bhv, acc[j], 0, 0, 0);
            }
        }
    };
    int64_t s = 0;
    // Twelve steps per trip first: the compiler lets all loads in flight land at a loop's head, and that wait
    // should come once in twelve steps, not once in three.  The steps fetched, up to s + 14, are whole.
    for (; s + 5 * kAhead <= full_steps; s += 4 * kAhead) {
#pragma unroll
        for (int rep = 0; rep < 4; ++rep) {
            step(std::integral_constant<int, 0>{}, s + 3 * rep, std::true_type{});
            step(std::integral_constant<int, 1>{}, s + 3 * rep + 1, std::true_type{});
            step(std::integral_constant<int, 2>{}, s + 3 * rep + 2, std::true_type{});
        }
    }
    for (; s + 2 * kAhead <= full_steps; s += kAhead) {     // the steps these three fetch, up to s + 5, are whole
        step(std::integral_constant<int, 0>{}, s, std::true_type{});
        step(std::integral_constant<int, 1>{}, s + 1, std::true_type{});
        step(std::integral_constant<int, 2>{}, s + 2, std::true_type{});
    }
    for (; s < steps; s += kAhead) {
        step(std::integral_constant<int, 0>{}, s, std::false_type{});
        if (s + 1 < steps) step(std::integral_constant<int, 1>{}, s + 1, std::false_type{});
        if (s + 2 < steps) step(std::integral_constant<int, 2>{}, s + 2, std::false_type{});
    }
    // the sums over slices 2, 3 (wavefronts 4 .. 7) join those over slices 0, 1 of the same tokens; the tile's
    // token scales go through LDS as well (one load per token instead of one per accumulator register)
    __syncthreads();
    float* part = (float*)smem;
    float* xsl = part + 4 * RB * 16 * 64;
    if (tid < 128) xsl[tid] = (T0 + tid < rows) ? xs[T0 + tid] : 0.f;
    if (sh == 1) {
#pragma unroll
        for (int j = 0; j < RB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) part[((tb * RB + j) * 16 + e) * 64 + lane] = acc[j][e];
    }
    __syncthreads();
    if (sh == 1) return;
#pragma unroll
    for (int j = 0; j < RB; ++j) {
        const int col = 32 * j + (lane & 31);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int64_t row = T0 + tb * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            if (row < rows) {
                const float pv = (acc[j][e] + part[((tb * RB + j) * 16 + e) * 64 + lane]) * xsl[row - T0];
                const uint32_t h = bf16_rne(pv);
                p_hi[row * ldp + col] = (uint16_t)h;
                if (SPLIT) p_lo[row * ldp + col] = (uint16_t)bf16_rne(pv - __uint_as_float(h << 16));
            }
        }
    }
}

struct FwdPlan {
    int r_pad;
    size_t off_p, off_lah, off_lal, off_lbh, off_lbl, total;
};

void fwd_plan(int64_t rows, int64_t n, int64_t m, int r, FwdPlan* p) {
    p->r_pad = (r + 31) / 32 * 32;
    size_t off = 0;
    p->off_p = off; off += align_up((size_t)rows * p->r_pad * 4, 256);
    p->off_lah = off; off += align_up((size_t)m * p->r_pad * 2, 256);
    p->off_lal = off; off += align_up((size_t)m * p->r_pad * 2, 256);
    p->off_lbh = off; off += align_up((size_t)p->r_pad * n * 2, 256);
    p->off_lbl = off; off += align_up((size_t)p->r_pad * n * 2, 256);
    p->total = r > 0 ? off : 0;
}

template <typename K>
int set_lds_once(aser_ctx* ctx, K kern, int bytes, bool* done) {
    if (ctx->device >= 0 && ctx->device < 16 && !done[ctx->device]) {
        ASER_HIP(ctx, hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
        done[ctx->device] = true;
    }
    return ASER_OK;
}

template <bool W4, bool SPLIT>
int launch_main(aser_ctx* ctx, const FwdArgs& g) {
    static bool done[16] = {false};
    constexpr int lds = 2 * (kFwdTM * 64 + kFwdTN * 64);
    auto kern = cf_main_kernel<W4, SPLIT>;
    ASER_TRY(set_lds_once(ctx, kern, lds, done));
    dim3 grid((unsigned)ceil_div64(g.m, kFwdTN), (unsigned)ceil_div64(g.rows, kFwdTM));
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, ctx->stream, g);
    return aser_check_launch(ctx, "compensated_forward");
}

template <bool W4, bool SPLIT>
int launch_dma(aser_ctx* ctx, const FwdArgs& g) {
    static bool done[16] = {false};
    constexpr int lds = kDmaStages * (kDmaTM * 64 + kDmaTN * (W4 ? 32 : 64));
    auto kern = cf_dma_kernel<W4, SPLIT>;
    ASER_TRY(set_lds_once(ctx, kern, lds, done));
    const int64_t tn = ceil_div64(g.m, kDmaTN), total = tn * ceil_div64(g.rows, kDmaTM);
    const int64_t per_xcd = ceil_div64(total, 8);
    hipLaunchKernelGGL(kern, dim3((unsigned)(8 * per_xcd)), dim3(256), lds, ctx->stream, g, (int)tn, total);
    return aser_check_launch(ctx, "compensated_forward");
}

template <int RB, bool SPLIT>
int launch_down(aser_ctx* ctx, const int8_t* xq, const float* xs, int64_t rows, int64_t n, const uint16_t* lbh,
                const uint16_t* lbl, uint16_t* p_hi, uint16_t* p_lo, int64_t ldp) {
    static bool done[16] = {false};
    constexpr int lds = 2 * (128 * 64 + 2 * (32 * RB * 128));   // two buffers of (codes, L_B hi, L_B lo)
    auto kern = cf_down_kernel<RB, SPLIT>;
    ASER_TRY(set_lds_once(ctx, kern, lds, done));
    hipLaunchKernelGGL(kern, dim3((unsigned)ceil_div64(rows, 128)), dim3(kDownThreads), lds, ctx->stream, xq, xs, rows, n, lbh, lbl, p_hi, p_lo, ldp);
    return aser_check_launch(ctx, "compensated_forward_down");
}

}  // namespace

extern "C" size_t aser_forward_workspace_bytes(int64_t rows, int64_t n, int64_t m, int32_t r) {
    if (rows <= 0 || n <= 0 || m <= 0 || r < 0) return 0;
    FwdPlan p;
    fwd_plan(rows, n, m, r, &p);
    return p.total + kAserWsTail;
}

extern "C" int aser_compensated_forward(aser_ctx* ctx, const int8_t* x_codes, const float* x_scales, int64_t rows, int64_t n,
                                        const void* w_codes, int32_t layout, const float* w_scales, int64_t m,
                                        const float* L_A, const float* L_B, int32_t r, int32_t lowrank_split,
                                        float* Y, int64_t ldy) {
    if (!ctx) return ASER_ERR_INVALID_ARG;
    if (!x_codes || !x_scales || !w_codes || !w_scales || !Y) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "compensated_forward: null pointer");
    if (rows < 0 || n <= 0 || m <= 0 || ldy < m) ASER_FAIL(ctx, ASER_ERR_SHAPE, "compensated_forward: bad shape");
    if (n % 32) ASER_FAIL(ctx, ASER_ERR_SHAPE, "compensated_forward: n must be a multiple of 32");
    if (layout != ASER_CODES_INT8 && layout != ASER_CODES_INT4_PACKED)
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "compensated_forward: unknown code layout");
    if (r < 0 || r > 128) ASER_FAIL(ctx, ASER_ERR_SHAPE, "compensated_forward: need 0 <= r <= 128");
    if (r > 0 && (!L_A || !L_B)) ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "compensated_forward: r > 0 needs L_A and L_B");
    if (((uintptr_t)x_codes & 15) || ((uintptr_t)w_codes & 15) || ((uintptr_t)x_scales & 3) || ((uintptr_t)w_scales & 3) ||
        ((uintptr_t)Y & 3))
        ASER_FAIL(ctx, ASER_ERR_INVALID_ARG, "compensated_forward: codes must be 16-byte aligned, scales and Y 4-byte aligned");
    FwdPlan pl;
    fwd_plan(rows > 0 ? rows : 1, n, m, r, &pl);
    if (r > 0 && (!ctx->ws || ctx->ws_bytes < pl.total + kAserWsTail))
        ASER_FAIL(ctx, ASER_ERR_WORKSPACE, "compensated_forward: workspace too small (%zu needed)", pl.total + kAserWsTail);
    if (rows == 0) return ASER_OK;
    ASER_TRY(aser_prepare_device(ctx));
    const bool split = lowrank_split != 0;
    FwdArgs g{};
    g.xq = x_codes; g.xs = x_scales; g.rows = rows; g.n = n;
    g.wq = w_codes; g.ws = w_scales; g.m = m;
    g.Y = Y; g.ldy = ldy;
    if (r > 0) {
        char* ws = (char*)ctx->ws;
        uint16_t* p_hi = (uint16_t*)(ws + pl.off_p);          // two bf16 planes in the room of one fp32 matrix
        uint16_t* p_lo = p_hi + (size_t)rows * pl.r_pad;
        uint16_t* lah = (uint16_t*)(ws + pl.off_lah);
        uint16_t* lal = (uint16_t*)(ws + pl.off_lal);
        uint16_t* lbh = (uint16_t*)(ws + pl.off_lbh);
        uint16_t* lbl = (uint16_t*)(ws + pl.off_lbl);
        const int rp = pl.r_pad;
        // the factors as bf16 planes: L_A (m x r) padded to r_pad columns, L_B (r x n) padded to r_pad rows
        {
            const int64_t total = (m + n) * rp, blocks = ceil_div64(total, 256);
            hipLaunchKernelGGL(split_factors_kernel, dim3((unsigned)(blocks < 2048 ? blocks : 2048)), dim3(256), 0, ctx->stream,
                               L_A, L_B, m, n, (int64_t)r, (int64_t)rp, lah, lal, lbh, lbl);
            ASER_TRY(aser_check_launch(ctx, "split_factors"));
        }
#define ASER_DOWN(RB)                                                                                   \
    (split ? launch_down<RB, true>(ctx, x_codes, x_scales, rows, n, lbh, lbl, p_hi, p_lo, rp)           \
           : launch_down<RB, false>(ctx, x_codes, x_scales, rows, n, lbh, lbl, p_hi, p_lo, rp))
        if (rp == 32) ASER_TRY(ASER_DOWN(1));
        else if (rp == 64) ASER_TRY(ASER_DOWN(2));
        else if (rp == 96) ASER_TRY(ASER_DOWN(3));
        else ASER_TRY(ASER_DOWN(4));
#undef ASER_DOWN
        g.p_hi = p_hi; g.p_lo = p_lo; g.la_hi = lah; g.la_lo = lal; g.r_pad = rp;
    }
    const bool w4 = layout == ASER_CODES_INT4_PACKED;
    if (rows >= kDmaTM && m >= kDmaTN) {                 // the 256 x 256 tiles without a register stage
        if (w4) return split ? launch_dma<true, true>(ctx, g) : launch_dma<true, false>(ctx, g);
        return split ? launch_dma<false, true>(ctx, g) : launch_dma<false, false>(ctx, g);
    }
    if (w4) return split ? launch_main<true, true>(ctx, g) : launch_main<true, false>(ctx, g);
    return split ? launch_main<false, true>(ctx, g) : launch_main<false, false>(ctx, g);
}
