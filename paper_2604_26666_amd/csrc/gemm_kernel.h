// bf16 GEMM main kernel for gfx950 (CDNA4): MFMA 32x32x16 bf16 -> fp32, LDS
// double-buffered operand staging with an XOR swizzle, 128-bit global loads,
// register-resident fused epilogue.  This is the tile-level / kernel-level /
// grid-level hierarchy of the paper (Section 4.2 Action 2) re-designed for
// 64-wide wavefronts: one work-group of WGM x WGN waves owns a BM x BN macro
// tile; each wave owns a (BM/WGM) x (BN/WGN) sub-tile made of 32x32 MFMA tiles
// whose fp32 accumulators stay in registers for the whole K loop.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fact {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

enum : int { ACT_NONE = 0, ACT_GELU_TANH = 1, ACT_SILU_GATE = 2 };

// Everything a launch needs.  Pointers are device pointers; ld* and strides in elements.
struct GemmArgs {
    const __bf16 *A;
    const __bf16 *B;        // trans_b=0: [K][N]; trans_b=1: [N][K] (gate rows when gated)
    const __bf16 *B_up;     // gated epilogue only: up-projection weights [N/2][K]
    __bf16 *C;              // [M][Nout]
    float *P;               // split-K partials [splits][M][N] (ld = N), or nullptr
    const __bf16 *bias;     // [Nout] or nullptr
    const __bf16 *res;      // [M][ldr] or nullptr
    int64_t lda, ldb, ldc, ldr;
    int64_t stride_a, stride_b, stride_c, stride_r;   // per grid.z when batched
    int M, N, K;            // N = columns of the contraction (2 x Nout when gated)
    int act;
    int splits;             // > 1: grid.z indexes a K range, output goes to P
    int k_per_split;        // multiple of 64
    int tiles_m, tiles_n;
    int group_m;            // tile rows walked together (L2 reuse)
    int vec_store;          // 1: C / residual / bias allow 8-byte vector access
};

constexpr int BK = 64;            // K elements staged per step
constexpr int LDS_ROW = BK * 2;   // bytes per staged row (one 128-byte line)

// Swizzle: the 16-byte chunk kc of staged row `row` lives at chunk position
// kc ^ swz(row).  Eight consecutive rows, and eight rows 8 apart, map one chunk
// column onto eight distinct positions, so both the fragment reads (lanes walk
// rows) and the transposing writes (lanes walk rows 8 apart) spread over all banks.
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ uint32_t lds_off(int row, int kc)
{
    return (uint32_t)(row * LDS_ROW + ((kc ^ swz(row)) << 4));
}

__device__ __forceinline__ float sigmoid_fast(float t)
{
    // 1 / (1 + e^-t); e^-t overflows to +inf for very negative t, giving 0.
    return __builtin_amdgcn_rcpf(1.0f + __expf(-t));
}

// tanh-form GELU: 0.5 z (1 + tanh(u)) = z * sigmoid(2u), u = sqrt(2/pi) (z + 0.044715 z^3)
__device__ __forceinline__ float gelu_tanh(float z)
{
    const float c = 0.7978845608028654f;
    float u = c * (z + 0.044715f * z * z * z);
    return z * sigmoid_fast(2.0f * u);
}

__device__ __forceinline__ float silu(float z) { return z * sigmoid_fast(z); }

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h16) { return __uint_as_float(h16 << 16); }

// fp32 -> bf16 bit pattern, round to nearest even; NaN -> quiet NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

__device__ __forceinline__ u32x2_t pack4_bf16(float a, float b, float c, float d)
{
    u32x2_t r;
    r.x = f32_to_bf16_bits(a) | (f32_to_bf16_bits(b) << 16);
    r.y = f32_to_bf16_bits(c) | (f32_to_bf16_bits(d) << 16);
    return r;
}

// Work-group id -> tile coordinates.  Consecutive work-group ids go to different
// XCDs (8 of them, each with its own L2), so id % 8 picks the XCD and every XCD
// gets one contiguous range of the tile order; inside that order tiles are walked
// group_m tile-rows at a time, column by column, so that the tiles resident on one
// XCD share A row-panels and B column-panels.
__device__ __forceinline__ void tile_coords(const GemmArgs &p, int pid, int &tm, int &tn)
{
    const int total = p.tiles_m * p.tiles_n;
    const int q = total >> 3, rem = total & 7;
    const int xcd = pid & 7, loc = pid >> 3;
    const int idx = xcd * q + (xcd < rem ? xcd : rem) + loc;
    const int per_group = p.group_m * p.tiles_n;
    const int grp = idx / per_group;
    const int first_m = grp * p.group_m;
    const int gsz = (p.tiles_m - first_m) < p.group_m ? (p.tiles_m - first_m) : p.group_m;
    const int in_grp = idx - grp * per_group;
    tm = first_m + in_grp % gsz;
    tn = in_grp / gsz;
}

template <int BM, int BN, int WGM, int WGN, bool TRANS_B>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_kernel(const GemmArgs p)
{
    constexpr int NTHR = WGM * WGN * 64;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int MT = WTM / 32, NT = WTN / 32;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 MFMA tiles");
    static_assert((BM * 8) % NTHR == 0, "A chunks must divide evenly over the threads");
    constexpr int A_CH = BM * 8 / NTHR;                       // 16-byte chunks per thread per step
    constexpr int B_CH = (BN * 8 + NTHR - 1) / NTHR;          // trans_b=1: chunks; may be partial
    constexpr int B_BLK = (BN + NTHR - 1) / NTHR;             // trans_b=0: 8x8 blocks per thread
    constexpr int STAGE = (BM + BN) * LDS_ROW;

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const int lr = lane & 31, g = lane >> 5;

    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    const int z = blockIdx.z;
    const bool gated = (p.act == ACT_SILU_GATE);
    const int nout = gated ? (p.N >> 1) : p.N;
    const int m0 = tm * BM;
    const int n0 = tn * (gated ? BN / 2 : BN);       // first OUTPUT column of this tile

    int k_begin = 0, k_end = p.K;
    int64_t batch_a = 0, batch_b = 0, batch_c = 0, batch_r = 0;
    if (p.splits > 1) {
        k_begin = z * p.k_per_split;
        k_end = k_begin + p.k_per_split < p.K ? k_begin + p.k_per_split : p.K;
    } else {
        batch_a = z * p.stride_a; batch_b = z * p.stride_b;
        batch_c = z * p.stride_c; batch_r = z * p.stride_r;
    }
    const int ksteps = (k_end - k_begin + BK - 1) / BK;

    // ---- global -> register -> LDS staging ------------------------------------------
    // A (and B when trans_b=1): thread owns chunks c = tid + i*NTHR; row = c/8, kc = c%8.
    const char *a_ptr[A_CH];
    uint32_t a_lds[A_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        const int c = tid + i * NTHR, row = c >> 3, kc = c & 7;
        int gr = m0 + row; gr = gr < p.M ? gr : p.M - 1;
        a_ptr[i] = (const char *)(p.A + batch_a + (int64_t)gr * p.lda + k_begin + kc * 8);
        a_lds[i] = lds_off(row, kc);
    }

    // staged B row r  <->  output column: plain: n0 + r.  gated: rows [0, BN/2) are gate
    // columns n0 + r, rows [BN/2, BN) the up columns n0 + r - BN/2 (read from B_up).
    const char *b_ptr[TRANS_B ? B_CH : B_BLK];
    uint32_t b_lds[TRANS_B ? B_CH : B_BLK];
    bool b_act[TRANS_B ? B_CH : B_BLK];
    if constexpr (TRANS_B) {
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            const int c = tid + i * NTHR, row = c >> 3, kc = c & 7;
            b_act[i] = (BN * 8) % NTHR == 0 ? true : (c < BN * 8);
            const __bf16 *base = p.B;
            int col = n0 + row;
            if (gated) {
                const bool up = row >= BN / 2;
                col = n0 + (up ? row - BN / 2 : row);
                base = up ? p.B_up : p.B;
            }
            col = col < nout ? col : nout - 1;
            b_ptr[i] = (const char *)(base + batch_b + (int64_t)col * p.ldb + k_begin + kc * 8);
            b_lds[i] = BM * LDS_ROW + lds_off(row < BN ? row : BN - 1, kc);
        }
    } else {
        // trans_b=0: thread owns 8(k) x 8(n) blocks c = tid + i*NTHR; nb = c % (BN/8), kb = c / (BN/8).
#pragma unroll
        for (int i = 0; i < B_BLK; ++i) {
            const int c = tid + i * NTHR;
            b_act[i] = BN % NTHR == 0 ? true : (c < BN);
            const int cc = c < BN ? c : BN - 1;
            const int nb = cc % (BN / 8), kb = cc / (BN / 8);
            int col = n0 + nb * 8; col = col < p.N ? col : p.N - 8;     // N % 8 == 0 on this path
            b_ptr[i] = (const char *)(p.B + batch_b + (int64_t)(k_begin + kb * 8) * p.ldb + col);
            b_lds[i] = (uint32_t)((kb << 8) | nb);                      // decoded at the store
        }
    }

    u32x4_t a_reg[A_CH];
    u32x4_t b_reg[TRANS_B ? B_CH : B_BLK * 8];

    auto load_global = [&](int kt) {
        const int k0 = k_begin + kt * BK;
        const bool full = k0 + BK <= k_end;
        if (full) {
#pragma unroll
            for (int i = 0; i < A_CH; ++i) a_reg[i] = *(const u32x4_t *)(a_ptr[i] + (int64_t)kt * (BK * 2));
            if constexpr (TRANS_B) {
#pragma unroll
                for (int i = 0; i < B_CH; ++i)
                    if (b_act[i]) b_reg[i] = *(const u32x4_t *)(b_ptr[i] + (int64_t)kt * (BK * 2));
            } else {
#pragma unroll
                for (int i = 0; i < B_BLK; ++i)
                    if (b_act[i]) {
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            b_reg[i * 8 + j] = *(const u32x4_t *)(b_ptr[i] + ((int64_t)kt * BK + j) * p.ldb * 2);
                    }
            }
        } else {
            // last, partial K step: chunks (rows of B) at or beyond k_end read as zero
            const u32x4_t zero = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < A_CH; ++i) {
                const int kc = (tid + i * NTHR) & 7;
                a_reg[i] = (k0 + kc * 8 < k_end) ? *(const u32x4_t *)(a_ptr[i] + (int64_t)kt * (BK * 2)) : zero;
            }
            if constexpr (TRANS_B) {
#pragma unroll
                for (int i = 0; i < B_CH; ++i) {
                    const int kc = (tid + i * NTHR) & 7;
                    if (b_act[i])
                        b_reg[i] = (k0 + kc * 8 < k_end) ? *(const u32x4_t *)(b_ptr[i] + (int64_t)kt * (BK * 2)) : zero;
                }
            } else {
#pragma unroll
                for (int i = 0; i < B_BLK; ++i)
                    if (b_act[i]) {
                        const int kb = (int)(b_lds[i] >> 8);
#pragma unroll
                        for (int j = 0; j < 8; ++j)
                            b_reg[i * 8 + j] = (k0 + kb * 8 + j < k_end)
                                ? *(const u32x4_t *)(b_ptr[i] + ((int64_t)kt * BK + j) * p.ldb * 2) : zero;
                    }
            }
        }
    };

    auto store_lds = [&](int stage) {
        char *s = smem + stage * STAGE;
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *(u32x4_t *)(s + a_lds[i]) = a_reg[i];
        if constexpr (TRANS_B) {
#pragma unroll
            for (int i = 0; i < B_CH; ++i)
                if (b_act[i]) *(u32x4_t *)(s + b_lds[i]) = b_reg[i];
        } else {
            // 8x8 transpose in registers: in[j] holds 8 n-values of k-row j; out[nn] holds
            // 8 k-values of column nn, i.e. the K-contiguous chunk the MFMA operand wants.
#pragma unroll
            for (int i = 0; i < B_BLK; ++i)
                if (b_act[i]) {
                    const int kb = (int)(b_lds[i] >> 8), nb = (int)(b_lds[i] & 0xFF);
#pragma unroll
                    for (int nn = 0; nn < 8; ++nn) {
                        u32x4_t o;
#pragma unroll
                        for (int d = 0; d < 4; ++d) {
                            const uint32_t lo = b_reg[i * 8 + 2 * d][nn >> 1];
                            const uint32_t hi = b_reg[i * 8 + 2 * d + 1][nn >> 1];
                            o[d] = (nn & 1) ? ((lo >> 16) | (hi & 0xFFFF0000u))
                                            : ((lo & 0xFFFFu) | (hi << 16));
                        }
                        *(u32x4_t *)(s + BM * LDS_ROW + lds_off(nb * 8 + nn, kb)) = o;
                    }
                }
        }
    };

    // ---- fragment addresses ------------------------------------------------------------
    // MFMA 32x32x16 operand: lane holds row (lane % 32) and the 8 K-values of K-group
    // (lane / 32), i.e. the 16-byte chunk kc = 2*kk + g of sub-step kk.  Because the
    // swizzle is an XOR, chunk (2*kk + g) ^ s sits at byte offset base ^ (kk << 5).
    uint32_t a_frag[MT], b_frag[NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) a_frag[mt] = lds_off(wm * WTM + mt * 32 + lr, g);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        int row = wn * WTN + nt * 32 + lr;
        if (gated) {
            // first NT/2 tiles: gate columns; last NT/2: the matching up columns
            const int h = nt < NT / 2 ? 0 : 1;
            row = h * (BN / 2) + wn * (WTN / 2) + (nt - h * (NT / 2)) * 32 + lr;
        }
        b_frag[nt] = BM * LDS_ROW + lds_off(row, g);
    }

    f32x16_t acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

    // ---- main loop: two LDS stages, next step's global loads in flight during the MFMAs ----
    if (ksteps > 0) {
        load_global(0);
        store_lds(0);
    }
    __syncthreads();
    for (int kt = 0; kt < ksteps; ++kt) {
        const bool more = kt + 1 < ksteps;
        if (more) load_global(kt + 1);
        const char *s = smem + (kt & 1) * STAGE;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8_t af[MT], bf[NT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) af[mt] = *(const bf16x8_t *)(s + (a_frag[mt] ^ (kk << 5)));
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) bf[nt] = *(const bf16x8_t *)(s + (b_frag[nt] ^ (kk << 5)));
            // Operand order (B-fragment first) makes the accumulator tile hold
            // D[n_local][m_local]: each lane then owns 4 consecutive output columns.
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[nt], af[mt], acc[mt][nt], 0, 0, 0);
        }
        if (more) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue ---------------------------------------------------------------------------
    // Accumulator register r of a tile, lane (lr, g): output row m = lr, output column
    // n = 8*(r/4) + 4*g + (r%4) inside the 32x32 tile.
    if (p.splits > 1) {
        float *P = p.P + (int64_t)z * p.M * p.N;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const int m = m0 + wm * WTM + mt * 32 + lr;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                int ncol = n0 + wn * WTN + nt * 32;           // contraction column of tile element 0
                if (gated) {
                    const int h = nt < NT / 2 ? 0 : 1;
                    ncol = h * nout + n0 + wn * (WTN / 2) + (nt - h * (NT / 2)) * 32;
                }
                const int nlim = gated ? ((nt < NT / 2 ? 0 : 1) * nout + nout) : p.N;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int n = ncol + q * 8 + g * 4;
                    if (m < p.M) {
                        float *dst = P + (int64_t)m * p.N + n;
                        if (n + 3 < nlim && (p.N & 3) == 0) {
                            f32x4_t v = {acc[mt][nt][q * 4], acc[mt][nt][q * 4 + 1],
                                         acc[mt][nt][q * 4 + 2], acc[mt][nt][q * 4 + 3]};
                            *(f32x4_t *)dst = v;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (n + e < nlim) dst[e] = acc[mt][nt][q * 4 + e];
                        }
                    }
                }
            }
        }
        return;
    }

    constexpr int NTO = NT;       // output tiles per wave along N when not gated
    const int nt_out = gated ? NT / 2 : NTO;
    __bf16 *C = p.C + batch_c;
    const __bf16 *R = p.res ? p.res + batch_r : nullptr;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = m0 + wm * WTM + mt * 32 + lr;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (nt >= nt_out) break;
            const int ncol = n0 + (gated ? wn * (WTN / 2) : wn * WTN) + nt * 32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = ncol + q * 8 + g * 4;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[mt][nt][q * 4 + e];
                if (gated) {
                    if constexpr (NT >= 2) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] = silu(v[e]) * acc[mt][(nt + NT / 2) % NT][q * 4 + e];
                    }
                }
                if (m >= p.M || n >= nout) continue;
                const bool vec = p.vec_store && (n + 3 < nout);
                if (p.bias) {
                    if (vec) {
                        const u32x2_t b = *(const u32x2_t *)(p.bias + n);
                        v[0] += bf16_bits_to_f32(b.x & 0xFFFFu); v[1] += bf16_bits_to_f32(b.x >> 16);
                        v[2] += bf16_bits_to_f32(b.y & 0xFFFFu); v[3] += bf16_bits_to_f32(b.y >> 16);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < nout) v[e] += (float)p.bias[n + e];
                    }
                }
                if (p.act == ACT_GELU_TANH) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = gelu_tanh(v[e]);
                }
                if (R) {
                    const __bf16 *rp = R + (int64_t)m * p.ldr + n;
                    if (vec) {
                        const u32x2_t b = *(const u32x2_t *)rp;
                        v[0] += bf16_bits_to_f32(b.x & 0xFFFFu); v[1] += bf16_bits_to_f32(b.x >> 16);
                        v[2] += bf16_bits_to_f32(b.y & 0xFFFFu); v[3] += bf16_bits_to_f32(b.y >> 16);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n + e < nout) v[e] += (float)rp[e];
                    }
                }
                __bf16 *cp = C + (int64_t)m * p.ldc + n;
                if (vec) {
                    *(u32x2_t *)cp = pack4_bf16(v[0], v[1], v[2], v[3]);
                } else {
                    uint16_t *cs = (uint16_t *)cp;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < nout) cs[e] = (uint16_t)f32_to_bf16_bits(v[e]);
                }
            }
        }
    }
}

}  // namespace fact
