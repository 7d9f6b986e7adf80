// Fused multi-head attention forward for gfx950: O = softmax(scale * Q K^T + causal mask) V per
// (batch entry, query head), grouped-query aware (a query head reads key/value head
// h / (Hq / Hkv); nothing is expanded in memory).  The paper's first block pattern (Section 5.2.4
// pattern p1; Section 5.2.5 pattern p1 for the grouped form) replaces this sub-graph with one
// kernel that tiles over keys and never writes the score matrix to HBM (Section 2.1); this is
// that kernel for 64-lane wavefronts and MFMA 16x16x32, written from the definition.
//
// Shape of the computation
//   A work-group owns BQ = NW * 64 consecutive queries of one (batch, query head): wave w owns
//   queries [q0 + 64 w, q0 + 64 w + 64) as 4 column tiles of 16.  Keys and values are walked in
//   blocks of 64, staged in LDS (double-buffered, global->LDS direct loads) and shared by the
//   waves.  Everything is computed TRANSPOSED so that a lane owns pieces of ONE query:
//     S^T (keys x queries) = K_block (A operand, rows = keys) x Q^T (B operand, columns = queries)
//     O^T (d    x queries) = V_block^T (A operand, rows = d)  x P^T (B operand, columns = queries)
//   MFMA 16x16x32 result layout: lane (r16 = lane % 16, q4 = lane / 16), register r holds
//   D[4 q4 + r][r16]: rows come from the A operand, the column is the lane's query.  Hence
//   * the running maximum of a query needs its 16 in-lane values per key block and one exchange
//     with the three other lanes that hold the same query (lane ^ 16, lane ^ 32);
//   * the softmax denominator is one more tile of the second contraction (V^T extended by a tile
//     of ones), which also adds up the four lanes;
//   * P^T in registers already IS the B operand of the second MFMA: a B operand lane holds 8
//     K-values (here: keys) of one column (query).  The 8 keys a lane holds after two S^T tiles are
//     {32u + 4 q4 + 0..3} and {32u + 16 + 4 q4 + 0..3}, not 8 consecutive ones, so the A operand
//     (V^T) is fetched with the same key permutation: the transposing LDS read takes one address
//     per 4-key group, so this costs nothing.
//   Q^T fragments (the B operand of the first MFMA: 8 consecutive d of one query) are 16-byte
//   pieces of Q rows: loaded once from global memory straight into registers.
//   Softmax runs in base 2: p = 2^(s * c - m * c) with c = scale * log2(e), fp32.  P is rounded to
//   bf16 (RNE) for the second MFMA; numerator and denominator sum the same rounded values.
//   One wave per SIMD (the accumulators take most of the 512 registers), so nothing hides a stall:
//   the key blocks are software-pipelined (scores of block j+1 under the softmax of block j, see
//   `step` below) and every instruction is placed by hand between the MFMAs.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace fact {
namespace attn {

#define FACT_ATTN_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x8_t __attribute__((ext_vector_type(8)));

struct AttnArgs {
    const __bf16 *Q, *K, *V;
    __bf16 *O;
    // element strides: batch entry, token, head (the head_dim elements of a row are contiguous)
    int64_t q_sb, k_sb, v_sb, o_sb, q_sh, k_sh, v_sh, o_sh;
    int q_st, k_st, v_st, o_st;
    int B, T, Hq, Hkv;
    int causal;
    float scale_log2;       // softmax scale * log2(e)
    int q_blocks;           // ceil(T / BQ)
    int total;              // q_blocks * Hq * B work-groups
    int group;              // (batch, query head) pairs per group of the work-group order; divides the pairs of an XCD
};

constexpr uint32_t kBufFlags = 0x00020000u;      // raw buffer descriptor word 3 (32-bit data format)

__device__ __forceinline__ const char *uniform_ptr(const char *ptr)
{
    const uint64_t v = (uint64_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char *)(((uint64_t)hi << 32) | lo);
}

// (Device-only builtins live in __device__ helpers: used directly in a __global__ template they
// make the host pass drop the kernel's launch stub without a diagnostic.)
__device__ __forceinline__ f32x4_t mfma_16x16x32(bf16x8_t a, bf16x8_t b, f32x4_t c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
// max over the four lanes lane, lane ^ 16, lane ^ 32, lane ^ 48, in every lane, without LDS:
// v_permlane16_swap exchanges the odd 16-lane rows of its first operand with the even rows of
// its second, v_permlane32_swap the upper half of the first with the lower half of the second;
// applied to two copies of x, the two results hold x and its partner's x in every lane.
__device__ __forceinline__ float max_with_lane_xor16(float x)
{
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (uint32_t)a[0]), __builtin_bit_cast(float, (uint32_t)a[1]));
}
__device__ __forceinline__ float max_with_lane_xor32(float x)
{
    const uint32_t w = __builtin_bit_cast(uint32_t, x);
    auto b = __builtin_amdgcn_permlane32_swap(w, w, false, false);
    return fmaxf(__builtin_bit_cast(float, (uint32_t)b[0]), __builtin_bit_cast(float, (uint32_t)b[1]));
}
__device__ __forceinline__ float max_over_lane_quads(float x) { return max_with_lane_xor32(max_with_lane_xor16(x)); }
// 16 bytes per lane from global memory straight into LDS at lds + 16 * lane (lds uniform over the wave)
__device__ __forceinline__ void load_to_lds_16(__amdgpu_buffer_rsrc_t rsrc, char *lds, uint32_t voffset, uint32_t soffset)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, FACT_ATTN_LDS_PTR(lds), 16, voffset, soffset, 0, 0);
}

template <int N, class F, int... I>
__device__ __forceinline__ void unroll_impl(F &&f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void unroll(F &&f) { unroll_impl<N>(static_cast<F &&>(f), std::make_integer_sequence<int, N>{}); }

// LDS layout of a key or value block: [64 rows][D] bf16, the 16-byte chunk c of row r stored at
// chunk position c ^ swz(r).
//  K (read as MFMA A operand: 16 consecutive rows x 4 consecutive chunks per instruction): the
//    XOR with the row number spreads the 16 rows, which all start at the same bank, over the banks.
//  V (read with the transposing 64-bit read: per 16 lanes, 4 rows x 32 bytes at the same column):
//    the XOR moves rows 4q..4q+3 (and the neighbouring group of 4) to different 32-byte windows.
template <int D> __device__ __forceinline__ int swz_keys(int row) { return row & (D / 8 - 1); }
template <int D> __device__ __forceinline__ int swz_vals(int row)
{
    if constexpr (D == 128) return ((row & 3) << 2) | (((row >> 2) & 1) << 1);
    else return (((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1);
}

template <int D, int NW>
__global__ void __launch_bounds__(NW * 64)
attn_fwd_kernel(const AttnArgs p)
{
    static_assert(D == 64 || D == 128, "head_dim");
    constexpr int QW = 64, QT = QW / 16, BQ = NW * QW;        // queries per wave, its column tiles, per work-group
    constexpr int BKV = 64, KT = BKV / 16, UB = BKV / 32;      // keys per block, its row tiles, 32-key groups
    constexpr int KB = D / 32, DT = D / 16;                    // 32-wide groups / 16-row tiles of head_dim
    constexpr int CPR = D / 8, ROWB = D * 2;                   // chunks and bytes per LDS row
    constexpr int TILE_BYTES = BKV * ROWB, STAGE_BYTES = 2 * TILE_BYTES;
    constexpr int RPL = 1024 / ROWB;                           // rows per wave-wide load
    constexpr int L = TILE_BYTES / 1024 / NW;                  // wave-wide loads per tile and wave
    static_assert(L >= 1 && L * NW * 1024 == TILE_BYTES, "tile split over the waves");

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = lane & 15, q4 = lane >> 4;

    // Work-group -> (batch, key/value head, query head, query block).  Consecutive work-group ids go
    // to different XCDs (each with its own L2): id % 8 picks the XCD, and every XCD gets its own
    // eighth of the (batch, head) pairs, the query heads that read the same K/V next to each other.
    // Within an XCD the pairs come in groups of p.group: a group's work-groups are ordered by query
    // block, the heaviest (last) first, all pairs of the group before the next lighter block.  So
    // runs of p.group consecutive work-groups carry the same amount of work, and the K/V of one
    // group (sized by the host to fit the L2) is what the XCD reads at any one time.
    // (The hardware hands consecutive work-groups of an XCD to its shader engines in turn and in
    // order; with a heavy .. light pattern whose period matched that turn, one engine got all the
    // heavy work-groups and the others idled between theirs - measured 30% of the time.)
    const int G = p.Hq / p.Hkv;
    const int pairs = p.total / p.q_blocks;                    // batch * query heads
    int qb, pair;
    {
        const int v = blockIdx.x;
        const bool split = (pairs & 7) == 0;                   // else: one sequence over all pairs
        const int pos = split ? v >> 3 : v, first = split ? (v & 7) * (pairs >> 3) : 0;
        const int per_group = p.group * p.q_blocks;
        const int gi = pos / per_group, within = pos - gi * per_group;
        qb = p.q_blocks - 1 - within / p.group;
        pair = first + gi * p.group + within % p.group;
    }
    const int kv = pair / G;
    const int b = kv / p.Hkv, hk = kv - b * p.Hkv;
    const int hq = hk * G + (pair - kv * G);
    const int q0 = qb * BQ, q0w = q0 + wave * QW;
    const int T = p.T;

    // key blocks this work-group walks, and how many of them this wave needs
    const int kend = p.causal ? (q0 + BQ < T ? q0 + BQ : T) : T;
    const int nb = (kend + BKV - 1) / BKV;
    int nbw = nb;
    if (p.causal) { const int e = q0w + QW < T ? q0w + QW : T; nbw = (e + BKV - 1) / BKV; }
    if (q0w >= T) nbw = 0;

    auto make_rsrc = [&](const __bf16 *base, int64_t st) {
        return __builtin_amdgcn_make_buffer_rsrc((void *)uniform_ptr((const char *)base), 0,
                                                 __builtin_amdgcn_readfirstlane((uint32_t)((((int64_t)T - 1) * st + D) * 2)), kBufFlags);
    };
    const __amdgpu_buffer_rsrc_t rsrc_q = make_rsrc(p.Q + (int64_t)b * p.q_sb + (int64_t)hq * p.q_sh, p.q_st);
    const __amdgpu_buffer_rsrc_t rsrc_k = make_rsrc(p.K + (int64_t)b * p.k_sb + (int64_t)hk * p.k_sh, p.k_st);
    const __amdgpu_buffer_rsrc_t rsrc_v = make_rsrc(p.V + (int64_t)b * p.v_sb + (int64_t)hk * p.v_sh, p.v_st);

    // ---- K / V block loads: wave w fills the 1 KB pieces w, w + NW, ... of each tile -------------
    // Lane l of a wave-wide load writes 16 bytes at piece + 16 l, i.e. row l / CPR of the piece,
    // chunk position l % CPR: it fetches the chunk that belongs there under the swizzle.  Rows at
    // or beyond T lie outside the descriptor's range and arrive as zeros.  A wave's pieces are
    // NW * RPL rows apart, a multiple of the swizzles' periods except for 128-wide K rows with two
    // waves (period 16, step 8): so one per-lane offset serves all of a wave's loads (two there),
    // the piece and the key block go into the scalar offset.
    // LDS: two K slots then two V slots; block j uses slot j % 2 of each.
    constexpr int KALT = (D == 128 && NW == 2) ? 2 : 1;
    uint32_t k_off[KALT], v_off;
    {
        const int row = wave * RPL + lane / CPR, pos = lane % CPR;
#pragma unroll
        for (int a = 0; a < KALT; ++a)
            k_off[a] = (uint32_t)(row * p.k_st * 2 + ((pos ^ swz_keys<D>(row + a * NW * RPL)) << 4));
        v_off = (uint32_t)(row * p.v_st * 2 + ((pos ^ swz_vals<D>(row)) << 4));
    }
    const uint32_t k_blk = (uint32_t)(BKV * p.k_st * 2), v_blk = (uint32_t)(BKV * p.v_st * 2);
    const uint32_t k_piece = (uint32_t)(NW * RPL * p.k_st * 2), v_piece = (uint32_t)(NW * RPL * p.v_st * 2);
    // (block j >= nb does not exist: its loads still run, with a scalar offset beyond every descriptor's
    // range, and bring zeros into a slot nobody reads - no branch around a load in the middle of the MFMAs)
    constexpr uint32_t kBeyond = 0x80000000u;
    // (per piece only one scalar addition for the offset and one for the LDS address: scalar
    // instructions take issue slots of this wave like any others)
    auto k_block_off = [&](int j) { return j < nb ? (uint32_t)j * k_blk : kBeyond; };
    auto v_block_off = [&](int j) { return j < nb ? (uint32_t)j * v_blk : kBeyond; };
    auto load_k_piece2 = [&](char *slot, uint32_t blk_off, int t) __attribute__((always_inline)) {
        load_to_lds_16(rsrc_k, slot + t * NW * 1024, k_off[t % KALT], blk_off + t * k_piece);
    };
    auto load_v_piece2 = [&](char *slot, uint32_t blk_off, int t) __attribute__((always_inline)) {
        load_to_lds_16(rsrc_v, slot + t * NW * 1024, v_off, blk_off + t * v_piece);
    };
    auto load_k_piece = [&](int j, int t) __attribute__((always_inline)) {
        load_k_piece2(smem + (j & 1) * TILE_BYTES + wave * 1024, k_block_off(j), t);
    };
    auto load_v_piece = [&](int j, int t) __attribute__((always_inline)) {
        load_v_piece2(smem + (2 + (j & 1)) * TILE_BYTES + wave * 1024, v_block_off(j), t);
    };
    auto load_k = [&](int j) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < L; ++t) load_k_piece(j, t);
    };
    auto load_v = [&](int j) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < L; ++t) load_v_piece(j, t);
    };
    load_k(0);
    load_v(0);
    if (nb > 1) load_k(1);

    // ---- Q^T fragments: query 16 qt + r16 of the wave, d = 32 kb + 8 q4 .. + 7 ----------------
    bf16x8_t qf[QT][KB];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const uint32_t off = (uint32_t)(((q0w + 16 * qt + r16) * p.q_st + 32 * kb + 8 * q4) * 2);
            qf[qt][kb] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc_q, off, 0, 0));
        }

    // ---- LDS fragment addresses (relative to the slot) -----------------------------------------
    // K tile kt, group kb: row 16 kt + r16, chunk (4 kb + q4) ^ swizzle(r16): kb sits in address bits
    // 6 and up, which the XOR leaves to it, so group kb is the group-0 address ^ (kb << 6).
    const uint32_t k_addr = (uint32_t)(r16 * ROWB + ((q4 ^ swz_keys<D>(r16)) << 4));
    // V^T tile dt, 32-key group u, half h: a transposing read hands lane i of a 16-lane group
    // column (= d) i of the 4 rows (= keys) whose addresses lanes 4 jj + cc supply for columns
    // 4 cc .. 4 cc + 3.  Keys 32 u + 16 h + 4 q4 + jj: the permutation P^T comes in.  Tile dt is the
    // tile-0 address ^ (dt << 5) (chunk 2 dt + cc / 2, swizzled by XOR; slots are 256-byte aligned).
    const int jj = (lane >> 2) & 3, cc = lane & 3;
    const uint32_t v_addr = (uint32_t)((4 * q4 + jj) * ROWB + (((cc >> 1) ^ swz_vals<D>(4 * q4 + jj)) << 4) + (cc & 1) * 8);
    const uint32_t lds0 = (uint32_t)(size_t)FACT_ATTN_LDS_PTR(smem);

    // ---- state ------------------------------------------------------------------------------------
    // The MFMAs are inline asm so that the register classes are fixed: O^T accumulators and the Q^T
    // fragments live in the accumulation registers for the whole kernel, S^T goes straight to
    // ordinary registers where the softmax works on it (through the builtin the compiler moved
    // ~900 registers per key block between the two files).  The compiler does not know these are
    // MFMAs, so the wait states between an MFMA and a vector-ALU read of its result are kept by
    // construction (see the s_nop's) instead.
    f32x4_t S[2][KT][QT];            // S^T of the block being consumed and of the one after it
    f32x4_t o[DT][QT];
    u32x4_t pf[UB][QT];              // P^T, bf16 pairs, in MFMA B-operand order
    bf16x8_t kf[4];                  // K fragments: ring, read two fragments ahead of their MFMAs
    s16x4_t vlo[3][UB], vhi[3][UB];   // V^T fragments: ring of three tiles, read two tiles ahead of their MFMAs
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            o[dt][qt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            asm volatile("" : "+a"(o[dt][qt]));
        }
    f32x4_t lsum[QT];                // row sums of P: one more tile of O^T, from a V^T tile of ones
    float m[QT], mx[QT], mc[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m[qt] = -__builtin_inff(); mx[qt] = 0.f; mc[qt] = 0.f;
        lsum[qt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        asm volatile("" : "+a"(lsum[qt]));
    }
    // a V^T fragment of ones: with it as the A operand, every row of the result tile is the sum of P
    // over the keys - the softmax denominator, from the same rounded probabilities the numerator
    // uses, on the matrix pipe instead of 64 vector additions per key block, and already summed
    // over the four lanes that share a query
    // (kept in registers for good: written right before its MFMA - which the compiler, not knowing
    // that the asm is an MFMA, did - the matrix pipe read the registers' previous contents)
    u32x4_t ones_frag = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    asm volatile("" : "+v"(ones_frag));
#pragma unroll
    for (int u = 0; u < UB; ++u)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) pf[u][qt] = u32x4_t{0u, 0u, 0u, 0u};
    const float c = p.scale_log2;

    constexpr int NS = KT * KB * QT;                 // MFMAs of one S^T block
    constexpr int EPM = KT * QT * 4 / NS;             // softmax elements worked off behind each of them
    constexpr int NF = KT * KB;                      // K fragments of a block
    constexpr int NE = KT * QT * 4;                  // softmax elements per lane and block

    // (lambdas that hold inline asm take plain integers, constant after inlining: asm operands
    // inside a generic lambda cannot name the enclosing function's variables)
    auto read_k = [&](int slot_off, int f) __attribute__((always_inline)) {
        const int kt = f / KB, kb = f % KB;
        kf[f & 3] = *(const bf16x8_t *)(smem + slot_off + (k_addr ^ (kb << 6)) + kt * 16 * ROWB);
    };
    // MFMA number i of S^T(block) into S[tb]: fragment f = i / QT (key tile kt, 32 d's kb), query tile i % QT
    auto s_mfma = [&](int tb, int slot_off, int i) __attribute__((always_inline)) {
        const int f = i / QT, qt = i % QT, kt = f / KB, kb = f % KB;
        if (qt == 0 && f + 2 < NF) read_k(slot_off, f + 2);
        // The softmax values worked on behind the previous MFMA (the other S buffer's registers in
        // their three stages, the packed pairs) ride along as dummy operands:
        // that is what keeps the compiler from moving the softmax out from between the MFMAs.
        const int e1 = (i + 1) * EPM < NE ? (i + 1) * EPM : NE - 1;      // an element stage 1 touched in slot i - 1
        const int e3 = i > 0 ? (i - 1) * EPM : 0;                        // an element stage 3 touched in slot i - 1
        const int q1 = e1 / (KT * 4), k1 = (e1 / 4) % KT, q3 = e3 / (KT * 4), k3 = (e3 / 4) % KT;
        // (inputs only: as outputs they would make the compiler put a wait state behind every MFMA,
        // which costs this wave an issue slot like any instruction)
        if (kb == 0)
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0"
                         : "=&v"(S[tb][kt][qt])
                         : "v"(kf[f & 3]), "a"(qf[qt][kb]), "v"(S[tb ^ 1][k1][q1]), "v"(S[tb ^ 1][k3][q3]), "v"(pf[k3 / 2][q3]));
        else
            asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0"
                         : "+v"(S[tb][kt][qt])
                         : "v"(kf[f & 3]), "a"(qf[qt][kb]), "v"(S[tb ^ 1][k1][q1]), "v"(S[tb ^ 1][k3][q3]), "v"(pf[k3 / 2][q3]));
    };
    // Softmax of S[sb], element e (query tile e / 16, key tile, register), in three stages that run
    // in consecutive MFMA slots for one element and side by side for three different elements: a
    // single wave per SIMD has nothing else to cover the latency of a dependent vector instruction
    // (measured: fma -> exp -> add back to back take 29 cycles, the same three independent 17).
    //   stage 1: t = s c - m c      stage 2: p = 2^t      stage 3: pack pairs to bf16
    auto sm1 = [&](auto sb_, auto e_) __attribute__((always_inline)) {
        constexpr int sb = decltype(sb_)::value, e = decltype(e_)::value;
        if constexpr (e < NE) {
            constexpr int qt = e / (KT * 4), kt = (e / 4) % KT, r = e % 4;
            S[sb][kt][qt][r] = __builtin_fmaf(S[sb][kt][qt][r], c, -mc[qt]);
        }
    };
    auto sm2 = [&](auto sb_, auto e_) __attribute__((always_inline)) {
        constexpr int sb = decltype(sb_)::value, e = decltype(e_)::value;
        if constexpr (e < NE) {
            constexpr int qt = e / (KT * 4), kt = (e / 4) % KT, r = e % 4;
            S[sb][kt][qt][r] = exp2_fast(S[sb][kt][qt][r]);
        }
    };
    auto sm3 = [&](auto sb_, auto e_) __attribute__((always_inline)) {
        constexpr int sb = decltype(sb_)::value, e = decltype(e_)::value;
        constexpr int qt = e / (KT * 4), kt = (e / 4) % KT, r = e % 4;
        if constexpr (r & 1) {
            const f32x2_t pr = {S[sb][kt][qt][r - 1], S[sb][kt][qt][r]};
            pf[kt / 2][qt][2 * (kt & 1) + r / 2] = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2_t));
        }
    };
    auto mask_block = [&](auto sb_, int j) __attribute__((always_inline)) {
        constexpr int sb = decltype(sb_)::value;
        const int j0 = j * BKV;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            const int last = p.causal ? q0w + 16 * qt + r16 : T - 1;         // last key this query sees
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (j0 + 16 * kt + 4 * q4 + r > last) S[sb][kt][qt][r] = -__builtin_inff();
            __builtin_amdgcn_sched_barrier(0);        // (16 compare masks at a time: all 64 at once spill scalar registers everywhere)
        }
    };
    auto needs_mask = [&](int j) { return p.causal ? (j * BKV + BKV - 1 > q0w) : (j * BKV + BKV > T); };
    // largest score of query tile qt in S[sb], over the four lanes that share a query
    auto max_of = [&](auto sb_, auto qt_) __attribute__((always_inline)) {
        constexpr int sb = decltype(sb_)::value, qt = decltype(qt_)::value;
        float t = S[sb][0][qt][0];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) t = fmaxf(t, S[sb][kt][qt][r]);
        mx[qt] = max_over_lane_quads(t);
    };
    // the same in pieces, to go between the MFMAs of the second contraction: piece p < KT folds in
    // key tile p, pieces KT and KT + 1 exchange with the lanes that share the query
    float mt = 0.f;
    auto max_piece = [&](auto sb_, auto qt_, auto p_) __attribute__((always_inline)) {
        constexpr int sb = decltype(sb_)::value, qt = decltype(qt_)::value, pc = decltype(p_)::value;
        if constexpr (pc < KT) {
            const f32x4_t x = S[sb][pc][qt];
            if constexpr (pc == 0) mt = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
            else mt = fmaxf(fmaxf(mt, x[0]), fmaxf(fmaxf(x[1], x[2]), x[3]));
        } else if constexpr (pc == KT) {
            mt = max_with_lane_xor16(mt);
        } else if constexpr (pc == KT + 1) {
            mt = max_with_lane_xor32(mt);
            mx[qt] = mt;
        }
    };
    // transposing reads of V^T tile dt into fragment set `set`: 32-key group u (both 16-key halves)
    auto read_v = [&](int set, uint32_t vbase, int dt, int u) __attribute__((always_inline)) {
        static_assert(UB == 2, "two 32-key groups");
        const uint32_t va = (vbase + v_addr) ^ (uint32_t)(dt << 5);
        if (u == 0) {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vlo[set][0]) : "v"(va), "n"(0));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vhi[set][0]) : "v"(va), "n"(16 * ROWB));
        } else {
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vlo[set][1]) : "v"(va), "n"(32 * ROWB));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(vhi[set][1]) : "v"(va), "n"(48 * ROWB));
        }
    };
    auto wait_v4 = [&](int set) __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(vlo[set][0]), "+v"(vhi[set][0]), "+v"(vlo[set][1]), "+v"(vhi[set][1]));
    };
    auto wait_v = [&](int set) __attribute__((always_inline)) {
        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(vlo[set][0]), "+v"(vhi[set][0]), "+v"(vlo[set][1]), "+v"(vhi[set][1]));
    };
    // MFMA number mi of O^T tile dt: 32-key group mi / QT, query tile mi % QT (the running maximum
    // of the piece worked off behind the previous MFMA rides along as a dummy operand, as above)
    auto pv_mfma = [&](int set, int dt, int mi) __attribute__((always_inline)) {
        const int u = mi / QT, qt = mi % QT;
        const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(vlo[set][u], vhi[set][u], 0, 1, 2, 3, 4, 5, 6, 7));
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(o[dt][qt]) : "v"(vf), "v"(pf[u][qt]), "v"(mt), "v"(mx[(dt + QT - 1) % QT]));
    };
    float gmax = __builtin_inff();
    auto sum_mfma = [&](int u, int qt) __attribute__((always_inline)) {
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(lsum[qt]) : "v"(ones_frag), "v"(pf[u][qt]), "v"(gmax));
    };
    auto nops = [&]() __attribute__((always_inline)) { asm volatile("s_nop 15\n\ts_nop 15" ::: "memory"); };

    // One key block: softmax of S[PAR] (block j) while S[PAR ^ 1] (block j + 1) is being computed,
    // then O^T += V_j^T P^T while the maxima of block j + 1 are found.
    auto step = [&](auto par_, int j) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_)::value;
        typedef std::integral_constant<int, PAR> cur_t;
        typedef std::integral_constant<int, PAR ^ 1> nxt_t;
        // Loads issued one step ago (K of block j+1, V of block j) have landed, for every wave; every
        // wave is done with K of block j and V of block j-1, whose slots the new loads overwrite.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        // The new loads: a wave with work issues them one by one between the MFMAs below (in a burst
        // right here, 4 waves x 2 L loads queue up at the compute unit's address unit and every wave
        // loses ~400 cycles of issue time).
        if (j >= nbw) {                                          // nothing (more) this wave's queries may see
            if (j + 2 < nb) load_k(j + 2);
            if (j + 1 < nb) load_v(j + 1);
            return;
        }

        // m[qt] is the REFERENCE exponent of the query's running sums, not always its running
        // maximum: it is raised (and the sums rescaled) only when a score exceeds it by more than
        // 2^kSlack in the base-2 domain, so the probabilities handed to the second MFMA stay below
        // 2^kSlack = 256 (harmless in bf16 and fp32) and the accumulators are left alone on most
        // key blocks.  The branch is uniform over the wave.
        constexpr float kSlack = 8.0f;
        // (gmax = largest (mx - m) c over the query tiles, found behind the previous step's last MFMAs;
        // +inf before the first block)
        if (__builtin_amdgcn_ballot_w64(gmax > kSlack) != 0) {
            nops();                                              // the previous block's MFMAs have written O
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                const float m_new = fmaxf(m[qt], mx[qt]);
                const float alpha = exp2_fast((m[qt] - m_new) * c);
                m[qt] = m_new;
                asm volatile("" : "+a"(lsum[qt]));
                lsum[qt] *= alpha;
                asm volatile("" : "+a"(lsum[qt]));
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    asm volatile("" : "+a"(o[dt][qt]));           // (keeps the copy out of the registers inside this branch)
                    o[dt][qt] *= alpha;
                    asm volatile("" : "+a"(o[dt][qt]));           // back in the accumulation registers before the paths join
                    __builtin_amdgcn_sched_barrier(0);            // one tile at a time: few registers in flight
                }
            }
        }
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) mc[qt] = m[qt] * c;

        // S^T of block j + 1, one softmax element of block j behind each MFMA.  On the wave's last
        // block this still runs, on whatever the other K slot holds: the result is never used, and
        // the softmax alone would take as long as the two together.
        {
            const int slot_off = ((j + 1) & 1) * TILE_BYTES;
            char *const k_dst = smem + (j & 1) * TILE_BYTES + wave * 1024, *const v_dst = smem + (2 + ((j + 1) & 1)) * TILE_BYTES + wave * 1024;
            const uint32_t k_src = k_block_off(j + 2), v_src = v_block_off(j + 1);
            read_k(slot_off, 0);
            read_k(slot_off, 1);
            unroll<EPM>([&](auto k_) __attribute__((always_inline)) {          // fill the softmax pipeline
                constexpr int k = decltype(k_)::value;
                sm1(cur_t{}, std::integral_constant<int, k>{});
                sm1(cur_t{}, std::integral_constant<int, EPM + k>{});
            });
            unroll<EPM>([&](auto k_) __attribute__((always_inline)) { sm2(cur_t{}, k_); });
            __builtin_amdgcn_sched_barrier(0);
            unroll<NS>([&](auto i_) __attribute__((always_inline)) {
                constexpr int i = decltype(i_)::value;
                s_mfma(PAR ^ 1, slot_off, i);
                constexpr int LOAD_EVERY = NS / (2 * L);
                if constexpr (i % LOAD_EVERY == LOAD_EVERY - 1) {
                    constexpr int t = i / LOAD_EVERY;
                    if constexpr (t < L) load_k_piece2(k_dst, k_src, t); else load_v_piece2(v_dst, v_src, t - L);
                }
                unroll<EPM>([&](auto k_) __attribute__((always_inline)) {
                    constexpr int k = decltype(k_)::value;
                    sm1(cur_t{}, std::integral_constant<int, (i + 2) * EPM + k>{});
                    __builtin_amdgcn_sched_barrier(0);      // fma first: an exponential right behind the asm gets a wait state
                    sm2(cur_t{}, std::integral_constant<int, (i + 1) * EPM + k>{});
                    sm3(cur_t{}, std::integral_constant<int, i * EPM + k>{});
                });
                __builtin_amdgcn_sched_barrier(0);
            });
            if (needs_mask(j + 1)) {
                nops();
                mask_block(nxt_t{}, j + 1);
            }
        }

        const uint32_t vbase = lds0 + (2 + (j & 1)) * TILE_BYTES;
        read_v(0, vbase, 0, 0);
        read_v(0, vbase, 0, 1);
        read_v(1, vbase, 1, 0);
        read_v(1, vbase, 1, 1);
        unroll<DT>([&](auto dt_) __attribute__((always_inline)) {
            constexpr int dt = decltype(dt_)::value;
            // tile dt has arrived when at most the 4 reads of tile dt + 1 are still in flight
            if constexpr (dt + 1 < DT) wait_v4(dt % 3); else wait_v(dt % 3);
            // 2 QT MFMAs; behind each: half of the reads of tile dt + 2, or a piece of the maximum of
            // query tile dt of block j + 1 (the S^T MFMAs of this step are >= 8 MFMAs back by then)
            unroll<UB * QT>([&](auto mi_) __attribute__((always_inline)) {
                constexpr int mi = decltype(mi_)::value;
                pv_mfma(dt % 3, dt, mi);
                if constexpr (mi < 2) {
                    if constexpr (dt + 2 < DT) read_v((dt + 2) % 3, vbase, dt + 2, mi);
                } else if constexpr (dt < QT && mi - 2 < KT + 2) {
                    max_piece(nxt_t{}, dt_, std::integral_constant<int, mi - 2>{});
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        // the row-sum tile; behind its first MFMAs: how far the new maxima exceed the reference
        unroll<UB * QT>([&](auto mi_) __attribute__((always_inline)) {
            constexpr int mi = decltype(mi_)::value;
            sum_mfma(mi / QT, mi % QT);
            if constexpr (mi < QT) {
                const float g = (mx[mi] - m[mi]) * c;
                gmax = mi == 0 ? g : fmaxf(gmax, g);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // first block: S^T(0), its mask and maxima, nothing to overlap with yet
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (nbw > 0) {
        read_k(0, 0);
        read_k(0, 1);
        unroll<NS>([&](auto i_) __attribute__((always_inline)) {
            s_mfma(0, 0, decltype(i_)::value);
            __builtin_amdgcn_sched_barrier(0);
        });
        nops();
        if (needs_mask(0)) mask_block(std::integral_constant<int, 0>{}, 0);
        unroll<QT>([&](auto qt_) __attribute__((always_inline)) { max_of(std::integral_constant<int, 0>{}, qt_); });
    }
    for (int j = 0; j < nb; j += 2) {
        step(std::integral_constant<int, 0>{}, j);
        if (j + 1 < nb) step(std::integral_constant<int, 1>{}, j + 1);
    }
    if (nbw == 0) return;
    nops();                                                      // the last MFMAs have written O
    // (new values for the compiler, so that it cannot read the registers before the wait states)
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        asm volatile("" : "+a"(lsum[qt]));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) asm volatile("" : "+a"(o[dt][qt]));
    }

    // ---- normalise and store: lane holds d = 16 dt + 4 q4 .. + 3 of query q0w + 16 qt + r16 ------
    __bf16 *obase = p.O + (int64_t)b * p.o_sb + (int64_t)hq * p.o_sh;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const float inv = 1.0f / lsum[qt][0];
        const int query = q0w + 16 * qt + r16;
        if (query < T) {
            __bf16 *row = obase + (int64_t)query * p.o_st + 4 * q4;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const f32x2_t a = {o[dt][qt][0] * inv, o[dt][qt][1] * inv}, bq = {o[dt][qt][2] * inv, o[dt][qt][3] * inv};
                u32x2_t w;
                w.x = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2_t));
                w.y = __builtin_bit_cast(uint32_t, __builtin_convertvector(bq, bf16x2_t));
                *(u32x2_t *)(row + 16 * dt) = w;
            }
        }
    }
}

}  // namespace attn
}  // namespace fact
