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
//   * the running sum stays per lane (the four lanes share the maximum, so their partial sums
//     have the same scale) and is added up once at the end;
//   * P^T in registers already IS the B operand of the second MFMA: a B operand lane holds 8
//     K-values (here: keys) of one column (query).  The 8 keys a lane holds after two S^T tiles are
//     {32u + 4 q4 + 0..3} and {32u + 16 + 4 q4 + 0..3}, not 8 consecutive ones, so the A operand
//     (V^T) is fetched with the same key permutation: the transposing LDS read takes one address
//     per 4-key group, so this costs nothing.
//   Q^T fragments (the B operand of the first MFMA: 8 consecutive d of one query) are 16-byte
//   pieces of Q rows: loaded once from global memory straight into registers.
//   Softmax runs in base 2: p = 2^(s * c - m * c) with c = scale * log2(e), fp32.  P is rounded to
//   bf16 (RNE) for the second MFMA; the row sum adds the unrounded values.
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
    int64_t q_sb, q_st, q_sh, k_sb, k_st, k_sh, v_sb, v_st, v_sh, o_sb, o_st, o_sh;
    int B, T, Hq, Hkv;
    int causal;
    float scale_log2;       // softmax scale * log2(e)
    int q_blocks;           // ceil(T / BQ)
    int total;              // q_blocks * Hq * B work-groups
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

    // Work-group -> (batch, key/value head, query block, query head).  Consecutive work-group ids
    // go to different XCDs (each with its own L2): id % 8 picks the XCD and every XCD gets one
    // contiguous range of the order below, in which the query heads and query blocks that read
    // the same K/V follow each other, heaviest (last) query block first.
    int v = blockIdx.x;
    if ((p.total & 7) == 0) v = (v & 7) * (p.total >> 3) + (v >> 3);
    const int G = p.Hq / p.Hkv;
    const int per_kv = p.q_blocks * G;
    const int kv = v / per_kv, rest = v - kv * per_kv;
    const int b = kv / p.Hkv, hk = kv - b * p.Hkv;
    const int qb = p.q_blocks - 1 - rest / G;
    const int hq = hk * G + rest % G;
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

    // ---- K / V block loads: wave w fills 1 KB pieces w*L .. w*L+L-1 of each tile -------------
    // Lane l of a wave-wide load writes 16 bytes at piece + 16 l, i.e. row l / CPR of the piece,
    // chunk position l % CPR: it fetches the chunk that belongs there under the swizzle.  Rows at
    // or beyond T lie outside the descriptor's range and arrive as zeros.
    uint32_t k_off[L], v_off[L];
#pragma unroll
    for (int t = 0; t < L; ++t) {
        const int row = (wave * L + t) * RPL + lane / CPR, pos = lane % CPR;
        k_off[t] = (uint32_t)(row * (int)p.k_st * 2 + ((pos ^ swz_keys<D>(row)) << 4));
        v_off[t] = (uint32_t)(row * (int)p.v_st * 2 + ((pos ^ swz_vals<D>(row)) << 4));
    }
    const uint32_t k_blk = (uint32_t)(BKV * (int)p.k_st * 2), v_blk = (uint32_t)(BKV * (int)p.v_st * 2);
    auto issue_loads = [&](int j, int stage) __attribute__((always_inline)) {
        char *sk = smem + stage * STAGE_BYTES + wave * L * 1024;
#pragma unroll
        for (int t = 0; t < L; ++t)
            load_to_lds_16(rsrc_k, sk + t * 1024, k_off[t], j * k_blk);
#pragma unroll
        for (int t = 0; t < L; ++t)
            load_to_lds_16(rsrc_v, sk + TILE_BYTES + t * 1024, v_off[t], j * v_blk);
    };
    issue_loads(0, 0);

    // ---- Q^T fragments: query 16 qt + r16 of the wave, d = 32 kb + 8 q4 .. + 7 ----------------
    bf16x8_t qf[QT][KB];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const uint32_t off = (uint32_t)(((q0w + 16 * qt + r16) * (int)p.q_st + 32 * kb + 8 * q4) * 2);
            qf[qt][kb] = __builtin_bit_cast(bf16x8_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc_q, off, 0, 0));
        }

    // ---- LDS fragment addresses ---------------------------------------------------------------
    // K tile kt, group kb: row 16 kt + r16, chunk 4 kb + q4 (the swizzle depends on r16 only).
    uint32_t k_addr[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
        k_addr[kb] = (uint32_t)(r16 * ROWB + (((4 * kb + q4) ^ swz_keys<D>(r16)) << 4));
    // V^T tile dt, 32-key group u, half h: a transposing read hands lane i of a 16-lane group
    // column (= d) i of the 4 rows (= keys) whose addresses lanes 4 jj + cc supply for columns
    // 4 cc .. 4 cc + 3.  Keys 32 u + 16 h + 4 q4 + jj: the permutation P^T comes in.
    const int jj = (lane >> 2) & 3, cc = lane & 3;
    uint32_t v_addr[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
        v_addr[dt] = (uint32_t)(TILE_BYTES + (4 * q4 + jj) * ROWB + (((2 * dt + (cc >> 1)) ^ swz_vals<D>(4 * q4 + jj)) << 4) + (cc & 1) * 8);

    f32x4_t o[DT][QT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) o[dt][qt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    float m[QT], l[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) { m[qt] = -__builtin_inff(); l[qt] = 0.f; }
    const float c = p.scale_log2;

    for (int j = 0; j < nb; ++j) {
        // the loads of block j (issued one iteration ago) have landed, for every wave; every wave
        // is done reading the other stage, which block j+1 now overwrites
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (j + 1 < nb) issue_loads(j + 1, (j + 1) & 1);
        if (j >= nbw) continue;                                  // nothing this wave's queries may see
        const char *st = smem + (j & 1) * STAGE_BYTES;
        const int j0 = j * BKV;

        // ---- S^T = K Q^T ----------------------------------------------------------------------
        f32x4_t s[KT][QT];
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) s[kt][qt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const bf16x8_t kf = *(const bf16x8_t *)(st + k_addr[kb] + kt * 16 * ROWB);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    s[kt][qt] = mfma_16x16x32(kf, qf[qt][kb], s[kt][qt]);
            }

        // ---- mask: lane holds keys j0 + 16 kt + 4 q4 + r of query q0w + 16 qt + r16 -------------
        const bool need_mask = p.causal ? (j0 + BKV - 1 > q0w) : (j0 + BKV > T);
        if (need_mask) {
#pragma unroll
            for (int qt = 0; qt < QT; ++qt) {
                const int last = p.causal ? q0w + 16 * qt + r16 : T - 1;     // last key this query sees
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (j0 + 16 * kt + 4 * q4 + r > last) s[kt][qt][r] = -__builtin_inff();
            }
        }

        // ---- online softmax, per query --------------------------------------------------------
        bf16x8_t pf[UB][QT];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            float mx = s[0][qt][0];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) mx = fmaxf(mx, s[kt][qt][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m[qt], mx);
            const float alpha = exp2_fast((m[qt] - m_new) * c);
            const float mc = m_new * c;
            m[qt] = m_new;
            float sum = 0.f;
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float e = exp2_fast(__builtin_fmaf(s[kt][qt][r], c, -mc));
                    s[kt][qt][r] = e;
                    sum += e;
                }
            l[qt] = l[qt] * alpha + sum;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt][qt] *= alpha;
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                u32x4_t w;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const f32x2_t a = {s[2 * u + h][qt][0], s[2 * u + h][qt][1]}, bq = {s[2 * u + h][qt][2], s[2 * u + h][qt][3]};
                    w[2 * h] = __builtin_bit_cast(uint32_t, __builtin_convertvector(a, bf16x2_t));
                    w[2 * h + 1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(bq, bf16x2_t));
                }
                pf[u][qt] = __builtin_bit_cast(bf16x8_t, w);
            }
        }

        // ---- O^T += V^T P^T ---------------------------------------------------------------------
        // Transposing reads through inline asm: the compiler would make each of them wait for the
        // global->LDS loads in flight.  It does not track them, so the wait is explicit and takes
        // the fragment registers as operands.
        const uint32_t vb = (uint32_t)(size_t)FACT_ATTN_LDS_PTR(st);
        unroll<DT>([&](auto dt_) __attribute__((always_inline)) {
            constexpr int dt = decltype(dt_)::value;
            static_assert(UB == 2, "reads and operand list below");
            const uint32_t va = vb + v_addr[dt];
            s16x4_t lo0, hi0, lo1, hi1;
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo0) : "v"(va), "n"(0));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi0) : "v"(va), "n"(16 * ROWB));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo1) : "v"(va), "n"(32 * ROWB));
            asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi1) : "v"(va), "n"(48 * ROWB));
            asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(lo0), "+v"(hi0), "+v"(lo1), "+v"(hi1));
            const s16x4_t lo[UB] = {lo0, lo1}, hi[UB] = {hi0, hi1};
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo[u], hi[u], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    o[dt][qt] = mfma_16x16x32(vf, pf[u][qt], o[dt][qt]);
            }
        });
    }

    // ---- normalise and store: lane holds d = 16 dt + 4 q4 .. + 3 of query q0w + 16 qt + r16 ------
    if (nbw == 0) return;
    __bf16 *obase = p.O + (int64_t)b * p.o_sb + (int64_t)hq * p.o_sh;
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        float lt = l[qt];
        lt += __shfl_xor(lt, 16);
        lt += __shfl_xor(lt, 32);
        const float inv = 1.0f / lt;
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
