// bf16 GEMM main kernel for gfx950 (CDNA4).
//
// The paper's three-level hierarchy (Section 4.2 Action 2: tile-level primitive,
// kernel-level pipelining, grid-level schedule) re-designed for 64-wide wavefronts:
//   tile level   : MFMA 16x16x32 bf16 -> fp32 (measured: with random operands this shape
//                  sustains about 16 % more FLOP/s under the chip's power limit than 32x32x16).
//                  A work-group of WGM x WGN waves owns a BM x BN macro tile; each wave owns a
//                  (BM/WGM) x (BN/WGN) sub-tile of 16x16 MFMA tiles whose accumulators stay in
//                  registers for the whole K loop.
//   kernel level : a ring of STAGES LDS buffers filled by 128-bit global->LDS direct loads
//                  (no staging registers) STAGES-1 K steps ahead of the MFMAs; the operand
//                  fragments of each 32-deep sub-step are read from LDS into a second register
//                  set while the MFMAs of the previous sub-step run; one barrier per K step.
//   grid level   : 2-D data-parallel tiling with an XCD-aware tile order; grid.z is the
//                  batch index or the split-K range; a tail split for a partly filled last
//                  round; a persistent instantiation whose work-groups walk several tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>
#include <utility>

namespace fact {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

#define FACT_LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))


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
    int vec_store;          // 1: C / residual / bias allow 16-byte vector access
    int pf_sa, pf_sb;       // L2 prefetch: work-groups that share an A row-panel / a B column-panel (0: off; else a power of two)
    int pf_dist;            // L2 prefetch: K steps ahead of the step being loaded into LDS (>= 1)
    // Tail split (the last, partly filled round of tiles): work-groups [0, tail_first) own one tile
    // each; the remaining tiles are shared by tail_g work-groups each, one K range apiece.
    int out_f32;            // fp32 output (written by the reduce pass; the main kernel then always stores partials)
    int c_f32;              // C holds fp32 and this kernel's epilogue writes it, unrounded (K not split)
    int f16;                // 1: A, B, bias, residual and a 16-bit C are IEEE binary16 (else bf16)
    int tail_first;         // number of tiles computed whole (== tiles_m * tiles_n when tail_g <= 1)
    int tail_g;             // K ranges per tail tile (0 or 1: off)
    float *tail_ws;         // fp32 partial accumulators, (tail_g - 1) per tail tile
    unsigned long long *tail_flags;   // one per partial
    unsigned long long *tail_status;  // workspace word that takes the launch's epoch when a hand-over wait gave up
    unsigned long long tail_epoch;    // value a flag takes when its partial of THIS launch is complete
    int tail_budget;                  // polls the collecting work-group of a tile spends on its partners' flags (< 0: gives up at once)
    // Persistent launch: grid.x work-groups walk persist_items work items (tiles x batch entries), work-group w
    // taking items w, w + grid.x, ...; 0: one item per work-group (grid.z = batch entry or K range).
    int persist_items;
    int persist_z;                    // batch entries of a persistent launch
    int persist_grid;                 // work-groups of a persistent launch (host side only)
};

constexpr uint32_t kBufferFlags = 0x00020000u;   // raw buffer descriptor word 3 (32-bit data format)
constexpr uint32_t kOobOffset = 0x80000000u;     // beyond any descriptor's num_records (< 2^31)

__device__ __forceinline__ float sigmoid_fast(float t)
{
    // 1 / (1 + e^-t); e^-t overflows to +inf for very negative t, giving 0.
    return __builtin_amdgcn_rcpf(1.0f + __expf(-t));
}

// tanh-form GELU: 0.5 z (1 + tanh(u)) = z * sigmoid(2u) = z / (1 + e^(-2u)), u = sqrt(2/pi) (z + 0.044715 z^3).
// Written as -2u log2(e) = z (k0 + k1 z^2) so that an element costs five plain vector instructions
// and the two transcendental ones (the epilogue of a 256 x 256 tile is 128 elements per lane, all
// of them vector-ALU time that no MFMA overlaps).  For z -> -inf the exponential overflows to
// +inf and the result is -0; for z -> +inf it underflows to 0 and the result is z.
__device__ __forceinline__ float gelu_tanh(float z)
{
    constexpr float k0 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
    constexpr float k1 = k0 * 0.044715f;
    const float t = __builtin_fmaf(z * z, k1, k0) * z;
    return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}

__device__ __forceinline__ float silu(float z) { return z * sigmoid_fast(z); }

// A pointer / integer that is the same in every lane of the wave, moved to scalar registers for
// good (buffer descriptors must be scalar; a descriptor the compiler takes for lane-dependent is
// applied lane group by lane group in a loop).
__device__ __forceinline__ const char *wave_uniform(const char *ptr)
{
    const uint64_t v = (uint64_t)ptr;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (const char *)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ uint32_t wave_uniform(uint32_t v) { return __builtin_amdgcn_readfirstlane(v); }

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

// The two 16-bit formats a launch may compute in.  F16 = false: bf16 (the workload definition's); F16 = true: IEEE
// binary16, the precision of the paper's own kernels (Listing 1; Sections 5.2.3 - 5.2.5).  Either way the
// accumulator is fp32 and the epilogue rounds once, to nearest even.
typedef __bf16 pk_bf16_t __attribute__((ext_vector_type(2)));
typedef _Float16 pk_f16_t __attribute__((ext_vector_type(2)));
typedef float pk_f32_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float f16_bits_to_f32(uint32_t h16) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h16); }
__device__ __forceinline__ uint32_t f32_to_f16_bits(float x) { return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)x); }
template <bool F16> __device__ __forceinline__ float in16(uint32_t bits)
{
    if constexpr (F16) return f16_bits_to_f32(bits);
    else return bf16_bits_to_f32(bits);
}
template <bool F16> __device__ __forceinline__ uint32_t out16(float x)
{
    if constexpr (F16) return f32_to_f16_bits(x);
    else return f32_to_bf16_bits(x);
}
template <bool F16> __device__ __forceinline__ uint32_t pack2(pk_f32_t f2)       // two values rounded to nearest even, low half first
{
    if constexpr (F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2, pk_f16_t));
    else return __builtin_bit_cast(uint32_t, __builtin_convertvector(f2, pk_bf16_t));
}

// Work-group id -> tile coordinates.  Consecutive work-group ids go to different
// XCDs (8 of them, each with its own L2), so id % 8 picks the XCD and every XCD
// gets one contiguous range of the tile order; inside that order tiles are walked
// group_m tile-rows at a time, column by column, so that the tiles resident on one
// XCD share A row-panels and B column-panels.
__device__ __forceinline__ void tile_index_to_coords(const GemmArgs &p, int idx, int &tm, int &tn);
__device__ __forceinline__ void tile_coords(const GemmArgs &p, int pid, int total, int &tm, int &tn)
{
    const int q = total >> 3, rem = total & 7;
    const int xcd = pid & 7, loc = pid >> 3;
    const int idx = xcd * q + (xcd < rem ? xcd : rem) + loc;
    tile_index_to_coords(p, idx, tm, tn);
}
// position idx of the tile order -> tile coordinates
__device__ __forceinline__ void tile_index_to_coords(const GemmArgs &p, int idx, int &tm, int &tn)
{
    const int per_group = p.group_m * p.tiles_n;
    const int grp = idx / per_group;
    const int first_m = grp * p.group_m;
    const int gsz = (p.tiles_m - first_m) < p.group_m ? (p.tiles_m - first_m) : p.group_m;
    const int in_grp = idx - grp * per_group;
    tm = first_m + in_grp % gsz;
    tn = in_grp / gsz;
}

// Compile-time loop: f(integral_constant<int, 0>{}), ..., f(integral_constant<int, N-1>{}).  The
// main loop's instruction order is built with it, so that it never depends on the optimizer's
// unrolling limits.
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// B given as [K][N] (trans_b = 0) is staged with loads that cover whole K-rows of the tile:
// the tile's N must hold a power-of-two number of 16-byte chunks.  Other tile widths serve
// trans_b = 1 only.
constexpr bool plain_b_supported(int bn) { return 64 % (bn / 8) == 0; }

// Epilogue staging geometry (shared with the host side, which sizes the dynamic LDS): each wave
// transposes its accumulators through an fp32 region of epi_rows rows with this pitch.
constexpr int epi_pitch(int wtn) { return wtn * 4 + 16; }
// Half a compute unit's LDS: a configuration that stays within it runs two work-groups per compute unit (its registers
// permitting), one's K loop under the other's prologue and epilogue.  Nothing optional may be what pushes a
// configuration over that line: the epilogue then stages 32 rows per pass instead of 64, and a ring of exactly this size
// does without the L2 prefetch and its sink (has_prefetch).
constexpr int kHalfLds = 80 * 1024;
constexpr int ring_bytes(int bm, int bn, int bk, int stages) { return stages * (bm + bn) * bk * 2; }
constexpr int epi_rows(int wtm, int wtn, int nwaves, int ring)
{
    const int r64 = nwaves * 64 * epi_pitch(wtn);
    return (wtm >= 64 && r64 <= 144 * 1024 && !(ring <= kHalfLds && r64 > kHalfLds)) ? 64 : 32;
}
constexpr int lds_bytes(int bm, int bn, int wgm, int wgn, int bk, int stages)
{
    const int ring = ring_bytes(bm, bn, bk, stages);
    const int epi = wgm * wgn * epi_rows(bm / wgm, bn / wgn, wgm * wgn, ring) * epi_pitch(bn / wgn);
    return ring > epi ? ring : epi;
}
// The L2 prefetch loads land in a small sink behind the operand ring (256 bytes per wave); the collecting work-group of a
// tail split also passes its verdict through a word of it.
constexpr bool has_prefetch(int bm, int bn, int wgm, int wgn, int bk, int stages)
{
    const int b = lds_bytes(bm, bn, wgm, wgn, bk, stages);
    return !(b <= kHalfLds && b + wgm * wgn * 256 > kHalfLds);
}
constexpr int lds_total(int bm, int bn, int wgm, int wgn, int bk, int stages)
{
    return lds_bytes(bm, bn, wgm, wgn, bk, stages) + (has_prefetch(bm, bn, wgm, wgn, bk, stages) ? wgm * wgn * 256 : 0);
}

// Wait until at most N of this wave's global->LDS loads are outstanding and all its LDS
// reads are done, then the work-group barrier.  "memory" keeps LDS accesses on their side.
template <int N>
__device__ __forceinline__ void wait_loads_and_barrier()
{
    __builtin_amdgcn_sched_barrier(0);       // nothing is scheduled across the barrier
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
    __builtin_amdgcn_sched_barrier(0);
}

// LDS layouts of one stage (all offsets in bytes, chunk = 16 bytes = 8 bf16):
//  K-contiguous operand (A always; B when trans_b=1): [rows][64] with the chunk kc of row r at
//  chunk position kc ^ swz_k(r).  A fragment read walks 16 consecutive rows at 4 consecutive
//  chunks; the XOR spreads them over the banks (measured: as fast as a contiguous read).  swz_k
//  has period 8 in r, so the MFMA tiles of a wave differ by constant offsets and a lane of a
//  global->LDS load (8 rows per load) sees the same swizzle in every load.
__device__ __forceinline__ int swz_k(int row) { return row & 7; }
//  N-contiguous operand (B when trans_b=0): [64][BN] with the chunk nc of K-row k at position
//  nc ^ swz_n(k).  The transposing 64-bit LDS reads of one 16-lane group touch 4 consecutive
//  K-rows x 32 bytes; rows are a multiple of 128 bytes apart, so unswizzled all four would hit
//  the same 32 banks.  The XOR puts them into the four 32-byte slots of one 128-byte line.
//  (An earlier version spread them 64 bytes apart, i.e. over two slots; this one is 0.7% faster
//  on 8192^3.  The bank-conflict counter reads one cycle per transposing read with either.)
template <int BN>
__device__ __forceinline__ int swz_n(int k)
{
    if constexpr ((BN / 8) % 16 == 0) return (k & 3) << 1;
    else return (k & 1) << 2;
}

// The accumulators are not C++ variables: tile T of a wave lives in the accumulation registers
// a[4T .. 4T+3] by name, and only the inline assembly below touches them.  (As variables, the
// compiler moved tiles between the two register files around the K loop whenever the code after
// the loop used their elements in vector arithmetic, and spilled.)  Every statement declares the
// registers it writes, so the compiler keeps nothing of its own there across the K loop and
// counts them in the kernel's register budget; the build checks that the compiler itself emits no
// write to an accumulation register in a GEMM kernel.
template <int T> struct AccTile;
#define FACT_ACC_TILE(T, R0, R1, R2, R3)                                                                                         \
    template <> struct AccTile<T> {                                                                                              \
        /* D = B-fragment x A-fragment + D */                                                                                    \
        static __device__ __forceinline__ void mfma(const bf16x8_t &b, const bf16x8_t &a)                                        \
        {                                                                                                                        \
            asm volatile("v_mfma_f32_16x16x32_bf16 a[" #R0 ":" #R3 "], %0, %1, a[" #R0 ":" #R3 "]"                               \
                         : : "v"(b), "v"(a) : "a" #R0, "a" #R1, "a" #R2, "a" #R3);                                               \
        }                                                                                                                        \
        static __device__ __forceinline__ void mfma_f16(const bf16x8_t &b, const bf16x8_t &a)   /* the same registers holding binary16 */ \
        {                                                                                                                        \
            asm volatile("v_mfma_f32_16x16x32_f16 a[" #R0 ":" #R3 "], %0, %1, a[" #R0 ":" #R3 "]"                                \
                         : : "v"(b), "v"(a) : "a" #R0, "a" #R1, "a" #R2, "a" #R3);                                               \
        }                                                                                                                        \
        static __device__ __forceinline__ void zero()                                                                            \
        {                                                                                                                        \
            asm volatile("v_accvgpr_write_b32 a" #R0 ", 0\n\tv_accvgpr_write_b32 a" #R1 ", 0\n\t"                                \
                         "v_accvgpr_write_b32 a" #R2 ", 0\n\tv_accvgpr_write_b32 a" #R3 ", 0"                                    \
                         : : : "a" #R0, "a" #R1, "a" #R2, "a" #R3);                                                              \
        }                                                                                                                        \
        /* the tile's 16 bytes per lane to LDS, straight from the accumulation registers */                                     \
        template <int OFFSET> static __device__ __forceinline__ void to_lds(uint32_t lds_addr)                                   \
        {                                                                                                                        \
            asm volatile("ds_write_b128 %0, a[" #R0 ":" #R3 "] offset:%1" : : "v"(lds_addr), "n"(OFFSET) : "memory");            \
        }                                                                                                                        \
        static __device__ __forceinline__ f32x4_t get()                                                                          \
        {                                                                                                                        \
            float x0, x1, x2, x3;                                                                                                \
            asm volatile("v_accvgpr_read_b32 %0, a" #R0 "\n\tv_accvgpr_read_b32 %1, a" #R1 "\n\t"                               \
                         "v_accvgpr_read_b32 %2, a" #R2 "\n\tv_accvgpr_read_b32 %3, a" #R3                                      \
                         : "=v"(x0), "=v"(x1), "=v"(x2), "=v"(x3));                                                              \
            return f32x4_t{x0, x1, x2, x3};                                                                                      \
        }                                                                                                                        \
    };
#include "acc_regs.inc"
#undef FACT_ACC_TILE

// The launch's parameters, read afresh from the kernel-argument segment.  A persistent work-group
// walks several tiles; with the by-value argument the compiler loads every field once at the
// kernel's start and carries all of them across the K loop for the next tile (some 60 scalar
// registers: it ran out and parked ~300 of them in vector-register lanes, +2.4 us per tile).  Behind
// this opaque pointer each tile's set-up and each epilogue load what they use where they use it.
__device__ __forceinline__ GemmArgs fresh_args()
{
#if defined(__HIP_DEVICE_COMPILE__)
    typedef const __attribute__((address_space(4))) GemmArgs *kernarg_ptr_t;
    kernarg_ptr_t k = (kernarg_ptr_t)__builtin_amdgcn_kernarg_segment_ptr();       // GemmArgs is the kernel's only argument
    asm volatile("" : "+s"(k));
    GemmArgs a;
    __builtin_memcpy(&a, k, sizeof a);
    return a;
#else
    return GemmArgs{};
#endif
}

// PERSIST: the work-group walks several work items (persistent launch; 4-wave configurations only).  The
// ordinary kernel is a separate instantiation in which the loop below is gone at compile time.
// F16: the operands, bias, residual and the 16-bit output are IEEE binary16 instead of bf16.
template <int BM, int BN, int WGM, int WGN, bool TRANS_B, int BK, int STAGES, bool PERSIST, bool F16 = false>
__global__ void __launch_bounds__(WGM * WGN * 64)
gemm_kernel(const GemmArgs p)
{
#if defined(__HIP_DEVICE_COMPILE__)      // the host pass only needs the kernel's symbol
    constexpr int NWAVES = WGM * WGN;
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int MT = WTM / 16, NT = WTN / 16;      // 16x16 MFMA tiles per wave
    constexpr int KC = BK / 8;                 // chunks per K-contiguous row
    constexpr int ROWB = BK * 2;               // bytes per K-contiguous row
    constexpr int KK = BK / 32;                // MFMA sub-steps (32 K-values) per K step
    constexpr int NCH = BN / 8;                // chunks per N-contiguous row
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
    constexpr int STAGE = A_BYTES + B_BYTES;
    constexpr int A_LD = A_BYTES / 1024 / NWAVES;     // direct loads (1 KB per wave each) per wave per step
    constexpr int B_LD = B_BYTES / 1024 / NWAVES;
    constexpr int LOADS = A_LD + B_LD;
    static_assert(WTM % 16 == 0 && WTN % 32 == 0, "wave tile must be made of 16x16 MFMA tiles, an even number along N");
    static_assert(A_BYTES % (1024 * NWAVES) == 0 && B_BYTES % (1024 * NWAVES) == 0, "tile must split into whole wave loads");
    static_assert(BK == 64, "BK");
    static_assert((STAGES - 2) * (LOADS + 1) + 1 <= 63 && STAGES >= 2, "vmcnt range");

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- what the epilogue needs of its tile ------------------------------------------------
    // A work-group may walk several tiles (persistent launch).  The epilogue of a tile runs when the
    // next tile's first operand stages have been requested, so it must not look at anything the
    // loop below derives for the tile in hand: these variables are set by hand_over() in the loop
    // (before the tile's K loop in a persistent work-group, after it in an ordinary one).
    int e_tm = 0, e_tn = 0, e_z = 0;                  // tile coordinates, batch entry or K range
    bool e_in_regs = false;                           // it takes the register path
    bool e_in_tail = false, tail_gave_up = false;     // tail split: a shared tile; its collecting wait gave up
    int e_tail_seg = 0, e_tail_tile = 0;              // tail split: K range number, tile number within the tail
    constexpr int TILE_FLOATS = BM * BN;
    constexpr int kSysScope = 17;                    // cache-policy bits sc0 | sc1 of buffer loads / stores
    // The 16-byte stores of finished C tiles: written through the XCD's L2 (sc0 | sc1) as non-temporal
    // data (nt).  C is not read again by this launch, and lines left dirty in the eight L2s have to be
    // written back before the launch can end.  Same-box A/B against plain stores, operands from the
    // memory-side cache / rotated out of it: 8192 x 2304 x 768 + bias 37.5 -> 36.6 / 48.1 -> 40.2 us,
    // 8192 x 3072 x 768 + bias + GELU 45.3 -> 41.6 / 48.0 -> 41.7 us, 128 x 512^3 43.5 -> 42.5 / 51.5 -> 48.5 us,
    // 8192^3 713 -> 708 us; no shape slower.  (Write-through alone: better from the cache, worse from HBM.)
    constexpr int kStoreThrough = 19;

    // ---- epilogue ---------------------------------------------------------------------------
    // Accumulator tile (mt, nt), lane (r16, q): output row mt*16 + r16, output columns
    // nt*16 + 4q .. + 3: a lane owns pieces of one row per tile, so a direct store would write
    // 16-byte pieces of 16 different rows per instruction.  Instead each wave transposes its
    // accumulators through its own LDS region (fp32, EPI_ROWS rows at a time) and reads them
    // back row-wise: a lane then holds 8 consecutive columns of one row and all epilogue
    // arithmetic happens there, in fp32, in registers:
    //     z = acc + bias[n];  z = act(z);  z = z + residual[m][n];  store bf16(z)
    // with 16-byte loads of bias / residual and 16-byte stores (whole 128-byte lines per row).
    // Region row pitch = row bytes + 16, which spreads the 16 rows a write instruction touches
    // over all banks.  Only the wave itself reads what it wrote: no work-group barrier inside.
    constexpr int EPI_PITCH = epi_pitch(WTN);
    constexpr int EPI_ROWS = epi_rows(WTM, WTN, NWAVES, ring_bytes(BM, BN, BK, STAGES));
    constexpr int EPI_TR = EPI_ROWS / 16;                       // tile-rows per pass
    constexpr int EPI_REGION = EPI_ROWS * EPI_PITCH;
    static_assert(lds_total(BM, BN, WGM, WGN, BK, STAGES) <= 160 * 1024 && NWAVES * EPI_REGION <= lds_bytes(BM, BN, WGM, WGN, BK, STAGES) && WTM % EPI_ROWS == 0, "LDS budget");
    // IN_REGS: the register path (interior tile, bf16 output, no hand-over); it touches no LDS, so the
    // operand ring may be filling for the next tile while it runs.  Otherwise the LDS-staged passes.
    auto epilogue = [&](auto in_regs_tag) __attribute__((always_inline)) {
    constexpr bool IN_REGS = decltype(in_regs_tag)::value;
    const bool gated = (p.act == ACT_SILU_GATE);
    const int nout = gated ? (p.N >> 1) : p.N;
    const bool partial = p.splits > 1 || p.out_f32;
    // The lane's position is derived anew here, so that nothing of it stays live in a vector register
    // across the K loop (the 8-wave kernels have no register to spare for that).
    const int tid = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) + wave * 64;
    const int lane = tid & 63;
    const int r16 = lane & 15, q = lane >> 4;
    if constexpr (!IN_REGS) __syncthreads();                    // every wave is done with the operand stages
    char *region = smem + wave * EPI_REGION;
    const int out_w = gated ? WTN / 2 : WTN;                    // output columns this wave owns
    const int lanes_per_row = out_w / 8;
    const int e_n0 = e_tn * (gated ? BN / 2 : BN);              // first OUTPUT column of the tile
    const int n_wave = e_n0 + wn * out_w;                       // first output column of this wave
    const int m_wave = e_tm * BM + wm * WTM;
    float *P = partial ? p.P + (int64_t)e_z * p.M * p.N : nullptr;       // split-K: this K range's plane of partials
    const bool batched = !e_in_tail && p.splits <= 1;            // e_z is a batch entry (a K range otherwise)
    __bf16 *C = p.C + (batched ? e_z * p.stride_c : 0);
    float *Cf = (float *)p.C + (batched ? e_z * p.stride_c : 0);       // the same matrix when it holds fp32 (c_f32)
    const __bf16 *R = p.res ? p.res + (batched ? e_z * p.stride_r : 0) : nullptr;
    // Fast path: the wave's whole tile lies inside C and everything allows 16-byte access.  Straight
    // code, no per-element guards: the general path spends most of its time in them.
    const bool fast = !partial && p.vec_store && m_wave + WTM <= p.M && n_wave + out_w <= nout;
    // (8-wave work-groups have half the registers per wave: they keep to the general path here)
    const bool fast_partial = NWAVES <= 4 && partial && (p.N & 3) == 0 && (nout & 3) == 0 && m_wave + WTM <= p.M && n_wave + out_w <= nout;
    const int tail_parts = e_in_tail ? p.tail_g - 1 : 0;
    const bool tail_producer = e_in_tail && e_tail_seg < tail_parts;
    const __amdgpu_buffer_rsrc_t rsrc_part = __builtin_amdgcn_make_buffer_rsrc(      // this tile's partials
        (void *)wave_uniform((const char *)(e_in_tail ? p.tail_ws + (int64_t)e_tail_tile * tail_parts * TILE_FLOATS : nullptr)), 0,
        (uint32_t)(tail_parts * TILE_FLOATS * 4), kBufferFlags);
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    auto fast_pass = [&](int pass, auto gated_tag) __attribute__((always_inline)) {
        constexpr bool GATED = decltype(gated_tag)::value;
        constexpr int OUT_W = GATED ? WTN / 2 : WTN;
        constexpr int LPR_USED = OUT_W / 8;                         // lanes a row needs
        constexpr int LPR = LPR_USED <= 1 ? 1 : LPR_USED <= 2 ? 2 : LPR_USED <= 4 ? 4 : LPR_USED <= 8 ? 8 : LPR_USED <= 16 ? 16 : 32;
        constexpr int TOTAL = EPI_ROWS * LPR;                       // (a power of two of lanes is set aside per row)
        constexpr int FU = NWAVES > 4 ? 2 : 4;                      // row-chunks per lane and batch
        static_assert(64 % LPR == 0 && TOTAL % 64 == 0, "a lane keeps its columns; batches are whole waves");
        const int c8 = lane % LPR;
        if constexpr (LPR != LPR_USED) { if (c8 >= LPR_USED) return; }      // 96- or 48-wide wave tiles: the lanes past a row's end idle
        const int n = n_wave + c8 * 8;
        float bv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) bv[e] = -0.0f;               // without a bias: the addend that leaves every value, a signed zero too, as it is
        if (p.bias) {
            const u32x4_t b4 = *(const u32x4_t *)(p.bias + n);
#pragma unroll
            for (int e = 0; e < 4; ++e) { bv[2 * e] = in16<F16>(b4[e] & 0xFFFFu); bv[2 * e + 1] = in16<F16>(b4[e] >> 16); }
        }
        const int act = p.act;
#pragma unroll
        for (int base = 0; base < TOTAL; base += 64 * FU) {
            u32x4_t rb[FU];
            f32x4_t x[FU][2], y[FU][2];
            int row[FU];
#pragma unroll
            for (int j = 0; j < FU; ++j) {
                if (base + 64 * j < TOTAL) {
                    row[j] = (base + 64 * j + lane) / LPR;
                    if (R) rb[j] = *(const u32x4_t *)(R + (int64_t)(m_wave + pass * EPI_ROWS + row[j]) * p.ldr + n);
                    const char *src = region + row[j] * EPI_PITCH + c8 * 32;
                    x[j][0] = *(const f32x4_t *)src; x[j][1] = *(const f32x4_t *)(src + 16);
                    if constexpr (GATED) { y[j][0] = *(const f32x4_t *)(src + OUT_W * 4); y[j][1] = *(const f32x4_t *)(src + OUT_W * 4 + 16); }
                    // last K range of a split tail tile: add the other ranges' partial sums, in range order
                    for (int sgm = 0; sgm < tail_parts; ++sgm) {
                        const int ps = ((wm * WTM + pass * EPI_ROWS + row[j]) * BN + wn * WTN + c8 * 8) * 4, so = sgm * TILE_FLOATS * 4;
                        auto ld = [&](int off) { return __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc_part, ps + off, so, kSysScope)); };
                        x[j][0] += ld(0); x[j][1] += ld(16);
                        if constexpr (GATED) { y[j][0] += ld(OUT_W * 4); y[j][1] += ld(OUT_W * 4 + 16); }
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < FU; ++j) {
                if (base + 64 * j < TOTAL) {
                    float z[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        z[e] = x[j][e >> 2][e & 3];
                        if constexpr (GATED) z[e] = silu(z[e]) * y[j][e >> 2][e & 3];
                        z[e] += bv[e];
                    }
                    if (act == ACT_GELU_TANH) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) z[e] = gelu_tanh(z[e]);
                    }
                    if (R) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { z[2 * e] += in16<F16>(rb[j][e] & 0xFFFFu); z[2 * e + 1] += in16<F16>(rb[j][e] >> 16); }
                    }
                    if (tail_gave_up) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) z[e] = __builtin_nanf("");
                    }
                    if (p.c_f32) {
                        float *cf = Cf + (int64_t)(m_wave + pass * EPI_ROWS + row[j]) * p.ldc + n;
                        *(f32x4_t *)cf = f32x4_t{z[0], z[1], z[2], z[3]};
                        *(f32x4_t *)(cf + 4) = f32x4_t{z[4], z[5], z[6], z[7]};
                        continue;
                    }
                    u32x4_t o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const f32x2_t f2 = {z[2 * e], z[2 * e + 1]};
                        o[e] = pack2<F16>(f2);     // round to nearest even
                    }
                    *(u32x4_t *)(C + (int64_t)(m_wave + pass * EPI_ROWS + row[j]) * p.ldc + n) = o;
                }
            }
        }
    };

    // The same pass as a short loop (bf16 output, no partial sums of other K ranges to add): the
    // read-back of a pass is not unrolled, so the whole epilogue is a few hundred instructions that
    // stay in the instruction cache from tile to tile (straight-line code of several thousand
    // instructions was measured to run at the speed of its instruction fetch: 9-15 us per
    // 256 x 256 tile on a compute unit's first tile).  C and the residual are addressed through
    // buffer descriptors of the wave's tile with one lane-offset register each that advances by a
    // constant per iteration (32-bit offsets: the host sets vec_store only if a tile's rows span
    // less than 2^31 bytes).
    auto compact_pass = [&](int pass, auto gated_tag) __attribute__((always_inline)) {
        constexpr bool GATED = decltype(gated_tag)::value;
        constexpr int OUT_W = GATED ? WTN / 2 : WTN;
        constexpr int LPR_USED = OUT_W / 8;
        constexpr int LPR = LPR_USED <= 1 ? 1 : LPR_USED <= 2 ? 2 : LPR_USED <= 4 ? 4 : LPR_USED <= 8 ? 8 : LPR_USED <= 16 ? 16 : 32;
        constexpr int RPB = 64 / LPR;                               // rows a wave-wide access covers
        constexpr int NB = EPI_ROWS / RPB;                          // such accesses per pass
        constexpr int FU0 = NWAVES > 4 ? 2 : 4, FU = NB < FU0 ? NB : FU0;       // of them per loop iteration
        static_assert(64 % LPR == 0 && NB % FU == 0, "a lane keeps its columns; iterations are whole");
        const int c8 = lane % LPR, lrow = lane / LPR;
        if constexpr (LPR != LPR_USED) { if (c8 >= LPR_USED) return; }      // 96- or 48-wide wave tiles: the lanes past a row's end idle
        // Tile edges: the columns of C end at a multiple of 8 here (16-byte access), so a lane's 8 columns lie
        // inside C or outside, and the lanes outside idle; rows past the last one fall outside the range of
        // the descriptors below, where the hardware drops stores and returns zero for loads.  (Edge tiles
        // used to take the guarded path further down: 16-20 us per wave tile against 4-5 us here.)
        const int cols_left = nout - n_wave, rows_left = p.M - (m_wave + pass * EPI_ROWS);
        if (rows_left <= 0 || c8 * 8 >= cols_left) return;
        const int valid_rows = rows_left < EPI_ROWS ? rows_left : EPI_ROWS, valid_cols = cols_left < OUT_W ? cols_left : OUT_W;
        float bv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) bv[e] = -0.0f;               // without a bias: the addend that leaves every value, a signed zero too, as it is
        if (p.bias) {
            const u32x4_t b4 = *(const u32x4_t *)(p.bias + n_wave + c8 * 8);
#pragma unroll
            for (int e = 0; e < 4; ++e) { bv[2 * e] = in16<F16>(b4[e] & 0xFFFFu); bv[2 * e + 1] = in16<F16>(b4[e] >> 16); }
        }
        const bool gelu = p.act == ACT_GELU_TANH, has_res = R != nullptr;
        const int64_t row0 = m_wave + pass * EPI_ROWS;
        const uint32_t nrec_c = wave_uniform((uint32_t)(((valid_rows - 1) * (int)p.ldc + valid_cols) * 2));       // (ldc, ldr < 2^21)
        const uint32_t nrec_r = wave_uniform((uint32_t)(((valid_rows - 1) * (int)(has_res ? p.ldr : p.ldc) + valid_cols) * 2));
        const __amdgpu_buffer_rsrc_t rsrc_c = __builtin_amdgcn_make_buffer_rsrc((void *)wave_uniform((const char *)(C + row0 * p.ldc + n_wave)), 0, nrec_c, kBufferFlags);
        const __amdgpu_buffer_rsrc_t rsrc_r = __builtin_amdgcn_make_buffer_rsrc(
            (void *)wave_uniform((const char *)(has_res ? R + row0 * p.ldr + n_wave : C + row0 * p.ldc + n_wave)), 0, nrec_r, kBufferFlags);
        uint32_t vo = (uint32_t)((lrow * (int)p.ldc + c8 * 8) * 2), vr = (uint32_t)((lrow * (int)p.ldr + c8 * 8) * 2);
        const uint32_t step_c = (uint32_t)(RPB * (int)p.ldc * 2), step_r = (uint32_t)(RPB * (int)p.ldr * 2);
        const char *src = region + lrow * EPI_PITCH + c8 * 32;
#pragma nounroll
        for (int it = 0; it < NB / FU; ++it) {
            u32x4_t rb[FU];
            f32x4_t x[FU][2], y[FU][2];
#pragma unroll
            for (int j = 0; j < FU; ++j) {
                if (has_res) rb[j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, vr + j * step_r, 0, 0);
                const char *sj = src + j * RPB * EPI_PITCH;
                x[j][0] = *(const f32x4_t *)sj; x[j][1] = *(const f32x4_t *)(sj + 16);
                if constexpr (GATED) { y[j][0] = *(const f32x4_t *)(sj + OUT_W * 4); y[j][1] = *(const f32x4_t *)(sj + OUT_W * 4 + 16); }
            }
#pragma unroll
            for (int j = 0; j < FU; ++j) {
                float z[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    z[e] = x[j][e >> 2][e & 3];
                    if constexpr (GATED) z[e] = silu(z[e]) * y[j][e >> 2][e & 3];
                    z[e] += bv[e];
                }
                if (gelu) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) z[e] = gelu_tanh(z[e]);
                }
                if (has_res) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { z[2 * e] += in16<F16>(rb[j][e] & 0xFFFFu); z[2 * e + 1] += in16<F16>(rb[j][e] >> 16); }
                }
                u32x4_t o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const f32x2_t f2 = {z[2 * e], z[2 * e + 1]};
                    o[e] = pack2<F16>(f2);     // round to nearest even
                }
                // (scalar offset operand: the constant 0, see the note at the partial-tile stores below)
                __builtin_amdgcn_raw_buffer_store_b128(o, rsrc_c, vo + j * step_c, 0, kStoreThrough);
            }
            vo += FU * step_c; vr += FU * step_r; src += FU * RPB * EPI_PITCH;
        }
    };

    // Register path (interior wave tiles with 16-byte access, bf16 output, no K hand-over): no LDS at
    // all (the transposing path above moves 1 MB through LDS per 256 x 256 tile, 4 us of LDS time).
    // Two neighbouring 16 x 16 accumulator tiles exchange 16-lane rows (v_permlane16_swap: the odd
    // rows of the first operand with the even rows of the second), after which lane (r16, q) holds 8
    // consecutive columns of output row r16: tile q & 1 of the pair, columns 8 (q >> 1) .. + 7.
    // Bias, activation, residual and the single rounding happen there, in fp32, and every lane
    // stores 16 bytes: the four lanes of a row write 64 consecutive bytes, the next pair of tiles
    // the other half of the 128-byte line.  (Gated: gate and up values of an element sit in the
    // same lane, so SiLU(gate) * up is formed before the exchange.)  What the epilogue adds is
    // fixed at compile time (one instance per combination, chosen once), so the code is straight;
    // C and the residual are addressed through buffer descriptors of the wave's tile with one
    // lane-offset register each (32-bit offsets: the host sets vec_store only if a tile's rows span
    // less than 2^31 bytes), a tile row adds one vector add, a pair an immediate offset.
    auto reg_epilogue = [&](auto gated_tag, auto bias_tag, auto gelu_tag, auto res_tag) __attribute__((always_inline)) {
        constexpr bool GATED = decltype(gated_tag)::value, BIAS = decltype(bias_tag)::value;
        constexpr bool GELU = decltype(gelu_tag)::value, RES = decltype(res_tag)::value;
        constexpr int OT = GATED ? NT / 2 : NT;                     // output tiles along N of this wave
        constexpr int NP = OT / 2;                                  // pairs of them
        static_assert(OT % 2 == 0, "tiles are exchanged in pairs");
        // 8-wave work-groups have half the registers per wave: the bias stays packed (unpacked at every
        // use) and the residual is loaded row by row instead of one row ahead
        constexpr bool LEAN = NWAVES > 4;
        const int col = (q & 1) * 16 + (q >> 1) * 8;                // the lane's first column inside a pair
        const __amdgpu_buffer_rsrc_t rsrc_c = __builtin_amdgcn_make_buffer_rsrc(
            (void *)wave_uniform((const char *)(C + (int64_t)m_wave * p.ldc + n_wave)), 0, 0x7FFFFFFF, kBufferFlags);
        const uint32_t voff_c = (uint32_t)((r16 * (int)p.ldc + col) * 2);
        const uint32_t row_c = (uint32_t)(16 * (int)p.ldc * 2);     // bytes per tile row of C
        __amdgpu_buffer_rsrc_t rsrc_r = rsrc_c;
        uint32_t voff_r = 0, row_r = 0;
        if constexpr (RES) {
            rsrc_r = __builtin_amdgcn_make_buffer_rsrc((void *)wave_uniform((const char *)(R + (int64_t)m_wave * p.ldr + n_wave)), 0, 0x7FFFFFFF, kBufferFlags);
            voff_r = (uint32_t)((r16 * (int)p.ldr + col) * 2);
            row_r = (uint32_t)(16 * (int)p.ldr * 2);
        }
        float bv[LEAN ? 1 : NP][8];
        u32x4_t bp[LEAN ? NP : 1];
        if constexpr (BIAS) {
#pragma unroll
            for (int pr = 0; pr < NP; ++pr) {
                const u32x4_t b4 = *(const u32x4_t *)(p.bias + n_wave + col + pr * 32);
                if constexpr (LEAN) bp[pr] = b4;
                else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { bv[pr][2 * e] = in16<F16>(b4[e] & 0xFFFFu); bv[pr][2 * e + 1] = in16<F16>(b4[e] >> 16); }
                }
            }
        }
        u32x4_t rb[LEAN ? 1 : 2][NP];                               // residual of the row in work (and of the next one)
        auto load_res = [&](int mt) __attribute__((always_inline)) {
            if constexpr (RES) {
#pragma unroll
                for (int pr = 0; pr < NP; ++pr)
                    rb[LEAN ? 0 : (mt & 1)][pr] = __builtin_amdgcn_raw_buffer_load_b128(rsrc_r, voff_r + mt * row_r + pr * 64, 0, 0);
            }
        };
        if constexpr (!LEAN) load_res(0);
        static_for<MT>([&](auto mt_) __attribute__((always_inline)) {
            constexpr int mt = decltype(mt_)::value;
            if constexpr (LEAN) load_res(mt);
            else if constexpr (mt + 1 < MT) load_res(mt + 1);
            const uint32_t vo = voff_c + mt * row_c;
            static_for<NP>([&](auto pr_) __attribute__((always_inline)) {
                constexpr int pr = decltype(pr_)::value;
                f32x4_t x0 = AccTile<mt * NT + 2 * pr>::get(), x1 = AccTile<mt * NT + 2 * pr + 1>::get();
                if constexpr (GATED) {
                    const f32x4_t u0 = AccTile<mt * NT + OT + 2 * pr>::get(), u1 = AccTile<mt * NT + OT + 2 * pr + 1>::get();
#pragma unroll
                    for (int e = 0; e < 4; ++e) { x0[e] = silu(x0[e]) * u0[e]; x1[e] = silu(x1[e]) * u1[e]; }
                }
                float z[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float a0 = x0[e], a1 = x1[e];      // (a bit cast applied to a vector element directly reads element 0)
                    const auto sw = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(uint32_t, a0), __builtin_bit_cast(uint32_t, a1), false, false);
                    z[e] = __builtin_bit_cast(float, (uint32_t)sw[0]);
                    z[4 + e] = __builtin_bit_cast(float, (uint32_t)sw[1]);
                }
                if constexpr (BIAS) {
                    if constexpr (LEAN) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { z[2 * e] += in16<F16>(bp[pr][e] & 0xFFFFu); z[2 * e + 1] += in16<F16>(bp[pr][e] >> 16); }
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) z[e] += bv[pr][e];
                    }
                }
                if constexpr (GELU) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) z[e] = gelu_tanh(z[e]);
                }
                if constexpr (RES) {
                    const u32x4_t r4 = rb[LEAN ? 0 : (mt & 1)][pr];
#pragma unroll
                    for (int e = 0; e < 4; ++e) { z[2 * e] += in16<F16>(r4[e] & 0xFFFFu); z[2 * e + 1] += in16<F16>(r4[e] >> 16); }
                }
                u32x4_t o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const f32x2_t f2 = {z[2 * e], z[2 * e + 1]};
                    o[e] = pack2<F16>(f2);     // round to nearest even
                }
                // (scalar offset operand: the constant 0, see the note at the partial-tile stores below)
                __builtin_amdgcn_raw_buffer_store_b128(o, rsrc_c, vo + pr * 64, 0, kStoreThrough);
            });
        });
    };
    if constexpr (IN_REGS) {
        const int what = (p.bias ? 1 : 0) | (p.act == ACT_GELU_TANH ? 2 : 0) | (R ? 4 : 0);
        constexpr std::true_type T{};
        constexpr std::false_type F{};
        if (!gated) {
            switch (what) {
            case 0: reg_epilogue(F, F, F, F); break;
            case 1: reg_epilogue(F, T, F, F); break;
            case 2: reg_epilogue(F, F, T, F); break;
            case 3: reg_epilogue(F, T, T, F); break;
            case 4: reg_epilogue(F, F, F, T); break;
            case 5: reg_epilogue(F, T, F, T); break;
            case 6: reg_epilogue(F, F, T, T); break;
            default: reg_epilogue(F, T, T, T); break;
            }
        } else if constexpr (NT % 4 == 0) {
            if (R) reg_epilogue(T, F, F, T); else reg_epilogue(T, F, F, F);
        }
    } else {
    static_for<WTM / EPI_ROWS>([&](auto pass_) __attribute__((always_inline)) {
        constexpr int pass = decltype(pass_)::value;
        if (pass > 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // previous pass's reads are done
        {
            const uint32_t dst = (uint32_t)(size_t)FACT_LDS_PTR(region + r16 * EPI_PITCH + q * 16);
            static_for<EPI_TR * NT>([&](auto w_) __attribute__((always_inline)) {
                constexpr int i = decltype(w_)::value / NT, nt = decltype(w_)::value % NT;
                AccTile<(pass * EPI_TR + i) * NT + nt>::template to_lds<i * 16 * EPI_PITCH + nt * 64>(dst);
            });
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                    // the wave's own writes have landed
        const int total = EPI_ROWS * lanes_per_row;
        if (tail_producer) {
            // partial tile, fp32 row-major [BM][BN] in accumulator column order (gated: gate columns,
            // then up columns, per wave); the wave's EPI_ROWS x WTN block of this pass, 16 bytes per lane
            constexpr int LPR4 = WTN / 4;
            const int dst = (e_tail_seg * TILE_FLOATS + (wm * WTM + pass * EPI_ROWS) * BN + wn * WTN) * 4;     // bytes
#pragma unroll
            for (int base = 0; base < EPI_ROWS * LPR4; base += 64) {
                const int idx = base + lane, row = idx / LPR4, c4 = idx % LPR4;
                const u32x4_t x = *(const u32x4_t *)(region + row * EPI_PITCH + c4 * 16);
                // The whole offset goes into the per-lane operand, the scalar one stays the constant 0:
                // with a scalar-register offset the compiler assumes that the data registers of a
                // 16-byte buffer store may be overwritten in the very next cycle, and on this chip
                // the last lanes of each 16 then stored the overwriting value (seen as the next
                // store's offset inside the partial tile).  With a constant it keeps the wait states.
                __builtin_amdgcn_raw_buffer_store_b128(x, rsrc_part, dst + (row * BN + c4 * 4) * 4, 0, kSysScope);
            }
            return;
        }
        if constexpr (NWAVES <= 4) if (fast_partial) {
            // split-K partials of an interior tile: raw fp32, 16-byte stores, both halves of a gated
            // tile at their contraction columns
            constexpr int LPR4 = WTN / 4;                             // lanes per row, 4 columns each
#pragma unroll
            for (int base = 0; base < EPI_ROWS * LPR4; base += 64) {
                const int idx = base + lane, row = idx / LPR4, c4 = idx % LPR4;
                const f32x4_t x = *(const f32x4_t *)(region + row * EPI_PITCH + c4 * 16);
                int nc = e_n0 + wn * WTN + c4 * 4;                       // plain: contraction column = output column
                if (gated) nc = e_n0 + wn * (WTN / 2) + (c4 * 4) % (WTN / 2) + ((c4 * 4) / (WTN / 2)) * nout;
                // streaming store: a partial is read once, by the reduction pass, and a line left dirty in
                // this XCD's L2 would have to be written back before the launch can end (large-K case with
                // operands from HBM: 43.6 -> 38.7 us for GEMM plus reduction, 30.2 -> 29.4 us from the cache)
                __builtin_nontemporal_store(x, (f32x4_t *)(P + (int64_t)(m_wave + pass * EPI_ROWS + row) * p.N + nc));
            }
            return;
        }
        if (!partial && p.vec_store && tail_parts == 0 && !p.c_f32) {      // interior and edge tiles alike
            if (gated) compact_pass(pass, std::true_type{}); else compact_pass(pass, std::false_type{});
            return;
        }
        if (fast) {
            if (gated) fast_pass(pass, std::true_type{}); else fast_pass(pass, std::false_type{});
            return;
        }
        // General path (tile edges, unaligned C / bias / residual, split-K partials), every access
        // guarded.  Read-back in batches of EPI_U row-chunks per lane: first every LDS read and every
        // bias / residual load of the batch is issued, then the arithmetic and the stores follow,
        // so the global-load latency is paid once per batch, not once per chunk.  (The residual
        // may alias C, which keeps the compiler from hoisting those loads over stores itself.)
        constexpr int EPI_U = NWAVES > 4 ? 2 : 4;                  // 8-wave work-groups have half the registers per wave
        for (int base = lane; base < total; base += 64 * EPI_U) {
            float v[EPI_U][8], u[EPI_U][8];
            u32x4_t rb[EPI_U], bb[EPI_U];
            int mm[EPI_U], nn[EPI_U];
            bool live[EPI_U], vec[EPI_U], whole[EPI_U];       // whole: all 8 columns inside C, whatever their alignment
#pragma unroll
            for (int j = 0; j < EPI_U; ++j) {
                const int idx = base + 64 * j;
                const int row = idx / lanes_per_row, c8 = idx - row * lanes_per_row;
                mm[j] = m_wave + pass * EPI_ROWS + row;
                nn[j] = n_wave + c8 * 8;
                live[j] = idx < total && mm[j] < p.M && nn[j] < nout;
                whole[j] = live[j] && (nn[j] + 7 < nout);
                vec[j] = whole[j] && p.vec_store;
                if (idx < total) {
                    const char *src = region + row * EPI_PITCH + c8 * 32;
                    const f32x4_t x0 = *(const f32x4_t *)src, x1 = *(const f32x4_t *)(src + 16);
                    v[j][0] = x0.x; v[j][1] = x0.y; v[j][2] = x0.z; v[j][3] = x0.w;
                    v[j][4] = x1.x; v[j][5] = x1.y; v[j][6] = x1.z; v[j][7] = x1.w;
                    if (gated) {
                        const char *su = src + out_w * 4;
                        const f32x4_t u0 = *(const f32x4_t *)su, u1 = *(const f32x4_t *)(su + 16);
                        u[j][0] = u0.x; u[j][1] = u0.y; u[j][2] = u0.z; u[j][3] = u0.w;
                        u[j][4] = u1.x; u[j][5] = u1.y; u[j][6] = u1.z; u[j][7] = u1.w;
                    }
                    for (int sgm = 0; sgm < tail_parts && !tail_producer; ++sgm) {       // see the fast path
                        const int ps = ((wm * WTM + pass * EPI_ROWS + row) * BN + wn * WTN + c8 * 8) * 4, so = sgm * TILE_FLOATS * 4;
                        auto ld = [&](int off) { return __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(rsrc_part, ps + off, so, kSysScope)); };
                        const f32x4_t a0 = ld(0), a1 = ld(16);
                        v[j][0] += a0.x; v[j][1] += a0.y; v[j][2] += a0.z; v[j][3] += a0.w;
                        v[j][4] += a1.x; v[j][5] += a1.y; v[j][6] += a1.z; v[j][7] += a1.w;
                        if (gated) {
                            const f32x4_t b0 = ld(out_w * 4), b1 = ld(out_w * 4 + 16);
                            u[j][0] += b0.x; u[j][1] += b0.y; u[j][2] += b0.z; u[j][3] += b0.w;
                            u[j][4] += b1.x; u[j][5] += b1.y; u[j][6] += b1.z; u[j][7] += b1.w;
                        }
                    }
                }
                if (!partial && vec[j]) {
                    if (p.bias) bb[j] = *(const u32x4_t *)(p.bias + nn[j]);
                    if (R) rb[j] = *(const u32x4_t *)(R + (int64_t)mm[j] * p.ldr + nn[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < EPI_U; ++j) {
                const int m = mm[j], n = nn[j];
                if (partial) {
                    // split-K: raw fp32 partials, both halves of a gated tile at their contraction columns
                    if (base + 64 * j < total && m < p.M) {
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            if (h == 1 && !gated) break;
                            const float *w = h ? u[j] : v[j];
                            const int nc = n + h * nout;                   // contraction column
                            const int nlim = gated ? (h + 1) * nout : p.N;
                            float *dst = P + (int64_t)m * p.N + nc;
                            if (nc + 7 < nlim && (p.N & 3) == 0) {
                                const f32x4_t y0 = {w[0], w[1], w[2], w[3]}, y1 = {w[4], w[5], w[6], w[7]};
                                __builtin_nontemporal_store(y0, (f32x4_t *)dst); __builtin_nontemporal_store(y1, (f32x4_t *)(dst + 4));
                            } else {
#pragma unroll
                                for (int e = 0; e < 8; ++e)
                                    if (nc + e < nlim) dst[e] = w[e];
                            }
                        }
                    }
                    continue;
                }
                if (!live[j]) continue;
                float z[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) z[e] = gated ? silu(v[j][e]) * u[j][e] : v[j][e];
                if (p.bias) {
                    if (vec[j]) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { z[2 * e] += in16<F16>(bb[j][e] & 0xFFFFu); z[2 * e + 1] += in16<F16>(bb[j][e] >> 16); }
                    } else if (whole[j]) {                       // (unaligned rows, e.g. an odd leading dimension: element accesses, no guards)
#pragma unroll
                        for (int e = 0; e < 8; ++e) z[e] += (float)p.bias[n + e];
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (n + e < nout) z[e] += (float)p.bias[n + e];
                    }
                }
                if (p.act == ACT_GELU_TANH) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) z[e] = gelu_tanh(z[e]);
                }
                if (R) {
                    if (vec[j]) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { z[2 * e] += in16<F16>(rb[j][e] & 0xFFFFu); z[2 * e + 1] += in16<F16>(rb[j][e] >> 16); }
                    } else {
                        const __bf16 *rp = R + (int64_t)m * p.ldr + n;
                        if (whole[j]) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) z[e] += (float)rp[e];
                        } else {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (n + e < nout) z[e] += (float)rp[e];
                        }
                    }
                }
                if (tail_gave_up) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) z[e] = __builtin_nanf("");
                }
                if (p.c_f32) {
                    float *cf = Cf + (int64_t)m * p.ldc + n;
                    if (vec[j]) {
                        *(f32x4_t *)cf = f32x4_t{z[0], z[1], z[2], z[3]};
                        *(f32x4_t *)(cf + 4) = f32x4_t{z[4], z[5], z[6], z[7]};
                    } else if (whole[j]) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) cf[e] = z[e];
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (n + e < nout) cf[e] = z[e];
                    }
                    continue;
                }
                __bf16 *cp = C + (int64_t)m * p.ldc + n;
                if (vec[j]) {
                    u32x4_t o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = out16<F16>(z[2 * e]) | (out16<F16>(z[2 * e + 1]) << 16);
                    *(u32x4_t *)cp = o;
                } else if (whole[j]) {
                    uint16_t *cs = (uint16_t *)cp;
#pragma unroll
                    for (int e = 0; e < 8; ++e) cs[e] = (uint16_t)out16<F16>(z[e]);
                } else {
                    uint16_t *cs = (uint16_t *)cp;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (n + e < nout) cs[e] = (uint16_t)out16<F16>(z[e]);
                }
            }
        }
    });
    if (tail_producer) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                 // this thread's write-through stores have reached memory
        __syncthreads();
        if (tid == 0)
            __hip_atomic_store(p.tail_flags + (int64_t)e_tail_tile * tail_parts + e_tail_seg, p.tail_epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    } else if (e_in_tail) {
        // The collecting work-group takes the flags down again once every thread has its partial sums
        // (each added them to its values before it got here).  A launch replayed from a captured graph
        // carries the same epoch every time: without this, the second replay would find the flags
        // of the first still raised and read partial tiles that are being rewritten.
        __syncthreads();
        if (tid == 0)
            for (int sgm = 0; sgm < tail_parts; ++sgm)
                __hip_atomic_store(p.tail_flags + (int64_t)e_tail_tile * tail_parts + sgm, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    }
    };

    bool owed = false;                               // a finished K loop's epilogue has not run yet
    // (8-wave work-groups never walk several items: they have no registers to carry anything across the K loop)
    static_assert(!PERSIST || NWAVES <= 4, "persistent launches are for 4-wave configurations");
    const int items = PERSIST ? p.persist_items : 0;            // > 0: a persistent launch
    const GemmArgs &p_launch = p;
    for (int round = 0;; ++round) {
    // Work item of this round.  An ordinary launch has one per work-group; a persistent one walks
    // items wg, wg + grid.x, ... in the same XCD-aware order (grid.x is a multiple of 8, so a
    // work-group stays on its XCD's part of the order).
    const bool persistent = items > 0;
    const int wg = (int)blockIdx.x + round * (int)gridDim.x;
    const bool has_tile = round == 0 || (PERSIST && wg < items);
    // Epilogues that run before anything of the next tile is touched: the LDS-staged ones (the ring
    // is their staging area) and the last tile's.
    if (round > 0 && (!has_tile || !e_in_regs)) {
        if (e_in_regs) epilogue(std::true_type{}); else epilogue(std::false_type{});
        owed = false;
        if (has_tile) __syncthreads();               // every wave has read its staging region back before the ring is refilled
    }
    if (!has_tile) break;
    // The tile's set-up reads the launch's parameters afresh (see fresh_args); the epilogue reads the
    // by-value copy, whose fields stay in registers across the K loop as far as it needs them.
    auto tile_args = [&]() __attribute__((always_inline)) -> GemmArgs { if constexpr (PERSIST) return fresh_args(); else return p_launch; };
    const GemmArgs p = tile_args();
    const bool gated = (p.act == ACT_SILU_GATE);
    const int nout = gated ? (p.N >> 1) : p.N;
    const bool partial = p.splits > 1 || p.out_f32;
    const int tid = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) + wave * 64;      // == threadIdx.x
    const int lane = tid & 63;
    const int r16 = lane & 15, q = lane >> 4;

    // Work-group -> tile (and, for a tile of the split tail, K range).  Tail work-groups are
    // numbered K range by K range, so that the work-groups holding a tile's last range - the ones
    // that wait for the others' partial sums - are dispatched after all they wait for.
    int tm, tn;
    const bool tail_mode = p.tail_g > 1;
    const bool in_tail = tail_mode && (int)blockIdx.x >= p.tail_first;
    int tail_tile = 0, tail_seg = 0;                 // tile number within the tail, K range number
    const int nz = persistent ? p.persist_z : (int)gridDim.z;
    int z = persistent ? 0 : (int)blockIdx.z;
    if (nz > 1) {
        // Split-K and batched launches: (K range or batch entry, tile) pairs in range-major order,
        // every XCD a contiguous run of them (the linear work-group id modulo 8 is the XCD).  The
        // tiles of one K range or batch entry then run side by side on one XCD and share its
        // operands through that XCD's L2.  With the plain grid.z mapping they sat on different
        // XCDs: 256 x 256 x 131072 on 128 x 256 tiles fetched B twice (202 MB of L2 fills against
        // 134 MB of operands), 128 x 512^3 on 256 x 256 tiles both operands twice (269 MB).
        const int tiles = p.tiles_m * p.tiles_n, total = tiles * nz;
        const int lin = persistent ? wg : (int)blockIdx.x + tiles * (int)blockIdx.z;
        const int qq = total >> 3, rem = total & 7, xcd = lin & 7, loc = lin >> 3;
        const int item = xcd * qq + (xcd < rem ? xcd : rem) + loc;
        z = item / tiles;
        tile_index_to_coords(p, item - z * tiles, tm, tn);
    } else if (!in_tail) {
        tile_coords(p, wg, tail_mode ? p.tail_first : p.tiles_m * p.tiles_n, tm, tn);
    } else {
        const int t_rem = p.tiles_m * p.tiles_n - p.tail_first;
        const int j = (int)blockIdx.x - p.tail_first;
        tail_seg = j / t_rem; tail_tile = j - tail_seg * t_rem;
        tile_index_to_coords(p, p.tail_first + tail_tile, tm, tn);
    }
    const int m0 = tm * BM;
    const int n0 = tn * (gated ? BN / 2 : BN);       // first OUTPUT column of this tile

    int k_begin = 0, k_end = p.K;
    int64_t batch_a = 0, batch_b = 0, batch_c = 0, batch_r = 0;
    if (in_tail) {
        const int steps = (p.K + BK - 1) / BK;
        k_begin = (int)((int64_t)tail_seg * steps / p.tail_g) * BK;
        const int e = (int)((int64_t)(tail_seg + 1) * steps / p.tail_g) * BK;
        k_end = e < p.K ? e : p.K;
    } else if (p.splits > 1) {
        k_begin = z * p.k_per_split;
        k_end = k_begin + p.k_per_split < p.K ? k_begin + p.k_per_split : p.K;
    } else {
        batch_a = z * p.stride_a; batch_b = z * p.stride_b;
        batch_c = z * p.stride_c; batch_r = z * p.stride_r;
    }
    const int klen = k_end - k_begin;
    const int ksteps = (klen + BK - 1) / BK;
    const int ktail = klen % BK;                     // > 0: the last step is partial

    // ---- global -> LDS direct loads ------------------------------------------------------
    // One wave-wide load moves 64 chunks (1 KB) to consecutive LDS addresses: lane l fills
    // physical chunk 64*block + l, so each lane fetches the global chunk that belongs there
    // under the swizzle.  A lane's byte offset is split into a per-lane part that is the same
    // for every load of an operand (one register) and a per-load block offset that is uniform
    // over the wave (scalar); K advances through the scalar offset (K-contiguous operands) or
    // the descriptor base (B, trans_b=0).  Rows past the matrix edge and K-rows past the K range
    // lie beyond the descriptor's num_records and chunks past the K range of the last step are
    // pushed there by an offset bit: the buffer hardware returns zero for all of them.
    //
    // The LDS address of such a load is M0 + immediate offset + 16*lane, and writing M0 costs
    // the wave about 8 cycles of matrix-pipe time.  A wave therefore fills runs of LOAD_RUN
    // consecutive blocks that share one M0 and differ in the immediate offset (< 4096).  The
    // immediate also counts towards the global address (measured, range check included); the
    // per-load offset takes it back, and every descriptor starts kOffBias bytes early (its
    // num_records that much larger) so that the offset never goes negative.
    auto clamp31 = [](int64_t v) -> uint32_t { return v > 0x7FFFFFFF ? 0x7FFFFFFFu : (uint32_t)v; };
    constexpr uint32_t kOffBias = 3072;
    constexpr auto run_of = [](int ld) { return ld % 4 == 0 ? 4 : ld % 3 == 0 ? 3 : ld % 2 == 0 ? 2 : 1; };
    constexpr int A_RUN = A_LD < 4 ? A_LD : run_of(A_LD), B_RUN = B_LD < 4 ? B_LD : run_of(B_LD);
    static_assert(A_LD % A_RUN == 0 && B_LD % B_RUN == 0, "loads split into whole runs");

    // K-contiguous rows: 8 rows x 8 chunks per load; lane -> row lane/8 of the block, chunk
    // (lane%8) ^ swz_k(row), the same in every block.
    const int kc_lane = (lane & 7) ^ swz_k(lane >> 3);
    const uint32_t tail_k = (ktail == 0 || kc_lane * 8 < ktail) ? 0u : kOobOffset;   // OR-ed in on the last step

    const int rows_a = (p.M - m0) < BM ? (p.M - m0) : BM;
    const char *base_a = (const char *)(p.A + batch_a + (int64_t)m0 * p.lda + k_begin) - kOffBias;
    const uint32_t nrec_a = clamp31((((int64_t)rows_a - 1) * p.lda + klen) * 2 + kOffBias);
    const __amdgpu_buffer_rsrc_t rsrc_a = __builtin_amdgcn_make_buffer_rsrc((void *)base_a, 0, nrec_a, kBufferFlags);
    const uint32_t a_lane = (uint32_t)(((int64_t)(lane >> 3) * p.lda + kc_lane * 8) * 2) + kOffBias;
    const uint32_t a_blk_bytes = (uint32_t)((int64_t)8 * p.lda * 2);            // bytes per 8-row block

    // B.  trans_b=1: as A, from rows of W.  Plain: LDS row r <-> output column n0 + r.  Gated:
    // the WTN rows a wave's fragments read hold its WTN/2 gate columns followed by the same
    // WTN/2 up columns (from B_up), so a wave's first NT/2 MFMA tiles are gate tiles and the last
    // NT/2 the matching up tiles.
    // trans_b=0: 64/NCH K-rows x NCH chunks per load; lane -> K-row lane/NCH, chunk
    // (lane%NCH) ^ swz_n(k); with fewer than 4 K-rows per load the swizzle, and with it the
    // per-lane part, alternates between loads (B_NV variants).
    constexpr int RPI = TRANS_B ? 8 : 64 / NCH;                            // rows per load
    constexpr int B_NV = TRANS_B ? 1 : (RPI >= 4 ? 1 : 4 / RPI);
    static_assert(TRANS_B || (64 % NCH == 0 && B_LD % B_NV == 0), "a load covers whole K-rows; swizzle variants cycle within a wave's loads");
    // One B descriptor per wave: in a gated launch the half (gate or up rows) a wave's loads fill
    // is the same for all of them, and so is the matrix they read.  The choice is made on the base
    // pointer, a scalar.
    constexpr int G = WTN / 16;                                            // 8-row blocks per half wave tile
    static_assert(!TRANS_B || G % B_LD == 0, "a wave's B loads lie inside one half of a wave tile");
    const char *base_b = nullptr, *base_b_up = nullptr;
    uint32_t nrec_b = 0;
    uint32_t b_lane[B_NV], b_blk_bytes;                                    // bytes per block of RPI rows
    const __bf16 *b_step_base = nullptr;             // trans_b=0: descriptor is rebuilt per step
    int64_t b_step_bytes = 0;
    if constexpr (TRANS_B) {
        const int ncols = gated ? nout : p.N;
        const int rows_b = (ncols - n0) < (gated ? BN / 2 : BN) ? (ncols - n0) : (gated ? BN / 2 : BN);
        nrec_b = clamp31((((int64_t)rows_b - 1) * p.ldb + klen) * 2 + kOffBias);
        base_b = (const char *)(p.B + batch_b + (int64_t)n0 * p.ldb + k_begin) - kOffBias;
        base_b_up = (const char *)((gated ? p.B_up : p.B) + batch_b + (int64_t)n0 * p.ldb + k_begin) - kOffBias;
        b_lane[0] = (uint32_t)(((int64_t)(lane >> 3) * p.ldb + kc_lane * 8) * 2) + kOffBias;
        b_blk_bytes = (uint32_t)((int64_t)8 * p.ldb * 2);
    } else {
        b_step_base = p.B + batch_b + (int64_t)k_begin * p.ldb + n0;
        b_step_bytes = (int64_t)BK * p.ldb * 2;
        base_b = base_b_up = (const char *)b_step_base - kOffBias;      // whole panel: used by the prefetch
        nrec_b = clamp31((((int64_t)klen - 1) * p.ldb + (p.N - n0)) * 2 + kOffBias);
        const int cols_b = (p.N - n0) < BN ? (p.N - n0) : BN;          // multiple of 8 on this path
#pragma unroll
        for (int v = 0; v < B_NV; ++v) {
            const int k_lane = v * RPI + lane / NCH;                   // K-row within a group of B_NV blocks
            const int nc = (lane % NCH) ^ swz_n<BN>(k_lane);
            const int cc = nc * 8 < cols_b ? nc * 8 : cols_b - 8;
            b_lane[v] = (uint32_t)(((int64_t)(lane / NCH) * p.ldb + cc) * 2) + kOffBias;
        }
        b_blk_bytes = (uint32_t)((int64_t)RPI * p.ldb * 2);
    }

    // gated: LDS block (2*wn + h)*G + x holds 8-row group x of half h (0: gate rows from B, 1: the up
    // rows of the same columns from B_up) of wave column wn; both halves read row block wn*G + x.
    // A wave fills blocks wave*B_LD .. wave*B_LD + B_LD - 1: inside one half when B_LD <= G.
    const int b_seg0 = (wave * B_LD) / G;
    const bool b_wave_up = TRANS_B && gated && B_LD <= G && (b_seg0 & 1);
    const __amdgpu_buffer_rsrc_t rsrc_bw = __builtin_amdgcn_make_buffer_rsrc((void *)wave_uniform(b_wave_up ? base_b_up : base_b), 0, wave_uniform(nrec_b), kBufferFlags);

    // ---- L2 prefetch ----------------------------------------------------------------------
    // The work-groups resident on one XCD at a time walk K in step, pf_sa of them sharing each A
    // row-panel and pf_sb each B column-panel.  One K step before a panel slab is loaded into LDS,
    // each of the sharers touches its share of the slab's 128-byte lines with a one-dword load
    // (into a sink behind the operand ring): the slab is then on its way into the XCD's L2 when
    // all of them ask for it, instead of every work-group waiting out the same miss.  First half
    // of the waves: A lines; second half: B lines; one load instruction per wave and K step.
    // Lines are prefetched for full steps inside the K range only, rows past an edge fall out
    // of the descriptor's range.
    uint32_t pf_voff = kOobOffset;
    uint32_t pf_step = 0;                                // byte advance per K step (scalar offset)
    const bool pf_is_a = wave < NWAVES / 2;
    bool pf_up = false;
    {
        constexpr int HT = NWAVES * 32;                   // threads per wave half
        constexpr int HT_LOG2 = NWAVES == 4 ? 7 : 8;
        static_assert((1 << HT_LOG2) == HT, "4 or 8 waves");
        const int hx = tid & (HT - 1);                    // index within the wave half
        // The sharer counts are powers of two (the host sees to that), so a share is L >> k lines of a
        // slab of L lines.  They are spread over the half's threads at a power-of-two stride, so that
        // every wave's load touches about the same number of lines; all of it in shifts (this runs
        // once per tile, on one wave per SIMD: the divisions it used to take were a third of the
        // 1.6 us between a work-group's start and its first load).
        auto pick = [&](auto l_tag, int k, int &li) __attribute__((always_inline)) {
            constexpr int L = decltype(l_tag)::value;
            constexpr int LC = L <= 16 ? 4 : L <= 32 ? 5 : L <= 64 ? 6 : L <= 128 ? 7 : 8;       // ceil(log2 L)
            static_assert(L >= 16 && L <= 256, "slab lines");
            const int sl = HT_LOG2 + k - LC;
            const int sh = sl > 0 ? sl : 0;
            li = hx >> sh;
            return (hx & ((1 << sh) - 1)) == 0 && li < (L >> k);
        };
        int li = 0;
        if (pf_is_a) {
            if (p.pf_sa > 0) {
                const int ka = __builtin_ctz((unsigned)p.pf_sa);
                if (pick(std::integral_constant<int, BM>{}, ka, li))
                    pf_voff = (uint32_t)((int64_t)((tn & (p.pf_sa - 1)) * (BM >> ka) + li) * p.lda * 2) + kOffBias;
            }
            pf_step = ROWB;
        } else if (p.pf_sb > 0) {
            const int kb = __builtin_ctz((unsigned)p.pf_sb);
            const int share = (tm % p.group_m) & (p.pf_sb - 1);
            if constexpr (TRANS_B) {
                bool mine;
                int row0;
                if (gated) {                              // shares alternate between the gate and the up rows
                    const int ks = kb > 0 ? kb - 1 : 0;
                    mine = pick(std::integral_constant<int, BN / 2>{}, ks, li);
                    row0 = (kb > 0 ? share >> 1 : 0) * ((BN / 2) >> ks); pf_up = (share & 1) != 0;
                } else {
                    mine = pick(std::integral_constant<int, BN>{}, kb, li);
                    row0 = share * (BN >> kb);
                }
                if (mine) pf_voff = (uint32_t)((int64_t)(row0 + li) * p.ldb * 2) + kOffBias;
                pf_step = ROWB;
            } else {
                constexpr int LPR = BN / 64;              // 128-byte lines per K-row of the slab
                if (pick(std::integral_constant<int, BN>{}, kb, li)) {
                    const int line = share * (BN >> kb) + li;
                    const int kr = line / LPR, col = (line % LPR) * 64;
                    if (col < p.N - n0) pf_voff = (uint32_t)(((int64_t)kr * p.ldb + col) * 2) + kOffBias;
                }
                pf_step = (uint32_t)b_step_bytes;         // the host enables this only if K * ldb * 2 < 2^31
            }
        }
    }
    const __amdgpu_buffer_rsrc_t rsrc_pf = __builtin_amdgcn_make_buffer_rsrc(
        (void *)wave_uniform(pf_is_a ? base_a : (pf_up ? base_b_up : base_b)), 0, wave_uniform(pf_is_a ? nrec_a : nrec_b), kBufferFlags);
    char *pf_sink = smem + lds_bytes(BM, BN, WGM, WGN, BK, STAGES) + wave * 256;
    const int pf_step_u = (int)wave_uniform(pf_step);          // the same in every lane: a scalar offset, no per-lane loop
    constexpr bool PF = has_prefetch(BM, BN, WGM, WGN, BK, STAGES);      // (without it there is no sink: nothing below may be issued)
    auto prefetch_step = [&](int step) __attribute__((always_inline)) {
        if constexpr (!PF) return;
        const uint32_t off = step < ksteps - 1 ? 0u : kOobOffset;
        const int st = step < ksteps - 1 ? step : 0;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_pf, FACT_LDS_PTR(pf_sink), 4, pf_voff | off, st * pf_step_u, 0, 0);
    };
    // The same inside the steady part of the K loop, without a per-lane operation: a step past the
    // range is clamped to the last one (a line touched twice costs an L2 hit; lines past a K range
    // or a matrix edge are outside the descriptor and touch nothing).
    auto prefetch_steady = [&](int step) __attribute__((always_inline)) {
        if constexpr (!PF) return;
        const int st = step < ksteps - 1 ? step : ksteps - 1;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_pf, FACT_LDS_PTR(pf_sink), 4, pf_voff, st * pf_step_u, 0, 0);
    };

    // The loads of K step `step` go to ring slot step % STAGES.  Every step index is legal: the
    // last step may be partial (its out-of-range chunks read as zero) and steps at or beyond
    // ksteps read nothing but zeros, so a phantom step adds exactly 0 to the accumulators and
    // the main loop needs no tail code.  Branch-free: setting the top offset bit puts a lane out
    // of the descriptor's range.
    struct StepCtx {
        char *s;
        uint32_t mask_k;          // per lane: out-of-range bit for K-contiguous operands
        uint32_t beyond;          // uniform: out-of-range bit of a phantom step
        int soff;
        __amdgpu_buffer_rsrc_t rb;
    };
    auto step_ctx = [&](int step, int slot) __attribute__((always_inline)) {
        StepCtx c;
        c.s = smem + slot * STAGE;
        c.beyond = step >= ksteps ? kOobOffset : 0u;
        c.mask_k = (step == ksteps - 1 ? tail_k : 0u) | c.beyond;
        const int st = step < ksteps ? step : 0;
        c.soff = st * ROWB;
        if constexpr (!TRANS_B) {
            const int ks = k_begin + st * BK;
            const int64_t rows_left = (int64_t)(k_end - 1 - ks);
            c.rb = __builtin_amdgcn_make_buffer_rsrc((void *)((const char *)b_step_base + st * b_step_bytes - kOffBias), 0,
                                                     clamp31((rows_left * p.ldb + (p.N - n0)) * 2 + kOffBias), kBufferFlags);
        } else {
            c.rb = rsrc_bw;
        }
        return c;
    };
    // load number idx of a step: 0 .. A_LD-1 fill the A part, A_LD .. LOADS-1 the B part.  Load i
    // of a wave fills LDS block wave * LD + i of the operand: run i / RUN, member i % RUN.
    auto issue_one = [&](const StepCtx &c, auto idx_) __attribute__((always_inline)) {
        constexpr int idx = decltype(idx_)::value;             // compile-time: it selects the immediate offset
        if constexpr (idx < A_LD) {
            constexpr int i = idx, run0 = (i / A_RUN) * A_RUN, t = i % A_RUN;
            const int blk = wave * A_LD + i;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, FACT_LDS_PTR(c.s + (wave * A_LD + run0) * 1024), 16,
                                                     a_lane + ((uint32_t)blk * a_blk_bytes - t * 1024) + c.mask_k, c.soff, t * 1024, 0);
        } else {
            constexpr int i = idx - A_LD, run0 = (i / B_RUN) * B_RUN, t = i % B_RUN;
            const int blk = wave * B_LD + i;
            char *dst = c.s + A_BYTES + (wave * B_LD + run0) * 1024;
            if constexpr (TRANS_B) {
                static_assert(!TRANS_B || B_LD <= G, "one descriptor per wave");
                const int seg = blk / G, x = blk % G;
                const uint32_t goff = (uint32_t)(gated ? (seg >> 1) * G + x : blk) * b_blk_bytes;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_bw, FACT_LDS_PTR(dst), 16,
                                                         b_lane[0] + (goff - t * 1024) + c.mask_k, c.soff, t * 1024, 0);
            } else {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(c.rb, FACT_LDS_PTR(dst), 16,
                                                         b_lane[i % B_NV] + ((uint32_t)blk * b_blk_bytes - t * 1024) + c.beyond, 0, t * 1024, 0);
            }
        }
    };

    // Steady part of the K loop (every step it loads is a whole step inside the K range): nothing
    // is computed per load.  Each load has its lane offset in a register of its own, fixed before
    // the loop; K advances through one scalar offset shared by the K-contiguous operands and, for a
    // [K][N] operand, through the descriptor's base (a 64-bit scalar add per step).  No range check
    // is needed there: every row of a steady step exists, and columns past the matrix edge were
    // clamped into it above.  The masked forms above serve the prologue and the last steps.
    uint32_t voff_a[A_LD], voff_b[B_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int blk = wave * A_LD + i, t = i % A_RUN;
        voff_a[i] = a_lane + ((uint32_t)blk * a_blk_bytes - t * 1024);
        asm volatile("" : "+v"(voff_a[i]));                    // kept in its register (not recomputed inside the loop)
    }
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int blk = wave * B_LD + i, t = i % B_RUN;
        if constexpr (TRANS_B) {
            const int seg = blk / G, x = blk % G;
            voff_b[i] = b_lane[0] + ((uint32_t)(gated ? (seg >> 1) * G + x : blk) * b_blk_bytes - t * 1024);
        } else {
            voff_b[i] = b_lane[i % B_NV] + ((uint32_t)blk * b_blk_bytes - t * 1024);
        }
        asm volatile("" : "+v"(voff_b[i]));
    }
    struct Steady {
        int koff;                          // byte offset of the step being loaded inside a K-contiguous row
        const char *bslab;                 // [K][N] operand: start of the step's slab (minus kOffBias)
        __amdgpu_buffer_rsrc_t rb;
    };
    auto steady_at = [&](int step) __attribute__((always_inline)) {
        Steady c;
        c.koff = step * ROWB;
        c.bslab = nullptr;
        c.rb = rsrc_bw;
        if constexpr (!TRANS_B) {
            c.bslab = (const char *)b_step_base + step * b_step_bytes - kOffBias;
            c.rb = __builtin_amdgcn_make_buffer_rsrc((void *)c.bslab, 0, 0x7FFFFFFF, kBufferFlags);
        }
        return c;
    };
    auto steady_next = [&](Steady &c) __attribute__((always_inline)) {
        c.koff += ROWB;
        if constexpr (!TRANS_B) {
            c.bslab += b_step_bytes;
            c.rb = __builtin_amdgcn_make_buffer_rsrc((void *)c.bslab, 0, 0x7FFFFFFF, kBufferFlags);
        }
    };
    auto issue_steady = [&](const Steady &c, char *stage, auto idx_) __attribute__((always_inline)) {
        constexpr int idx = decltype(idx_)::value;
        if constexpr (idx < A_LD) {
            constexpr int i = idx, run0 = (i / A_RUN) * A_RUN, t = i % A_RUN;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_a, FACT_LDS_PTR(stage + (wave * A_LD + run0) * 1024), 16, voff_a[i], c.koff, t * 1024, 0);
        } else {
            constexpr int i = idx - A_LD, run0 = (i / B_RUN) * B_RUN, t = i % B_RUN;
            char *dst = stage + A_BYTES + (wave * B_LD + run0) * 1024;
            if constexpr (TRANS_B) __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc_bw, FACT_LDS_PTR(dst), 16, voff_b[i], c.koff, t * 1024, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(c.rb, FACT_LDS_PTR(dst), 16, voff_b[i], 0, t * 1024, 0);
        }
    };

    // ---- fragment addresses ------------------------------------------------------------
    // MFMA 16x16x32 operand: lane holds row/column r16 = lane % 16 and the 8 K-values of K-group
    // q = lane / 16 of the sub-step.
    //  K-contiguous: one 128-bit read of chunk 4*kk + q of the lane's row.  The swizzle depends on
    //  r16 only, so one address per sub-step serves every MFMA tile through a constant offset.
    //  N-contiguous B: two transposing 64-bit reads.  Within a 16-lane group, lane 4*j + c
    //  supplies the address of K-row j, columns 4c..4c+3, and receives column (lane % 16) of
    //  K-rows 0..3: four consecutive K-values of its own column.  Sub-step and half select
    //  K-rows through constant offsets because the swizzle depends on k & 3 = j only.
    // trans_b=0: the swizzle XORs bits 1 and 2 of a K-row's chunk index, so two tiles whose chunk
    // indices differ only above bit 2 (4 tiles = 128 bytes apart) share one per-lane address and
    // differ by an immediate; wave tiles of fewer than 8 tiles keep one address per tile.
    constexpr int BF_N = NT >= 8 ? NT / 2 : NT;              // addresses kept
    constexpr int BF_STRIDE = NT >= 8 ? NT / 2 : NT;         // tile t uses address t % BF_STRIDE, immediate (t / BF_STRIDE) * BF_STRIDE * 32
    static_assert(TRANS_B || NT < 8 || (NT / 2) % 4 == 0, "paired tiles are a multiple of 128 bytes apart");
    uint32_t a_addr[KK], b_addr[KK], b_frag[BF_N];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const uint32_t ch = (uint32_t)(((4 * kk + q) ^ swz_k(r16)) << 4);
        a_addr[kk] = (uint32_t)((wm * WTM + r16) * ROWB) + ch;
        b_addr[kk] = (uint32_t)(A_BYTES + (wn * WTN + r16) * ROWB) + ch;
    }
#pragma unroll
    for (int t = 0; t < BF_N; ++t) {
        const int j = (lane >> 2) & 3, c = lane & 3;
        const int k = 8 * q + j;                                     // + 32*kk + 4*half
        const int n = wn * WTN + t * 16 + 4 * c;
        b_frag[t] = (uint32_t)(A_BYTES + k * (BN * 2) + ((((n >> 3) ^ swz_n<BN>(k))) << 4) + (c & 1) * 8);
    }

    // accumulator tile (mt, nt) is AccTile<mt * NT + nt>
    static_assert(MT * NT <= 64, "accumulator tiles");

    // A K step is consumed in U = KK * PH units: sub-step kk (32 K-values) x part h of the wave's
    // tile rows (MTH of them).  Register sets: two of MTH A fragments (alternating per unit), two
    // of NT B fragments (alternating per sub-step).  While the MFMAs of one unit run, the LDS
    // reads of the next unit fill the other A set and, when a new sub-step begins, the other B set.
    constexpr int PH = MT >= 4 ? 2 : 1;
    constexpr int MTH = MT / PH;
    constexpr int U = KK * PH;
    static_assert(U % 2 == 0 && KK % 2 == 0, "register sets alternate with period 2");
    bf16x8_t af[2][MTH], bf[2][NT];

    // Fragment read number t of unit u of the stage at s: its MTH A fragments, then (first part
    // of a sub-step only) the NT B fragments of the sub-step.
    auto read_one = [&](const char *s, int u, auto t_) __attribute__((always_inline)) {
        constexpr int t = decltype(t_)::value;                // compile-time: it selects an immediate offset
        const int kk = u / PH, h = u % PH;
        if constexpr (t < MTH) {
            af[u & 1][t] = *(const bf16x8_t *)(s + a_addr[kk] + (h * MTH + t) * 16 * ROWB);
        } else {
            constexpr int nt = t - MTH;
            if constexpr (TRANS_B) {
                bf[kk & 1][nt] = *(const bf16x8_t *)(s + b_addr[kk] + nt * 16 * ROWB);
            } else {
                // Inline asm, not the builtin: the compiler cannot tell that these LDS reads do not
                // alias the global->LDS loads in flight and would wait for all of them (vmcnt(0))
                // before every read.  The price: it does not track these reads either, so the
                // consumer waits explicitly (wait_frags below), and a build whose register
                // allocation spills is refused (a spill could store a register before its data
                // has arrived).
                const uint32_t a = (uint32_t)(size_t)FACT_LDS_PTR(s + b_frag[nt % BF_STRIDE]) + kk * 32 * (BN * 2);
                s16x4_t lo, hi;
                asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(a), "n"((nt / BF_STRIDE) * BF_STRIDE * 32));
                asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a), "n"((nt / BF_STRIDE) * BF_STRIDE * 32 + 4 * (BN * 2)));
                typedef short s16x8_t __attribute__((ext_vector_type(8)));
                const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                bf[kk & 1][nt] = __builtin_bit_cast(bf16x8_t, both);
            }
        }
    };
    // trans_b=0 only: all LDS reads issued so far have returned; the fragment registers are
    // operands so that no MFMA using them can be scheduled above the wait.
    auto wait_frags = [&](int set) __attribute__((always_inline)) {
        if constexpr (!TRANS_B) {
            static_assert(TRANS_B || NT == 2 || NT == 4 || NT == 8, "operand lists below");
            if constexpr (NT == 8)
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[set][0]), "+v"(bf[set][1]), "+v"(bf[set][2]), "+v"(bf[set][3]),
                                                      "+v"(bf[set][4]), "+v"(bf[set][5]), "+v"(bf[set][6]), "+v"(bf[set][7]));
            else if constexpr (NT == 4)
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[set][0]), "+v"(bf[set][1]), "+v"(bf[set][2]), "+v"(bf[set][3]));
            else
                asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bf[set][0]), "+v"(bf[set][1]));
        }
    };
    // MFMA number idx of unit u.  The tiles of a unit are walked column by column, up one column and
    // down the next, so that consecutive MFMAs share one operand: the B fragment for a whole column,
    // the A fragment across a column change.  The chip is power-limited under this load, and the
    // order is worth 1-1.8 % on 8192^3 against row by row from the left (same-box A/B: [K][N]
    // 1556 -> 1571, [N][K] 1556 -> 1582 TFLOP/s; rows walked to and fro: 1567 / 1569; columns always
    // from the top: no gain).
    // Operand order (B fragment first) makes the accumulator tile hold D[n_local][m_local]:
    // lane (r16, q) owns output row r16 and the 4 consecutive output columns 4q .. 4q+3.
    constexpr int NMFMA = MTH * NT;
    auto mfma_one = [&](auto u_, auto idx_) __attribute__((always_inline)) {
        constexpr int u = decltype(u_)::value, idx = decltype(idx_)::value;     // compile-time: they name the accumulator's registers
        constexpr int kk = u / PH, h = u % PH;
        constexpr int nt = idx / MTH, x = (nt & 1) ? MTH - 1 - idx % MTH : idx % MTH;
        if constexpr (F16) AccTile<(h * MTH + x) * NT + nt>::mfma_f16(bf[kk & 1][nt], af[u & 1][x]);
        else AccTile<(h * MTH + x) * NT + nt>::mfma(bf[kk & 1][nt], af[u & 1][x]);
    };

    // ---- main loop -----------------------------------------------------------------------
    // Ring of STAGES slots; step kt lives in slot kt % STAGES.  The loop body for step kt starts
    // right after a barrier that guarantees (a) step kt has landed in LDS for the whole
    // work-group and (b) every wave has read its last fragments of step kt-1, so slot
    // (kt-1) % STAGES is free.  The body runs U phases of MTH*NT MFMAs:
    //   phase 0      : MFMAs of the LAST unit of step kt-1 (fragments already in registers),
    //                  while the fragments of unit 0 of step kt are read;
    //   phase j >= 1 : MFMAs of unit j-1 of step kt, while unit j is read.
    // The global->LDS loads of step kt+STAGES-1 (into the freed slot) are spread over the step's
    // MFMAs.  The body ends with: wait for step kt+1 (all but the
    // newest STAGES-2 steps' loads done) and for this wave's LDS reads; barrier.
    // Before the first body the "previous last unit" fragments are zero, after the last body
    // one more MFMA phase drains the real last unit.  Every body issues the same number of
    // loads (phantom, all-zero ones past the K range), so the wait count is the same throughout.
    // Instruction issue is in order and a 16x16x32 MFMA occupies the matrix pipe for only 16
    // cycles, so the LDS reads of a phase are spread evenly over the first 7/8 of its MFMAs, with
    // a scheduling fence after every MFMA to keep every memory instruction where it was put.
    // every step's loads are followed by one prefetch load; a wave may leave outstanding the
    // newest STAGES-2 such groups and the prefetch behind the group it waits for
    constexpr int WAIT_N = (STAGES - 2) * (LOADS + (PF ? 1 : 0)) + (PF ? 1 : 0);
    // The address unit is shared by the CU's waves and takes one wave-wide load per 16 cycles, so a
    // step's loads are spread evenly: over the first half of the step's MFMAs with a two-slot
    // ring (they must have landed by its end: a step of such a ring lasts about as long as the loads'
    // latency, so the last load's issue time adds to it), over nearly all of it with a deeper ring.
    // Same-box A/B of the two-slot span, 3/4 -> 1/2: 2048 x 6144 x 4096 on 256 x 192 tiles 72.6 -> 70.3 us
    // (operands from HBM 79.7 -> 76.6), 8192^3 from HBM 713.7 -> 700.8 us, from the memory-side cache
    // unchanged; 3/8 and 1/4 are slower again (address-unit contention stalls the matrix pipe).  Deeper
    // rings: 15/16, 3/4 and 1/2 measure the same or worse in that order.
    constexpr int TG = U * NMFMA;                        // MFMAs (= gaps) per K step
    constexpr int LOAD_SPAN = STAGES > 2 ? (TG * 15) / 16 : TG / 2;
    auto load_gap = [](int l) constexpr { const int g = 1 + (l * LOAD_SPAN) / LOADS; return g < TG ? g : TG - 1; };
    constexpr int SPAN = (NMFMA * 7) / 8 > 0 ? (NMFMA * 7) / 8 : 1;
    Steady sc = steady_at(STAGES - 1);
    auto body = [&](int kt, auto slot_tag, auto steady_tag) __attribute__((always_inline)) {
        constexpr int SLOT = decltype(slot_tag)::value;            // kt % STAGES, known at compile time
        constexpr bool STEADY = decltype(steady_tag)::value;       // the step loaded here is a whole one inside the K range
        constexpr int LSLOT = (SLOT + STAGES - 1) % STAGES;
        StepCtx c;
        if constexpr (!STEADY) c = step_ctx(kt + STAGES - 1, LSLOT);
        char *lstage = smem + LSLOT * STAGE;
        const char *s = smem + SLOT * STAGE;
        static_for<U>([&](auto j_) __attribute__((always_inline)) {
            constexpr int j = decltype(j_)::value;
            constexpr int cu = (j + U - 1) % U;                    // the unit the MFMAs consume
            constexpr int nreads = MTH + (j % PH == 0 ? NT : 0);
            wait_frags((cu / PH) & 1);
            static_for<NMFMA>([&](auto i_) __attribute__((always_inline)) {
                constexpr int i = decltype(i_)::value;
                static_for<nreads>([&](auto t_) __attribute__((always_inline)) {
                    constexpr int t = decltype(t_)::value;
                    if constexpr ((t * SPAN) / nreads == i) read_one(s, j, t_);
                });
                static_for<LOADS>([&](auto l_) __attribute__((always_inline)) {
                    constexpr int l = decltype(l_)::value;
                    if constexpr (load_gap(l) == j * NMFMA + i) {
                        if constexpr (STEADY) issue_steady(sc, lstage, l_); else issue_one(c, l_);
                    }
                });
                if constexpr (load_gap(LOADS - 1) == j * NMFMA + i) {
                    if constexpr (STEADY) { prefetch_steady(kt + STAGES - 1 + p.pf_dist); steady_next(sc); }
                    else prefetch_step(kt + STAGES - 1 + p.pf_dist);
                }
                mfma_one(std::integral_constant<int, cu>{}, i_);
                __builtin_amdgcn_sched_barrier(0);
            });
        });
        wait_loads_and_barrier<WAIT_N>();
    };

    // The prefetch behind the loads of step x covers step x + pf_dist; the steps between the
    // prologue's loads and the first of those are touched here, ahead of the loads (older than
    // them, so the wait counts are unaffected).
    if constexpr (PF)
        for (int x = STAGES - 1; x < p.pf_dist; ++x) prefetch_step(x);
    if (ksteps >= STAGES) {
        // every step of the prologue is a whole step inside the K range: the steady form of the loads
        // (offsets already in registers) instead of some fifteen instructions of range arithmetic per load
        static_for<STAGES - 1>([&](auto s_) __attribute__((always_inline)) {
            constexpr int s = decltype(s_)::value;
            const Steady c = steady_at(s);
            static_for<LOADS>([&](auto i_) __attribute__((always_inline)) { issue_steady(c, smem + s * STAGE, i_); });
            prefetch_steady(s + p.pf_dist);
        });
    } else {
        static_for<STAGES - 1>([&](auto s_) __attribute__((always_inline)) {
            constexpr int s = decltype(s_)::value;
            const StepCtx c = step_ctx(s, s);
            static_for<LOADS>([&](auto i_) __attribute__((always_inline)) { issue_one(c, i_); });
            prefetch_step(s + p.pf_dist);
        });
    }
    // The previous tile's register epilogue, while this tile's first stages are on their way.  Its
    // loads and stores are younger than those stages' loads, and the wait counts of the K loop
    // assume that nothing else is outstanding: wait for all of it (the stores have left within
    // ~0.3 us of the last one; the stages were requested before the epilogue began).
    if (owed) {
        epilogue(std::true_type{});
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        owed = false;
    }
    // ---- what this tile's epilogue will need (the previous tile's has run by now) -----------------
    auto hand_over = [&]() __attribute__((always_inline)) {
        e_tm = tm; e_tn = tn; e_z = z;
        e_in_tail = in_tail; e_tail_seg = tail_seg; e_tail_tile = tail_tile;
        // register epilogue: the whole tile inside C, bf16 output, no hand-over; gated tiles only where a
        // wave's output tiles pair up
        // (the same answer in every wave of the work-group: the two kinds of epilogue meet different
        // barriers and run at different points of a persistent work-group's loop)
        const bool inside = m0 + BM <= p_launch.M && n0 + (gated ? BN / 2 : BN) <= nout;
        e_in_regs = !partial && p_launch.vec_store && inside && !in_tail && !p_launch.c_f32 && (!gated || NT % 4 == 0);
    };
    // (a persistent work-group sets these before the K loop, so that nothing of the tile's set-up is needed after
    // it; an ordinary one after it, where its 8-wave form has the registers)
    if constexpr (PERSIST) hand_over();
    // accumulators and the "previous last unit" fragments start from zero
    static_for<MT * NT>([&](auto t_) __attribute__((always_inline)) { AccTile<decltype(t_)::value>::zero(); });
#pragma unroll
    for (int x = 0; x < MTH; ++x)
#pragma unroll
        for (int e = 0; e < 8; ++e) af[(U - 1) & 1][x][e] = (__bf16)0.0f;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int e = 0; e < 8; ++e) bf[(KK - 1) & 1][nt][e] = (__bf16)0.0f;
    wait_loads_and_barrier<WAIT_N>();
    // Unrolled over the ring so that each body knows its slot.  Rounds whose loads are all whole
    // steps inside the K range (the last body of a round loads step kt + 2 STAGES - 2) run the
    // steady form; the remaining rounds the masked one, where an incomplete last round runs phantom
    // (all-zero) steps.
    int kt = 0;
    for (; kt + 2 * STAGES - 1 < ksteps; kt += STAGES) {
        static_for<STAGES>([&](auto s_) __attribute__((always_inline)) { body(kt + decltype(s_)::value, s_, std::true_type{}); });
    }
    for (; kt < ksteps; kt += STAGES) {
        static_for<STAGES>([&](auto s_) __attribute__((always_inline)) { body(kt + decltype(s_)::value, s_, std::false_type{}); });
    }
    // drain: the last unit of the last step
    wait_frags((KK - 1) & 1);
    static_for<NMFMA>([&](auto i_) __attribute__((always_inline)) { mfma_one(std::integral_constant<int, U - 1>{}, i_); });
    // The compiler does not see the MFMAs inside the asm statements, so it cannot pad the gap the
    // hardware needs between a matrix instruction and the first ordinary read of its result.
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // phantom loads still target LDS

    // (From here to the end of the item the launch's parameters are read from the by-value copy, as in the
    // epilogue: the set-up's own copy of them is then dead before the K loop.)
    // ---- split tail: hand over or collect partial sums ------------------------------------------
    // A tile of the tail is accumulated by tail_g work-groups, one K range each.  All but the last
    // store their accumulators as an fp32 tile (row-major, through the epilogue's LDS transpose)
    // and then raise a flag; the last one waits for the flags and adds the partial tiles, in
    // ascending K-range order, to its own sums as it reads them back in the epilogue.  The order is
    // fixed, so the result is bit-reproducible.  Producers never wait and are dispatched before the
    // work-group that waits for them; the wait is bounded all the same (what a wait that gives
    // up does is described below).
    // The partners may sit on different XCDs, whose L2 caches are not coherent with each other.
    // Partial tiles and flags therefore move with system-scope accesses (write-through stores,
    // cache-bypassing loads): a cache-wide write-back and invalidate around the hand-over, which is
    // what a device-scope fence amounts to here, was measured to cost more than the split saves.
    const int tail_parts = in_tail ? p_launch.tail_g - 1 : 0;
    const bool tail_producer = in_tail && tail_seg < tail_parts;
    // A wait that gives up is an error, never a quietly wrong tile: the work-group then writes NaN to
    // every element of its tile and stores the launch's epoch into the workspace's status word,
    // which fact_tail_timeouts reads.  (Every thread learns of it through a word of the first
    // wave's prefetch sink: the operand stages may still be read by slower waves.)
    tail_gave_up = false;
    if (PF && in_tail && !tail_producer) {          // (the host never splits the tail of a configuration without a sink)
        unsigned long long *flags = p_launch.tail_flags + (int64_t)tail_tile * tail_parts;
        volatile int *verdict = (volatile int *)(smem + lds_bytes(BM, BN, WGM, WGN, BK, STAGES));
        const int tid = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u)) + wave * 64;      // (derived anew: not kept across the K loop)
        if (tid == 0) {
            int budget = p_launch.tail_budget;
            bool gave_up = budget < 0;
            for (int sgm = 0; sgm < tail_parts && !gave_up; ++sgm)
                while (__hip_atomic_load(flags + sgm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM) != p_launch.tail_epoch) {
                    if (budget <= 0) { gave_up = true; break; }
                    __builtin_amdgcn_s_sleep(8);
                    --budget;
                }
            if (gave_up) __hip_atomic_store(p_launch.tail_status, p_launch.tail_epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
            *verdict = gave_up ? 1 : 0;
        }
        __syncthreads();
        tail_gave_up = *verdict != 0;
    }

    if constexpr (!PERSIST) hand_over();
    owed = true;
    if constexpr (!PERSIST) {                        // one item per work-group: straight to its epilogue (no loop for the compiler to carry state around)
        if (e_in_regs) epilogue(std::true_type{}); else epilogue(std::false_type{});
        break;
    }
    }   // next work item

#else
    (void)p;
#endif
}

}  // namespace fact
