// Split-K reduction pass with the fused epilogue, and the guarded fallback GEMM for
// shapes the MFMA path does not take (unaligned pointers or dimensions).
#include "launch.h"

namespace fact {

// 16-bit pattern <-> fp32 in the launch's format (these kernels are bound by memory traffic: a run-time choice)
__device__ __forceinline__ float in16_rt(int f16, uint32_t bits) { return f16 ? f16_bits_to_f32(bits) : bf16_bits_to_f32(bits); }
__device__ __forceinline__ uint32_t out16_rt(int f16, float x) { return f16 ? f32_to_f16_bits(x) : f32_to_bf16_bits(x); }

// ---- split-K reduction -----------------------------------------------------------------
// P holds `splits` fp32 partial products [M][N].  A lane owns 4 consecutive output columns of
// one row; the W waves of a work-group own the same 64 such column groups and a W-th of the K
// ranges each (consecutive ranges, added in ascending order); the W sums are then added in
// ascending order by the first wave, which applies the epilogue and rounds once.  W depends on
// the problem's M, N and number of ranges only (reduce_waves below), so the order of additions is
// fixed for a given problem and the result is bit-reproducible.  Many ranges of a small output want W = 8 (one wave
// per column group adding all ranges in turn was bound by its trips to memory: 8.5 us for the
// 17 MB of 64 ranges of a 256 x 256 output, whatever the number of loads in flight per wave);
// few ranges of a large output want W = 1 (with W = 8 six of the eight waves idled and every
// 64 column groups paid two barriers: 61 us for 2 ranges of a 256 x 8192 output).  The paper's
// counterpart is the fix-up step of its Stream-K schedule (Section 5.2.3).
template <int kReduceWaves>
__global__ void __launch_bounds__(64 * kReduceWaves) splitk_reduce_kernel(const GemmArgs p)
{
    __shared__ float part[kReduceWaves > 1 ? kReduceWaves - 1 : 1][2][4][64];        // sums of waves 1..: [wave-1][gate|up][column][lane]
    const bool gated = p.act == ACT_SILU_GATE;
    const int nout = gated ? (p.N >> 1) : p.N;
    const int groups = (nout + 3) >> 2;
    const int64_t total = (int64_t)p.M * groups;
    const int64_t plane = (int64_t)p.M * p.N;
    const bool vec_p = (p.N & 3) == 0 && (!gated || (nout & 3) == 0);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int per = (p.splits + kReduceWaves - 1) / kReduceWaves;      // K ranges per wave
    const int s_begin = wave * per < p.splits ? wave * per : p.splits;
    const int s_end = s_begin + per < p.splits ? s_begin + per : p.splits;
    for (int64_t t0 = (int64_t)blockIdx.x * 64; t0 < total; t0 += (int64_t)gridDim.x * 64) {
        const int64_t t = t0 + lane;
        const bool live = t < total;
        int m = 0, n = 0;
        if (live) {
            if (total <= 0x7FFFFFFF) { m = (int)((uint32_t)t / (uint32_t)groups); n = (int)((uint32_t)t - (uint32_t)m * (uint32_t)groups) * 4; }
            else { m = (int)(t / groups); n = (int)(t % groups) * 4; }
        }
        float v[4] = {0.f, 0.f, 0.f, 0.f}, u[4] = {0.f, 0.f, 0.f, 0.f};
        const float *src = p.P + (int64_t)m * p.N + n + (int64_t)s_begin * plane;
        const bool full = n + 3 < nout;
        const int cnt = live ? s_end - s_begin : 0;
        if (full && vec_p) {
            // whole batches with every load issued before the first add, then the rest one by one
            constexpr int NB = 8;
            int s0 = 0;
            for (; s0 + NB <= cnt; s0 += NB) {
                f32x4_t a[NB], b[NB];
#pragma unroll
                for (int j = 0; j < NB; ++j) a[j] = *(const f32x4_t *)(src + (s0 + j) * plane);
                if (gated) {
#pragma unroll
                    for (int j = 0; j < NB; ++j) b[j] = *(const f32x4_t *)(src + (s0 + j) * plane + nout);
                }
#pragma unroll
                for (int j = 0; j < NB; ++j) { v[0] += a[j].x; v[1] += a[j].y; v[2] += a[j].z; v[3] += a[j].w; }
                if (gated) {
#pragma unroll
                    for (int j = 0; j < NB; ++j) { u[0] += b[j].x; u[1] += b[j].y; u[2] += b[j].z; u[3] += b[j].w; }
                }
            }
            for (; s0 < cnt; ++s0) {
                const f32x4_t a = *(const f32x4_t *)(src + s0 * plane);
                v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
                if (gated) { const f32x4_t b = *(const f32x4_t *)(src + s0 * plane + nout); u[0] += b.x; u[1] += b.y; u[2] += b.z; u[3] += b.w; }
            }
        } else {
            for (int s0 = 0; s0 < cnt; ++s0)
                for (int e = 0; e < 4; ++e)
                    if (n + e < nout) {
                        v[e] += src[s0 * plane + e];
                        if (gated) u[e] += src[s0 * plane + nout + e];
                    }
        }
        if (kReduceWaves > 1) {
            if (wave > 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) { part[wave - 1][0][e][lane] = v[e]; part[wave - 1][1][e][lane] = u[e]; }
            }
            __syncthreads();
        }
        if (wave == 0 && live) {
#pragma unroll
            for (int w = 0; w < kReduceWaves - 1; ++w)
#pragma unroll
                for (int e = 0; e < 4; ++e) { v[e] += part[w][0][e][lane]; u[e] += part[w][1][e][lane]; }
            for (int e = 0; e < 4; ++e) {
                if (n + e >= nout) continue;
                float zv = v[e];
                if (gated) zv = silu(zv) * u[e];
                if (p.bias) zv += in16_rt(p.f16, ((const uint16_t *)p.bias)[n + e]);
                if (p.act == ACT_GELU_TANH) zv = gelu_tanh(zv);
                if (p.res) zv += in16_rt(p.f16, ((const uint16_t *)p.res)[(int64_t)m * p.ldr + n + e]);
                v[e] = zv;
            }
            if (p.out_f32) {                                   // fp32 output: no rounding at all
                float *cf = (float *)p.C + (int64_t)m * p.ldc + n;
                if (full && p.vec_store) {
                    *(f32x4_t *)cf = f32x4_t{v[0], v[1], v[2], v[3]};
                } else {
                    for (int e = 0; e < 4; ++e)
                        if (n + e < nout) cf[e] = v[e];
                }
            } else {
                __bf16 *cp = p.C + (int64_t)m * p.ldc + n;
                if (full && p.vec_store) {
                    *(u32x2_t *)cp = u32x2_t{out16_rt(p.f16, v[0]) | (out16_rt(p.f16, v[1]) << 16), out16_rt(p.f16, v[2]) | (out16_rt(p.f16, v[3]) << 16)};
                } else {
                    uint16_t *cs = (uint16_t *)cp;
                    for (int e = 0; e < 4; ++e)
                        if (n + e < nout) cs[e] = (uint16_t)out16_rt(p.f16, v[e]);
                }
            }
        }
        if (kReduceWaves > 1) __syncthreads();                 // the waves' sums are read before the next round overwrites them
    }
}

// Waves that share a column group's K ranges: as many (1, 2, 4 or 8) as it takes to have some 2048 waves
// at work, each with at least four ranges.  A function of the problem alone (M, N, split factor).
static int reduce_waves(int splits, int64_t blocks)
{
    int w = 1;
    while (w < 8 && blocks * w < 2048 && splits >= 8 * w) w *= 2;
    return w;
}

hipError_t launch_splitk_reduce(const GemmArgs &args, hipStream_t stream)
{
    const int nout = args.act == ACT_SILU_GATE ? args.N / 2 : args.N;
    const int64_t total = (int64_t)args.M * ((nout + 3) / 4);
    // 64 column groups per work-group: even a 256 x 256 output spreads over all CUs
    int64_t blocks = (total + 63) / 64;
    if (blocks > 256 * 256) blocks = 256 * 256;
    switch (reduce_waves(args.splits, (total + 63) / 64)) {
    case 8: hipLaunchKernelGGL(splitk_reduce_kernel<8>, dim3((unsigned)blocks), dim3(512), 0, stream, args); break;
    case 4: hipLaunchKernelGGL(splitk_reduce_kernel<4>, dim3((unsigned)blocks), dim3(256), 0, stream, args); break;
    case 2: hipLaunchKernelGGL(splitk_reduce_kernel<2>, dim3((unsigned)blocks), dim3(128), 0, stream, args); break;
    default: hipLaunchKernelGGL(splitk_reduce_kernel<1>, dim3((unsigned)blocks), dim3(64), 0, stream, args); break;
    }
    return hipGetLastError();
}

// ---- guarded fallback ---------------------------------------------------------------------
// One thread per output element, ascending-k fp32 FMA.  No alignment or divisibility
// requirement; every access is bounds-guarded.  Slow by design: it exists so that no
// shape is silently wrong or rejected.
template <bool TRANS_B>
__global__ void __launch_bounds__(256) fallback_gemm_kernel(const GemmArgs p)
{
    const bool gated = p.act == ACT_SILU_GATE;
    const int nout = gated ? (p.N >> 1) : p.N;
    const int tiles_n = (nout + 15) >> 4;
    const int n = (int)(blockIdx.x % tiles_n) * 16 + (threadIdx.x & 15);
    const int m = (int)(blockIdx.x / tiles_n) * 16 + (threadIdx.x >> 4);
    const int z = blockIdx.z;
    if (m >= p.M || n >= nout) return;
    const uint16_t *A = (const uint16_t *)(p.A + z * p.stride_a) + (int64_t)m * p.lda;
    const uint16_t *B = (const uint16_t *)(p.B + z * p.stride_b);
    float acc = 0.f, acc_up = 0.f;
    if (TRANS_B) {
        const uint16_t *w = B + (int64_t)n * p.ldb;
        const uint16_t *wu = gated ? (const uint16_t *)(p.B_up + z * p.stride_b) + (int64_t)n * p.ldb : nullptr;
        for (int k = 0; k < p.K; ++k) {
            const float a = in16_rt(p.f16, A[k]);
            acc = __builtin_fmaf(a, in16_rt(p.f16, w[k]), acc);
            if (gated) acc_up = __builtin_fmaf(a, in16_rt(p.f16, wu[k]), acc_up);
        }
    } else {
        for (int k = 0; k < p.K; ++k)
            acc = __builtin_fmaf(in16_rt(p.f16, A[k]), in16_rt(p.f16, B[(int64_t)k * p.ldb + n]), acc);
    }
    float zv = acc;
    if (gated) zv = silu(zv) * acc_up;
    if (p.bias) zv += in16_rt(p.f16, ((const uint16_t *)p.bias)[n]);
    if (p.act == ACT_GELU_TANH) zv = gelu_tanh(zv);
    if (p.res) zv += in16_rt(p.f16, ((const uint16_t *)(p.res + z * p.stride_r))[(int64_t)m * p.ldr + n]);
    ((uint16_t *)(p.C + z * p.stride_c))[(int64_t)m * p.ldc + n] = (uint16_t)out16_rt(p.f16, zv);
}

hipError_t launch_fallback_gemm(const GemmArgs &args, bool trans_b, int grid_z, hipStream_t stream)
{
    const int nout = args.act == ACT_SILU_GATE ? args.N / 2 : args.N;
    const int64_t blocks = (int64_t)((nout + 15) / 16) * ((args.M + 15) / 16);
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidConfiguration;
    dim3 grid((unsigned)blocks, 1, (unsigned)grid_z);
    if (trans_b)
        hipLaunchKernelGGL(fallback_gemm_kernel<true>, grid, dim3(256), 0, stream, args);
    else
        hipLaunchKernelGGL(fallback_gemm_kernel<false>, grid, dim3(256), 0, stream, args);
    return hipGetLastError();
}

}  // namespace fact
