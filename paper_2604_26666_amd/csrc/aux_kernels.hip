// Split-K reduction pass with the fused epilogue, and the guarded fallback GEMM for
// shapes the MFMA path does not take (unaligned pointers or dimensions).
#include "launch.h"

namespace fact {

// ---- split-K reduction -----------------------------------------------------------------
// P holds `splits` fp32 partial products [M][N].  Each thread owns 4 consecutive output
// columns of one row, adds the partials in ascending split order (fixed order, so the
// result is bit-reproducible), applies the epilogue and rounds once.  The paper's
// counterpart is the fix-up step of its Stream-K schedule (Section 5.2.3).
__global__ void __launch_bounds__(64) splitk_reduce_kernel(const GemmArgs p)
{
    const bool gated = p.act == ACT_SILU_GATE;
    const int nout = gated ? (p.N >> 1) : p.N;
    const int groups = (nout + 3) >> 2;
    const int64_t total = (int64_t)p.M * groups;
    const int64_t plane = (int64_t)p.M * p.N;
    const bool vec_p = (p.N & 3) == 0 && (!gated || (nout & 3) == 0);
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        const int m = (int)(t / groups);
        const int n = (int)(t % groups) * 4;
        float v[4] = {0.f, 0.f, 0.f, 0.f}, u[4] = {0.f, 0.f, 0.f, 0.f};
        const float *src = p.P + (int64_t)m * p.N + n;
        const bool full = n + 3 < nout;
        if (full && vec_p) {
            // batches of 8 partials: all loads of a batch are issued before the first add, the adds
            // keep the ascending split order
            for (int s0 = 0; s0 < p.splits; s0 += 8) {
                f32x4_t a[8], b[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (s0 + j < p.splits) {
                        a[j] = *(const f32x4_t *)(src + (s0 + j) * plane);
                        if (gated) b[j] = *(const f32x4_t *)(src + (s0 + j) * plane + nout);
                    }
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (s0 + j < p.splits) {
                        v[0] += a[j].x; v[1] += a[j].y; v[2] += a[j].z; v[3] += a[j].w;
                        if (gated) { u[0] += b[j].x; u[1] += b[j].y; u[2] += b[j].z; u[3] += b[j].w; }
                    }
                }
            }
        } else {
            for (int s = 0; s < p.splits; ++s)
                for (int e = 0; e < 4; ++e)
                    if (n + e < nout) {
                        v[e] += src[s * plane + e];
                        if (gated) u[e] += src[s * plane + nout + e];
                    }
        }
        for (int e = 0; e < 4; ++e) {
            if (n + e >= nout) continue;
            float zv = v[e];
            if (gated) zv = silu(zv) * u[e];
            if (p.bias) zv += (float)p.bias[n + e];
            if (p.act == ACT_GELU_TANH) zv = gelu_tanh(zv);
            if (p.res) zv += (float)p.res[(int64_t)m * p.ldr + n + e];
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
            continue;
        }
        __bf16 *cp = p.C + (int64_t)m * p.ldc + n;
        if (full && p.vec_store) {
            *(u32x2_t *)cp = pack4_bf16(v[0], v[1], v[2], v[3]);
        } else {
            uint16_t *cs = (uint16_t *)cp;
            for (int e = 0; e < 4; ++e)
                if (n + e < nout) cs[e] = (uint16_t)f32_to_bf16_bits(v[e]);
        }
    }
}

hipError_t launch_splitk_reduce(const GemmArgs &args, hipStream_t stream)
{
    const int nout = args.act == ACT_SILU_GATE ? args.N / 2 : args.N;
    const int64_t total = (int64_t)args.M * ((nout + 3) / 4);
    // one-wave work-groups: even a 256 x 256 output spreads over all CUs
    int64_t blocks = (total + 63) / 64;
    if (blocks > 256 * 256) blocks = 256 * 256;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)blocks), dim3(64), 0, stream, args);
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
            const float a = bf16_bits_to_f32(A[k]);
            acc = __builtin_fmaf(a, bf16_bits_to_f32(w[k]), acc);
            if (gated) acc_up = __builtin_fmaf(a, bf16_bits_to_f32(wu[k]), acc_up);
        }
    } else {
        for (int k = 0; k < p.K; ++k)
            acc = __builtin_fmaf(bf16_bits_to_f32(A[k]), bf16_bits_to_f32(B[(int64_t)k * p.ldb + n]), acc);
    }
    float zv = acc;
    if (gated) zv = silu(zv) * acc_up;
    if (p.bias) zv += (float)p.bias[n];
    if (p.act == ACT_GELU_TANH) zv = gelu_tanh(zv);
    if (p.res) zv += (float)(p.res + z * p.stride_r)[(int64_t)m * p.ldr + n];
    ((uint16_t *)(p.C + z * p.stride_c))[(int64_t)m * p.ldc + n] = (uint16_t)f32_to_bf16_bits(zv);
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
