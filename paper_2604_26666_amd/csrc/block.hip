// The pieces of a transformer block around attention and the feed-forward network - LayerNorm /
// RMSNorm and the rotary embedding, two small memory-bound kernels - and the composition of the
// whole block from this library's entry points.  The paper composes its patterns into one module
// that keeps the sub-graph's interface (Section 4.3) and evaluates two blocks (Section 5.1: a
// GPT-style block with LayerNorm and GELU, a Llama-3-8B decoder block with RMSNorm, grouped-query
// attention and SwiGLU); fact_block_forward is that composition with every stage on the GPU.
#include "../../include/fact.h"

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <cmath>

namespace fact {

int record_hip_failure(hipError_t e, const char *what);      // fact_api.hip

namespace blockk {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float lo16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi16(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}
__device__ __forceinline__ uint32_t pack2(float a, float b) { return bf16_rne(a) | (bf16_rne(b) << 16); }
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s);
    return v;
}

// One wave per row: the row is read once (16 bytes per lane and piece), kept in registers in fp32,
// reduced across the wave, normalised and written once.  d <= 8192, a multiple of 8.
// The number of 512-element pieces is a template parameter: a short row takes few registers, so
// many waves fit on a SIMD and cover each other's memory latency.
constexpr int kMaxPieces = 16;           // 16 pieces x 64 lanes x 8 elements
template <bool RMS, int PIECES>
__global__ void __launch_bounds__(256)
norm_kernel(const uint16_t *X, int64_t ldx, const uint16_t *gamma, const uint16_t *beta, float eps,
            uint16_t *Y, int64_t ldy, int T, int d)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= T) return;
    const uint16_t *x = X + (int64_t)row * ldx;
    float v[PIECES][8];
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
        const int c = p * 512 + lane * 8;
        if (c < d) {
            const u32x4_t w = *(const u32x4_t *)(x + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) { v[p][2 * e] = lo16(w[e]); v[p][2 * e + 1] = hi16(w[e]); }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[p][e] = 0.f;
        }
        if (!RMS) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s += v[p][e];
        }
    }
    float mean = 0.f;
    if (!RMS) mean = wave_sum(s) / (float)d;
    float q = 0.f;
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
        const int c = p * 512 + lane * 8;
        if (c < d) {
#pragma unroll
            for (int e = 0; e < 8; ++e) { const float t = v[p][e] - mean; q += t * t; }
        }
    }
    const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)d + eps);
    uint16_t *y = Y + (int64_t)row * ldy;
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
        const int c = p * 512 + lane * 8;
        if (c < d) {
            const u32x4_t g = *(const u32x4_t *)(gamma + c);
            u32x4_t b = {0u, 0u, 0u, 0u};
            if (!RMS && beta) b = *(const u32x4_t *)(beta + c);
            u32x4_t o;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                o[e] = pack2((v[p][2 * e] - mean) * rstd * lo16(g[e]) + lo16(b[e]),
                             (v[p][2 * e + 1] - mean) * rstd * hi16(g[e]) + hi16(b[e]));
            *(u32x4_t *)(y + c) = o;
        }
    }
}

// Rotary embedding in place, "rotate-half" pairing: one thread takes 8 consecutive i < D/2 of one
// (batch entry, token) - the 16-byte piece at i and the one at i + D/2 - and walks a group of up to
// kRopeHeads heads (blockIdx.y), so the eight sines and cosines are computed once per group.
constexpr int kRopeHeads = 8;
__global__ void __launch_bounds__(256)
rope_kernel(uint16_t *X, int64_t sb, int64_t st, int64_t sh, int B, int T, int H, int D, float log2_base)
{
    const int per_head = D / 16;
    const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)B * T * per_head;
    if (gid >= total) return;
    const int piece = (int)(gid % per_head);
    const int64_t bt = gid / per_head;
    const int t = (int)(bt % T), b = (int)(bt / T);
    float sn[8], cs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int i = piece * 8 + e;
        const float inv_freq = exp2f(-2.0f * (float)i / (float)D * log2_base);
        sincosf((float)t * inv_freq, &sn[e], &cs[e]);
    }
    const int h0 = blockIdx.y * kRopeHeads, h1 = h0 + kRopeHeads < H ? h0 + kRopeHeads : H;
    uint16_t *p = X + (int64_t)b * sb + (int64_t)t * st + (int64_t)h0 * sh + piece * 8;
    for (int h = h0; h < h1; ++h, p += sh) {
        const u32x4_t lo = *(const u32x4_t *)p, hi = *(const u32x4_t *)(p + D / 2);
        u32x4_t olo, ohi;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a0 = lo16(lo[e]), a1 = hi16(lo[e]), c0 = lo16(hi[e]), c1 = hi16(hi[e]);
            olo[e] = pack2(a0 * cs[2 * e] - c0 * sn[2 * e], a1 * cs[2 * e + 1] - c1 * sn[2 * e + 1]);
            ohi[e] = pack2(c0 * cs[2 * e] + a0 * sn[2 * e], c1 * cs[2 * e + 1] + a1 * sn[2 * e + 1]);
        }
        *(u32x4_t *)p = olo;
        *(u32x4_t *)(p + D / 2) = ohi;
    }
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
static size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Layout {
    size_t n1, qkv, a, x1, n2, h, ws, ws_bytes, total;
};

static int plan(const fact_block *b, Layout &L)
{
    if (!b) return FACT_ERR_NULL;
    if (b->batch <= 0 || b->tokens <= 0 || b->d_model <= 0 || b->n_q_heads <= 0 || b->n_kv_heads <= 0 || b->d_ff <= 0) return FACT_ERR_DIM;
    if (b->n_q_heads % b->n_kv_heads) return FACT_ERR_DIM;
    if (b->head_dim != 64 && b->head_dim != 128) return FACT_ERR_UNSUPPORTED;
    if (b->d_model % 8 || b->d_model > 8192 || b->d_ff % 8) return FACT_ERR_UNSUPPORTED;
    if (b->act != FACT_ACT_GELU_TANH && b->act != FACT_ACT_SILU_GATE && b->act != FACT_ACT_NONE) return FACT_ERR_EPILOGUE;
    if (!b->norm1_g || !b->norm2_g || !b->Wqkv || !b->Wo || !b->W1 || !b->W2) return FACT_ERR_NULL;
    if (b->act == FACT_ACT_SILU_GATE && (!b->W1u || b->b1)) return FACT_ERR_EPILOGUE;
    if (b->act != FACT_ACT_SILU_GATE && b->W1u) return FACT_ERR_EPILOGUE;
    const int64_t T = b->batch * b->tokens, d = b->d_model, nq = b->n_q_heads * b->head_dim;
    const int64_t nqkv = (b->n_q_heads + 2 * b->n_kv_heads) * b->head_dim;
    // what the later stages would refuse is refused here, before anything is launched: the attention
    // kernel's 32-bit row offsets inside a batch entry of the packed projection and its grid limit,
    // the norm kernels' 16-byte access to their parameters
    if ((b->tokens + 512) * nqkv * 2 >= (int64_t)1 << 31 || b->tokens > 0x7FFFFFFF - 1024) return FACT_ERR_UNSUPPORTED;
    if (b->batch * b->n_q_heads * ((b->tokens + 127) / 128) > 0x7FFFFFFF || T > 0x7FFFFFFF) return FACT_ERR_UNSUPPORTED;
    if (!aligned16(b->norm1_g) || !aligned16(b->norm2_g) || (!b->norm_rms && ((b->norm1_b && !aligned16(b->norm1_b)) || (b->norm2_b && !aligned16(b->norm2_b)))))
        return FACT_ERR_ALIGN;
    if (b->norm_rms != 0 && b->norm_rms != 1) return FACT_ERR_LAYOUT;
    size_t off = 0;
    L.n1 = off; off += up256((size_t)T * d * 2);
    L.qkv = off; off += up256((size_t)T * nqkv * 2);
    L.a = off; off += up256((size_t)T * nq * 2);
    L.x1 = off; off += up256((size_t)T * d * 2);
    L.n2 = off; off += up256((size_t)T * d * 2);
    L.h = off; off += up256((size_t)T * b->d_ff * 2);
    size_t w = fact_gemm_splitk_workspace_bytes(T, nqkv, d, 0);
    const size_t w2 = fact_gemm_splitk_workspace_bytes(T, d, nq, 0), w3 = fact_block_mlp_workspace_bytes(T, d, b->d_ff, b->act);
    if (w2 > w) w = w2;
    if (w3 > w) w = w3;
    L.ws = off; L.ws_bytes = w; off += up256(w);
    L.total = off;
    return FACT_OK;
}

}  // namespace blockk
}  // namespace fact

extern "C" {

int fact_norm(int64_t T, int64_t d, const void *X, int64_t ldx, const void *gamma, const void *beta, float eps, int rms,
              void *Y, int64_t ldy, void *stream)
{
    using namespace fact::blockk;
    if (!X || !gamma || !Y) return FACT_ERR_NULL;
    if (T <= 0 || d <= 0 || ldx < d || ldy < d || T > 0x7FFFFFFF) return FACT_ERR_DIM;
    if (rms != 0 && rms != 1) return FACT_ERR_LAYOUT;
    if (rms && beta) return FACT_ERR_EPILOGUE;
    if (d % 8 || d > 512 * kMaxPieces) return FACT_ERR_UNSUPPORTED;
    if (!aligned16(X) || !aligned16(Y) || !aligned16(gamma) || (beta && !aligned16(beta)) || (ldx & 7) || (ldy & 7)) return FACT_ERR_ALIGN;
    if (!(eps >= 0.f)) return FACT_ERR_DIM;
    const unsigned grid = (unsigned)((T + 3) / 4);
    hipStream_t s = (hipStream_t)stream;
    const int pieces = (int)((d + 511) / 512);
#define FACT_NORM_LAUNCH(R, P) hipLaunchKernelGGL((norm_kernel<R, P>), dim3(grid), dim3(256), 0, s, (const uint16_t *)X, ldx, \
        (const uint16_t *)gamma, (const uint16_t *)(R ? nullptr : beta), eps, (uint16_t *)Y, ldy, (int)T, (int)d)
#define FACT_NORM_PICK(R) do { if (pieces <= 1) FACT_NORM_LAUNCH(R, 1); else if (pieces <= 2) FACT_NORM_LAUNCH(R, 2); \
        else if (pieces <= 4) FACT_NORM_LAUNCH(R, 4); else if (pieces <= 8) FACT_NORM_LAUNCH(R, 8); else FACT_NORM_LAUNCH(R, 16); } while (0)
    if (rms) FACT_NORM_PICK(true); else FACT_NORM_PICK(false);
#undef FACT_NORM_PICK
#undef FACT_NORM_LAUNCH
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? FACT_OK : fact::record_hip_failure(e, "norm launch");
}

int fact_rope(int64_t batch, int64_t T, int64_t n_heads, int64_t head_dim, void *X, const int64_t *strides, float base, void *stream)
{
    using namespace fact::blockk;
    if (!X || !strides) return FACT_ERR_NULL;
    if (batch <= 0 || T <= 0 || n_heads <= 0 || strides[1] < head_dim || strides[0] < 0 || strides[2] < 0) return FACT_ERR_DIM;
    if (head_dim <= 0 || head_dim % 16) return FACT_ERR_UNSUPPORTED;
    if (!aligned16(X) || (strides[0] & 7) || (strides[1] & 7) || (strides[2] & 7)) return FACT_ERR_ALIGN;
    if (!(base > 1.0f)) return FACT_ERR_DIM;
    const int64_t total = batch * T * (head_dim / 16);
    if (batch > 0x7FFFFFFF || T > 0x7FFFFFFF || n_heads > 65535 * kRopeHeads || (total + 255) / 256 > 0x7FFFFFFF) return FACT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(rope_kernel, dim3((unsigned)((total + 255) / 256), (unsigned)((n_heads + kRopeHeads - 1) / kRopeHeads)), dim3(256), 0, (hipStream_t)stream, (uint16_t *)X,
                       strides[0], strides[1], strides[2], (int)batch, (int)T, (int)n_heads, (int)head_dim, std::log2(base));
    const hipError_t e = hipGetLastError();
    return e == hipSuccess ? FACT_OK : fact::record_hip_failure(e, "rope launch");
}

size_t fact_block_scratch_bytes(const fact_block *blk)
{
    fact::blockk::Layout L;
    return fact::blockk::plan(blk, L) == FACT_OK ? L.total : 0;
}

int fact_block_scratch_offsets(const fact_block *blk, size_t *offsets)
{
    fact::blockk::Layout L;
    const int rc = fact::blockk::plan(blk, L);
    if (rc != FACT_OK) return rc;
    if (!offsets) return FACT_ERR_NULL;
    offsets[0] = L.n1; offsets[1] = L.qkv; offsets[2] = L.a; offsets[3] = L.x1; offsets[4] = L.n2; offsets[5] = L.h; offsets[6] = L.ws;
    return FACT_OK;
}

int fact_block_forward(const fact_block *blk, const void *X, void *Y, void *scratch, size_t scratch_bytes, void *stream)
{
    using namespace fact::blockk;
    Layout L;
    int rc = plan(blk, L);
    if (rc != FACT_OK) return rc;
    if (!X || !Y || !scratch) return FACT_ERR_NULL;
    if (scratch_bytes < L.total) return FACT_ERR_WORKSPACE;
    if (!aligned16(X) || !aligned16(Y) || ((uintptr_t)scratch & 255u)) return FACT_ERR_ALIGN;
    const fact_block &b = *blk;
    const int64_t T = b.batch * b.tokens, d = b.d_model, D = b.head_dim, nq = b.n_q_heads * D;
    const int64_t nqkv = (b.n_q_heads + 2 * b.n_kv_heads) * D;
    char *s = (char *)scratch;
    void *N1 = s + L.n1, *QKV = s + L.qkv, *A = s + L.a, *X1 = s + L.x1, *N2 = s + L.n2, *H = s + L.h, *ws = s + L.ws;
    const float eps = b.eps > 0.f ? b.eps : 1e-5f;

    rc = fact_norm(T, d, X, d, b.norm1_g, b.norm_rms ? nullptr : b.norm1_b, eps, b.norm_rms, N1, d, stream);
    if (rc != FACT_OK) return rc;
    fact_epilogue e1 = {b.bqkv, nullptr, 0, 0, FACT_ACT_NONE};
    rc = fact_gemm_splitk(T, nqkv, d, N1, d, b.Wqkv, d, 1, QKV, nqkv, &e1, 0, ws, L.ws_bytes, stream);
    if (rc != FACT_OK) return rc;
    const int64_t st[3] = {b.tokens * nqkv, nqkv, D};
    if (b.rope) {
        rc = fact_rope(b.batch, b.tokens, b.n_q_heads + b.n_kv_heads, D, QKV, st, b.rope_base > 1.f ? b.rope_base : 500000.f, stream);
        if (rc != FACT_OK) return rc;
    }
    const int64_t so[3] = {b.tokens * nq, nq, D};
    rc = fact_attention(b.batch, b.tokens, b.n_q_heads, b.n_kv_heads, D, QKV, st, (char *)QKV + 2 * nq, st,
                        (char *)QKV + 2 * (nq + b.n_kv_heads * D), st, A, so, 1, 0.f, stream);
    if (rc != FACT_OK) return rc;
    fact_epilogue e2 = {b.bo, X, d, 0, FACT_ACT_NONE};
    rc = fact_gemm_splitk(T, d, nq, A, nq, b.Wo, nq, 1, X1, d, &e2, 0, ws, L.ws_bytes, stream);
    if (rc != FACT_OK) return rc;
    rc = fact_norm(T, d, X1, d, b.norm2_g, b.norm_rms ? nullptr : b.norm2_b, eps, b.norm_rms, N2, d, stream);
    if (rc != FACT_OK) return rc;
    return fact_block_mlp(T, d, b.d_ff, N2, b.W1, b.W1u, b.b1, b.act, b.W2, b.b2, X1, H, Y, ws, L.ws_bytes, stream);
}

}  // extern "C"
