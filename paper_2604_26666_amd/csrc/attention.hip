// fact_attention: argument validation and launch of the fused attention kernel.  Host code only;
// the computation runs in attention_kernel.h.
#include "../../include/fact.h"
#include <atomic>
#include "attention_kernel.h"

#include <cmath>
#include <cstdlib>

namespace fact {

int record_hip_failure(hipError_t e, const char *what);      // fact_api.hip: text for fact_last_error()

namespace attn {

template <int D, int NW>
static hipError_t launch(AttnArgs a, hipStream_t stream)
{
    auto kern = attn_fwd_kernel<D, NW>;
    constexpr int lds = 2 * 2 * 64 * D * 2;                   // two stages of a K and a V block
    static std::atomic<bool> attr_set[64];         // (two host threads may make a kernel's first launch at once: setting the limit twice is harmless)
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
    }
    constexpr int BQ = NW * 64;
    a.q_blocks = (a.T + BQ - 1) / BQ;
    a.total = a.q_blocks * a.Hq * a.B;
    // Pairs per group of the work-group order (see the kernel): a multiple of 4, so that each of an
    // XCD's shader engines gets the same mix of heavy and light work-groups; as large as the K/V of
    // the group's heads still fits an XCD's L2 (4 MB), which also starts the heavy work-groups early.
    {
        const int pairs = a.Hq * a.B, per = (pairs & 7) == 0 ? pairs >> 3 : pairs, G = a.Hq / a.Hkv;
        int best = 0, smallest = 0;
        for (int r = 4; r <= per; r += 4) {
            if (per % r) continue;
            if (!smallest) smallest = r;
            const int64_t kv_heads = r >= G ? (r + G - 1) / G : 1;
            if (kv_heads * a.T * D * 4 <= (int64_t)4 << 20) best = r;
        }
        a.group = best ? best : smallest ? smallest : per;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)a.total), dim3(NW * 64), lds, stream, a);
    return hipGetLastError();
}

}  // namespace attn
}  // namespace fact

extern "C" int fact_attention(int64_t batch, int64_t T, int64_t n_q_heads, int64_t n_kv_heads, int64_t head_dim,
                              const void *Q, const int64_t *q_strides, const void *K, const int64_t *k_strides,
                              const void *V, const int64_t *v_strides, void *O, const int64_t *o_strides,
                              int causal, float scale, void *stream)
{
    using namespace fact::attn;
    if (!Q || !K || !V || !O || !q_strides || !k_strides || !v_strides || !o_strides) return FACT_ERR_NULL;
    if (batch <= 0 || T <= 0 || n_q_heads <= 0 || n_kv_heads <= 0) return FACT_ERR_DIM;
    if (n_q_heads % n_kv_heads) return FACT_ERR_DIM;
    if (head_dim != 64 && head_dim != 128) return FACT_ERR_UNSUPPORTED;
    if (causal != 0 && causal != 1) return FACT_ERR_LAYOUT;
    if (!(scale == scale) || std::isinf(scale)) return FACT_ERR_DIM;
    // a row's head_dim elements are contiguous; the kernel addresses rows with 32-bit byte offsets
    // inside one (batch entry, head) and moves 16 bytes (inputs) or 8 bytes (output) at a time
    const int64_t *in[3] = {q_strides, k_strides, v_strides};
    const void *ptr[3] = {Q, K, V};
    for (int i = 0; i < 3; ++i) {
        const int64_t sb = in[i][0], st = in[i][1], sh = in[i][2];
        if (st < head_dim || sb < 0 || sh < 0) return FACT_ERR_DIM;
        if ((T + 512) * st * 2 >= (int64_t)1 << 31) return FACT_ERR_UNSUPPORTED;
        if (((uintptr_t)ptr[i] & 15u) || (sb & 7) || (st & 7) || (sh & 7)) return FACT_ERR_ALIGN;
    }
    if (o_strides[1] < head_dim || o_strides[0] < 0 || o_strides[2] < 0) return FACT_ERR_DIM;
    if (o_strides[1] > 0x7FFFFFFF) return FACT_ERR_UNSUPPORTED;
    if (((uintptr_t)O & 7u) || (o_strides[0] & 3) || (o_strides[1] & 3) || (o_strides[2] & 3)) return FACT_ERR_ALIGN;
    if (batch * n_q_heads * ((T + 127) / 128) > 0x7FFFFFFF || T > 0x7FFFFFFF - 1024) return FACT_ERR_UNSUPPORTED;

    AttnArgs a;
    a.Q = (const __bf16 *)Q; a.K = (const __bf16 *)K; a.V = (const __bf16 *)V; a.O = (__bf16 *)O;
    a.q_sb = q_strides[0]; a.q_st = (int)q_strides[1]; a.q_sh = q_strides[2];
    a.k_sb = k_strides[0]; a.k_st = (int)k_strides[1]; a.k_sh = k_strides[2];
    a.v_sb = v_strides[0]; a.v_st = (int)v_strides[1]; a.v_sh = v_strides[2];
    a.o_sb = o_strides[0]; a.o_st = (int)o_strides[1]; a.o_sh = o_strides[2];
    a.B = (int)batch; a.T = (int)T; a.Hq = (int)n_q_heads; a.Hkv = (int)n_kv_heads;
    a.causal = causal;
    const float sc = scale > 0.f ? scale : 1.0f / std::sqrt((float)head_dim);
    a.scale_log2 = sc * 1.4426950408889634f;
    a.q_blocks = 0; a.total = 0; a.group = 1;

    // 128 queries per work-group (two waves; two work-groups share a compute unit, and fewer of a
    // causal work-group's key blocks lie partly above the diagonal).  256 queries halve the K/V
    // traffic into LDS per query, which pays only for long sequences of wide heads (measured: from
    // T = 8192 at head_dim 128, 3-4%; below that the smaller work-groups are 5-20% faster), and
    // only with enough work-groups to give every compute unit two.
    const int64_t wgs256 = ((T + 255) / 256) * n_q_heads * batch;
    const bool four = head_dim == 128 && T >= 8192 && wgs256 >= 512;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (head_dim == 128) e = four ? launch<128, 4>(a, s) : launch<128, 2>(a, s);
    else e = launch<64, 2>(a, s);
    return e == hipSuccess ? FACT_OK : fact::record_hip_failure(e, "attention launch");
}
