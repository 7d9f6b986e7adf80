// One tile configuration's kernels (both B layouts).  Built once per row of configs.def with
// -DFACT_ID=.. -DFACT_BM=.. -DFACT_BN=.. -DFACT_WM=.. -DFACT_WN=.. -DFACT_BK=.. -DFACT_STAGES=..
#include "launch.h"
#include <atomic>

namespace fact {

#define FACT_CAT2(a, b) a##b
#define FACT_CAT(a, b) FACT_CAT2(a, b)

template <bool TRANS_B>
static hipError_t launch_one(const GemmArgs &args, int grid_z, hipStream_t stream)
{
    if constexpr (!TRANS_B && !plain_b_supported(FACT_BN)) {
        (void)args; (void)grid_z; (void)stream;
        return hipErrorInvalidConfiguration;          // (the host side never selects such a tile for this layout)
    } else {
    constexpr bool CAN_PERSIST = FACT_WM * FACT_WN <= 4;      // the persistent form exists for 4-wave configurations
    auto kern = gemm_kernel<FACT_BM, FACT_BN, FACT_WM, FACT_WN, TRANS_B, FACT_BK, FACT_STAGES, false>;
    auto kern_p = gemm_kernel<FACT_BM, FACT_BN, FACT_WM, FACT_WN, TRANS_B, FACT_BK, FACT_STAGES, CAN_PERSIST>;
    auto kern_h = gemm_kernel<FACT_BM, FACT_BN, FACT_WM, FACT_WN, TRANS_B, FACT_BK, FACT_STAGES, false, true>;      // binary16 operands (ordinary launches only)
    const bool persist = CAN_PERSIST && args.persist_items > 0;
    if (args.persist_items > 0 && (!CAN_PERSIST || args.f16)) return hipErrorInvalidConfiguration;     // (the host side never asks for it)
    constexpr int lds = lds_total(FACT_BM, FACT_BN, FACT_WM, FACT_WN, FACT_BK, FACT_STAGES);
    static std::atomic<bool> attr_set[64];         // (two host threads may make a kernel's first launch at once: setting the limit twice is harmless)
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!attr_set[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        if (CAN_PERSIST) {
            e = hipFuncSetAttribute((const void *)kern_p, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
        }
        e = hipFuncSetAttribute((const void *)kern_h, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_set[dev].store(true, std::memory_order_release);
    }
    const int tiles = args.tiles_m * args.tiles_n;
    const int grid_x = args.tail_g > 1 ? args.tail_first + (tiles - args.tail_first) * args.tail_g : tiles;
    dim3 grid((unsigned)grid_x, 1, (unsigned)grid_z);
    if (args.persist_items > 0) grid = dim3((unsigned)args.persist_grid, 1, 1);
    dim3 block(FACT_WM * FACT_WN * 64, 1, 1);
    if (args.f16) hipLaunchKernelGGL(kern_h, grid, block, lds, stream, args);
    else if (persist) hipLaunchKernelGGL(kern_p, grid, block, lds, stream, args);
    else hipLaunchKernelGGL(kern, grid, block, lds, stream, args);
    return hipGetLastError();
    }
}

hipError_t FACT_CAT(fact_launch_cfg, FACT_ID)(const GemmArgs &args, bool trans_b, int grid_z, hipStream_t stream)
{
    return trans_b ? launch_one<true>(args, grid_z, stream) : launch_one<false>(args, grid_z, stream);
}

}  // namespace fact
