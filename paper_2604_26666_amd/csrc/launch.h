// Host-side interface between the C ABI and the per-configuration translation units.
#pragma once
#include <hip/hip_runtime.h>
#include "gemm_kernel.h"

namespace fact {

// Launches configuration `id`'s kernel.  Defined once per configuration (inst.hip).
typedef hipError_t (*launch_fn)(const GemmArgs &args, bool trans_b, int grid_z, hipStream_t stream);

#define FACT_CFG(id, bm, bn, wm, wn, bk, st) hipError_t fact_launch_cfg##id(const GemmArgs &, bool, int, hipStream_t);
#include "configs.def"
#undef FACT_CFG

struct ConfigDesc {
    int id, bm, bn, wm, wn, bk, stages;
    launch_fn launch;
    // operand ring, or the epilogue's per-wave fp32 staging regions if those are larger
    int lds_bytes() const { return fact::lds_total(bm, bn, wm, wn, bk, stages); }
    int threads() const { return wm * wn * 64; }
    bool has_prefetch() const { return fact::has_prefetch(bm, bn, wm, wn, bk, stages); }      // and with it the sink a tail split's collector needs
    bool gate_capable() const { return true; }      // every wave tile has an even number of MFMA tiles along N
    bool serves(int trans_b) const { return trans_b || plain_b_supported(bn); }      // 192-wide tiles: B as [N][K] only
};

// Split-K reduction + epilogue, and the guarded fallback GEMM (aux_kernels.hip).
hipError_t launch_splitk_reduce(const GemmArgs &args, hipStream_t stream);
hipError_t launch_fallback_gemm(const GemmArgs &args, bool trans_b, int grid_z, hipStream_t stream);

}  // namespace fact
