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
    int lds_bytes() const
    {
        const int ring = stages * (bm + bn) * bk * 2;
        const int mt = bm / wm / 32, wtn = bn / wn;
        const int pitch = wtn * 4 + 16;
        const int epi_mt = (mt % 2 == 0 && wm * wn * 64 * pitch <= 144 * 1024) ? 2 : 1;
        const int epi = wm * wn * epi_mt * 32 * pitch;
        return ring > epi ? ring : epi;
    }
    int threads() const { return wm * wn * 64; }
    int nt() const { return bn / wn / 32; }              // MFMA tiles per wave along N
    bool gate_capable() const { return nt() % 2 == 0; }  // gate and up tiles pair up inside a wave
};

// Split-K reduction + epilogue, and the guarded fallback GEMM (aux_kernels.hip).
hipError_t launch_splitk_reduce(const GemmArgs &args, hipStream_t stream);
hipError_t launch_fallback_gemm(const GemmArgs &args, bool trans_b, int grid_z, hipStream_t stream);

}  // namespace fact
