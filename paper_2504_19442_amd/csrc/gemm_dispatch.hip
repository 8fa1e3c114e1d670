// Dispatch of a GEMM launch to the translation unit that holds the kernels of its tile configuration.
#include "agg_internal.h"

namespace agg {

#define AGG_DECL(BM, BN, MF) hipError_t launch_gemm_##BM##x##BN##_mf##MF(const GemmParams& p, bool grouped, int grid, hipStream_t s);
AGG_DECL(256, 224, 32) AGG_DECL(256, 256, 32) AGG_DECL(128, 256, 32) AGG_DECL(128, 128, 32)
AGG_DECL(256, 224, 16) AGG_DECL(256, 256, 16) AGG_DECL(128, 256, 16) AGG_DECL(128, 128, 16)
#undef AGG_DECL

static hipError_t launch_any(const GemmParams& p, bool grouped, int cfg, int grid, hipStream_t stream)
{
    switch (cfg) {
        case TILE_256x224: return launch_gemm_256x224_mf32(p, grouped, grid, stream);
        case TILE_256x256: return launch_gemm_256x256_mf32(p, grouped, grid, stream);
        case TILE_128x256: return launch_gemm_128x256_mf32(p, grouped, grid, stream);
        case TILE_128x128: return launch_gemm_128x128_mf32(p, grouped, grid, stream);
        case TILE_256x224 | TILE_K32: return launch_gemm_256x224_mf16(p, grouped, grid, stream);
        case TILE_256x256 | TILE_K32: return launch_gemm_256x256_mf16(p, grouped, grid, stream);
        case TILE_128x256 | TILE_K32: return launch_gemm_128x256_mf16(p, grouped, grid, stream);
        case TILE_128x128 | TILE_K32: return launch_gemm_128x128_mf16(p, grouped, grid, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm(const GemmParams& p, int cfg, int grid, hipStream_t stream)
{
    return launch_any(p, false, cfg, grid, stream);
}

hipError_t launch_gemm_grouped(const GemmParams& p, int cfg, int grid, hipStream_t stream)
{
    return launch_any(p, true, cfg, grid, stream);
}

}  // namespace agg
