// The 256 x 256 tile of the block-scaled FP4 GEMM (Sec. 2.2 / 3.1): every epilogue variant of
// gemm_regdq_kernel<256, 256, ...>.
#include "nvfp4_gemm_tile.h"

namespace nvfp4 {

hipError_t launch_tile_256x256(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s)
{
    return launch_tile<256, 256>(epi, g, tiles, s);
}

}  // namespace nvfp4
