// The 64 x 64 tile of the block-scaled FP4 GEMM (Sec. 2.2 / 3.1): every epilogue variant of
// gemm_regdq_kernel<64, 64, ...>.
#include "nvfp4_gemm_tile.h"

namespace nvfp4 {

hipError_t launch_tile_64x64(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s)
{
    return launch_tile<64, 64>(epi, g, tiles, s);
}

}  // namespace nvfp4
