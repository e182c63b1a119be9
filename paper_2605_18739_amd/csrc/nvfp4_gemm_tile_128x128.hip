// The 128 x 128 tile of the block-scaled FP4 GEMM (Sec. 2.2 / 3.1): every epilogue variant of
// gemm_regdq_kernel<128, 128, ...>.
#include "nvfp4_gemm_tile.h"

namespace nvfp4 {

hipError_t launch_tile_128x128(int epi, const GemmArgs &g, int64_t tiles, hipStream_t s)
{
    return launch_tile<128, 128>(epi, g, tiles, s);
}

}  // namespace nvfp4
