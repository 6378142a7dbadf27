// Instantiations of the bf16 matrix-core GEMM for 64 x 64 output tiles (2 x 2 wavefronts), for
// layers with few channels: a 128-wide tile would be mostly empty there.
#include "gemm_mfma_impl.h"

namespace lbp {

hipError_t mfma_tile_64x64(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s)
{
    return mfma::launch_tile<64, 64, 2, 2, 2, true>(p, a_kfast, out, lp, splits, s);
}

}  // namespace lbp
