// Instantiations of the bf16 matrix-core GEMM for 256 x 192 output tiles (4 x 2 wavefronts),
// 2 reduction steps of loads in flight.
#include "gemm_mfma_impl.h"

namespace lbp {

hipError_t mfma_tile_256x192(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s)
{
    return mfma::launch_tile<256, 192, 4, 2, 2, false>(p, a_kfast, out, lp, splits, s);
}

}  // namespace lbp
