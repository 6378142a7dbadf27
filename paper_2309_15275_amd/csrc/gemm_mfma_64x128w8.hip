// Instantiations of the bf16 matrix-core GEMM for 64 x 128 output tiles (2 x 4 wavefronts),
// 2 reduction steps of loads in flight.
#include "gemm_mfma_impl.h"

namespace lbp {

hipError_t mfma_tile_64x128w8(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s)
{
    return mfma::launch_tile<64, 128, 2, 4, 2, true>(p, a_kfast, out, lp, splits, s);
}

}  // namespace lbp
