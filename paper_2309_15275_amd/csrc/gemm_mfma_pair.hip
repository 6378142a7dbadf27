// Instantiations of the grouped launch (input-gradient product + weight-gradient product in one
// grid) for the tiles the planner gives the low-rank products: the 8-wavefront ones, and 64 x 64
// for layers with few channels.
#include "gemm_mfma_impl.h"
namespace lbp {
namespace {
using namespace mfma;

template <int BMX, int EPIX, int LPX, bool JOINX = false>
hipError_t pair(const Params &x, int splits_x, const Params &w, int splits_w, hipStream_t s, bool w_leads)
{
    return launch_pair<2, 4, 2, BMX, 128, true, EPIX, LPX, 128, 128, false, EPI_PLAIN, 0, JOINX>(x, splits_x, w, splits_w, s,
                                                                                                 w_leads);
}

template <int BMX>
hipError_t pair_bm(const Params &x, GemmOut out_x, int splits_x, const Params &w, int splits_w, hipStream_t s,
                   bool w_leads)
{
    if (out_x == GemmOut::kUnproject) {
        if (splits_x != 1) {        // the slices of a tile combine inside the launch, the last one runs the epilogue
            if (!x.parts || !x.counters || x.splits != splits_x) return hipErrorInvalidValue;
            if (x.mfma_epilogue) return pair<BMX, EPI_UNPROJECT_MFMA, 3, true>(x, splits_x, w, splits_w, s, w_leads);
            return pair<BMX, EPI_UNPROJECT, 3, true>(x, splits_x, w, splits_w, s, w_leads);
        }
        if (x.mfma_epilogue) return pair<BMX, EPI_UNPROJECT_MFMA, 3>(x, 1, w, splits_w, s, w_leads);
        return pair<BMX, EPI_UNPROJECT, 3>(x, 1, w, splits_w, s, w_leads);
    }
    return pair<BMX, EPI_PLAIN, 0>(x, splits_x, w, splits_w, s, w_leads);
}
}  // namespace

// thin layers: 64 x 64 tiles with 4 wavefronts for both products
hipError_t mfma_pair_64x64(const mfma::Params &x, GemmOut out_x, int splits_x, const mfma::Params &w, int splits_w,
                           hipStream_t s, bool w_leads)
{
    if (out_x == GemmOut::kUnproject) {
        if (splits_x != 1 || x.mfma_epilogue) return hipErrorInvalidValue;
        return launch_pair<2, 2, 2, 64, 64, true, EPI_UNPROJECT, 3, 64, 64, false, EPI_PLAIN, 0>(x, 1, w, splits_w, s, w_leads);
    }
    return launch_pair<2, 2, 2, 64, 64, true, EPI_PLAIN, 0, 64, 64, false, EPI_PLAIN, 0>(x, splits_x, w, splits_w, s, w_leads);
}

hipError_t mfma_pair_w8(const mfma::Params &x, int bm_x, GemmOut out_x, int splits_x, const mfma::Params &w,
                        int splits_w, hipStream_t s, bool w_leads)
{
    if (bm_x == 128) return pair_bm<128>(x, out_x, splits_x, w, splits_w, s, w_leads);
    if (bm_x == 64) return pair_bm<64>(x, out_x, splits_x, w, splits_w, s, w_leads);
    return hipErrorInvalidValue;
}
}  // namespace lbp
