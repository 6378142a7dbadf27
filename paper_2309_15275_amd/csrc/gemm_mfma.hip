// Host side of the bf16 matrix-core GEMM: parameter set-up and the choice of tile shape.
#include <cstdlib>

#include "gemm_mfma_impl.h"

namespace lbp {
namespace {

int round_up(int v, int m) { return (v + m - 1) / m * m; }

struct TileShape {
    int bm, bn;
    bool fused;   // has the fused reverse-projection epilogue
    hipError_t (*launch)(const mfma::Params &, bool, GemmOut, int, int, hipStream_t);
};

const TileShape kTiles[] = {
    {128, 128, true, mfma_tile_128x128},
    {64, 128, true, mfma_tile_64x128},
    {256, 128, false, mfma_tile_256x128},
    {256, 256, false, mfma_tile_256x256},
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

int tile_from_env()
{
    const char *s = std::getenv("LBP_GEMM_TILE");
    if (!s || !*s) return -1;
    int v = std::atoi(s);
    return v >= 0 && v < kNumTiles ? v : -1;
}

// Workgroups needed by a tile shape.
long workgroups(const TileShape &t, long M, long N, int splits)
{
    return ((M + t.bm - 1) / t.bm) * ((N + t.bn - 1) / t.bn) * splits;
}

// Picks the tile shape: large tiles need fewer bytes per FLOP from L2 (a compute unit's L1 takes
// in 64 bytes a clock, which a 128x128 tile just balances against the matrix cores), small tiles
// give more workgroups when the output is small.  The cost is the number of rounds the
// workgroups take over the compute units times the time of one workgroup.
int choose_tile(const GemmArgs &a, int num_cus)
{
    int best = 0;
    double best_cost = 1e300;
    for (int i = 0; i < kNumTiles; ++i) {
        const TileShape &t = kTiles[i];
        if (a.out == GemmOut::kUnproject && !t.fused) continue;
        long wgs = workgroups(t, a.M, a.N, a.splits);
        double rounds = (double)((wgs + num_cus - 1) / num_cus);
        double mfma_clk = 2.0 * t.bm * t.bn * mfma::BK / 4096.0;
        double fill_clk = (double)(t.bm + t.bn) * mfma::BK * 2 / 64.0;
        double step = mfma_clk > fill_clk ? mfma_clk : fill_clk;
        double steps = (double)((a.K + a.splits - 1) / a.splits + mfma::BK - 1) / mfma::BK;
        double cost = rounds * (steps * step + 4000.0);
        if (cost < best_cost) {
            best_cost = cost;
            best = i;
        }
    }
    return best;
}

int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            cus = v;
        else
            cus = 256;
    }
    return cus;
}

}  // namespace

bool gemm_can_fuse_unproject(const BasisPlan &plan, int dtype, GemmPath path)
{
    if (path == GemmPath::kSimple || dtype != LBP_BF16) return false;
    if (plan.patch != 4 && plan.patch != 8) return false;
    int nc = (plan.patch >> plan.mh) * (plan.patch >> plan.mw);
    return nc <= 16;     // r <= patch^2 <= 64 always fits the smallest tile
}

hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t stream)
{
    if (a.dtype != LBP_BF16) return hipErrorInvalidValue;
    if (a.M < 8 || a.N < 8 || a.K < 1) return hipErrorInvalidValue;
    if (a.N % 8 || a.ldb % 8 || a.lda % 8 || (a.a_kfast ? a.K % 8 : a.M % 8)) return hipErrorInvalidValue;
    if (a.out != GemmOut::kF32 && a.splits != 1) return hipErrorInvalidValue;
    int tile = tile_from_env();
    if (tile >= 0 && a.out == GemmOut::kUnproject && !kTiles[tile].fused) tile = -1;
    if (tile < 0) tile = a.tile >= 0 && a.tile < kNumTiles ? a.tile : choose_tile(a, device_cus());
    const TileShape &t = kTiles[tile];

    mfma::Params p{};
    p.A = (const unsigned short *)a.A;
    p.B = (const unsigned short *)a.B;
    p.M = a.M; p.N = a.N; p.K = a.K;
    p.lda = a.lda; p.ldb = a.ldb;
    p.k_per_split = round_up((a.K + a.splits - 1) / a.splits, mfma::BK);
    p.bm_step = t.bm;
    p.tiles_n = (a.N + t.bn - 1) / t.bn;
    p.C = a.C;
    p.scale = a.scale;
    int lp = 0;
    if (a.out == GemmOut::kUnproject) {
        if (!a.plan || !a.a_kfast || !t.fused || !gemm_can_fuse_unproject(*a.plan, a.dtype, GemmPath::kAuto))
            return hipErrorInvalidValue;
        const BasisPlan &bp = *a.plan;
        lp = bp.log2p;
        p.r = bp.r; p.mh = bp.mh; p.mw = bp.mw;
        p.bm_step = t.bm / bp.r * bp.r;
        p.sel.mask = bp.pooled_mask;
        for (int j = 0; j < 64; ++j) p.sel.pos[j] = bp.pooled_pos[j];
        p.geom.Wt = a.grid_w;
        p.geom.HWt = a.grid_h * a.grid_w;
        p.geom.PW = a.grid_w / bp.patch;
        p.geom.PHW = (a.grid_h / bp.patch) * (a.grid_w / bp.patch);
        p.geom.patch = bp.patch;
        p.Q = a.M / bp.r;
    }
    p.tiles_m = (a.M + p.bm_step - 1) / p.bm_step;
    return t.launch(p, a.a_kfast, a.out, lp, a.splits, stream);
}

}  // namespace lbp
