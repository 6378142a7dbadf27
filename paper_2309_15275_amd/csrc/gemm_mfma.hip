// Host side of the bf16 matrix-core GEMM: parameter set-up and the choice of tile shape.
#include <cstdlib>

#include "gemm_mfma_impl.h"

namespace lbp {
// Tile counters of the split reductions that combine inside a launch: zero whenever no such launch is
// running (the device image loads them as zeros and every launch leaves them so).  Each device has its
// own copy, found on first use.  Launches that overlap in time on one device must not both use them.
static __device__ unsigned join_counters[kJoinMaxTiles];

namespace {

unsigned *join_counter_ptr()
{
    static unsigned *ptrs[mfma::kMaxLaunchDevices] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= mfma::kMaxLaunchDevices) return nullptr;
    if (!ptrs[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(join_counters)) != hipSuccess) return nullptr;
        ptrs[dev] = static_cast<unsigned *>(ptr);
    }
    return ptrs[dev];
}

int round_up(int v, int m) { return (v + m - 1) / m * m; }

typedef hipError_t (*TileLaunch)(const mfma::Params &, bool, GemmOut, int, int, hipStream_t);

// same order as kGemmTiles
const TileLaunch kLaunch[kNumGemmTiles] = {mfma_tile_128x128, mfma_tile_64x128, mfma_tile_256x128,
                                           mfma_tile_256x256, mfma_tile_128x128w8, mfma_tile_64x128w8, mfma_tile_64x64,
                                           mfma_tile_256x192};

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
    // Up to 16 pooled coefficients per channel the epilogue expands them with the register
    // butterfly; beyond that (selections that cannot be pooled) an 8 x 8 patch goes through the
    // matrix-core epilogue.  r <= patch^2 <= 64 always fits the smallest tile.
    return gemm_unproject_pooled(plan) || plan.patch == 8;
}

bool gemm_unproject_pooled(const BasisPlan &plan)
{
    return (plan.patch >> plan.mh) * (plan.patch >> plan.mw) <= 16;
}

namespace {

// Checks one product, picks its tile and fills the kernel parameters.
hipError_t prepare(const GemmArgs &a, int *tile_out, mfma::Params *out, int *lp_out)
{
    if (a.dtype != LBP_BF16) return hipErrorInvalidValue;
    // rows of a k-fast A are clamped one by one (any M); a k-slow A and B are read in 8-element pieces
    if (a.M < (a.a_kfast ? 1 : 8) || a.N < 8 || a.K < 1) return hipErrorInvalidValue;
    if (a.N % 8 || a.ldb % 8 || a.lda % 8 || (a.a_kfast ? a.K % 8 : a.M % 8)) return hipErrorInvalidValue;
    // split reductions: fp32 slices for a reduction kernel, or a fused reverse projection whose slices combine in the launch
    if (a.out != GemmOut::kF32 && a.splits != 1 && !(a.out == GemmOut::kUnproject && a.join_parts && a.splits <= 16))
        return hipErrorInvalidValue;
    int tile = options().gemm_tile;     // testing: force one tile shape for every product
    if (tile >= 0 && a.out == GemmOut::kUnproject &&
        (!kGemmTiles[tile].fused || (a.plan && !gemm_unproject_pooled(*a.plan) && kGemmTiles[tile].bn != 128)))
        tile = -1;
    if (tile < 0) tile = a.tile;
    if (tile < 0 || tile >= kNumGemmTiles) {
        const bool fused = a.out == GemmOut::kUnproject;
        tile = plan_gemm(a.M, a.N, a.K / a.splits, a.out == GemmOut::kF32 ? 4 : 2, false,
                         fused && a.plan ? a.plan->r : 0, fused && a.plan ? a.plan->patch : 0, device_cus(),
                         fused && a.plan && !gemm_unproject_pooled(*a.plan)).tile;
    }
    const GemmTileInfo &t = kGemmTiles[tile];

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
    p.store_bf16 = a.out == GemmOut::kBF16 ? 1 : 0;
    int lp = 0;
    if (a.out == GemmOut::kUnproject) {
        if (!a.plan || !a.a_kfast || !t.fused || a.plan->r > t.bm || !gemm_can_fuse_unproject(*a.plan, a.dtype, GemmPath::kAuto))
            return hipErrorInvalidValue;
        const BasisPlan &bp = *a.plan;
        lp = bp.log2p;
        p.r = bp.r; p.mh = bp.mh; p.mw = bp.mw;
        p.bm_step = t.bm / bp.r * bp.r;
        p.mfma_epilogue = gemm_unproject_pooled(bp) ? 0 : 1;
        if (p.mfma_epilogue && t.bn != 128) return hipErrorInvalidValue;
        for (int k = 0; k < 64; ++k) p.nat[k] = k < bp.r ? (unsigned char)bp.nat[k] : (unsigned char)0;
        p.sel.mask = bp.pooled_mask;
        for (int j = 0; j < 64; ++j) p.sel.pos[j] = bp.pooled_pos[j];
        if (a.extra_rows < 0 || a.extra_rows > a.M || (a.extra_rows > 0 && (a.extra < 1 || a.extra_rows % a.extra)) ||
            (a.M - a.extra_rows) % bp.r)
            return hipErrorInvalidValue;
        p.geom = make_geom(a.grid_h, a.grid_w, bp.patch, a.extra);
        p.Q = (a.M - a.extra_rows) / bp.r;     // = patches of the zero-padded grids
        p.extra_rows = a.extra_rows;
        p.extra = a.extra > 0 ? a.extra : 1;
    }
    p.tiles_m = (a.M + p.bm_step - 1) / p.bm_step;
    p.splits = 1;
    if (a.out == GemmOut::kUnproject && a.splits > 1) {
        if ((long)p.tiles_m * p.tiles_n > kJoinMaxTiles) return hipErrorInvalidValue;
        if ((long)(a.splits - 1) * p.k_per_split >= a.K) return hipErrorInvalidValue;       // no empty slice
        if ((size_t)p.tiles_m * p.tiles_n * a.splits * t.bm * t.bn * sizeof(float) > a.join_bytes) return hipErrorInvalidValue;
        p.splits = a.splits;
        p.parts = static_cast<float *>(a.join_parts);
        p.counters = join_counter_ptr();
        if (!p.counters) return hipErrorInvalidSymbol;
    }
    // The tiles of one XCD (T / 8 of them) as an xcd_a x xcd_b block of the output: the block shape
    // whose strips of A and B together are the fewest bytes for that XCD's L2 to fetch.
    p.xcd_a = p.xcd_b = 0;
    const int T = p.tiles_m * p.tiles_n;
    if (T % 8 == 0) {
        double best = 1e300;
        for (int xa = 1; xa <= p.tiles_m; ++xa) {
            if ((T / 8) % xa || p.tiles_m % xa) continue;
            const int xb = T / 8 / xa;
            if (xb > p.tiles_n || p.tiles_n % xb) continue;
            const double bytes = (double)xa * p.bm_step + (double)xb * t.bn;      // times K * 2 bytes
            if (bytes < best) {
                best = bytes;
                p.xcd_a = xa;
                p.xcd_b = xb;
            }
        }
    }
    *tile_out = tile;
    *out = p;
    *lp_out = lp;
    return hipSuccess;
}

// Tiles of the grouped launch: 128x128 with 8 wavefronts for the weight gradient, that or 64x128
// with 8 wavefronts for the input gradient.
constexpr int kPairTileW = 4, kPairTileX0 = 4, kPairTileX1 = 5;
// ... and 64x64 for both on thin layers
constexpr int kPairTileThin = 6;

bool pair_tiles_ok(int tx, int tw)
{
    return (tw == kPairTileW && (tx == kPairTileX0 || tx == kPairTileX1)) || (tw == kPairTileThin && tx == kPairTileThin);
}

}  // namespace

size_t gemm_join_bytes(int tile, long M_rows, long N, int r, int splits)
{
    if (tile < 0 || tile >= kNumGemmTiles || r < 1 || splits < 2) return 0;
    const GemmTileInfo &t = kGemmTiles[tile];
    const long bm_step = t.bm / r * r;
    if (bm_step < 1) return 0;
    const long tiles = ((M_rows + bm_step - 1) / bm_step) * ((N + t.bn - 1) / t.bn);
    return (size_t)tiles * splits * t.bm * t.bn * sizeof(float);
}

bool gemm_join_supported(const GemmArgs &a, GemmPath path)
{
    if (path == GemmPath::kSimple || a.out != GemmOut::kUnproject || a.splits < 2 || !a.plan || a.plan->patch != 8) return false;
    int tile, lp;
    mfma::Params p;
    if (prepare(a, &tile, &p, &lp) != hipSuccess) return false;
    return tile == kPairTileX0 || tile == kPairTileX1;
}

hipError_t launch_gemm_mfma(const GemmArgs &a, hipStream_t stream)
{
    int tile, lp;
    mfma::Params p;
    hipError_t e = prepare(a, &tile, &p, &lp);
    if (e != hipSuccess) return e;
    // slices of a fused product join inside the launch on the 8-wavefront 128-wide tiles only
    if (a.out == GemmOut::kUnproject && a.splits != 1 && tile != kPairTileX0 && tile != kPairTileX1) return hipErrorInvalidValue;
    return kLaunch[tile](p, a.a_kfast, a.out, lp, a.splits, stream);
}

bool gemm_pair_supported(const GemmArgs &x, const GemmArgs &w, GemmPath path)
{
    if (path == GemmPath::kSimple) return false;
    if (x.dtype != LBP_BF16 || w.dtype != LBP_BF16 || !x.a_kfast || w.a_kfast) return false;
    if (w.out == GemmOut::kUnproject) return false;
    if (x.out == GemmOut::kUnproject && (!x.plan || x.plan->patch != 8)) return false;
    int tx, tw, lp;
    mfma::Params p;
    if (prepare(x, &tx, &p, &lp) != hipSuccess || prepare(w, &tw, &p, &lp) != hipSuccess) return false;
    if (tw == kPairTileThin && x.out == GemmOut::kUnproject && (!gemm_unproject_pooled(*x.plan) || x.splits != 1)) return false;
    return pair_tiles_ok(tx, tw);
}

hipError_t launch_gemm_pair(const GemmArgs &x, const GemmArgs &w, hipStream_t stream)
{
    int tx, tw, lpx, lpw;
    mfma::Params px, pw;
    hipError_t e = prepare(x, &tx, &px, &lpx);
    if (e != hipSuccess) return e;
    e = prepare(w, &tw, &pw, &lpw);
    if (e != hipSuccess) return e;
    if (!pair_tiles_ok(tx, tw) || !x.a_kfast || w.a_kfast || w.out == GemmOut::kUnproject ||
        (x.out == GemmOut::kUnproject && lpx != 3))
        return hipErrorInvalidValue;
    // Dispatch order.  When the launch has more workgroups than the device holds at once (two of these
    // per compute unit), those with the higher indices start late; the input-gradient workgroups end with
    // long bursts of stores (the whole g^x goes through them), and weight-gradient workgroups that start
    // during those bursts crawl.  So the weight-gradient product goes first then: its short, store-free
    // workgroups run beside the first input-gradient ones (measured: -7 % on 131072 tokens x 768 channels
    // at r = 4 and 8; +7 % to +17 % where everything is resident anyway, hence the condition).
    const long blocks = (long)px.tiles_m * px.tiles_n * x.splits + (long)pw.tiles_m * pw.tiles_n * w.splits;
    const bool w_leads = options().gemm_group == 2 || (tw != kPairTileThin && blocks > 2L * device_cus());
    if (tw == kPairTileThin) return mfma_pair_64x64(px, x.out, x.splits, pw, w.splits, stream, w_leads);
    return mfma_pair_w8(px, kGemmTiles[tx].bm, x.out, x.splits, pw, w.splits, stream, w_leads);
}

}  // namespace lbp
