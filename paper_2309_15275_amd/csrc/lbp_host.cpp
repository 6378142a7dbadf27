// Host-side logic: validation, basis selection (Section 3.2, Eq. 8-9), sequency -> natural
// index conversion, workspace planning.  No HIP calls in this file.
#include "lbp_host.h"

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <tuple>
#include <vector>

namespace lbp {

int patch_log2(int patch)
{
    switch (patch) {
        case 2: return 1;
        case 4: return 2;
        case 8: return 3;
        case 16: return 4;
        default: return -1;
    }
}

int sequency_to_natural(int s, int log2p)
{
    // Walsh function number s (s sign changes) is Sylvester row bitreverse(gray(s)).
    unsigned gray = (unsigned)s ^ ((unsigned)s >> 1);
    unsigned nat = 0;
    for (int b = 0; b < log2p; ++b)
        if (gray & (1u << b)) nat |= 1u << (log2p - 1 - b);
    return (int)nat;
}

int select_bases(int patch, int r, int order, int32_t *basis_idx)
{
    if (patch_log2(patch) < 0) return LBP_ERR_PATCH;
    if (r < 1 || r > patch * patch) return LBP_ERR_RANK;
    if (order != LBP_ORDER_L1 && order != LBP_ORDER_LINF) return LBP_ERR_ORDER;
    if (!basis_idx) return LBP_ERR_NULL;
    // (shell, tie-break towards the diagonal, smaller u first, index)
    std::vector<std::tuple<int, int, int, int>> all;
    all.reserve((size_t)patch * patch);
    for (int u = 0; u < patch; ++u)
        for (int v = 0; v < patch; ++v) {
            int sum = u + v, mx = std::max(u, v);
            if (order == LBP_ORDER_L1)
                all.emplace_back(sum, mx, u, u * patch + v);
            else
                all.emplace_back(mx, sum, u, u * patch + v);
        }
    std::sort(all.begin(), all.end());
    for (int k = 0; k < r; ++k) basis_idx[k] = std::get<3>(all[(size_t)k]);
    return LBP_OK;
}

int select_lhe(const double *energy, int patch, int r, int32_t *basis_idx)
{
    if (patch_log2(patch) < 0) return LBP_ERR_PATCH;
    if (r < 1 || r > patch * patch) return LBP_ERR_RANK;
    if (!energy || !basis_idx) return LBP_ERR_NULL;
    const int pp = patch * patch;
    std::vector<int32_t> order((size_t)pp);
    int rc = select_bases(patch, pp, LBP_ORDER_L1, order.data());
    if (rc) return rc;
    // stable: bases of equal energy stay in LP_L1 order
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return energy[a] > energy[b]; });
    for (int k = 0; k < r; ++k) basis_idx[k] = order[(size_t)k];
    return LBP_OK;
}

static int trailing_zeros_capped(int v, int cap)
{
    int n = 0;
    while (n < cap && !(v & (1 << n))) ++n;
    return n;
}

int make_basis_plan(int patch, const int32_t *basis_idx, int r, BasisPlan *plan)
{
    int lp = patch_log2(patch);
    if (lp < 0) return LBP_ERR_PATCH;
    if (r < 1 || r > patch * patch) return LBP_ERR_RANK;
    if (!basis_idx || !plan) return LBP_ERR_NULL;
    bool seen[kMaxBases];
    std::memset(seen, 0, sizeof seen);
    std::memset(plan, 0, sizeof *plan);
    plan->patch = patch;
    plan->log2p = lp;
    plan->r = r;
    int mh = lp, mw = lp;
    int nat_u[kMaxBases], nat_v[kMaxBases];
    for (int k = 0; k < r; ++k) {
        int idx = basis_idx[k];
        if (idx < 0 || idx >= patch * patch || seen[idx]) return LBP_ERR_BASIS;
        seen[idx] = true;
        nat_u[k] = sequency_to_natural(idx / patch, lp);
        nat_v[k] = sequency_to_natural(idx % patch, lp);
        plan->nat[k] = (uint8_t)(nat_u[k] * patch + nat_v[k]);
        mh = std::min(mh, trailing_zeros_capped(nat_u[k], lp));
        mw = std::min(mw, trailing_zeros_capped(nat_v[k], lp));
    }
    plan->mh = mh;
    plan->mw = mw;
    if (patch <= 8) {
        int wbits = lp - mw;   // bits of the pooled width index
        for (int k = 0; k < r; ++k) {
            int j = ((nat_u[k] >> mh) << wbits) | (nat_v[k] >> mw);
            plan->pooled_mask |= 1ull << j;
            plan->pooled_pos[j] = (uint8_t)k;
        }
    }
    return LBP_OK;
}

size_t dtype_size(int dtype)
{
    return dtype == LBP_F32 ? 4 : dtype == LBP_BF16 ? 2 : 0;
}

static int channel_multiple(int dtype) { return dtype == LBP_BF16 ? 8 : 4; }

int validate_grid(int N, int H, int W, int C, int dtype, int patch)
{
    if (dtype_size(dtype) == 0) return LBP_ERR_DTYPE;
    if (N < 1 || H < 1 || W < 1 || C < 1) return LBP_ERR_SHAPE;
    if (patch != 0) {
        if (patch_log2(patch) < 0) return LBP_ERR_PATCH;
    }
    long long tokens = (long long)N * H * W;
    if (tokens >= (1ll << 31)) return LBP_ERR_SHAPE;
    if (C % channel_multiple(dtype)) return LBP_ERR_ALIGN;
    return LBP_OK;
}

int validate_shape(const lbp_shape_t *s, int patch)
{
    if (!s) return LBP_ERR_NULL;
    if (dtype_size(s->dtype) == 0) return LBP_ERR_DTYPE;
    if (s->gw_dtype != LBP_F32 && s->gw_dtype != s->dtype) return LBP_ERR_DTYPE;
    int rc = validate_grid(s->N, s->H, s->W, s->Cin, s->dtype, patch);
    if (rc) return rc;
    return validate_grid(s->N, s->H, s->W, s->Cout, s->dtype, patch);
}

int validate_alignment(const void *const *ptrs, int n)
{
    for (int i = 0; i < n; ++i)
        if (ptrs[i] && (reinterpret_cast<uintptr_t>(ptrs[i]) & 15u)) return LBP_ERR_ALIGN;
    return LBP_OK;
}

bool ranges_overlap(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b || na == 0 || nb == 0) return false;
    uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + nb && b0 < a0 + na;
}

const GemmTileInfo kGemmTiles[kNumGemmTiles] = {
    {128, 128, true, 1.0, 0, "128x128 (4 wavefronts)"},
    {64, 128, true, 1.0, 0, "64x128 (4 wavefronts)"},
    {256, 128, false, 1.15, 0, "256x128 (8 wavefronts)"},
    {256, 256, false, 1.4, 0, "256x256 (8 wavefronts)"},
    {128, 128, true, 0.92, 0, "128x128 (8 wavefronts)"},    // 8 wavefronts: hides more of the LDS -> matrix-core latency
    {64, 128, true, 0.88, 0, "64x128 (8 wavefronts)"},      // 8 wavefronts
    {64, 64, true, 1.0, 64, "64x64 (4 wavefronts)"},        // thin layers only: on wide ones it measured 10-15 % behind 64 x 128
    // 768 columns are four of these: the exact backward's gx at ViT-B is then 256 equal workgroups
    // (82 us against 93-98 us for the other tiles; behind them on every split-K product measured)
    {256, 192, false, 1.4, 0, "256x192 (8 wavefronts)", true},
};

GemmPlan plan_gemm(long M, long N, long K, int out_elem_bytes, bool allow_split, int fused_r,
                   int fused_patch, int num_cus, bool fused_wide, int only_tile)
{
    const double kFill = 20.0;            // bytes per clock a compute unit takes in from L2
    const double kClkPerUs = 2400.0;
    const double kWgFixed = 3000.0;       // clocks of prologue and drain per workgroup
    const int kStep = 64;                 // reduction elements per step of the kernel
    if (num_cus < 1) num_cus = 256;
    GemmPlan best{0, 1, 1e300};
    for (int t = 0; t < kNumGemmTiles; ++t) {
        const GemmTileInfo &ti = kGemmTiles[t];
        if (only_tile >= 0 && t != only_tile) continue;
        if (fused_r > 0 && (!ti.fused || fused_r > ti.bm)) continue;
        if (ti.max_n > 0 && N > ti.max_n) continue;
        if (ti.whole_k && allow_split) continue;
        if (fused_r > 0 && fused_wide && ti.bn != 128) continue;
        if (N <= 64 && ti.bn > 64 && !(fused_r > 0 && fused_wide)) continue;      // a thin product takes the 64-wide tile (measured)
        const long bm_step = fused_r > 0 ? ti.bm / fused_r * fused_r : ti.bm;
        const long tiles = ((M + bm_step - 1) / bm_step) * ((N + ti.bn - 1) / ti.bn);
        const int max_splits = (allow_split && fused_r == 0) ? 64 : 1;
        for (int sp = 1; sp <= max_splits; ++sp) {
            const long k_slice = (K + sp - 1) / sp;
            if (sp > 1 && k_slice < 4 * kStep) break;
            const double steps = (double)((k_slice + kStep - 1) / kStep);
            const double fill = steps * (ti.bm + ti.bn) * kStep * 2.0;
            double out;
            if (fused_r > 0)
                out = (double)(bm_step / fused_r) * fused_patch * fused_patch * ti.bn * 2.0;
            else
                out = (double)ti.bm * ti.bn * (sp > 1 ? 4 : out_elem_bytes);
            const double mfma = steps * 2.0 * ti.bm * ti.bn * kStep / 4096.0;
            double wg = (fill + out) / kFill;
            if (mfma > wg) wg = mfma;
            wg = wg * ti.slowdown + kWgFixed;
            const double rounds = (double)((tiles * sp + num_cus - 1) / num_cus);
            double clk = rounds * wg;
            if (sp > 1)   // the reduction kernel: about 3 us of launch and ramp, then ~7 TB/s
                clk += kClkPerUs * (3.0 + (double)(sp * 4 + out_elem_bytes) * M * N / 7.0e6);
            if (clk < best.est_us) best = GemmPlan{t, sp, clk};
        }
    }
    best.est_us /= kClkPerUs;
    return best;
}

long gemm_workgroups(const GemmPlan &g, long M, long N, int fused_r)
{
    const GemmTileInfo &ti = kGemmTiles[g.tile];
    const long bm_step = fused_r > 0 ? ti.bm / fused_r * fused_r : ti.bm;
    return ((M + bm_step - 1) / bm_step) * ((N + ti.bn - 1) / ti.bn) * g.splits;
}

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

double grouped_launch_estimate(long n_x, double cost_x, long n_w, double cost_w, int num_cus, bool w_first)
{
    if (num_cus < 1) num_cus = 256;
    // unit j gets the workgroups j, j + num_cus, j + 2 num_cus, ... of the dispatch order; count how many of
    // each kind that is for the fullest unit of each residue class
    const long n_first = w_first ? n_w : n_x, n_second = w_first ? n_x : n_w;
    const double c_first = w_first ? cost_w : cost_x, c_second = w_first ? cost_x : cost_w;
    double worst = 0.0;
    for (int j = 0; j < num_cus; ++j) {
        // indices i = j + k num_cus below n_first are of the first kind, the rest up to n_first + n_second of the second
        const long total = n_first + n_second;
        if (j >= total) break;
        const long mine = (total - 1 - j) / num_cus + 1;
        const long mine_first = j < n_first ? (n_first - 1 - j) / num_cus + 1 : 0;
        const double load = mine_first * c_first + (mine - mine_first) * c_second;
        if (load > worst) worst = load;
    }
    return worst;
}

static int plan_workspace_uncached(const lbp_shape_t *s, int patch, int r, int num_cus, bool can_fuse,
                                   bool force_fuse, WorkspacePlan *ws, bool fused_wide, bool allow_group, int extra,
                                   int coef16, int gx_join)
{
    std::memset(ws, 0, sizeof *ws);
    ws->gx_join = 1;
    if (num_cus < 1) num_cus = 256;
    const size_t esz = dtype_size(s->dtype);
    const int gw_bytes = (int)dtype_size(s->gw_dtype);
    if (extra < 0) return LBP_ERR_SHAPE;
    const long M = (long)s->N * ((long)s->H * s->W + extra);      // tokens, those outside the grid included
    size_t off = 0;
    if (patch == 0) {
        // full-rank backward: only the split-K partial sums of gW
        ws->gw = plan_gemm(s->Cout, s->Cin, M, gw_bytes, true, 0, 0, num_cus);
        ws->gx = plan_gemm(M, s->Cin, s->Cout, (int)esz, false, 0, 0, num_cus);
        ws->splitk = off;
        off += align_up((size_t)ws->gw.splits * s->Cout * s->Cin * 4, 256);
        ws->total = off;
        return LBP_OK;
    }
    // rows of the projected tensors: (patch, basis) pairs, then the tokens outside the grid as they are
    const long Mr = patch_count(s->N, s->H, s->W, patch) * r + (long)s->N * extra;
    ws->gw = plan_gemm(s->Cout, s->Cin, Mr, gw_bytes, true, 0, 0, num_cus);
    // gx: fused epilogue (no split, few workgroups when Mr is small) against split-K partial sums
    // that the reverse-projection kernel adds up while it reads them
    GemmPlan unfused = plan_gemm(Mr, s->Cin, s->Cout, 4, false, 0, 0, num_cus);
    for (int sp = 2; sp <= 16; ++sp) {      // slices are summed by the reverse-projection kernel
        if (s->Cout / sp < 256) break;
        GemmPlan g = plan_gemm(Mr, s->Cin, (s->Cout + sp - 1) / sp, 4, false, 0, 0, num_cus);
        // the planner sees one slice: scale its rounds to sp times the workgroups
        GemmPlan whole = plan_gemm(Mr * sp, s->Cin, (s->Cout + sp - 1) / sp, 4, false, 0, 0, num_cus);
        g.est_us = whole.est_us;
        g.splits = sp;
        if (g.est_us + 1.0 * sp < unfused.est_us) unfused = g;
    }
    // the reverse-projection kernel: about 8 us of launch, ramp and tail at these sizes, then
    // (slices read + tokens written) at ~4 TB/s
    unfused.est_us += 8.0 + ((double)unfused.splits * Mr * s->Cin * 4 + (double)M * s->Cin * esz) / 4.0e6;
    ws->gx = unfused;
    ws->gx_fused = false;
    if (can_fuse && s->dtype == LBP_BF16) {
        GemmPlan fused = plan_gemm(Mr, s->Cin, s->Cout, 2, false, r, patch, num_cus, fused_wide);
        if (force_fuse || fused.est_us <= unfused.est_us) {
            ws->gx = fused;
            ws->gx_fused = true;
        }
    }
    // Both products in one launch (kernels exist for the 8-wavefront tiles: 128 x 128 for gW, that
    // or 64 x 128 for gx; and for 64 x 64 tiles on layers with few channels).  Measured on the benchmark layers: the grouped launch takes 0.65-0.9 of
    // the two launches' sum while the two grids together are below about four workgroups per
    // compute unit, and the better gx tile is the one that fills the chip once (else twice) with
    // the most workgroups, else the larger tile.
    if (allow_group && s->dtype == LBP_BF16 && (patch == 8 || !(can_fuse && ws->gx_fused))) {
        const bool thin = s->Cin <= 64;                  // 64 x 64 tiles for both
        const int kTileW = thin ? 6 : 4, kTileX[2] = {thin ? 6 : 5, thin ? 6 : 4};       // indices into kGemmTiles
        // (the matrix-core epilogue pays inside a grouped launch up to two 16-basis steps: measured)
        const bool fuse = can_fuse && patch == 8 && (ws->gx_fused || force_fuse || !fused_wide || r <= 32);
        const GemmPlan w = plan_gemm(s->Cout, s->Cin, Mr, gw_bytes, true, 0, 0, num_cus, false, kTileW);
        const long n_w = gemm_workgroups(w, s->Cout, s->Cin, 0);
        GemmPlan x[2];
        long n_x[2];
        for (int i = 0; i < 2; ++i) {
            x[i] = fuse ? plan_gemm(Mr, s->Cin, s->Cout, 2, false, r, patch, num_cus, fused_wide, kTileX[i])
                        : plan_gemm(Mr, s->Cin, s->Cout, 4, false, 0, 0, num_cus, false, kTileX[i]);
            n_x[i] = gemm_workgroups(x[i], Mr, s->Cin, fuse ? r : 0);
        }
        int pick;
        if (n_w + n_x[0] <= num_cus) pick = 0;
        else if (n_w + n_x[1] <= num_cus) pick = 1;
        else if (n_w + n_x[0] <= 2 * num_cus) pick = 0;
        else pick = 1;
        // A fused input-gradient product cannot hand split-K slices to a reduction kernel, so with few
        // low-rank rows and many output channels it is a handful of workgroups walking a long reduction
        // while the rest of the device waits.  Its kernel can split the reduction over workgroups that
        // combine inside the launch (the last one of a tile to finish adds the parts and runs the
        // epilogue).  Whether that pays is decided with a model of the launch fitted to measurements
        // (times in microseconds: a 64-deep step of a 64- or 128-row tile 0.40 / 0.60, of the weight
        // gradient 0.70; the epilogue's stores at 45 GB/s per workgroup; storing a part 2, reading the
        // parts back 3 + s / 4): ViT-L fc1 r=4 32.2 -> 23.0 us with four slices, r=8 38.4 -> 33.7 with
        // two, ViT-B fc1 with 8 images 23.4 -> 16.3 with four; ViT-B fc1 with 64 images, ViT-L fc1 r=16
        // and ViT-L fc2 lose 10-30 % with any split and the model keeps them whole.
        int join = 1;
        double join_gain = 1.0;          // estimated time with the chosen slices over the time in one piece
        if (fuse && !thin && n_x[pick] <= 16384) {
            const GemmTileInfo &tx = kGemmTiles[x[pick].tile];
            const long bm_step = tx.bm / r * r;
            const long steps_w = ((Mr + w.splits - 1) / w.splits + 63) / 64;
            const double t_x = tx.bm <= 64 ? 0.40 : 0.60;
            const double epi_x = (double)(bm_step / r) * patch * patch * tx.bn * esz / 45.0e3;
            const double cost_w = steps_w * 0.70 + 2.0;
            auto estimate = [&](int sl) {
                const long st = ((s->Cout + sl - 1) / sl + 63) / 64;
                const double cost_x = st * t_x + epi_x + (sl > 1 ? 5.0 + 0.25 * sl : 0.0);
                const long n = n_x[pick] * sl;      // (n_w counts the weight gradient's own slices)
                return grouped_launch_estimate(n, cost_x, n_w, cost_w, num_cus, n + n_w > 2L * num_cus);
            };
            const double whole_us = estimate(1);
            double best_us = whole_us;
            for (int sl = 2; sl <= 8; ++sl) {
                if (gx_join > 0 && sl != gx_join) continue;
                const long k_slice = ((s->Cout + sl - 1) / sl + 63) / 64 * 64;
                if (k_slice < 4 * 64 || (long)(sl - 1) * k_slice >= s->Cout) continue;     // no short or empty slice
                const double us = estimate(sl);
                if (gx_join > 0 || us < best_us) {
                    best_us = us;
                    join = sl;
                }
            }
            if (gx_join == 0 && best_us > 0.9 * whole_us) join = 1;       // a split has to gain a tenth
            if (join > 1 && gx_join == 0) join_gain = best_us / whole_us;     // (a forced count leaves the grouping as it was)
        }
        double est = 0.85 * (w.est_us + x[pick].est_us) * join_gain;
        if (!fuse) est += 8.0 + ((double)Mr * s->Cin * 4 + (double)M * s->Cin * esz) / 4.0e6;
        const double launch_gap = 3.0;
        // Larger launches (up to eight workgroups per unit) are grouped too when the weight-gradient
        // product has to be split along its reduction: that means few output tiles with long
        // reductions and no stores, which, dispatched first, run beside the input-gradient
        // workgroups and fill the matrix cores during their store bursts (measured: -7 % at 131072
        // tokens x 768 channels r=16 and at the 49-token maps r=36; an unsplit weight-gradient product
        // fills the device by itself and loses 5 % in a launch of that size).  Only where the
        // input-gradient product keeps the tile and epilogue it would have had on its own: trading
        // its 256-row tile for the pair's 128 x 128 costs more than the overlap gains (ViT-B fc1, r=36
        // and 48: +5 to +7 %).
        // Nor where the weight-gradient product on its own would run on 256 x 256 tiles (r=48: +4 %).
        const bool same_gx = ws->gx.tile == x[pick].tile && ws->gx_fused == fuse;
        const bool big_gw = kGemmTiles[ws->gw.tile].bm * kGemmTiles[ws->gw.tile].bn >= 256 * 256;
        const long group_limit = (w.splits > 1 && same_gx && !big_gw ? 8L : 4L) * num_cus;
        if (w.est_us < 1e200 && x[pick].est_us < 1e200 && n_w + n_x[pick] <= group_limit &&
            est < ws->gw.est_us + ws->gx.est_us + launch_gap) {
            ws->gw = w;
            ws->gx = x[pick];
            ws->gx.est_us = est - w.est_us;
            ws->gx_fused = fuse;
            ws->grouped = true;
            ws->gx_join = join;
        }
    }
    // A fused input-gradient product launched on its own (only g~x wanted, or the grouped launch was not
    // taken) can cut its reduction the same way, on the 8-wavefront tiles: same model, no second product.
    if (!ws->grouped && can_fuse && patch == 8 && s->dtype == LBP_BF16 && s->Cin > 64 && gx_join != 1) {
        int best_tile = -1, best_join = 1;
        double best_us = 1e300;
        auto model = [&](int t, int sl) {
            const GemmTileInfo &tx = kGemmTiles[t];
            const long bm_step = tx.bm / r * r;
            const long tiles = ((Mr + bm_step - 1) / bm_step) * ((s->Cin + tx.bn - 1) / tx.bn);
            const long st = ((s->Cout + sl - 1) / sl + 63) / 64;
            const double cost = st * (tx.bm <= 64 ? 0.40 : 0.60) + (double)(bm_step / r) * patch * patch * tx.bn * esz / 45.0e3 +
                                (sl > 1 ? 5.0 + 0.25 * sl : 0.0);
            return tiles > 16384 ? 1e300 : grouped_launch_estimate(tiles * sl, cost, 0, 0.0, num_cus, false) + 3.0;
        };
        for (int t : {5, 4}) {
            if (r > kGemmTiles[t].bm) continue;
            for (int sl = 2; sl <= 8; ++sl) {
                if (gx_join > 0 && sl != gx_join) continue;
                const long k_slice = ((s->Cout + sl - 1) / sl + 63) / 64 * 64;
                if (k_slice < 4 * 64 || (long)(sl - 1) * k_slice >= s->Cout) continue;
                const double us = model(t, sl);
                if (us < best_us) {
                    best_us = us;
                    best_tile = t;
                    best_join = sl;
                }
            }
        }
        // against what the plan has: the same model for a fused product on one of these tiles, else the plan's own estimate
        double cur_us = ws->gx.est_us;
        if (ws->gx_fused && (ws->gx.tile == 4 || ws->gx.tile == 5)) cur_us = model(ws->gx.tile, 1);
        if (best_tile >= 0 && (gx_join > 1 || best_us < 0.9 * cur_us)) {
            ws->gx = GemmPlan{best_tile, 1, best_us};
            ws->gx_fused = true;
            ws->gx_join = best_join;
        }
    }
    // Where the reverse projection stays a kernel of its own, the product can hand it bf16
    // coefficients in one piece instead of fp32 split-K slices: a quarter of the bytes on the way
    // there and back, and any tile.  (Decided last, so that it only ever replaces the fp32 hand-over.)
    if (!ws->gx_fused && coef16 > 0 && s->dtype == LBP_BF16 && extra == 0) {
        if (ws->grouped) {
            ws->gx_coef16 = true;       // the same tile, half the store
        } else {
            GemmPlan g = plan_gemm(Mr, s->Cin, s->Cout, 2, false, 0, 0, num_cus);
            g.est_us += 8.0 + ((double)Mr * s->Cin * 2 + (double)M * s->Cin * esz) / 4.0e6;
            if (coef16 > 1 || g.est_us < ws->gx.est_us) {
                ws->gx = g;
                ws->gx_coef16 = true;
            }
        }
    }
    ws->gy_r = off;
    off += align_up((size_t)Mr * s->Cout * esz, 256);
    ws->x_r = off;
    off += align_up((size_t)Mr * s->Cin * esz, 256);
    ws->gx_r = off;
    if (!ws->gx_fused) off += align_up((size_t)ws->gx.splits * Mr * s->Cin * (ws->gx_coef16 ? 2 : 4), 256);
    else if (ws->gx_join > 1) {      // the slices' partial tiles, for either tile the grouped launch may run them on
        size_t need = 0;
        for (int t : {4, 5}) {
            const GemmTileInfo &tx = kGemmTiles[t];
            const long bm_step = tx.bm / r * r;
            if (bm_step < 1) continue;
            const long tiles = ((Mr + bm_step - 1) / bm_step) * ((s->Cin + tx.bn - 1) / tx.bn);
            const size_t bytes = (size_t)tiles * ws->gx_join * tx.bm * tx.bn * 4;
            if (bytes > need) need = bytes;
        }
        ws->gx_join_bytes = need;
        off += align_up(need, 256);
    }
    ws->splitk = off;
    off += align_up((size_t)ws->gw.splits * s->Cout * s->Cin * 4, 256);
    ws->total = off;
    return LBP_OK;
}

// The plan is a pure function of its arguments and costs dozens of sweeps over tiles and split
// factors; a training loop calls with the same few layers over and over, so the last plans are kept.
namespace {
struct PlanKey {
    int32_t v[20];
    bool operator==(const PlanKey &o) const { return std::memcmp(v, o.v, sizeof v) == 0; }
};
struct PlanSlot {
    bool used = false;
    PlanKey key;
    WorkspacePlan plan;
};
constexpr int kPlanSlots = 32;
std::mutex g_plan_mutex;
PlanSlot g_plan_cache[kPlanSlots];
unsigned g_plan_next = 0;
}  // namespace

int plan_workspace(const lbp_shape_t *s, int patch, int r, int num_cus, bool can_fuse,
                   bool force_fuse, WorkspacePlan *ws, bool fused_wide, bool allow_group, int extra, int coef16,
                   int gx_join)
{
    if (!s || !ws) return LBP_ERR_NULL;
    if (gx_join < 0 || gx_join > 8) return LBP_ERR_OPTION;
    const PlanKey key{{s->N, s->H, s->W, s->Cin, s->Cout, s->dtype, s->gw_dtype, patch, r, num_cus, can_fuse,
                       force_fuse, fused_wide, allow_group, extra, coef16, gx_join}};
    {
        std::lock_guard<std::mutex> lock(g_plan_mutex);
        for (const PlanSlot &slot : g_plan_cache)
            if (slot.used && slot.key == key) {
                *ws = slot.plan;
                return LBP_OK;
            }
    }
    const int rc = plan_workspace_uncached(s, patch, r, num_cus, can_fuse, force_fuse, ws, fused_wide, allow_group,
                                           extra, coef16, gx_join);
    if (rc != LBP_OK) return rc;
    std::lock_guard<std::mutex> lock(g_plan_mutex);
    PlanSlot &slot = g_plan_cache[g_plan_next++ % kPlanSlots];
    slot.used = true;
    slot.key = key;
    slot.plan = *ws;
    return LBP_OK;
}

namespace {

std::mutex g_opt_mutex;
Options g_opt;
bool g_opt_env_read = false;

const char *const kOptionNames[] = {"LBP_WHT_PATH", "LBP_GEMM_PATH", "LBP_GEMM_TILE", "LBP_FUSE_UNPROJECT",
                                    "LBP_GEMM_GROUP", "LBP_GX_COEF", "LBP_GX_JOIN"};

// Applies one switch to `o`; value NULL or "" restores the default.
int apply_option(Options *o, const char *name, const char *value)
{
    const Options def;
    const bool reset = !value || !*value;
    auto is = [&](const char *v) { return !reset && !std::strcmp(value, v); };
    if (!std::strcmp(name, "LBP_WHT_PATH")) {
        if (reset || is("auto")) o->wht_path = def.wht_path;
        else if (is("generic")) o->wht_path = 1;
        else if (is("register")) o->wht_path = 2;
        else if (is("mfma")) o->wht_path = 3;
        else return LBP_ERR_OPTION;
    } else if (!std::strcmp(name, "LBP_GEMM_PATH")) {
        if (reset || is("auto")) o->gemm_simple = 0;
        else if (is("simple")) o->gemm_simple = 1;
        else return LBP_ERR_OPTION;
    } else if (!std::strcmp(name, "LBP_GEMM_TILE")) {
        if (reset) {
            o->gemm_tile = def.gemm_tile;
            return LBP_OK;
        }
        char *end = nullptr;
        const long v = std::strtol(value, &end, 10);
        if (*end || v < 0 || v >= kNumGemmTiles) return LBP_ERR_OPTION;
        o->gemm_tile = (int)v;
    } else if (!std::strcmp(name, "LBP_FUSE_UNPROJECT")) {
        if (reset) o->fuse_unproject = def.fuse_unproject;
        else if (is("0")) o->fuse_unproject = 0;
        else if (is("1")) o->fuse_unproject = 1;
        else return LBP_ERR_OPTION;
    } else if (!std::strcmp(name, "LBP_GEMM_GROUP")) {
        if (reset || is("1")) o->gemm_group = 1;
        else if (is("0")) o->gemm_group = 0;
        else if (is("2")) o->gemm_group = 2;
        else return LBP_ERR_OPTION;
    } else if (!std::strcmp(name, "LBP_GX_JOIN")) {
        if (reset) o->gx_join = def.gx_join;
        else {
            char *end = nullptr;
            const long v = std::strtol(value, &end, 10);
            if (*end || end == value || v < 1 || v > 8) return LBP_ERR_OPTION;
            o->gx_join = (int)v;
        }
    } else if (!std::strcmp(name, "LBP_GX_COEF")) {
        if (reset) o->gx_coef = def.gx_coef;
        else if (is("f32")) o->gx_coef = 0;
        else if (is("bf16")) o->gx_coef = 2;
        else return LBP_ERR_OPTION;
    } else {
        return LBP_ERR_OPTION;
    }
    return LBP_OK;
}

// The only place the environment is read: once per process (g_opt_mutex held).  A value a switch
// does not take is ignored.
void read_env_once()
{
    if (g_opt_env_read) return;
    g_opt_env_read = true;
    for (const char *name : kOptionNames)
        if (const char *v = std::getenv(name)) (void)apply_option(&g_opt, name, v);
}

}  // namespace

Options options()
{
    std::lock_guard<std::mutex> lock(g_opt_mutex);
    read_env_once();
    return g_opt;
}

int set_option(const char *name, const char *value)
{
    if (!name) return LBP_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_opt_mutex);
    read_env_once();
    return apply_option(&g_opt, name, value);
}

const char *status_string(int code)
{
    switch (code) {
        case LBP_OK: return "success";
        case LBP_ERR_NULL: return "a required pointer is NULL";
        case LBP_ERR_SHAPE: return "bad shape: non-positive dimension or too many tokens";
        case LBP_ERR_PATCH: return "patch must be 2, 4, 8 or 16";
        case LBP_ERR_RANK: return "rank r must be in [1, patch^2]";
        case LBP_ERR_BASIS: return "basis index out of range or listed twice";
        case LBP_ERR_DTYPE: return "dtype or gw_dtype not recognised, or an unsupported combination";
        case LBP_ERR_ALIAS: return "an output buffer overlaps an input or the other output";
        case LBP_ERR_ALIGN: return "device pointers must be 16-byte aligned and channel counts a multiple of 8 (bf16) or 4 (fp32)";
        case LBP_ERR_ORDER: return "order must be LBP_ORDER_L1 or LBP_ORDER_LINF";
        case LBP_ERR_WORKSPACE: return "caller-provided workspace is too small";
        case LBP_ERR_HIP: return "a HIP call failed (see lbp_last_hip_error)";
        case LBP_ERR_OPTION: return "unknown option name or value";
        default: return "unknown status code";
    }
}

}  // namespace lbp
