// Host-side logic of the LBP-WHT library: argument validation, basis bookkeeping and the
// small tables the kernels receive by value.  Plain C++, no HIP calls, so that every function
// here can run (and be tested) on a machine without a GPU.
#pragma once
#include <cstddef>
#include <cstdint>

#include "../../include/lbp_wht.h"

namespace lbp {

constexpr int kMaxPatch = 16;
constexpr int kMaxBases = kMaxPatch * kMaxPatch;

// Sylvester (natural-order) row index of the Walsh function with `s` sign changes, for an
// order-2^log2p transform: the Gray code of s, bit-reversed.
int sequency_to_natural(int s, int log2p);

// -1 if p is not one of 2, 4, 8, 16, else log2(p).
int patch_log2(int patch);

// Patches of a batch of H x W token grids.  A grid that is not a multiple of the patch is treated
// as zero-padded at its bottom and right edges up to the next multiple (the paper's own maps are
// 7 x 7 = 49 tokens, Section 3.3).
inline long patch_count(int N, int H, int W, int patch)
{
    return (long)N * ((H + patch - 1) / patch) * ((W + patch - 1) / patch);
}
inline bool grid_is_ragged(int H, int W, int patch) { return H % patch != 0 || W % patch != 0; }

// Everything the projection kernels need to know about the selected bases, passed to them by
// value in the kernel arguments (no device copy, no host/device synchronisation).
//
// A 2-D basis (u, v) in sequency order is natural-order coefficient nat(u)*p + nat(v) of the
// length-p^2 Hadamard transform of the row-major flattened patch.  If every selected nat(u) has
// its `mh` lowest bits clear and every nat(v) its `mw` lowest bits clear, the wanted coefficients
// equal those of the (p>>mh) x (p>>mw) transform of the patch sum-pooled over 2^mh x 2^mw token
// groups; `pooled_mask`/`pooled_pos` describe the selection in that smaller transform.
struct BasisPlan {
    int32_t patch;
    int32_t log2p;
    int32_t r;
    int32_t mh, mw;                 // pooling levels along H and W (0..log2p)
    uint8_t nat[kMaxBases];         // nat[k]: natural-order index of basis k in the p^2 transform
    uint64_t pooled_mask;           // bit j set: pooled natural coefficient j is selected (p <= 8)
    uint8_t pooled_pos[64];         // pooled natural coefficient j -> its position k (p <= 8)
};

// Checks patch / r / basis_idx and fills `plan`.  Returns LBP_OK or the matching error.
int make_basis_plan(int patch, const int32_t *basis_idx, int r, BasisPlan *plan);

int select_bases(int patch, int r, int order, int32_t *basis_idx);

// Low-heuristic-error selection (Section 3.2): the r bases of largest energy, by decreasing energy;
// equal energies keep the LP_L1 order.  energy has patch^2 entries indexed u*patch + v.
int select_lhe(const double *energy, int patch, int r, int32_t *basis_idx);

// Element size in bytes of a dtype code, 0 if unknown.
size_t dtype_size(int dtype);

// Shape / dtype / divisibility checks shared by the entry points.  patch == 0 skips the patch
// related checks (full-rank backward).
int validate_shape(const lbp_shape_t *shape, int patch);

// One tensor of a projection call.
int validate_grid(int N, int H, int W, int C, int dtype, int patch);

// LBP_ERR_ALIGN unless every listed pointer is 16-byte aligned (NULL entries are skipped).
int validate_alignment(const void *const *ptrs, int n);

// [a, a+na) and [b, b+nb) overlap?
bool ranges_overlap(const void *a, size_t na, const void *b, size_t nb);

// Tile shapes of the bf16 matrix-core GEMM (gemm_mfma_*.hip instantiates them in this order):
// 128x128, 64x128, 256x128, 256x256, then 128x128 and 64x128 with 8 instead of 4 wavefronts.
struct GemmTileInfo {
    int bm, bn;        // output tile of one workgroup
    bool fused;        // has the fused reverse-projection epilogue
    double slowdown;   // measured factor over the simple cost model below
    int max_n;         // only offered to products with at most this many columns (0: any)
    const char *name;  // for diagnostics
    bool whole_k = false;   // only offered to products the caller will not split along the reduction
};
constexpr int kNumGemmTiles = 8;
extern const GemmTileInfo kGemmTiles[kNumGemmTiles];

// How one matrix product is run.
struct GemmPlan {
    int tile;          // index into kGemmTiles
    int splits;        // split-K slices (1 = the kernel writes the final output itself)
    double est_us;     // cost-model estimate, for diagnostics
};

// Picks tile shape and split-K factor for C[M][N] = A * B with reduction length K.
//   out_elem_bytes  size of one output element when the kernel stores the result itself
//   allow_split     the caller can reduce fp32 partial results afterwards
//   fused_r/patch   non-zero: the reverse projection is fused into the epilogue (rows are
//                   (patch, basis) pairs, r bases kept); implies no split
// The model: a compute unit takes in about 20 bytes a clock from L2 however many loads are in
// flight, so a workgroup's time is its operand and output bytes over that rate (or its matrix-core
// time if larger), and the workgroups run in ceil(count / compute units) rounds.
// fused_wide: the fused epilogue is the matrix-core one, which needs a 128-column tile.
// only_tile >= 0: consider that tile shape alone (est_us is 1e300 / clock when it cannot run the product).
GemmPlan plan_gemm(long M, long N, long K, int out_elem_bytes, bool allow_split, int fused_r,
                   int fused_patch, int num_cus, bool fused_wide = false, int only_tile = -1);

// Workgroups the plan launches for an M x N output (fused_r as in plan_gemm).
long gemm_workgroups(const GemmPlan &g, long M, long N, int fused_r);

// Workspace layout of one backward call; offsets in bytes from the workspace base, each
// 256-byte aligned.  Sizes of 0 mean "not used".
struct WorkspacePlan {
    size_t gy_r, x_r, gx_r, splitk;   // offsets
    size_t total;                      // bytes
    GemmPlan gw;                       // the weight-gradient product
    GemmPlan gx;                       // the input-gradient product
    bool gx_fused;                     // reverse projection fused into that product's epilogue
    bool grouped;                      // both products run in one launch (tiles chosen for that)
    bool gx_coef16;                    // not fused: the product stores its coefficients as bf16 in one
                                       // piece (no split-K) and the reverse projection reads those
    int gx_join;                       // fused and grouped: slices of the input-gradient product's reduction that
                                       // combine inside the launch (1: none); their partial tiles live at gx_r,
    size_t gx_join_bytes;              // in this many bytes
};

// num_cus: compute units of the device (the GEMM plans depend on it); pass 256 when unknown.
// can_fuse: the selection allows the fused reverse projection (false gives the larger workspace);
// force_fuse: take it whenever allowed instead of comparing estimates; fused_wide: see plan_gemm;
// allow_group: the caller wants both gradients and can launch the two products as one grid;
// extra: tokens per image in front of the grid (tensors are [N][extra + H*W][C]);
// coef16: 1 = the caller has a reverse projection that reads bf16 coefficients (gx_coef16 may be
// chosen), 2 = take it whenever the reverse projection is not fused, 0 = never.
// gx_join: 0 = choose the number of joined slices of a fused, grouped input-gradient product, n = take n.
int plan_workspace(const lbp_shape_t *shape, int patch, int r, int num_cus, bool can_fuse,
                   bool force_fuse, WorkspacePlan *ws, bool fused_wide = false, bool allow_group = false,
                   int extra = 0, int coef16 = 0, int gx_join = 0);

// Estimated length in microseconds of a grouped launch on `num_cus` compute units: n_x workgroups of the
// input-gradient product (cost_x each) and n_w of the weight-gradient product (cost_w each), dispatched
// in that order (or the other way round), the i-th workgroup to unit i mod num_cus, workgroups on one
// unit sharing it.
double grouped_launch_estimate(long n_x, double cost_x, long n_w, double cost_w, int num_cus, bool w_first);

const char *status_string(int code);

// Kernel-choice switches (tests and measurement; see lbp_set_option in the public header).
struct Options {
    int wht_path = 0;          // 0 chosen per selection, 1 generic, 2 register, 3 matrix-core
    int gemm_simple = 0;       // 1: plain cross-check products
    int gemm_tile = -1;        // >= 0: one tile shape for every product
    int fuse_unproject = -1;   // -1 planner, 0 never, 1 wherever the kernel supports the selection
    int gemm_group = 1;        // 0: the two products of a call in separate launches; 2: one launch, weight gradient first
    int gx_coef = 1;           // 1 planner, 0 fp32 slices, 2 bf16 wherever the kernels allow
    int gx_join = 0;           // 0 planner, 1..8: that many joined slices wherever the grouped fused launch runs
};
// The current switches; the first call reads the LBP_* environment variables, once per process.
Options options();
// One switch by name; value NULL restores the default.  LBP_OK, LBP_ERR_NULL or LBP_ERR_OPTION.
int set_option(const char *name, const char *value);

}  // namespace lbp
