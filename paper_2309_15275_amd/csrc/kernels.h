// Internal launch interface between the C-ABI layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "lbp_host.h"

namespace lbp {

// Which implementation of a step to use.  kAuto picks the fastest one that supports the shape;
// the others exist so that tests can run every kernel on every shape it supports.
enum class WhtPath { kAuto = 0, kGeneric = 1, kRegister = 2, kMfma = 3 };
enum class GemmPath { kAuto = 0, kSimple = 1 };

// `extra` in the launchers below: tokens of every image in front of its grid (a class token, ...);
// tensors are then [N][extra + H*W][C] and those tokens belong to no patch (the projections skip
// them, see launch_gather_extra / launch_scatter_extra).
//
// p(.) of Eq. 6 per patch: in [N][H][W][C] -> out [P*r][C], both of `dtype`.  With extra > 0
// the N*extra tokens outside the grid follow as rows P*r ..., multiplied by extra_scale (0: they are
// skipped and nothing is appended).
hipError_t launch_project(const void *in, void *out, int N, int H, int W, int C, int dtype,
                          const BasisPlan &plan, WhtPath path, hipStream_t stream, int extra = 0,
                          float extra_scale = 1.0f);

// The same for two tensors on one token grid (gy and x of a backward call) in ONE launch where
// the kernels allow it, so that the second, smaller tensor fills the tail of the first.
hipError_t launch_project_pair(const void *in0, void *out0, int C0, const void *in1, void *out1, int C1,
                               int N, int H, int W, int dtype, const BasisPlan &plan, WhtPath path,
                               hipStream_t stream, int extra = 0, float extra_scale0 = 1.0f,
                               float extra_scale1 = 1.0f);

// p^-1(.) of Eq. 7 per patch with the 1/p^2 factor: in fp32 [slices][P*r][C] (the slices are
// summed first: split-K partial results) -> out [N][H][W][C] of `dtype`.  slice_rows > 0: rows
// of one slice when it holds more than the P*r coefficient rows.
hipError_t launch_unproject(const float *in, int slices, void *out, int N, int H, int W, int C,
                            int dtype, const BasisPlan &plan, WhtPath path, hipStream_t stream, int extra = 0,
                            long slice_rows = 0);
// The same from bf16 coefficients [P*r][C] in one piece (a product stored them, rounded once), for
// bf16 tensors and the selections the matrix-core form takes (unproject_bf16_supported).
bool unproject_bf16_supported(const BasisPlan &plan, WhtPath path, int dtype, int C);
hipError_t launch_unproject_bf16(const void *in, void *out, int N, int H, int W, int C, const BasisPlan &plan,
                                 hipStream_t stream, int extra = 0);

// Tokens outside the grid.  gather: out[n*extra + e][c] = scale * in[n][e][c] (rows appended to
// a projected tensor so that the products treat them exactly); scatter: the reverse for the
// input gradient, out[n][e][c] = scale * sum over slices of in[slice][n*extra + e][c] (fp32 in).
hipError_t launch_gather_extra(const void *in, void *out, int N, int extra, long img_tokens, int C, int dtype,
                               float scale, hipStream_t stream);
hipError_t launch_scatter_extra(const float *in, int slices, size_t slice_stride, void *out, int N, int extra,
                                long img_tokens, int C, int dtype, float scale, hipStream_t stream);

// Which projection kernel launch_project / launch_unproject take for this selection: "register",
// "matrix-core" or "generic" (host logic only).
const char *projection_kernel_name(const BasisPlan &plan, WhtPath path, int dtype, int C);

// Matrix-core form of the two projections (bf16 tensors, any selection, any patch up to 16).
bool wht_mfma_supported(const BasisPlan &plan, int dtype, int C);
hipError_t launch_project_mfma(const void *in0, void *out0, int C0, const void *in1, void *out1, int C1,
                               int N, int H, int W, const BasisPlan &plan, hipStream_t stream, int extra = 0,
                               float extra_scale0 = 1.0f, float extra_scale1 = 1.0f);
hipError_t launch_unproject_mfma(const float *in, int slices, void *out, int N, int H, int W, int C,
                                 const BasisPlan &plan, hipStream_t stream, int extra = 0, long slice_rows = 0,
                                 bool in_bf16 = false);

// energy[j] += sum over patches q and channels of coef[q*pp + j][c]^2 for all pp = p^2 bases; `partial`
// is scratch of pp * energy_chunks(Q) doubles.
int energy_chunks(long Q);
hipError_t launch_energy(const void *coef, long Q, int pp, int C, int dtype, double *partial, double *energy,
                         hipStream_t stream);

// What a matrix product does with its accumulators.
enum class GemmOut {
    kF32 = 0,        // C[z][M][N] fp32 = scale * partial product of split-K slice z
    kBF16 = 1,       // C[M][N] bf16 = scale * product            (splits must be 1)
    kUnproject = 2   // rows of the product are (patch, basis) pairs: apply p^-1(.) of Eq. 7 per
                     // patch in the epilogue and write bf16 tokens [N][H][W][Ncols]   (splits 1)
};

// Operand descriptions for the matrix products.  All matrices are row-major and dense along
// their fast axis; `ld` is the row pitch in elements.
//   a_kfast  true : A is stored [M][K] (K contiguous)      false: A is stored [K][M]
//   B is always stored [K][N] (N contiguous).
struct GemmArgs {
    const void *A = nullptr;
    const void *B = nullptr;
    int M = 0, N = 0, K = 0;
    long lda = 0, ldb = 0;
    bool a_kfast = true;
    int dtype = LBP_BF16;      // operand type; accumulation is fp32
    int splits = 1;            // split-K slices
    int tile = -1;             // tile shape of the bf16 matrix-core kernel, -1 = choose
    GemmOut out = GemmOut::kF32;
    void *C = nullptr;
    float scale = 1.0f;
    // kUnproject only: token grid of one image and the selected bases
    int grid_h = 0, grid_w = 0;
    const BasisPlan *plan = nullptr;
    // kUnproject only: `extra` tokens per image in front of the grid; the last extra_rows rows of A
    // are theirs (image-major) and their rows of the product go to those tokens, scaled by 1/patch^2
    int extra = 0, extra_rows = 0;
    // kUnproject with splits > 1 (8-wavefront 128-wide tiles, patch 8): gemm_join_bytes(...) bytes of device memory in
    // which the slices of a tile leave their partial sums for the one that finishes the tile
    void *join_parts = nullptr;
    size_t join_bytes = 0;     // size of that memory: a launch that needs more is refused
};

// True if launch_gemm runs this kUnproject product with its reduction in a.splits slices that join inside the launch.
bool gemm_join_supported(const GemmArgs &a, GemmPath path);
// Bytes of GemmArgs::join_parts for a kUnproject product of `tile` shape, M_rows x N with r bases, in `splits` slices.
size_t gemm_join_bytes(int tile, long M_rows, long N, int r, int splits);
// Most tiles such a product may have (one counter each).
constexpr int kJoinMaxTiles = 16384;

// True if launch_gemm supports GemmOut::kUnproject for this selection and dtype.
bool gemm_can_fuse_unproject(const BasisPlan &plan, int dtype, GemmPath path);
// True if the fused epilogue is the pooled register butterfly (else the matrix-core form, which
// needs a tile 128 columns wide).
bool gemm_unproject_pooled(const BasisPlan &plan);

hipError_t launch_gemm(const GemmArgs &g, GemmPath path, hipStream_t stream);

// The two products of one backward call in a single launch (bf16 matrix-core path only): `x` is
// the input-gradient product (A reduction-fast), `w` the weight-gradient product (A reduction-slow).
// gemm_pair_supported says whether the tiles chosen for the two have a grouped kernel; results
// are bit-identical to two launch_gemm calls.
bool gemm_pair_supported(const GemmArgs &x, const GemmArgs &w, GemmPath path);
hipError_t launch_gemm_pair(const GemmArgs &x, const GemmArgs &w, hipStream_t stream);

// out[i] = scale * sum_z part[z][i], i < count (count % 4 == 0), written as `out_dtype`.
hipError_t launch_splitk_reduce(const float *part, int splits, long count, float scale, void *out,
                                int out_dtype, hipStream_t stream);

// Implementation hooks between the two GEMM source files.
hipError_t launch_gemm_mfma(const GemmArgs &g, hipStream_t stream);
hipError_t launch_gemm_simple(const GemmArgs &g, hipStream_t stream);

}  // namespace lbp
