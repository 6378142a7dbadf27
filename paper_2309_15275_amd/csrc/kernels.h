// Internal launch interface between the C-ABI layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>

#include "lbp_host.h"

namespace lbp {

// Which implementation of a step to use.  kAuto picks the fastest one that supports the shape;
// the others exist so that tests can run every kernel on every shape it supports.
enum class WhtPath { kAuto = 0, kGeneric = 1, kRegister = 2 };

// p(.) of Eq. 6 per patch: in [N][H][W][C] -> out [P*r][C], both of `dtype`.
hipError_t launch_project(const void *in, void *out, int N, int H, int W, int C, int dtype,
                          const BasisPlan &plan, WhtPath path, hipStream_t stream);

// p^-1(.) of Eq. 7 per patch with the 1/p^2 factor: in fp32 [P*r][C] -> out [N][H][W][C] of `dtype`.
hipError_t launch_unproject(const float *in, void *out, int N, int H, int W, int C, int dtype,
                            const BasisPlan &plan, WhtPath path, hipStream_t stream);

// Operand descriptions for the matrix products.  All matrices are row-major and dense along
// their fast axis; `ld` is the row pitch in elements.
//   a_kfast  true : A is stored [M][K] (K contiguous)      false: A is stored [K][M]
//   B is always stored [K][N] (N contiguous).
struct GemmArgs {
    const void *A;
    const void *B;
    int M, N, K;
    long lda, ldb;
    bool a_kfast;
    int dtype;          // LBP_F32 or LBP_BF16 operands; accumulation is fp32 in both cases
    int splits;         // split-K slices; slice z writes C + z*M*N (fp32), unscaled
    float *C;           // fp32 output [splits][M][N]
};

// C[z] = A[:, Kz] * B[Kz, :] for every split-K slice z.
hipError_t launch_gemm(const GemmArgs &g, hipStream_t stream);

// out[i] = scale * sum_z part[z][i], i < count (count % 4 == 0), written as `out_dtype`.
hipError_t launch_splitk_reduce(const float *part, int splits, long count, float scale, void *out,
                                int out_dtype, hipStream_t stream);

}  // namespace lbp
