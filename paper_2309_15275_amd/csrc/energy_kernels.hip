// Energy of every WHT basis of a tensor (Section 3.2, low-heuristic-error selection; the spectrum
// of Section 4.5): E[j] = sum over patches and channels of (coefficient j)^2.
//
// The coefficients of ALL p^2 bases are first produced by the projection kernels (row q*p^2 + j of
// the coefficient matrix is basis j of patch q); the kernels here square and add them up.  Sums
// are formed in a fixed order (per-thread fp32 over at most a few thousand terms, then fp64 within
// a workgroup and across workgroups), so the result is repeatable run to run.
#include "device_utils.h"
#include "kernels.h"

namespace lbp {
namespace {

constexpr int kEnergyThreads = 256;

// grid (p^2, NB): workgroup (j, b) covers basis j of patches [b*per, (b+1)*per)
template <bool BF16>
__global__ __launch_bounds__(kEnergyThreads) void energy_partial_kernel(const void *__restrict__ coef, long Q,
                                                                       int pp, int C, long per,
                                                                       double *__restrict__ partial)
{
    __shared__ double red[kEnergyThreads];
    const int j = blockIdx.x, b = blockIdx.y;
    const long q0 = (long)b * per, q1 = min(Q, q0 + per);
    const int vecs = BF16 ? C / 8 : C / 4;      // 16-byte vectors per row
    double total = 0.0;
    for (long q = q0; q < q1; ++q) {
        const uint4 *row = reinterpret_cast<const uint4 *>(coef) + ((size_t)q * pp + j) * vecs;
        float s = 0.f;
        for (int v = threadIdx.x; v < vecs; v += kEnergyThreads) {
            uint4 u = row[v];
            if (BF16) {
                float f[8] = {bf16_lo_to_f32(u.x), bf16_hi_to_f32(u.x), bf16_lo_to_f32(u.y), bf16_hi_to_f32(u.y),
                              bf16_lo_to_f32(u.z), bf16_hi_to_f32(u.z), bf16_lo_to_f32(u.w), bf16_hi_to_f32(u.w)};
#pragma unroll
                for (int e = 0; e < 8; ++e) s = fmaf(f[e], f[e], s);
            } else {
                float f[4] = {__uint_as_float(u.x), __uint_as_float(u.y), __uint_as_float(u.z), __uint_as_float(u.w)};
#pragma unroll
                for (int e = 0; e < 4; ++e) s = fmaf(f[e], f[e], s);
            }
        }
        total += (double)s;
    }
    red[threadIdx.x] = total;
    __syncthreads();
    for (int h = kEnergyThreads / 2; h > 0; h >>= 1) {
        if ((int)threadIdx.x < h) red[threadIdx.x] += red[threadIdx.x + h];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[(size_t)j * gridDim.y + b] = red[0];
}

// energy[j] += sum_b partial[j][b], one thread per basis, fixed order
__global__ void energy_final_kernel(const double *__restrict__ partial, int pp, int nb, double *energy)
{
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= pp) return;
    double s = 0.0;
    for (int b = 0; b < nb; ++b) s += partial[(size_t)j * nb + b];
    energy[j] += s;
}

}  // namespace

int energy_chunks(long Q)
{
    long nb = Q < 64 ? Q : 64;
    return (int)(nb < 1 ? 1 : nb);
}

hipError_t launch_energy(const void *coef, long Q, int pp, int C, int dtype, double *partial, double *energy,
                         hipStream_t stream)
{
    const int nb = energy_chunks(Q);
    const long per = (Q + nb - 1) / nb;
    dim3 grid((unsigned)pp, (unsigned)nb);
    if (dtype == LBP_BF16)
        hipLaunchKernelGGL(energy_partial_kernel<true>, grid, dim3(kEnergyThreads), 0, stream, coef, Q, pp, C, per, partial);
    else
        hipLaunchKernelGGL(energy_partial_kernel<false>, grid, dim3(kEnergyThreads), 0, stream, coef, Q, pp, C, per, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(energy_final_kernel, dim3((pp + 63) / 64), dim3(64), 0, stream, partial, pp, nb, energy);
    return hipGetLastError();
}

}  // namespace lbp
