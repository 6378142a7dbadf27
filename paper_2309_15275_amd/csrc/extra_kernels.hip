// Tokens that are not on the grid (a class token in front of the patch tokens): they belong to no
// patch, so nothing is projected for them.  Their rows are appended, as they are, to the projected
// tensors (gather) so that the two products of the backward pass treat them exactly, and their rows
// of the input gradient are copied out of the product (scatter).  Tiny, bandwidth-trivial kernels:
// N * extra rows of C channels.
#include "device_utils.h"
#include "kernels.h"
#include "wht_device.h"

namespace lbp {
namespace {

template <bool BF16>
__global__ __launch_bounds__(256) void gather_extra_kernel(ExtraRows x)
{
    copy_extra_rows<BF16>(x, blockIdx.x, threadIdx.x);
}

// one thread: 4 consecutive channels of one row, summed over the slices in a fixed order
template <bool BF16>
__global__ __launch_bounds__(256) void scatter_extra_kernel(const float4 *__restrict__ in, int slices,
                                                            size_t slice_stride4, void *__restrict__ out, long items,
                                                            int C4, int extra, long img_tokens, float scale)
{
    const long item = (long)blockIdx.x * 256 + threadIdx.x;
    if (item >= items) return;
    const long row = item / C4;
    const int c4 = (int)(item - row * C4);
    const long n = row / extra;
    const int e = (int)(row - n * extra);
    float4 s = in[item];
    for (int z = 1; z < slices; ++z) {
        const float4 t = in[(size_t)z * slice_stride4 + item];
        s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    const size_t o = ((size_t)n * img_tokens + e) * C4 + c4;       // in units of 4 channels
    if (BF16)
        reinterpret_cast<uint2 *>(out)[o] = make_uint2(pack_bf16x2(s.x * scale, s.y * scale), pack_bf16x2(s.z * scale, s.w * scale));
    else
        reinterpret_cast<float4 *>(out)[o] = make_float4(s.x * scale, s.y * scale, s.z * scale, s.w * scale);
}

}  // namespace

hipError_t launch_gather_extra(const void *in, void *out, int N, int extra, long img_tokens, int C, int dtype,
                               float scale, hipStream_t stream)
{
    if (extra <= 0 || N <= 0) return hipSuccess;
    ExtraRows x{};
    set_extra_rows(x, 0, in, out, N, extra, img_tokens, C, dtype, scale);
    set_extra_rows(x, 1, nullptr, nullptr, N, extra, img_tokens, C, dtype, scale);
    if (dtype == LBP_BF16)
        hipLaunchKernelGGL(gather_extra_kernel<true>, dim3(x.blocks[0]), dim3(256), 0, stream, x);
    else
        hipLaunchKernelGGL(gather_extra_kernel<false>, dim3(x.blocks[0]), dim3(256), 0, stream, x);
    return hipGetLastError();
}

hipError_t launch_scatter_extra(const float *in, int slices, size_t slice_stride, void *out, int N, int extra,
                                long img_tokens, int C, int dtype, float scale, hipStream_t stream)
{
    if (extra <= 0 || N <= 0) return hipSuccess;
    if (slices < 1 || C % 4 || slice_stride % 4) return hipErrorInvalidValue;
    const int C4 = C / 4;
    const long items = (long)N * extra * C4;
    const unsigned blocks = (unsigned)((items + 255) / 256);
    if (dtype == LBP_BF16)
        hipLaunchKernelGGL(scatter_extra_kernel<true>, dim3(blocks), dim3(256), 0, stream, (const float4 *)in, slices,
                           slice_stride / 4, out, items, C4, extra, img_tokens, scale);
    else
        hipLaunchKernelGGL(scatter_extra_kernel<false>, dim3(blocks), dim3(256), 0, stream, (const float4 *)in, slices,
                           slice_stride / 4, out, items, C4, extra, img_tokens, scale);
    return hipGetLastError();
}

}  // namespace lbp
