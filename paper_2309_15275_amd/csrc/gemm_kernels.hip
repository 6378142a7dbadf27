// Matrix products of the backward pass on gfx950, the plain kernels:
//   gx_r = gy_r * W      (Algorithm 1, fourth statement)    A stored [M][K], B stored [K][N]
//   gW   = gy_r^T * x_r  (Algorithm 1, third statement)     A stored [K][M], B stored [K][N]
// and the same two shapes at full rank for Eq. 2.  B is always stored with the reduction index
// as its slow axis (W is [Cout][Cin], x_r is [rows][Cin]), A either way.
//
// fp32 operands: a 64x64x16 FMA kernel (the fp32 path exists for exactness checks, not speed).
// bf16 operands, "simple" path: 128x128x32 tiles with v_mfma_f32_32x32x16_bf16 and element-wise
// LDS transposition.  It is the slow, easy-to-read cross-check of the tuned kernel in
// gemm_mfma.hip and is only used when asked for.
// Split-K: slice z of the reduction writes its own fp32 partial result; a second kernel sums the
// slices in a fixed order, so results do not depend on scheduling.  This file also holds the
// dispatcher between the implementations.
#include "device_utils.h"
#include "kernels.h"

namespace lbp {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDA_KFAST = BK + 8;     // bf16 elements per LDS row of a [m][k] tile (80 bytes)
constexpr int LD_KSLOW = BM + 8;      // bf16 elements per LDS row of a [k][m] tile (272 bytes)

struct GemmDev {
    const unsigned short *A;
    const unsigned short *B;
    float *C;
    int M, N, K;
    long lda, ldb;
    int k_per_split;     // multiple of BK
    float scale;
};

__device__ __forceinline__ uint4 load16_or_zero(const unsigned short *p, bool ok)
{
    return ok ? *reinterpret_cast<const uint4 *>(p) : make_uint4(0u, 0u, 0u, 0u);
}

template <bool A_KFAST>
__global__ __launch_bounds__(256) void gemm_bf16_simple_kernel(GemmDev g)
{
    __shared__ __attribute__((aligned(16))) unsigned short As[A_KFAST ? BM * LDA_KFAST : BK * LD_KSLOW];
    __shared__ __attribute__((aligned(16))) unsigned short Bs[BK * LD_KSLOW];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int kbeg = blockIdx.z * g.k_per_split;
    const int kend = min(g.K, kbeg + g.k_per_split);

    f32x16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    uint4 ra[2], rb[2];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int c = tid + i * 256;
            if (A_KFAST) {
                int row = c >> 2, kc = c & 3;
                int m = m0 + row, k = k0 + kc * 8;
                ra[i] = load16_or_zero(g.A + (size_t)m * g.lda + k, m < g.M && k < kend);
            } else {
                int krow = c >> 4, cc = c & 15;
                int k = k0 + krow, m = m0 + cc * 8;
                ra[i] = load16_or_zero(g.A + (size_t)k * g.lda + m, k < kend && m < g.M);
            }
            int krow = c >> 4, cc = c & 15;
            int k = k0 + krow, n = n0 + cc * 8;
            rb[i] = load16_or_zero(g.B + (size_t)k * g.ldb + n, k < kend && n < g.N);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            int c = tid + i * 256;
            if (A_KFAST) {
                int row = c >> 2, kc = c & 3;
                *reinterpret_cast<uint4 *>(&As[row * LDA_KFAST + kc * 8]) = ra[i];
            } else {
                int krow = c >> 4, cc = c & 15;
                *reinterpret_cast<uint4 *>(&As[krow * LD_KSLOW + cc * 8]) = ra[i];
            }
            int krow = c >> 4, cc = c & 15;
            *reinterpret_cast<uint4 *>(&Bs[krow * LD_KSLOW + cc * 8]) = rb[i];
        }
    };

    const int li = lane & 31, kg = lane >> 5;
    if (kbeg < kend) {
        fetch(kbeg);
        for (int k0 = kbeg; k0 < kend; k0 += BK) {
            __syncthreads();          // previous tile fully consumed
            stage();
            __syncthreads();
            if (k0 + BK < kend) fetch(k0 + BK);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int kk = ks * 16 + kg * 8;
                bf16x8_t a[2], b[2];
#pragma unroll
                for (int mi = 0; mi < 2; ++mi) {
                    int row = wm * 64 + mi * 32 + li;
                    u16x8_t t;
                    if (A_KFAST) {
                        t = *reinterpret_cast<const u16x8_t *>(&As[row * LDA_KFAST + kk]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 8; ++e) t[e] = As[(kk + e) * LD_KSLOW + row];
                    }
                    a[mi] = __builtin_bit_cast(bf16x8_t, t);
                }
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    int col = wn * 64 + ni * 32 + li;
                    u16x8_t t;
#pragma unroll
                    for (int e = 0; e < 8; ++e) t[e] = Bs[(kk + e) * LD_KSLOW + col];
                    b[ni] = __builtin_bit_cast(bf16x8_t, t);
                }
#pragma unroll
                for (int mi = 0; mi < 2; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
            }
        }
    }

    // accumulator element 4*grp + e of a 32x32 tile is row 8*grp + 4*(lane/32) + e, column lane%32
    float *Cz = g.C + (size_t)blockIdx.z * g.M * g.N;
#pragma unroll
    for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            int col = n0 + wn * 64 + ni * 32 + li;
#pragma unroll
            for (int grp = 0; grp < 4; ++grp)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int row = m0 + wm * 64 + mi * 32 + grp * 8 + kg * 4 + e;
                    if (row < g.M && col < g.N) Cz[(size_t)row * g.N + col] = acc[mi][ni][grp * 4 + e] * g.scale;
                }
        }
}

// ---- fp32 operands -------------------------------------------------------------------------

constexpr int FM = 64, FN = 64, FK = 16;

struct GemmDevF32 {
    const float *A;
    const float *B;
    float *C;
    int M, N, K;
    long lda, ldb;
    int k_per_split;
    float scale;
};

template <bool A_KFAST>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmDevF32 g)
{
    __shared__ __attribute__((aligned(16))) float As[FK][FM + 4];
    __shared__ __attribute__((aligned(16))) float Bs[FK][FN + 4];
    const int tid = threadIdx.x;
    const int ty = tid >> 4, tx = tid & 15;
    const int m0 = blockIdx.y * FM, n0 = blockIdx.x * FN;
    const int kbeg = blockIdx.z * g.k_per_split;
    const int kend = min(g.K, kbeg + g.k_per_split);
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = kbeg; k0 < kend; k0 += FK) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int idx = tid + i * 256;
            int m, k;
            if (A_KFAST) { m = idx >> 4; k = idx & 15; } else { k = idx >> 6; m = idx & 63; }
            int gm = m0 + m, gk = k0 + k;
            float v = 0.f;
            if (gm < g.M && gk < kend)
                v = A_KFAST ? g.A[(size_t)gm * g.lda + gk] : g.A[(size_t)gk * g.lda + gm];
            As[k][m] = v;
            int kb = idx >> 6, n = idx & 63;
            int gn = n0 + n, gkb = k0 + kb;
            Bs[kb][n] = (gn < g.N && gkb < kend) ? g.B[(size_t)gkb * g.ldb + gn] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < FK; ++k) {
            float4 a = *reinterpret_cast<const float4 *>(&As[k][ty * 4]);
            float4 b = *reinterpret_cast<const float4 *>(&Bs[k][tx * 4]);
            float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
    float *Cz = g.C + (size_t)blockIdx.z * g.M * g.N;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = m0 + ty * 4 + i;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int col = n0 + tx * 4 + j;
            if (row < g.M && col < g.N) Cz[(size_t)row * g.N + col] = acc[i][j] * g.scale;
        }
    }
}

// ---- split-K reduction ------------------------------------------------------------------------

// out[i] = scale * sum_z part[z][i] in a FIXED order (results repeat bit for bit).  A workgroup
// owns 64 consecutive float4 elements; its four wavefronts take every fourth slice each, with all
// loads of a wavefront independent of one another (a small output split into many slices is bound
// by load latency, not bandwidth), and the four partial sums are combined through LDS:
// ((w0 + w1) + (w2 + w3)), w_g = part[g] + part[g+4] + ...
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float4 *__restrict__ part, int splits,
                                                            long count4, float scale, void *out)
{
    __shared__ float4 partial[3][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6;
    const long i = (long)blockIdx.x * 64 + lane;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < count4) {
        int z = g;
        for (; z + 12 < splits; z += 16) {          // four slices of this wavefront in flight together
            float4 t0 = part[(size_t)z * count4 + i], t1 = part[(size_t)(z + 4) * count4 + i];
            float4 t2 = part[(size_t)(z + 8) * count4 + i], t3 = part[(size_t)(z + 12) * count4 + i];
            s.x += t0.x; s.y += t0.y; s.z += t0.z; s.w += t0.w;
            s.x += t1.x; s.y += t1.y; s.z += t1.z; s.w += t1.w;
            s.x += t2.x; s.y += t2.y; s.z += t2.z; s.w += t2.w;
            s.x += t3.x; s.y += t3.y; s.z += t3.z; s.w += t3.w;
        }
        for (; z < splits; z += 4) {
            float4 t = part[(size_t)z * count4 + i];
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
    }
    if (g > 0) partial[g - 1][lane] = s;
    __syncthreads();
    if (g != 0 || i >= count4) return;
    const float4 w1 = partial[0][lane], w2 = partial[1][lane], w3 = partial[2][lane];
    s.x = (s.x + w1.x) + (w2.x + w3.x);
    s.y = (s.y + w1.y) + (w2.y + w3.y);
    s.z = (s.z + w1.z) + (w2.z + w3.z);
    s.w = (s.w + w1.w) + (w2.w + w3.w);
    s.x *= scale; s.y *= scale; s.z *= scale; s.w *= scale;
    if (OUT_BF16)
        reinterpret_cast<uint2 *>(out)[i] = make_uint2(pack_bf16x2(s.x, s.y), pack_bf16x2(s.z, s.w));
    else
        reinterpret_cast<float4 *>(out)[i] = s;
}

int round_up(int v, int m) { return (v + m - 1) / m * m; }

}  // namespace

hipError_t launch_gemm(const GemmArgs &a, GemmPath path, hipStream_t stream)
{
    if (a.M < 1 || a.N < 1 || a.K < 1 || a.splits < 1 || !a.A || !a.B || !a.C) return hipErrorInvalidValue;
    if (a.dtype == LBP_BF16 && path != GemmPath::kSimple) return launch_gemm_mfma(a, stream);
    return launch_gemm_simple(a, stream);
}

hipError_t launch_gemm_simple(const GemmArgs &a, hipStream_t stream)
{
    if (a.out != GemmOut::kF32) return hipErrorInvalidValue;   // the plain kernels only store fp32
    if (a.dtype == LBP_BF16) {
        // 16-byte vector loads: the fast axis of every operand must be a multiple of 8 elements
        if (a.N % 8 || a.ldb % 8 || a.lda % 8 || (a.a_kfast ? a.K % 8 : a.M % 8)) return hipErrorInvalidValue;
        GemmDev g;
        g.A = (const unsigned short *)a.A;
        g.B = (const unsigned short *)a.B;
        g.C = (float *)a.C;
        g.scale = a.scale;
        g.M = a.M; g.N = a.N; g.K = a.K;
        g.lda = a.lda; g.ldb = a.ldb;
        g.k_per_split = round_up((a.K + a.splits - 1) / a.splits, BK);
        dim3 grid((a.N + BN - 1) / BN, (a.M + BM - 1) / BM, a.splits);
        if (a.a_kfast) hipLaunchKernelGGL(gemm_bf16_simple_kernel<true>, grid, dim3(256), 0, stream, g);
        else hipLaunchKernelGGL(gemm_bf16_simple_kernel<false>, grid, dim3(256), 0, stream, g);
    } else if (a.dtype == LBP_F32) {
        GemmDevF32 g;
        g.A = (const float *)a.A;
        g.B = (const float *)a.B;
        g.C = (float *)a.C;
        g.scale = a.scale;
        g.M = a.M; g.N = a.N; g.K = a.K;
        g.lda = a.lda; g.ldb = a.ldb;
        g.k_per_split = round_up((a.K + a.splits - 1) / a.splits, FK);
        dim3 grid((a.N + FN - 1) / FN, (a.M + FM - 1) / FM, a.splits);
        if (a.a_kfast) hipLaunchKernelGGL(gemm_f32_kernel<true>, grid, dim3(256), 0, stream, g);
        else hipLaunchKernelGGL(gemm_f32_kernel<false>, grid, dim3(256), 0, stream, g);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_splitk_reduce(const float *part, int splits, long count, float scale, void *out,
                                int out_dtype, hipStream_t stream)
{
    if (count % 4 || splits < 1) return hipErrorInvalidValue;
    long count4 = count / 4;
    unsigned blocks = (unsigned)((count4 + 63) / 64);
    if (out_dtype == LBP_BF16)
        hipLaunchKernelGGL(splitk_reduce_kernel<true>, dim3(blocks), dim3(256), 0, stream,
                           (const float4 *)part, splits, count4, scale, out);
    else
        hipLaunchKernelGGL(splitk_reduce_kernel<false>, dim3(blocks), dim3(256), 0, stream,
                           (const float4 *)part, splits, count4, scale, out);
    return hipGetLastError();
}

}  // namespace lbp
