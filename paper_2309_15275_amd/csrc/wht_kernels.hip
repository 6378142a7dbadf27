// Walsh-Hadamard projection p(.) (Eq. 6) and reverse projection p^-1(.) (Eq. 7) per token patch,
// for gfx950.  Both are HBM-bandwidth bound: every input element is read once and every output
// element written once, with additions and subtractions only in between (Section 3, fourth
// property of the WHT) plus one exact power-of-two scale in the reverse direction.
//
// Two implementations of each direction:
//   * "register" kernels (patch 2, 4, 8): one lane owns one 32-bit column of channels (two bf16 or
//     one fp32) of one patch, loads the patch's p*p tokens straight into registers (every load of
//     a wavefront covers 256 contiguous bytes), sum-pools away the butterfly stages that no
//     selected basis needs, runs the remaining butterfly in registers and stores the r selected
//     coefficients.  Lanes are numbered (patch, channel column) so that thin layers (few
//     channels) still fill wavefronts: neighbouring patches of one patch-row are neighbours in
//     memory.
//   * "generic" kernels (any patch up to 16, any selection): the matrix form of Eq. 6 / Eq. 7,
//     signs from the parity of popcount(natural index & token index).  Slower, used for patch 16
//     and kept selectable for testing.
#include "device_utils.h"
#include "kernels.h"
#include "wht_device.h"

namespace lbp {
namespace {

// ------------------------------------------------------------------------------------------
// register kernels
// ------------------------------------------------------------------------------------------

// One tensor of a projection launch.  A launch can carry two (gy and x of one backward call):
// the first `blocks` workgroups belong to tensor 0, the rest to tensor 1.
struct ProjTensor {
    const uint32_t *in;
    uint32_t *out;
    long items;         // patches * 32-bit channel columns
    int Cd;             // 32-bit channel columns per token
    unsigned blocks;    // workgroups of this tensor
};

template <int LP, int MH, int MW, bool BF16>
__global__ __launch_bounds__(256) void wht_project_reg_kernel(ProjTensor t0, ProjTensor t1, GridGeom g,
                                                              PooledSel sel, int r, ExtraRows xr)
{
    constexpr int P = 1 << LP;
    constexpr int NC = (P >> MH) * (P >> MW);
    if (blockIdx.x >= t0.blocks + t1.blocks) {      // appended workgroups: tokens outside the grid
        copy_extra_rows<BF16>(xr, blockIdx.x - (t0.blocks + t1.blocks), threadIdx.x);
        return;
    }
    const bool second = blockIdx.x >= t0.blocks;
    const ProjTensor &t = second ? t1 : t0;
    const int Cd = t.Cd;
    long item = (long)(blockIdx.x - (second ? t0.blocks : 0u)) * 256 + threadIdx.x;
    if (item >= t.items) return;
    long q;
    if (t.items <= 0xffffffffLL) q = (long)((unsigned)item / (unsigned)Cd);      // a 64-bit division costs ~100 instructions
    else q = item / Cd;
    int cd = (int)(item - q * Cd);
    long n;
    int a0, b0;
    g.origin(q, n, a0, b0);
    const uint32_t *src = t.in + g.token(n, a0, b0) * Cd + cd;

    uint32_t raw[P * P];
    if (a0 + P <= g.Ht && b0 + P <= g.Wt) {
#pragma unroll
        for (int h = 0; h < P; ++h) {
#pragma unroll
            for (int w = 0; w < P; ++w)
                raw[h * P + w] = __builtin_nontemporal_load(src + ((size_t)h * g.Wt + w) * Cd);   // read once
        }
    } else {
        // a patch that hangs over the bottom or right edge of the grid: the missing tokens are zeros
        const int hv = g.Ht - a0, wv = g.Wt - b0;
#pragma unroll
        for (int h = 0; h < P; ++h) {
#pragma unroll
            for (int w = 0; w < P; ++w) {
                uint32_t v = 0u;
                if (h < hv && w < wv) v = __builtin_nontemporal_load(src + ((size_t)h * g.Wt + w) * Cd);
                raw[h * P + w] = v;
            }
        }
    }

    uint32_t *dst = t.out + (size_t)q * r * Cd + cd;
    if (BF16) {
        // low halves first; their coefficients wait as rounded bf16 pairs (half the registers)
        // while the high halves go through the same transform
        float c[NC];
        pooled_transform_raw<P, MH, MW, 0>(raw, c);
        uint32_t lo[(NC + 1) / 2];
#pragma unroll
        for (int j = 0; j < NC; j += 2) lo[j / 2] = f32_to_bf16_bits(c[j]) | (f32_to_bf16_bits(c[j + 1 < NC ? j + 1 : j]) << 16);
        pooled_transform_raw<P, MH, MW, 1>(raw, c);
#pragma unroll
        for (int j = 0; j < NC; ++j)
            if ((sel.mask >> j) & 1ull) {
                uint32_t l = (j & 1) ? (lo[j / 2] >> 16) : (lo[j / 2] & 0xffffu);
                dst[(size_t)sel.pos[j] * Cd] = l | (f32_to_bf16_bits(c[j]) << 16);
            }
    } else {
        float c[NC];
        pooled_transform_raw<P, MH, MW, 2>(raw, c);
#pragma unroll
        for (int j = 0; j < NC; ++j)
            if ((sel.mask >> j) & 1ull) dst[(size_t)sel.pos[j] * Cd] = __float_as_uint(c[j]);
    }
}

// Reverse direction: lane = (patch, 32-bit output column).  Reads the r selected fp32
// coefficients, zero-fills the others, transforms, replicates over the pooled token groups.
template <int LP, int MH, int MW, bool BF16>
__global__ __launch_bounds__(256) void wht_unproject_reg_kernel(const float *__restrict__ in,
                                                                uint32_t *__restrict__ out,
                                                                long items, int Cd, GridGeom g,
                                                                PooledSel sel, int r, int slices,
                                                                size_t slice_stride)
{
    constexpr int P = 1 << LP;
    constexpr int PWd = P >> MW;
    constexpr int NC = (P >> MH) * PWd;
    constexpr float scale = 1.0f / (float)(P * P);
    long item = (long)blockIdx.x * 256 + threadIdx.x;
    if (item >= items) return;
    long q;
    if (items <= 0xffffffffLL) q = (long)((unsigned)item / (unsigned)Cd);      // a 64-bit division costs ~100 instructions
    else q = item / Cd;
    int cd = (int)(item - q * Cd);
    long n;
    int a0, b0;
    g.origin(q, n, a0, b0);
    uint32_t *dst = out + g.token(n, a0, b0) * Cd + cd;
    const int hv = g.Ht - a0, wv = g.Wt - b0;      // tokens of the patch that exist (>= P: all of them)

    if (BF16) {
        const int C = Cd * 2;
        const float2 *src = reinterpret_cast<const float2 *>(in + (size_t)q * r * C) + cd;
        float c0[NC], c1[NC];
#pragma unroll
        for (int j = 0; j < NC; ++j) c0[j] = c1[j] = 0.f;
        // slice by slice (fixed order: deterministic sums), all coefficients of a slice in flight
        // together
        for (int z = 0; z < slices; ++z) {
            const float2 *sz = reinterpret_cast<const float2 *>(reinterpret_cast<const float *>(src) + z * slice_stride);
#pragma unroll
            for (int j = 0; j < NC; ++j) {
                if ((sel.mask >> j) & 1ull) {
                    float2 t = sz[(size_t)sel.pos[j] * Cd];
                    c0[j] += t.x;
                    c1[j] += t.y;
                }
            }
        }
        fwht_inplace<NC>(c0);
        fwht_inplace<NC>(c1);
        if (hv >= P && wv >= P) {                 // the whole patch is inside the grid
#pragma unroll
            for (int h = 0; h < P; ++h) {
#pragma unroll
                for (int w = 0; w < P; ++w) {
                    int j = (h >> MH) * PWd + (w >> MW);
                    __builtin_nontemporal_store(pack_bf16x2(c0[j] * scale, c1[j] * scale), dst + ((size_t)h * g.Wt + w) * Cd);
                }
            }
        } else {
#pragma unroll
            for (int h = 0; h < P; ++h) {
#pragma unroll
                for (int w = 0; w < P; ++w) {
                    int j = (h >> MH) * PWd + (w >> MW);
                    if (h < hv && w < wv)
                        __builtin_nontemporal_store(pack_bf16x2(c0[j] * scale, c1[j] * scale), dst + ((size_t)h * g.Wt + w) * Cd);
                }
            }
        }
    } else {
        const float *src = in + (size_t)q * r * Cd + cd;
        float c0[NC];
#pragma unroll
        for (int j = 0; j < NC; ++j) c0[j] = 0.f;
        for (int z = 0; z < slices; ++z) {
            const float *sz = src + z * slice_stride;
#pragma unroll
            for (int j = 0; j < NC; ++j)
                if ((sel.mask >> j) & 1ull) c0[j] += sz[(size_t)sel.pos[j] * Cd];
        }
        fwht_inplace<NC>(c0);
#pragma unroll
        for (int h = 0; h < P; ++h) {
#pragma unroll
            for (int w = 0; w < P; ++w) {
                int j = (h >> MH) * PWd + (w >> MW);
                if (h < hv && w < wv)
                    __builtin_nontemporal_store(__float_as_uint(c0[j] * scale), dst + ((size_t)h * g.Wt + w) * Cd);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// generic kernels (matrix form)
// ------------------------------------------------------------------------------------------

template <bool BF16>
struct Vec16;   // one 16-byte vector of channels as fp32 lanes
template <>
struct Vec16<false> {
    static constexpr int N = 4;
    __device__ static void load(const uint4 &u, float (&f)[4])
    {
        f[0] = __uint_as_float(u.x); f[1] = __uint_as_float(u.y);
        f[2] = __uint_as_float(u.z); f[3] = __uint_as_float(u.w);
    }
};
template <>
struct Vec16<true> {
    static constexpr int N = 8;
    __device__ static void load(const uint4 &u, float (&f)[8])
    {
        f[0] = bf16_lo_to_f32(u.x); f[1] = bf16_hi_to_f32(u.x);
        f[2] = bf16_lo_to_f32(u.y); f[3] = bf16_hi_to_f32(u.y);
        f[4] = bf16_lo_to_f32(u.z); f[5] = bf16_hi_to_f32(u.z);
        f[6] = bf16_lo_to_f32(u.w); f[7] = bf16_hi_to_f32(u.w);
    }
};

__device__ __forceinline__ uint4 store_vec(const float (&f)[4])
{
    return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]),
                      __float_as_uint(f[3]));
}
__device__ __forceinline__ uint4 store_vec(const float (&f)[8])
{
    return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                      pack_bf16x2(f[6], f[7]));
}

// grid.x = patch, grid.y * blockDim.x covers the 16-byte channel vectors of a token.
template <bool BF16>
__global__ __launch_bounds__(128) void wht_project_generic_kernel(const uint4 *__restrict__ in,
                                                                  uint4 *__restrict__ out, int Cv,
                                                                  GridGeom g, NatTable nat, int r)
{
    constexpr int VN = Vec16<BF16>::N;
    constexpr int KC = 4;
    int cv = blockIdx.y * blockDim.x + threadIdx.x;
    if (cv >= Cv) return;
    long q = blockIdx.x;
    int p = g.patch, pp = p * p;
    long n;
    int a0, b0;
    g.origin(q, n, a0, b0);
    const uint4 *src = in + g.token(n, a0, b0) * Cv + cv;
    for (int k0 = 0; k0 < r; k0 += KC) {
        float acc[KC][VN];
#pragma unroll
        for (int kk = 0; kk < KC; ++kk)
#pragma unroll
            for (int e = 0; e < VN; ++e) acc[kk][e] = 0.f;
        for (int t = 0; t < pp; ++t) {
            int h = t / p, w = t - h * p;
            if (a0 + h >= g.Ht || b0 + w >= g.Wt) continue;      // zero padding past the grid's edge
            float f[VN];
            Vec16<BF16>::load(src[((size_t)h * g.Wt + w) * Cv], f);
#pragma unroll
            for (int kk = 0; kk < KC; ++kk) {
                int k = k0 + kk < r ? k0 + kk : r - 1;
                bool neg = __popc((unsigned)nat.v[k] & (unsigned)t) & 1;
#pragma unroll
                for (int e = 0; e < VN; ++e) acc[kk][e] += neg ? -f[e] : f[e];
            }
        }
#pragma unroll
        for (int kk = 0; kk < KC; ++kk)
            if (k0 + kk < r) out[((size_t)q * r + k0 + kk) * Cv + cv] = store_vec(acc[kk]);
    }
}

// Reverse, matrix form.  Input is fp32 [P*r][C]; thread = (patch, 16-byte OUTPUT vector).
template <bool BF16>
__global__ __launch_bounds__(128) void wht_unproject_generic_kernel(const float *__restrict__ in,
                                                                    uint4 *__restrict__ out, int Cv,
                                                                    GridGeom g, NatTable nat, int r,
                                                                    int slices, size_t slice_stride)
{
    constexpr int VN = Vec16<BF16>::N;
    constexpr int TC = 4;
    int cv = blockIdx.y * blockDim.x + threadIdx.x;
    if (cv >= Cv) return;
    long q = blockIdx.x;
    int p = g.patch, pp = p * p;
    const int C = Cv * VN;
    const float scale = 1.0f / (float)pp;
    const float *src = in + (size_t)q * r * C + (size_t)cv * VN;
    long n;
    int a0, b0;
    g.origin(q, n, a0, b0);
    uint4 *dst = out + g.token(n, a0, b0) * Cv + cv;
    for (int t0 = 0; t0 < pp; t0 += TC) {     // pp is a multiple of 4 for every legal patch
        float acc[TC][VN];
#pragma unroll
        for (int tt = 0; tt < TC; ++tt)
#pragma unroll
            for (int e = 0; e < VN; ++e) acc[tt][e] = 0.f;
        for (int k = 0; k < r; ++k) {
            float f[VN];
#pragma unroll
            for (int e = 0; e < VN; e += 4) {
                float4 t4 = *reinterpret_cast<const float4 *>(src + (size_t)k * C + e);
                for (int z = 1; z < slices; ++z) {
                    float4 u4 = *reinterpret_cast<const float4 *>(src + z * slice_stride + (size_t)k * C + e);
                    t4.x += u4.x; t4.y += u4.y; t4.z += u4.z; t4.w += u4.w;
                }
                f[e] = t4.x; f[e + 1] = t4.y; f[e + 2] = t4.z; f[e + 3] = t4.w;
            }
#pragma unroll
            for (int tt = 0; tt < TC; ++tt) {
                bool neg = __popc((unsigned)nat.v[k] & (unsigned)(t0 + tt)) & 1;
#pragma unroll
                for (int e = 0; e < VN; ++e) acc[tt][e] += neg ? -f[e] : f[e];
            }
        }
#pragma unroll
        for (int tt = 0; tt < TC; ++tt) {
            int t = t0 + tt;
            int h = t / p, w = t - h * p;
#pragma unroll
            for (int e = 0; e < VN; ++e) acc[tt][e] *= scale;
            if (a0 + h < g.Ht && b0 + w < g.Wt) dst[((size_t)h * g.Wt + w) * Cv] = store_vec(acc[tt]);
        }
    }
}

// ------------------------------------------------------------------------------------------
// dispatch
// ------------------------------------------------------------------------------------------

// Slices of the reverse direction's input (split-K partial sums) and their pitch in floats.
struct Slices {
    int count = 1;
    size_t stride = 0;
};

// Second tensor of a projection launch (unused by the reverse direction).
struct Second {
    const void *in = nullptr;
    void *out = nullptr;
    long items = 0;
    int Cd = 0;
    ExtraRows xr{};      // tokens outside the grid, copied by workgroups appended to the launch
};

template <bool UNPROJECT, int LP, int MH, int MW, bool BF16>
void launch_reg_one(const void *in, void *out, long items, int Cd, const GridGeom &g,
                    const PooledSel &sel, int r, Slices sl, Second sec, hipStream_t stream)
{
    unsigned blocks = (unsigned)((items + 255) / 256);
    if (!UNPROJECT) {
        ProjTensor t0{(const uint32_t *)in, (uint32_t *)out, items, Cd, blocks};
        ProjTensor t1{(const uint32_t *)sec.in, (uint32_t *)sec.out, sec.items, sec.Cd > 0 ? sec.Cd : 1,
                      (unsigned)((sec.items + 255) / 256)};
        hipLaunchKernelGGL((wht_project_reg_kernel<LP, MH, MW, BF16>),
                           dim3(t0.blocks + t1.blocks + sec.xr.blocks[0] + sec.xr.blocks[1]), dim3(256), 0, stream, t0,
                           t1, g, sel, r, sec.xr);
        return;
    }
    if (UNPROJECT)
        hipLaunchKernelGGL((wht_unproject_reg_kernel<LP, MH, MW, BF16>), dim3(blocks), dim3(256), 0,
                           stream, (const float *)in, (uint32_t *)out, items, Cd, g, sel, r, sl.count,
                           sl.stride);
}

template <bool UNPROJECT, int LP, int MH, bool BF16>
void launch_reg_mw(int mw, const void *in, void *out, long items, int Cd, const GridGeom &g,
                   const PooledSel &sel, int r, Slices sl, Second sec, hipStream_t s)
{
    switch (mw) {
        case 0: launch_reg_one<UNPROJECT, LP, MH, 0, BF16>(in, out, items, Cd, g, sel, r, sl, sec, s); break;
        case 1: launch_reg_one<UNPROJECT, LP, MH, (LP >= 1 ? 1 : 0), BF16>(in, out, items, Cd, g, sel, r, sl, sec, s); break;
        case 2: launch_reg_one<UNPROJECT, LP, MH, (LP >= 2 ? 2 : 0), BF16>(in, out, items, Cd, g, sel, r, sl, sec, s); break;
        default: launch_reg_one<UNPROJECT, LP, MH, (LP >= 3 ? 3 : 0), BF16>(in, out, items, Cd, g, sel, r, sl, sec, s); break;
    }
}

template <bool UNPROJECT, int LP, bool BF16>
void launch_reg_mh(int mh, int mw, const void *in, void *out, long items, int Cd, const GridGeom &g,
                   const PooledSel &sel, int r, Slices sl, Second sec, hipStream_t s)
{
    switch (mh) {
        case 0: launch_reg_mw<UNPROJECT, LP, 0, BF16>(mw, in, out, items, Cd, g, sel, r, sl, sec, s); break;
        case 1: launch_reg_mw<UNPROJECT, LP, (LP >= 1 ? 1 : 0), BF16>(mw, in, out, items, Cd, g, sel, r, sl, sec, s); break;
        case 2: launch_reg_mw<UNPROJECT, LP, (LP >= 2 ? 2 : 0), BF16>(mw, in, out, items, Cd, g, sel, r, sl, sec, s); break;
        default: launch_reg_mw<UNPROJECT, LP, (LP >= 3 ? 3 : 0), BF16>(mw, in, out, items, Cd, g, sel, r, sl, sec, s); break;
    }
}

// in2/out2/C2: optional second tensor on the same token grid (projection only).
template <bool UNPROJECT>
hipError_t launch_reg(const void *in, void *out, int N, int H, int W, int C, int dtype,
                      const BasisPlan &plan, Slices sl, hipStream_t s, int extra, const void *in2 = nullptr,
                      void *out2 = nullptr, int C2 = 0, float extra_scale = 1.0f, float extra_scale2 = 1.0f)
{
    const bool bf16 = dtype == LBP_BF16;
    const int Cd = bf16 ? C / 2 : C;
    const long Q = patch_count(N, H, W, plan.patch);
    const long items = Q * Cd;
    Second sec;
    if (in2) {
        sec.in = in2;
        sec.out = out2;
        sec.Cd = bf16 ? C2 / 2 : C2;
        sec.items = Q * sec.Cd;
    }
    if (!UNPROJECT && extra > 0) {
        const size_t esz = dtype_size(dtype);
        const size_t rows = (size_t)Q * plan.r;
        const long img_tokens = (long)H * W + extra;
        set_extra_rows(sec.xr, 0, in, (char *)out + rows * C * esz, N, extra, img_tokens, C, dtype, extra_scale);
        set_extra_rows(sec.xr, 1, in2, in2 ? (char *)out2 + rows * C2 * esz : nullptr, N, extra, img_tokens,
                       in2 ? C2 : C, dtype, extra_scale2);
    }
    GridGeom g = make_geom(H, W, plan.patch, extra);
    PooledSel sel;
    sel.mask = plan.pooled_mask;
    for (int j = 0; j < 64; ++j) sel.pos[j] = plan.pooled_pos[j];
    // mh <= log2p and mw <= log2p always hold for a plan made by make_basis_plan
    const int mh = plan.mh, mw = plan.mw, r = plan.r;
    switch (plan.log2p) {
        case 1:
            if (bf16) launch_reg_mh<UNPROJECT, 1, true>(mh, mw, in, out, items, Cd, g, sel, r, sl, sec, s);
            else launch_reg_mh<UNPROJECT, 1, false>(mh, mw, in, out, items, Cd, g, sel, r, sl, sec, s);
            break;
        case 2:
            if (bf16) launch_reg_mh<UNPROJECT, 2, true>(mh, mw, in, out, items, Cd, g, sel, r, sl, sec, s);
            else launch_reg_mh<UNPROJECT, 2, false>(mh, mw, in, out, items, Cd, g, sel, r, sl, sec, s);
            break;
        case 3:
            if (bf16) launch_reg_mh<UNPROJECT, 3, true>(mh, mw, in, out, items, Cd, g, sel, r, sl, sec, s);
            else launch_reg_mh<UNPROJECT, 3, false>(mh, mw, in, out, items, Cd, g, sel, r, sl, sec, s);
            break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <bool UNPROJECT>
hipError_t launch_generic(const void *in, void *out, int N, int H, int W, int C, int dtype,
                          const BasisPlan &plan, Slices sl, hipStream_t s, int extra)
{
    const bool bf16 = dtype == LBP_BF16;
    const int Cv = bf16 ? C / 8 : C / 4;
    const long Q = patch_count(N, H, W, plan.patch);
    GridGeom g = make_geom(H, W, plan.patch, extra);
    NatTable nat;
    for (int k = 0; k < kMaxBases; ++k) nat.v[k] = plan.nat[k];
    dim3 grid((unsigned)Q, (unsigned)((Cv + 127) / 128));
    if (UNPROJECT) {
        if (bf16)
            hipLaunchKernelGGL(wht_unproject_generic_kernel<true>, grid, dim3(128), 0, s,
                               (const float *)in, (uint4 *)out, Cv, g, nat, plan.r, sl.count, sl.stride);
        else
            hipLaunchKernelGGL(wht_unproject_generic_kernel<false>, grid, dim3(128), 0, s,
                               (const float *)in, (uint4 *)out, Cv, g, nat, plan.r, sl.count, sl.stride);
    } else {
        if (bf16)
            hipLaunchKernelGGL(wht_project_generic_kernel<true>, grid, dim3(128), 0, s,
                               (const uint4 *)in, (uint4 *)out, Cv, g, nat, plan.r);
        else
            hipLaunchKernelGGL(wht_project_generic_kernel<false>, grid, dim3(128), 0, s,
                               (const uint4 *)in, (uint4 *)out, Cv, g, nat, plan.r);
    }
    return hipGetLastError();
}

bool use_register_path(const BasisPlan &plan, WhtPath path)
{
    if (plan.patch > 8) return false;
    return path != WhtPath::kGeneric;
}

// The matrix-core form takes over where the pooled butterfly cannot prune (more than 16 pooled
// coefficients per channel) and for patch 16.
bool use_mfma_path(const BasisPlan &plan, WhtPath path, int dtype, int C)
{
    if (!wht_mfma_supported(plan, dtype, C)) return false;
    if (path == WhtPath::kMfma) return true;
    if (path != WhtPath::kAuto) return false;
    if (plan.patch > 8) return true;
    return (plan.patch >> plan.mh) * (plan.patch >> plan.mw) > 16;
}

// The generic kernels have a two-dimensional grid: the tokens outside the grid get a launch of their own.
hipError_t gather_after_generic(const void *in, void *out, int N, int H, int W, int C, int dtype, const BasisPlan &plan,
                                int extra, float scale, hipStream_t stream)
{
    if (extra <= 0 || scale == 0.0f) return hipSuccess;
    const size_t rows = (size_t)patch_count(N, H, W, plan.patch) * plan.r;
    return launch_gather_extra(in, (char *)out + rows * C * dtype_size(dtype), N, extra, (long)H * W + extra, C, dtype,
                               scale, stream);
}

}  // namespace

const char *projection_kernel_name(const BasisPlan &plan, WhtPath path, int dtype, int C)
{
    if (use_mfma_path(plan, path, dtype, C)) return "matrix-core";
    if (use_register_path(plan, path)) return "register";
    return "generic";
}

hipError_t launch_project(const void *in, void *out, int N, int H, int W, int C, int dtype,
                          const BasisPlan &plan, WhtPath path, hipStream_t stream, int extra, float extra_scale)
{
    if (use_mfma_path(plan, path, dtype, C))
        return launch_project_mfma(in, out, C, nullptr, nullptr, 0, N, H, W, plan, stream, extra, extra_scale, 1.0f);
    if (use_register_path(plan, path))
        return launch_reg<false>(in, out, N, H, W, C, dtype, plan, Slices{}, stream, extra, nullptr, nullptr, 0,
                                 extra_scale, 1.0f);
    hipError_t e = launch_generic<false>(in, out, N, H, W, C, dtype, plan, Slices{}, stream, extra);
    if (e != hipSuccess) return e;
    return gather_after_generic(in, out, N, H, W, C, dtype, plan, extra, extra_scale, stream);
}

hipError_t launch_project_pair(const void *in0, void *out0, int C0, const void *in1, void *out1, int C1,
                               int N, int H, int W, int dtype, const BasisPlan &plan, WhtPath path,
                               hipStream_t stream, int extra, float extra_scale0, float extra_scale1)
{
    if (use_mfma_path(plan, path, dtype, C0) && use_mfma_path(plan, path, dtype, C1))
        return launch_project_mfma(in0, out0, C0, in1, out1, C1, N, H, W, plan, stream, extra, extra_scale0,
                                   extra_scale1);
    if (use_register_path(plan, path))
        return launch_reg<false>(in0, out0, N, H, W, C0, dtype, plan, Slices{}, stream, extra, in1, out1, C1,
                                 extra_scale0, extra_scale1);
    hipError_t e = launch_generic<false>(in0, out0, N, H, W, C0, dtype, plan, Slices{}, stream, extra);
    if (e != hipSuccess) return e;
    e = launch_generic<false>(in1, out1, N, H, W, C1, dtype, plan, Slices{}, stream, extra);
    if (e != hipSuccess) return e;
    e = gather_after_generic(in0, out0, N, H, W, C0, dtype, plan, extra, extra_scale0, stream);
    if (e != hipSuccess) return e;
    return gather_after_generic(in1, out1, N, H, W, C1, dtype, plan, extra, extra_scale1, stream);
}

hipError_t launch_unproject(const float *in, int slices, void *out, int N, int H, int W, int C,
                            int dtype, const BasisPlan &plan, WhtPath path, hipStream_t stream, int extra,
                            long slice_rows)
{
    if (slices < 1) return hipErrorInvalidValue;
    if (use_mfma_path(plan, path, dtype, C))
        return launch_unproject_mfma(in, slices, out, N, H, W, C, plan, stream, extra, slice_rows);
    Slices sl;
    sl.count = slices;
    sl.stride = (size_t)(slice_rows > 0 ? slice_rows : patch_count(N, H, W, plan.patch) * plan.r) * C;
    if (use_register_path(plan, path))
        return launch_reg<true>(in, out, N, H, W, C, dtype, plan, sl, stream, extra);
    return launch_generic<true>(in, out, N, H, W, C, dtype, plan, sl, stream, extra);
}

bool unproject_bf16_supported(const BasisPlan &plan, WhtPath path, int dtype, int C)
{
    return use_mfma_path(plan, path, dtype, C);
}

hipError_t launch_unproject_bf16(const void *in, void *out, int N, int H, int W, int C, const BasisPlan &plan,
                                 hipStream_t stream, int extra)
{
    if (!wht_mfma_supported(plan, LBP_BF16, C)) return hipErrorInvalidValue;
    return launch_unproject_mfma((const float *)in, 1, out, N, H, W, C, plan, stream, extra, 0, true);
}

}  // namespace lbp
