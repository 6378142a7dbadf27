// Device-side pieces of the Walsh-Hadamard projections that more than one kernel file uses:
// the per-launch tables passed by value and the pooled in-register transform.
#pragma once
#include "device_utils.h"
#include "lbp_host.h"

namespace lbp {

struct NatTable {
    uint8_t v[kMaxBases];
};

struct PooledSel {
    uint64_t mask;
    uint8_t pos[64];
};

// Decomposition of a patch number into its place on the token grid.  The grid may end inside the
// last patch row / column (zero padding): tokens with row >= Ht or column >= Wt do not exist.
struct GridGeom {
    int Wt;        // tokens per grid row (W)
    int Ht;        // grid rows (H)
    int HWt;       // tokens per image (H*W)
    int PW;        // patches per grid row, ceil(W / patch)
    int PHW;       // patches per image
    int patch;
    int img;       // tokens one image occupies in memory: tokens in front of the grid + H*W
    int tok0;      // tokens of an image in front of its grid (class token ...), not part of any patch
    // image n, first grid row a0 and first grid column b0 of patch q (patch numbers fit 31 bits:
    // the token count does; 32-bit divisions are several times cheaper than 64-bit ones)
    __device__ __forceinline__ void origin(long q, long &n, int &a0, int &b0) const
    {
        const unsigned uq = (unsigned)q;
        const unsigned un = uq / (unsigned)PHW;
        const unsigned rem = uq - un * (unsigned)PHW;
        const unsigned a = rem / (unsigned)PW;
        n = (long)un;
        a0 = (int)(a * (unsigned)patch);
        b0 = (int)((rem - a * (unsigned)PW) * (unsigned)patch);
    }
    // index, among all tokens of the tensor, of grid token (a0, b0) of image n
    __device__ __forceinline__ size_t token(long n, int a0, int b0) const
    {
        return (size_t)n * img + tok0 + (size_t)a0 * Wt + b0;
    }
};

inline GridGeom make_geom(int H, int W, int patch, int extra = 0)
{
    GridGeom g;
    g.Wt = W;
    g.Ht = H;
    g.HWt = H * W;
    g.PW = (W + patch - 1) / patch;
    g.PHW = ((H + patch - 1) / patch) * g.PW;
    g.patch = patch;
    g.img = extra + H * W;
    g.tok0 = extra;
    return g;
}

// Tokens outside the grid (a class token in front of the patch tokens) belong to no patch: their
// rows are copied, scaled, behind the projected rows of their tensor.  Up to two tensors; in a
// projection launch the copies are done by workgroups appended to the grid (256 threads each,
// one thread per 16 bytes), so that they cost no launch of their own.
struct ExtraRows {
    const uint4 *in[2];     // the token tensors
    uint4 *out[2];          // first appended row of each projected tensor
    long items[2];          // 16-byte pieces to copy: N * extra * Cv
    long img_vecs[2];       // 16-byte pieces of one image: tokens per image * Cv
    int Cv[2];              // 16-byte pieces of one token
    float scale[2];
    unsigned blocks[2];     // workgroups per tensor
    int extra;              // tokens per image in front of the grid
};

template <bool BF16>
__device__ __forceinline__ void copy_extra_rows(const ExtraRows &x, unsigned block, int tid)
{
    const int i = block >= x.blocks[0] ? 1 : 0;
    const long item = (long)(block - (i ? x.blocks[0] : 0u)) * 256 + tid;
    if (item >= x.items[i]) return;
    const int Cv = x.Cv[i];
    const long row = item / Cv;
    const int cv = (int)(item - row * Cv);
    const long n = row / x.extra;
    const int e = (int)(row - n * x.extra);
    const float scale = x.scale[i];
    uint4 v = x.in[i][(size_t)n * x.img_vecs[i] + (size_t)e * Cv + cv];
    if (BF16) {
        v.x = pack_bf16x2(bf16_lo_to_f32(v.x) * scale, bf16_hi_to_f32(v.x) * scale);
        v.y = pack_bf16x2(bf16_lo_to_f32(v.y) * scale, bf16_hi_to_f32(v.y) * scale);
        v.z = pack_bf16x2(bf16_lo_to_f32(v.z) * scale, bf16_hi_to_f32(v.z) * scale);
        v.w = pack_bf16x2(bf16_lo_to_f32(v.w) * scale, bf16_hi_to_f32(v.w) * scale);
    } else {
        v.x = __float_as_uint(__uint_as_float(v.x) * scale);
        v.y = __float_as_uint(__uint_as_float(v.y) * scale);
        v.z = __float_as_uint(__uint_as_float(v.z) * scale);
        v.w = __float_as_uint(__uint_as_float(v.w) * scale);
    }
    x.out[i][item] = v;
}

// Fills one slot of an ExtraRows: tensor `in` [N][img_tokens][C] of `dtype`, rows appended at `out_rows`.
inline void set_extra_rows(ExtraRows &x, int slot, const void *in, void *out_rows, int N, int extra, long img_tokens,
                           int C, int dtype, float scale)
{
    const int Cv = dtype == LBP_BF16 ? C / 8 : C / 4;
    x.in[slot] = (const uint4 *)in;
    x.out[slot] = (uint4 *)out_rows;
    x.items[slot] = (in && scale != 0.0f) ? (long)N * extra * Cv : 0;      // scale 0: nothing is appended
    x.img_vecs[slot] = img_tokens * Cv;
    x.Cv[slot] = Cv > 0 ? Cv : 1;
    x.scale[slot] = scale;
    x.blocks[slot] = (unsigned)((x.items[slot] + 255) / 256);
    x.extra = extra > 0 ? extra : 1;
}

// Sum-pool a P x P patch over 2^MH x 2^MW token groups, then transform the pooled patch.
template <int P, int MH, int MW>
__device__ __forceinline__ void pooled_transform(const float (&v)[P * P],
                                                 float (&c)[(P >> MH) * (P >> MW)])
{
    constexpr int PH = P >> MH, PWd = P >> MW;
#pragma unroll
    for (int hh = 0; hh < PH; ++hh) {
#pragma unroll
        for (int ww = 0; ww < PWd; ++ww) {
            float s = 0.f;
#pragma unroll
            for (int dh = 0; dh < (1 << MH); ++dh) {
#pragma unroll
                for (int dw = 0; dw < (1 << MW); ++dw)
                    s += v[((hh << MH) + dh) * P + (ww << MW) + dw];
            }
            c[hh * PWd + ww] = s;
        }
    }
    fwht_inplace<PH * PWd>(c);
}

// The same from raw 32-bit words, converting on the fly: HALF 0 = low bf16 of each word, 1 = high
// bf16, 2 = the word is an fp32 value.  No array of converted tokens is kept.
template <int P, int MH, int MW, int HALF>
__device__ __forceinline__ void pooled_transform_raw(const uint32_t (&raw)[P * P],
                                                     float (&c)[(P >> MH) * (P >> MW)])
{
    constexpr int PH = P >> MH, PWd = P >> MW;
#pragma unroll
    for (int hh = 0; hh < PH; ++hh) {
#pragma unroll
        for (int ww = 0; ww < PWd; ++ww) {
            float s = 0.f;
#pragma unroll
            for (int dh = 0; dh < (1 << MH); ++dh) {
#pragma unroll
                for (int dw = 0; dw < (1 << MW); ++dw) {
                    uint32_t u = raw[((hh << MH) + dh) * P + (ww << MW) + dw];
                    float f = HALF == 0 ? bf16_lo_to_f32(u) : HALF == 1 ? bf16_hi_to_f32(u) : __uint_as_float(u);
                    s = (dh == 0 && dw == 0) ? f : s + f;
                }
            }
            c[hh * PWd + ww] = s;
        }
    }
    fwht_inplace<PH * PWd>(c);
}

}  // namespace lbp
