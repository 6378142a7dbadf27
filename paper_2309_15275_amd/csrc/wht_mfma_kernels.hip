// Projection (Eq. 6) and reverse projection (Eq. 7) in their matrix form on the matrix cores, for
// bf16 tensors and ANY selection of bases (any r, any patch up to 16).
//
// The register kernels of wht_kernels.hip prune the butterfly by sum-pooling, which needs all
// selected bases to have even natural indices; selections without that structure (LP_L1 with
// r >= 15, all bases, profiled selections) would run a full 64-point butterfly per lane and are
// register bound.  Here the p^2 x r matrix of +1/-1 (exact in bf16) is the A operand of
// v_mfma_f32_32x32x16_bf16, generated in registers from the natural indices of the bases (the sign
// of basis j at token t is the parity of popcount(j & t)); the patch is staged [token][channel] in
// LDS with 16-byte copies and reaches the matrix cores through the transposing LDS read
// (ds_read_b64_tr_b16), exactly like a reduction-slow GEMM operand.  Products of +-1 with bf16
// values are exact and accumulate in fp32, so the result equals the butterfly's up to summation
// order.  The matrix-core work is a few percent of the time; the kernels are memory bound.
//
// One workgroup (4 wavefronts) handles items of (patch, 128-channel chunk); each wavefront owns 32
// channels.  Results go back through LDS so that global stores are 16 bytes per lane, 256
// contiguous bytes per row.
#include "device_utils.h"
#include "kernels.h"
#include "wht_device.h"

namespace lbp {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short i16x4_t __attribute__((ext_vector_type(4)));
typedef unsigned short u16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));   // 16 bytes, usable with the non-temporal builtins

#define LBP_LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int CB = 128;                 // channels per workgroup item
constexpr int S_IN = CB * 2 + 64;       // LDS row pitch of a [k][channel] bf16 tile read with tr16_b64
constexpr int S_OUT = CB * 2 + 16;      // LDS row pitch of the staged result rows
constexpr unsigned short kPlusOne = 0x3F80, kMinusOne = 0xBF80;

struct MfmaTensor {
    const unsigned short *in;   // forward: tokens (bf16)
    unsigned short *out;        // forward: coefficients (bf16)
    int C;
    int chunks;                 // ceil(C / CB)
    long items;                 // patches * chunks
    unsigned blocks;            // workgroups of this tensor
};

// 8 consecutive reduction entries of one row of the sign matrix, as a matrix-core operand.
// forward:  row = basis (natural index `fixed`), entries = tokens t0..t0+7
// reverse:  row = token `fixed`, entries = bases k0..k0+7 (natural indices from the LDS table)
__device__ __forceinline__ bf16x8_t signs_over_tokens(unsigned nat, int t0, int p2, bool row_ok)
{
    u16x8_t v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        int t = t0 + e;
        unsigned short s = (__popc(nat & (unsigned)t) & 1) ? kMinusOne : kPlusOne;
        v[e] = (row_ok && t < p2) ? s : (unsigned short)0;
    }
    return __builtin_bit_cast(bf16x8_t, v);
}

__device__ __forceinline__ bf16x8_t signs_over_bases(const unsigned char *lds_nat, int k0, int r, unsigned t,
                                                     bool row_ok)
{
    u16x8_t v;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        int k = k0 + e;
        unsigned nat = lds_nat[k < r ? k : 0];
        unsigned short s = (__popc(nat & t) & 1) ? kMinusOne : kPlusOne;
        v[e] = (row_ok && k < r) ? s : (unsigned short)0;
    }
    return __builtin_bit_cast(bf16x8_t, v);
}

// B operand (reduction index slow in LDS): 8 k-values of one column through two transposing reads.
__device__ __forceinline__ bf16x8_t read_b_frag(const unsigned char *tile, int ks, int wave, int lane)
{
    const int grp = lane >> 4, i16 = lane & 15;
    const unsigned char *q = tile + (ks * 16 + 8 * (grp >> 1) + (i16 >> 2)) * S_IN +
                             (wave * 32 + 16 * (grp & 1) + 4 * (i16 & 3)) * 2;
    i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, q));
    i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, q + 4 * S_IN));
    return __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// ---------------------------------------------------------------------------------------------
// forward: coefficients[k][c] = sum_t sign(nat_k, t) * tokens[t][c]
// KSTEPS = padded tokens per patch / 16; MTILES = ceil(r / 32) upper bound for cached operands
// ---------------------------------------------------------------------------------------------
// A_LDS: the cached sign operands live in LDS instead of registers (more than 32 bases: two
// accumulator tiles per wavefront leave no room for them beside the prefetched item).
// Occupancy is asked for explicitly: a workgroup has one 16 KB item in flight, so bandwidth follows
// the number of resident workgroups.  Left alone the compiler takes 134 registers for the A_LDS
// form (3 wavefronts per SIMD) and 98 for the patch-8 form with up to 32 bases (4); held to 4 and
// 5 they fit in 100 and 84 without spilling: 3.9 -> 5.0 TB/s at 36 bases, +2-3 % at 15 and 21.
template <int KSTEPS, int MTILES, bool CACHE_A, bool A_LDS = false>
__global__ __launch_bounds__(256, (A_LDS ? 4 : (KSTEPS == 4 && MTILES == 1 ? 5 : 1))) void wht_project_mfma_kernel(MfmaTensor t0, MfmaTensor t1, GridGeom g,
                                                               NatTable nat, int r, int items_per_wg, ExtraRows xr)
{
    constexpr int P2PAD = KSTEPS * 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    if (blockIdx.x >= t0.blocks + t1.blocks) {      // appended workgroups: tokens outside the grid
        copy_extra_rows<true>(xr, blockIdx.x - (t0.blocks + t1.blocks), threadIdx.x);
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int p = g.patch, p2 = p * p;
    const int li = lane & 31, kg = lane >> 5;
    const int mtiles = (r + 31) >> 5;

    const bool second = blockIdx.x >= t0.blocks;
    const MfmaTensor &t = second ? t1 : t0;
    const long wg = blockIdx.x - (second ? t0.blocks : 0u);

    static_assert(!A_LDS || CACHE_A, "sign operands in LDS are cached operands");
    bf16x8_t afrag[CACHE_A && !A_LDS ? MTILES : 1][CACHE_A && !A_LDS ? KSTEPS : 1];
    // sign operands in LDS: behind the token / result rows, [m-tile][k-step][lane] 16 bytes each
    unsigned char *const sgn = smem + (P2PAD > r ? P2PAD : r) * S_IN;
    if (CACHE_A) {
#pragma unroll
        for (int mt = 0; mt < MTILES; ++mt) {
            int k = mt * 32 + li;
            unsigned nk = nat.v[k < r ? k : 0];
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks) {
                if (A_LDS) {
                    if (((mt * KSTEPS + ks) & 3) == wave)      // the four wavefronts share the work; first barrier of the loop below
                        *reinterpret_cast<bf16x8_t *>(sgn + ((mt * KSTEPS + ks) * 64 + lane) * 16) =
                            signs_over_tokens(nk, ks * 16 + kg * 8, p2, k < r);
                } else {
                    afrag[mt][ks] = signs_over_tokens(nk, ks * 16 + kg * 8, p2, k < r);
                }
            }
        }
    }

    // The loads of the next item are issued before the current one is multiplied, so that a
    // workgroup always has one item (16 KB) on its way from HBM (not for patch 16: no registers left).
    constexpr bool PREFETCH = KSTEPS <= 4 && (MTILES == 1 || A_LDS);
    constexpr int LOADS = P2PAD * (CB / 8) / 256 > 0 ? P2PAD * (CB / 8) / 256 : 1;      // 16-byte loads per lane per item
    static_assert(P2PAD * (CB / 8) % 256 == 0 || P2PAD * (CB / 8) < 256, "loads must divide over the lanes");
    const long item_end = min(t.items, (wg + 1) * (long)items_per_wg);
    u32x4_t stage_regs[PREFETCH ? LOADS : 1];
    const int lp = 31 - __clz(p);             // patch is a power of two
    // per-lane constants of the staging loads: element offset inside a patch, token row/column
    size_t ld_off[PREFETCH ? LOADS : 1];
    int ld_h[PREFETCH ? LOADS : 1], ld_w[PREFETCH ? LOADS : 1];
    const int cc8 = (tid & 15) * 8;
#pragma unroll
    for (int j = 0; j < (PREFETCH ? LOADS : 1); ++j) {
        const int tk = (tid + j * 256) >> 4;
        ld_h[j] = tk < p2 ? tk >> lp : 0x7fffffff;        // rows past the patch never pass the edge test
        ld_w[j] = tk & (p - 1);
        ld_off[j] = ((size_t)(tk >> lp) * g.Wt + (tk & (p - 1))) * t.C + cc8;
    }
    auto fetch = [&](unsigned q, int chunk) {
        const int c0 = chunk * CB;
        long n;
        int a0, b0;
        g.origin(q, n, a0, b0);
        const unsigned short *base = t.in + g.token(n, a0, b0) * t.C + c0;
        const int hv = g.Ht - a0, wv = g.Wt - b0;         // tokens of the patch inside the grid
        const bool chan_ok = c0 + cc8 < t.C;
        if (hv >= p && wv >= p && P2PAD == p2) {
#pragma unroll
            for (int j = 0; j < (PREFETCH ? LOADS : 1); ++j) {
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (chan_ok) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(base + ld_off[j]));
                stage_regs[j] = v;
            }
        } else {
#pragma unroll
            for (int j = 0; j < (PREFETCH ? LOADS : 1); ++j) {
                u32x4_t v = {0u, 0u, 0u, 0u};           // zero padding past the patch, the grid or the channels
                if (chan_ok && ld_h[j] < hv && ld_w[j] < wv && tid + j * 256 < P2PAD * (CB / 8))
                    v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(base + ld_off[j]));
                stage_regs[j] = v;
            }
        }
    };
    // (patch, chunk) of the items of this workgroup: one division, then counting
    long item = wg * items_per_wg;
    unsigned q = (unsigned)(item / t.chunks);
    int chunk = (int)(item - (long)q * t.chunks);
    if (PREFETCH && item < item_end) fetch(q, chunk);
    for (; item < item_end; ++item) {
        const int c0 = chunk * CB;
        unsigned q_next = q;
        int chunk_next = chunk + 1;
        if (chunk_next == t.chunks) {
            chunk_next = 0;
            ++q_next;
        }
        __syncthreads();                      // the previous item's stores have left LDS
        // ---- tokens -> LDS [token][channel]
        if constexpr (PREFETCH) {
#pragma unroll
            for (int j = 0; j < LOADS; ++j) {
                const int c = tid + j * 256;
                if (c < P2PAD * (CB / 8)) *reinterpret_cast<u32x4_t *>(smem + (c >> 4) * S_IN + (c & 15) * 16) = stage_regs[j];
            }
            if (item + 1 < item_end) fetch(q_next, chunk_next);
        } else {
            long n;
            int a0, b0;
            g.origin(q, n, a0, b0);
            const size_t tok0 = g.token(n, a0, b0);
            for (int c = tid; c < P2PAD * (CB / 8); c += 256) {
                int tk = c >> 4, cc = c & 15;
                u32x4_t v = {0u, 0u, 0u, 0u};
                int h = tk >> lp, w = tk & (p - 1);
                if (tk < p2 && c0 + cc * 8 < t.C && a0 + h < g.Ht && b0 + w < g.Wt) {   // else zero padding
                    v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(
                        t.in + (tok0 + (size_t)h * g.Wt + w) * t.C + c0 + cc * 8));
                }
                *reinterpret_cast<u32x4_t *>(smem + tk * S_IN + cc * 16) = v;
            }
        }
        __syncthreads();
        // ---- matrix cores: each wavefront 32 channels, all bases
        f32x16_t acc[MTILES];
#pragma unroll
        for (int mt = 0; mt < MTILES; ++mt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mt][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            bf16x8_t b = read_b_frag(smem, ks, wave, lane);
#pragma unroll
            for (int mt = 0; mt < MTILES; ++mt) {
                if (mt < mtiles) {
                    bf16x8_t a;
                    if (A_LDS) {
                        a = *reinterpret_cast<const bf16x8_t *>(sgn + ((mt * KSTEPS + ks) * 64 + lane) * 16);
                    } else if (CACHE_A) {
                        a = afrag[mt][ks];
                    } else {
                        int k = mt * 32 + li;
                        a = signs_over_tokens(nat.v[k < r ? k : 0], ks * 16 + kg * 8, p2, k < r);
                    }
                    // operands swapped: rows of the product are channels, columns are bases, so
                    // that a lane ends up with 4 consecutive channels of one basis
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[mt], 0, 0, 0);
                }
            }
        }
        __syncthreads();                      // everyone is done reading the tokens
        // ---- coefficients -> LDS [basis][channel] as bf16; accumulator element 4*g4+e is
        //      channel 8*g4+4*kg+e (row) of basis li (column): 4 channels = one 8-byte write
#pragma unroll
        for (int mt = 0; mt < MTILES; ++mt) {
            const int k = mt * 32 + li;
            if (mt < mtiles && k < r) {
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
                    *reinterpret_cast<uint2 *>(smem + k * S_OUT + (wave * 32 + g4 * 8 + kg * 4) * 2) =
                        make_uint2(pack_bf16x2(acc[mt][g4 * 4], acc[mt][g4 * 4 + 1]),
                                   pack_bf16x2(acc[mt][g4 * 4 + 2], acc[mt][g4 * 4 + 3]));
            }
        }
        __syncthreads();
        // ---- 16-byte stores, a basis row of 128 channels is 256 contiguous bytes
        for (int c = tid; c < r * (CB / 8); c += 256) {
            int k = c >> 4, cc = c & 15;
            if (c0 + cc * 8 < t.C)
                *reinterpret_cast<uint4 *>(t.out + ((size_t)q * r + k) * t.C + c0 + cc * 8) =
                    *reinterpret_cast<const uint4 *>(smem + k * S_OUT + cc * 16);
        }
        q = q_next;
        chunk = chunk_next;
    }
}

// ---------------------------------------------------------------------------------------------
// reverse: tokens[t][c] = (1/p^2) * sum_k sign(nat_k, t) * coefficients[k][c]
// MTILES = padded tokens per patch / 32; KSTEPS = ceil(r / 16) upper bound
// ---------------------------------------------------------------------------------------------
// IN_BF16: the coefficients arrive as one bf16 tensor [P*r][C] (a product that stored them itself,
// rounded once from its fp32 accumulators: what this kernel does to fp32 input anyway) instead of
// fp32 split-K slices; `in` is then read as bf16, 16 bytes a lane, and `slices` is ignored.  That form
// has few, short items (one patch x 128 channels per workgroup, 1536 of them at ViT-B fc1), so it is
// bound by the length of one item's load -> LDS -> matrix core -> LDS -> store chain and gains from
// residency: held to 5 wavefronts per SIMD (94 registers, no spills; 3 when left alone, because
// the accumulators then go to AGPRs) it takes 14 instead of 17 us at 36 bases.
template <int MTILES, int KSTEPS, bool CACHE_A, bool IN_BF16 = false>
__global__ __launch_bounds__(256, (IN_BF16 && MTILES == 2 ? 5 : 1)) void wht_unproject_mfma_kernel(const float *__restrict__ in, int slices,
                                                                 size_t slice_stride, unsigned short *out,
                                                                 int C, int chunks, long items, GridGeom g,
                                                                 NatTable nat, int r, int items_per_wg)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    __shared__ unsigned char lds_nat[kMaxBases];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int p = g.patch, p2 = p * p;
    const int li = lane & 31, kg = lane >> 5;
    const int ksteps = (r + 15) >> 4;
    const float scale = 1.0f / (float)p2;
    lds_nat[tid] = nat.v[tid];
    __syncthreads();

    bf16x8_t afrag[CACHE_A ? MTILES : 1][CACHE_A ? KSTEPS : 1];
    if (CACHE_A) {
#pragma unroll
        for (int mt = 0; mt < MTILES; ++mt) {
            int tk = mt * 32 + li;
#pragma unroll
            for (int ks = 0; ks < KSTEPS; ++ks)
                afrag[mt][ks] = signs_over_bases(lds_nat, ks * 16 + kg * 8, r, (unsigned)tk, tk < p2);
        }
    }

    const long wg = blockIdx.x;
    const int lp = 31 - __clz(p);             // patch is a power of two
    // per-lane constants of the token stores (16 bytes each): element offset inside a patch, row, column
    // (only where registers allow: up to 32 bases of an 8 x 8 patch)
    constexpr bool HOIST = MTILES <= 2 && KSTEPS <= 2;
    constexpr int STORES = HOIST ? MTILES * 32 * (CB / 8) / 256 : 1;
    size_t st_off[STORES];
    int st_h[STORES], st_w[STORES];
    const int cc8 = (tid & 15) * 8;
#pragma unroll
    for (int j = 0; j < STORES; ++j) {
        const int tk = (tid + j * 256) >> 4;
        st_h[j] = tk < p2 ? tk >> lp : 0x7fffffff;        // rows past the patch never pass the edge test
        st_w[j] = tk & (p - 1);
        st_off[j] = ((size_t)(tk >> lp) * g.Wt + (tk & (p - 1))) * C + cc8;
    }
    // (patch, chunk) of the items of this workgroup: one division, then counting
    long item = wg * items_per_wg;
    const long item_end = min(items, (wg + 1) * (long)items_per_wg);
    unsigned q = (unsigned)(item / chunks);
    int chunk = (int)(item - (long)q * chunks);
    for (; item < item_end; ++item) {
        const int c0 = chunk * CB;
        long n;
        int a0, b0;
        g.origin(q, n, a0, b0);
        const size_t tok0 = g.token(n, a0, b0);
        __syncthreads();
        // ---- coefficients (fp32, split-K slices summed in fixed order) -> bf16 -> LDS [basis][channel]
        // lane: 4 channels (cc4) of basis rows tid/32, tid/32 + 8, ...: all loads of a slice are issued
        // before any is used (patch 16 has no registers for that and keeps the plain loop)
        if constexpr (IN_BF16) {
            const unsigned short *inb = reinterpret_cast<const unsigned short *>(in);
            for (int c = tid; c < ksteps * 16 * (CB / 8); c += 256) {
                const int k = c >> 4, cc = c & 15;
                u32x4_t v = {0u, 0u, 0u, 0u};
                if (k < r && c0 + cc * 8 < C)
                    v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(inb + ((size_t)q * r + k) * C + c0 + cc * 8));
                *reinterpret_cast<u32x4_t *>(smem + k * S_IN + cc * 16) = v;
            }
        } else if constexpr (KSTEPS > 4) {
            for (int c = tid; c < ksteps * 16 * (CB / 4); c += 256) {
                int k = c >> 5, cc = c & 31;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < r && c0 + cc * 4 < C) {
                    const float *src = in + ((size_t)q * r + k) * C + c0 + cc * 4;
                    v = *reinterpret_cast<const float4 *>(src);
                    for (int z = 1; z < slices; ++z) {
                        float4 u = *reinterpret_cast<const float4 *>(src + z * slice_stride);
                        v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
                    }
                }
                *reinterpret_cast<uint2 *>(smem + k * S_IN + cc * 8) = make_uint2(pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w));
            }
        } else {
            const int cc4 = (tid & 31) * 4, k0 = tid >> 5;
            const bool chan_ok = c0 + cc4 < C;
            const float *src = in + ((size_t)q * r + k0) * C + c0 + cc4;
            float4 v[2 * KSTEPS];
#pragma unroll
            for (int j = 0; j < 2 * KSTEPS; ++j) {
                v[j] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (j * 8 < ksteps * 16 && chan_ok && k0 + j * 8 < r) v[j] = *reinterpret_cast<const float4 *>(src + (size_t)j * 8 * C);
            }
            for (int z = 1; z < slices; ++z) {
                const float *sz = src + z * slice_stride;
#pragma unroll
                for (int j = 0; j < 2 * KSTEPS; ++j) {
                    if (j * 8 < ksteps * 16 && chan_ok && k0 + j * 8 < r) {
                        float4 u = *reinterpret_cast<const float4 *>(sz + (size_t)j * 8 * C);
                        v[j].x += u.x; v[j].y += u.y; v[j].z += u.z; v[j].w += u.w;
                    }
                }
            }
#pragma unroll
            for (int j = 0; j < 2 * KSTEPS; ++j)
                if (j * 8 < ksteps * 16)
                    *reinterpret_cast<uint2 *>(smem + (k0 + j * 8) * S_IN + cc4 * 2) =
                        make_uint2(pack_bf16x2(v[j].x, v[j].y), pack_bf16x2(v[j].z, v[j].w));
        }
        __syncthreads();
        f32x16_t acc[MTILES];
#pragma unroll
        for (int mt = 0; mt < MTILES; ++mt)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[mt][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KSTEPS; ++ks) {
            if (ks < ksteps) {
                bf16x8_t b = read_b_frag(smem, ks, wave, lane);
#pragma unroll
                for (int mt = 0; mt < MTILES; ++mt) {
                    bf16x8_t a;
                    if (CACHE_A) {
                        a = afrag[mt][ks];
                    } else {
                        int tk = mt * 32 + li;
                        a = signs_over_bases(lds_nat, ks * 16 + kg * 8, r, (unsigned)tk, tk < p2);
                    }
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[mt], 0, 0, 0);   // rows = channels
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int mt = 0; mt < MTILES; ++mt) {
            const int tk = mt * 32 + li;          // column of the product = token
            if (tk < p2) {
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
                    *reinterpret_cast<uint2 *>(smem + tk * S_OUT + (wave * 32 + g4 * 8 + kg * 4) * 2) =
                        make_uint2(pack_bf16x2(acc[mt][g4 * 4] * scale, acc[mt][g4 * 4 + 1] * scale),
                                   pack_bf16x2(acc[mt][g4 * 4 + 2] * scale, acc[mt][g4 * 4 + 3] * scale));
            }
        }
        __syncthreads();
        if constexpr (!HOIST) {
            for (int c = tid; c < p2 * (CB / 8); c += 256) {
                int tk = c >> 4, cc = c & 15;
                int h = tk >> lp, w = tk & (p - 1);
                if (c0 + cc * 8 < C && a0 + h < g.Ht && b0 + w < g.Wt) {
                    u32x4_t v = *reinterpret_cast<const u32x4_t *>(smem + tk * S_OUT + cc * 16);
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(out + (tok0 + (size_t)h * g.Wt + w) * C + c0 + cc * 8));
                }
            }
        } else if (c0 + cc8 < C) {
            unsigned short *base = out + tok0 * C + c0;
            const int hv = g.Ht - a0, wv = g.Wt - b0;     // tokens of the patch inside the grid
            const unsigned char *row = smem + (tid >> 4) * S_OUT + (tid & 15) * 16;
#pragma unroll
            for (int j = 0; j < STORES; ++j) {
                if (st_h[j] < hv && st_w[j] < wv) {
                    u32x4_t v = *reinterpret_cast<const u32x4_t *>(row + j * 16 * S_OUT);
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(base + st_off[j]));
                }
            }
        }
        if (++chunk == chunks) {
            chunk = 0;
            ++q;
        }
    }
}

NatTable make_nat(const BasisPlan &plan)
{
    NatTable nat;
    for (int k = 0; k < kMaxBases; ++k) nat.v[k] = plan.nat[k];
    return nat;
}

int items_per_wg(long items)
{
    // enough workgroups to fill the chip several times over, few enough that the per-workgroup
    // set-up of the sign operands is amortised
    long wgs_wanted = 256L * 16;
    long ipw = (items + wgs_wanted - 1) / wgs_wanted;
    return (int)(ipw < 1 ? 1 : ipw > 8 ? 8 : ipw);
}

template <typename K>
hipError_t set_lds(K kern, int bytes)
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

}  // namespace

bool wht_mfma_supported(const BasisPlan &plan, int dtype, int C)
{
    return dtype == LBP_BF16 && C % 8 == 0 && plan.patch >= 2 && plan.patch <= 16 && plan.r >= 1;
}

hipError_t launch_project_mfma(const void *in0, void *out0, int C0, const void *in1, void *out1, int C1,
                               int N, int H, int W, const BasisPlan &plan, hipStream_t stream, int extra,
                               float extra_scale0, float extra_scale1)
{
    const long Q = patch_count(N, H, W, plan.patch);
    GridGeom g = make_geom(H, W, plan.patch, extra);
    NatTable nat = make_nat(plan);
    MfmaTensor t[2] = {};
    const void *ins[2] = {in0, in1};
    void *outs[2] = {out0, out1};
    const int Cs[2] = {C0, C1};
    long all_items = 0;
    for (int i = 0; i < 2; ++i) {
        if (!ins[i]) continue;
        t[i].in = (const unsigned short *)ins[i];
        t[i].out = (unsigned short *)outs[i];
        t[i].C = Cs[i];
        t[i].chunks = (Cs[i] + CB - 1) / CB;
        t[i].items = Q * t[i].chunks;
        all_items += t[i].items;
    }
    if (t[1].chunks == 0) t[1].chunks = 1;
    const int ipw = items_per_wg(all_items);
    for (int i = 0; i < 2; ++i) t[i].blocks = (unsigned)((t[i].items + ipw - 1) / ipw);
    ExtraRows xr{};
    if (extra > 0) {
        const size_t rows = (size_t)Q * plan.r;
        const long img_tokens = (long)H * W + extra;
        set_extra_rows(xr, 0, in0, (char *)out0 + rows * C0 * 2, N, extra, img_tokens, C0, LBP_BF16, extra_scale0);
        set_extra_rows(xr, 1, in1, in1 ? (char *)out1 + rows * C1 * 2 : nullptr, N, extra, img_tokens, in1 ? C1 : C0,
                       LBP_BF16, extra_scale1);
    }
    const unsigned blocks = t[0].blocks + t[1].blocks + xr.blocks[0] + xr.blocks[1];
    const int p2 = plan.patch * plan.patch;
    const int p2pad = p2 < 16 ? 16 : p2;
    const int lds = (p2pad > plan.r ? p2pad : plan.r) * S_IN;     // S_IN >= S_OUT: covers both uses
#define LBP_LAUNCH(KS, MT, CACHE, ALDS)                                                             \
    do {                                                                                            \
        auto kern = wht_project_mfma_kernel<KS, MT, CACHE, ALDS>;                                   \
        const int bytes = lds + (ALDS ? MT * KS * 64 * 16 : 0);                                     \
        hipError_t e = set_lds(kern, bytes);                                                        \
        if (e != hipSuccess) return e;                                                              \
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), bytes, stream, t[0], t[1], g, nat, plan.r, ipw, xr); \
    } while (0)
    if (p2pad == 16) LBP_LAUNCH(1, 1, true, false);
    else if (p2pad == 64 && plan.r <= 32) LBP_LAUNCH(4, 1, true, false);
    else if (p2pad == 64) LBP_LAUNCH(4, 2, true, true);
    else LBP_LAUNCH(16, 8, false, false);
#undef LBP_LAUNCH
    return hipGetLastError();
}

hipError_t launch_unproject_mfma(const float *in, int slices, void *out, int N, int H, int W, int C,
                                 const BasisPlan &plan, hipStream_t stream, int extra, long slice_rows, bool in_bf16)
{
    const long Q = patch_count(N, H, W, plan.patch);
    GridGeom g = make_geom(H, W, plan.patch, extra);
    NatTable nat = make_nat(plan);
    const int chunks = (C + CB - 1) / CB;
    const long items = Q * chunks;
    const int ipw = items_per_wg(items);
    const unsigned blocks = (unsigned)((items + ipw - 1) / ipw);
    const size_t slice_stride = (size_t)(slice_rows > 0 ? slice_rows : Q * plan.r) * C;
    const int p2 = plan.patch * plan.patch;
    const int kpad = (plan.r + 15) / 16 * 16;
    const int rows = p2 > kpad ? p2 : kpad;
    const int lds = rows * S_IN;
#define LBP_LAUNCH_T(MT, KS, CACHE, INB)                                                            \
    do {                                                                                            \
        auto kern = wht_unproject_mfma_kernel<MT, KS, CACHE, INB>;                                  \
        hipError_t e = set_lds(kern, lds);                                                          \
        if (e != hipSuccess) return e;                                                              \
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), lds, stream, in, slices, slice_stride,    \
                           (unsigned short *)out, C, chunks, items, g, nat, plan.r, ipw);           \
    } while (0)
#define LBP_LAUNCH(MT, KS, CACHE)                       \
    do {                                                \
        if (in_bf16) LBP_LAUNCH_T(MT, KS, CACHE, true); \
        else LBP_LAUNCH_T(MT, KS, CACHE, false);        \
    } while (0)
    if (p2 <= 32) LBP_LAUNCH(1, 1, true);                       // patch 2 and 4: at most 16 bases
    else if (p2 == 64 && plan.r <= 32) LBP_LAUNCH(2, 2, true);
    else if (p2 == 64) LBP_LAUNCH(2, 4, true);
    else LBP_LAUNCH(8, 16, false);
#undef LBP_LAUNCH
#undef LBP_LAUNCH_T
    return hipGetLastError();
}

}  // namespace lbp
