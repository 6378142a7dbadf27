// bf16 matrix-core GEMM kernel template for gfx950 (fp32 accumulation); instantiated per tile
// shape by the gemm_mfma_*.hip files.
//
// One workgroup owns a BM x BN tile of the output and walks the reduction in steps of BK = 64.
//   * Global -> registers (16-byte loads, issued PF steps ahead) -> LDS (two stages, one barrier
//     per step).  Loads are never predicated in the steady state: rows and columns past the edge
//     of a matrix are clamped to the last valid ones (they only feed outputs that are never
//     stored); only a final partial step of the reduction zero-fills.
//   * Operands whose reduction index is contiguous in memory are stored [row][k] in LDS and read
//     back with 16-byte reads.  Operands whose reduction index is the slow axis (W, and both
//     operands of gW) are stored as they arrive, [k][row], and transposed on the way to the
//     matrix cores with ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the
//     address of 4 consecutive elements of row k = i/4 starting at column 4*(i%4), and lane j
//     receives the 4 k-values of column j.  Two such reads give the 8 consecutive k-values per
//     lane that v_mfma_f32_32x32x16_bf16 takes.  Row pitches are padded so that both access
//     patterns spread over all LDS banks.
//   * Each wavefront owns a (BM/WGM) x (BN/WGN) block of 32x32 accumulator tiles.
//   * Epilogues: scaled fp32 store (per split-K slice), scaled bf16 store, or the reverse
//     projection of Eq. 7 fused in: the tile's rows are (patch, basis) pairs, the accumulators go
//     through LDS, and every lane expands the r coefficients of one (patch, channel pair) into
//     the p x p tokens of that patch with the same pooled butterfly the stand-alone kernel uses.
//   * Workgroups are numbered so that each of the 8 XCDs (private L2 each) works on a contiguous
//     run of tiles that share the same rows of A.
//   * A fused product with few tiles under a long reduction can cut the reduction into slices, one
//     workgroup each, that combine inside the launch (JOIN instantiations): see store_part below.
#pragma once
#include "device_utils.h"
#include "kernels.h"
#include "wht_device.h"

namespace lbp {
namespace mfma {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short i16x4_t __attribute__((ext_vector_type(4)));
typedef short i16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

#define LBP_LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

constexpr int BK = 64;

// EPI_PLAIN: fp32 or bf16 store chosen at run time by Params::store_bf16 (grouped launches)
enum { EPI_F32 = 0, EPI_BF16 = 1, EPI_UNPROJECT = 2, EPI_UNPROJECT_MFMA = 3, EPI_PLAIN = 4 };

struct Params {
    const unsigned short *A;
    const unsigned short *B;
    int M, N, K;
    long lda, ldb;
    int k_per_split;      // multiple of BK
    int bm_step;          // rows of the output one tile advances by (BM, or a multiple of r below BM)
    int tiles_m, tiles_n;
    int xcd_a, xcd_b;     // tiles of one XCD form an xcd_a x xcd_b block of the output (0: plain numbering)
    void *C;
    float scale;
    // fused reverse projection
    GridGeom geom;
    PooledSel sel;
    int r, mh, mw;
    long Q;               // number of patches
    int extra_rows;       // rows of A after the Q*r (patch, basis) rows: tokens outside the grid, extra per image
    int extra;            // such tokens per image; their rows of the product are stored scaled by 1/patch^2
    unsigned char nat[64];   // natural (Sylvester) index of every selected basis (matrix-core epilogue, patch 8)
    int mfma_epilogue;    // 1: the selection cannot be pooled, Eq. 7 runs on the matrix cores in the epilogue
    int store_bf16;       // EPI_PLAIN: 1 stores bf16, 0 stores fp32 (slice by slice)
    // reduction split over `splits` workgroups per tile that combine inside the launch (JOIN kernels only)
    int splits;           // slices per tile
    float *parts;         // [tile][slice][BM * BN] partial accumulators
    unsigned *counters;   // one per tile, zero between launches
};

// Scheduling hint for one sub-step of the main loop: N matrix instructions with R LDS reads spread
// evenly between them (the arguments of the builtin must be constants, hence the recursion).
template <int I, int N, int R>
__device__ __forceinline__ void interleave_mfma_with_lds_reads()
{
    if constexpr (I < N) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);          // one matrix instruction
        constexpr int share = (R * (I + 1)) / N - (R * I) / N;
        if constexpr (share > 0) __builtin_amdgcn_sched_group_barrier(0x100, share, 0);      // its share of the LDS reads
        interleave_mfma_with_lds_reads<I + 1, N, R>();
    }
}

// Reverse projection of one tile held in LDS as fp32 ct[row][cts]; rows are (patch, basis).
template <int LP, int MH, int MW, int BN, int NT>
__device__ __forceinline__ void unproject_tile(const float *ct, int cts, const Params &p, int m0,
                                               int n0, int tid)
{
    constexpr int P = 1 << LP;
    constexpr int PWd = P >> MW;
    constexpr int NC = (P >> MH) * PWd;
    constexpr float scale = 1.0f / (float)(P * P);
    constexpr int HALF = BN / 2;
    const int patches = p.bm_step / p.r;
    const int Cd = p.N >> 1;
    for (int it = tid; it < patches * HALF; it += NT) {
        int pt = it / HALF, cp = it - pt * HALF;
        long q = (long)(m0 / p.r) + pt;
        if (q >= p.Q || n0 + 2 * cp >= p.N) continue;
        const float *src = ct + (size_t)(pt * p.r) * cts + 2 * cp;
        float c0[NC], c1[NC];
#pragma unroll
        for (int j = 0; j < NC; ++j) {
            float2 t = make_float2(0.f, 0.f);
            if ((p.sel.mask >> j) & 1ull) t = *reinterpret_cast<const float2 *>(src + (size_t)p.sel.pos[j] * cts);
            c0[j] = t.x;
            c1[j] = t.y;
        }
        fwht_inplace<NC>(c0);
        fwht_inplace<NC>(c1);
        long img;
        int a0, b0;
        p.geom.origin(q, img, a0, b0);
        uint32_t *dst = reinterpret_cast<uint32_t *>(p.C) + p.geom.token(img, a0, b0) * Cd + (n0 >> 1) + cp;
        const int hv = p.geom.Ht - a0, wv = p.geom.Wt - b0;     // tokens of the patch inside the grid (>= P: all)
        if (hv >= P && wv >= P) {                 // the whole patch is inside the grid
#pragma unroll
            for (int h = 0; h < P; ++h) {
#pragma unroll
                for (int w = 0; w < P; ++w) {
                    int j = (h >> MH) * PWd + (w >> MW);
                    __builtin_nontemporal_store(pack_bf16x2(c0[j] * scale, c1[j] * scale), dst + ((size_t)h * p.geom.Wt + w) * Cd);
                }
            }
        } else {
#pragma unroll
            for (int h = 0; h < P; ++h) {
#pragma unroll
                for (int w = 0; w < P; ++w) {
                    int j = (h >> MH) * PWd + (w >> MW);
                    if (h < hv && w < wv)
                        __builtin_nontemporal_store(pack_bf16x2(c0[j] * scale, c1[j] * scale), dst + ((size_t)h * p.geom.Wt + w) * Cd);
                }
            }
        }
    }
}

// Rows [lo, hi) of the tile that belong to tokens outside the grid (global row >= Q*r): empty
// for all but the last tiles.
__device__ __forceinline__ void extra_row_range(const Params &p, int m0, int &lo, int &hi)
{
    const long first = p.Q * p.r;
    const long l = first - m0, h = (long)p.M - m0;
    lo = l < 0 ? 0 : (int)(l < p.bm_step ? l : p.bm_step);
    hi = (int)(h < p.bm_step ? h : p.bm_step);
}

// LDS layout of one stage.  A reduction-slow operand keeps its rows [k][row]; the transposing reads
// of one instruction touch 64 consecutive bytes of four consecutive k-rows, which must fall into
// different banks: rows of 128 bytes are padded to a pitch of 192, rows of 256 bytes or more are
// not padded but have their 64-byte pieces permuted per row (piece index xor k % 4), which keeps
// two workgroups of the 128-wide tiles inside one compute unit's LDS.
template <int BM, int BN, bool A_KFAST>
struct Smem {
    static constexpr bool A_SWZ = !A_KFAST && BM >= 128;
    static constexpr bool B_SWZ = BN % 128 == 0;      // the permutation works on rows of whole 256-byte groups
    static constexpr int SA = A_KFAST ? (BK + 8) * 2 : (A_SWZ ? BM * 2 : BM * 2 + 64);   // row pitch of A in bytes
    static constexpr int SB = B_SWZ ? BN * 2 : BN * 2 + 64;
    static constexpr int A_BYTES = (A_KFAST ? BM : BK) * SA;
    static constexpr int B_BYTES = BK * SB;
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int TOTAL = 2 * STAGE;
};

// Split reductions that are combined inside the launch.  Every workgroup of a tile stores its partial
// accumulators, then counts itself in on the tile's counter; whichever comes last adds all the parts
// in slice order (so the sum does not depend on who came last) and goes on to the epilogue.  Nobody
// waits.  Parts travel from one XCD's L2 to another's: they are written and read with device-scope
// accesses (8 bytes per lane), which go to the point where the XCDs are coherent, so that no cache has
// to be written back or invalidated as a whole, which is what a device-scope fence would cost
// (measured: tens of microseconds per launch).  The last workgroup leaves the counter at zero.
template <int TM, int TN>
__device__ __forceinline__ void store_part(float *slot, const f32x16_t (&acc)[TM][TN])
{
    unsigned long long *dst = reinterpret_cast<unsigned long long *>(slot) + threadIdx.x;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                const unsigned long long v = (unsigned long long)__float_as_uint(acc[i][j][2 * g]) |
                                             ((unsigned long long)__float_as_uint(acc[i][j][2 * g + 1]) << 32);
                __hip_atomic_store(dst + (size_t)((i * TN + j) * 8 + g) * blockDim.x, v, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            }
}

template <int TM, int TN>
__device__ __forceinline__ void add_part(float *slot, f32x16_t (&sum)[TM][TN])
{
    unsigned long long *src = reinterpret_cast<unsigned long long *>(slot) + threadIdx.x;
    unsigned long long v[TM * TN * 8];            // all loads of the part in flight together
#pragma unroll
    for (int q = 0; q < TM * TN * 8; ++q)
        v[q] = __hip_atomic_load(src + (size_t)q * blockDim.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                sum[i][j][2 * g] += __uint_as_float((unsigned)v[(i * TN + j) * 8 + g]);
                sum[i][j][2 * g + 1] += __uint_as_float((unsigned)(v[(i * TN + j) * 8 + g] >> 32));
            }
}

// One workgroup's share of a product: output tile `tile_id` (before the XCD renumbering), split-K
// slice `slice`; `smem` is the workgroup's dynamic LDS (at least Smem<BM, BN, A_KFAST>::TOTAL bytes).
template <int BM, int BN, int WGM, int WGN, int PF, bool A_KFAST, int EPI, int LP, bool JOIN = false>
__device__ __forceinline__ void gemm_body(const Params &p, const int tile_id, const int slice, unsigned char *smem)
{
    static_assert(PF == 2 || PF == 4, "prefetch depth must be even");
    using S = Smem<BM, BN, A_KFAST>;
    constexpr int NT = 64 * WGM * WGN;
    constexpr int WM = BM / WGM, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int SA = S::SA, SB = S::SB, A_BYTES = S::A_BYTES, STAGE = S::STAGE;
    constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;       // 16-byte chunks per thread per step
    static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile does not divide over the threads");
    static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be made of 32x32 tiles");
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave - wm * WGN;

    // XCD-aware tile numbering: workgroup ids go round-robin over the 8 XCDs, each of which has an
    // L2 of its own; the tiles of one XCD form an xcd_a x xcd_b block of the output, so that they
    // share xcd_a strips of A and xcd_b strips of B (chosen on the host to make that sum smallest)
    int tm, tn;
    if (p.xcd_a > 0) {
        const int x = tile_id & 7, i = tile_id >> 3;
        const int bn = p.tiles_n / p.xcd_b;           // blocks along n
        const int xm = x / bn, xn = x - xm * bn;
        const int im = i / p.xcd_b, in = i - im * p.xcd_b;
        tm = xm * p.xcd_a + im;
        tn = xn * p.xcd_b + in;
    } else {
        const int T = p.tiles_m * p.tiles_n;          // no such block: a contiguous run of tiles per XCD
        int t = tile_id;
        if ((T & 7) == 0) t = (t & 7) * (T >> 3) + (t >> 3);
        tm = t / p.tiles_n;
        tn = t - tm * p.tiles_n;
    }
    const int m0 = tm * p.bm_step, n0 = tn * BN;
    const int kbeg = slice * p.k_per_split;
    const int kend = min(p.K, kbeg + p.k_per_split);

    // ---- per-thread load descriptors (rows / columns clamped into the matrix)
    const unsigned short *ga[A_CH];
    const unsigned short *gb[B_CH];
    int sa_off[A_CH], sb_off[B_CH];     // LDS byte offsets inside a stage
    int ka[A_CH], kb[B_CH];             // k offset of the chunk inside a step
#pragma unroll
    for (int i = 0; i < A_CH; ++i) {
        int c = tid + i * NT;
        if (A_KFAST) {
            int row = c >> 3, kc = c & 7;
            sa_off[i] = row * SA + kc * 16;
            ka[i] = kc * 8;
            ga[i] = p.A + (size_t)min(m0 + row, p.M - 1) * p.lda + kc * 8;
        } else {
            int krow = c / (BM / 8), cc = c - krow * (BM / 8);
            sa_off[i] = krow * SA + ((cc * 16) ^ (S::A_SWZ ? (krow & 3) << 6 : 0));
            ka[i] = krow;
            ga[i] = p.A + (size_t)krow * p.lda + min(m0 + cc * 8, p.M - 8);
        }
    }
#pragma unroll
    for (int i = 0; i < B_CH; ++i) {
        int c = tid + i * NT;
        int krow = c / (BN / 8), cc = c - krow * (BN / 8);
        sb_off[i] = A_BYTES + krow * SB + ((cc * 16) ^ (S::B_SWZ ? (krow & 3) << 6 : 0));
        kb[i] = krow;
        gb[i] = p.B + (size_t)krow * p.ldb + min(n0 + cc * 8, p.N - 8);
    }

    // PF register sets: while step s is multiplied out of LDS, the loads of steps s+1 .. s+PF are
    // in flight (one step of a tile is far shorter than a trip to L2 or HBM, so a small problem
    // with one workgroup per compute unit needs several steps in flight).  The steady state has no
    // predication and no branches around loads, so the compiler's wait counters only wait for
    // the oldest set.
    uint4 ra[PF][A_CH], rb[PF][B_CH];
    auto fetch_full = [&](int set, int k0) {        // needs k0 + BK <= kend
#pragma unroll
        for (int i = 0; i < A_CH; ++i)
            ra[set][i] = *reinterpret_cast<const uint4 *>(ga[i] + (A_KFAST ? (size_t)k0 : (size_t)k0 * p.lda));
#pragma unroll
        for (int i = 0; i < B_CH; ++i)
            rb[set][i] = *reinterpret_cast<const uint4 *>(gb[i] + (size_t)k0 * p.ldb);
    };
    auto fetch_tail = [&](int set, int k0) {        // a partial step: zero-fill k >= kend
#pragma unroll
        for (int i = 0; i < A_CH; ++i) {
            ra[set][i] = make_uint4(0u, 0u, 0u, 0u);
            if (k0 + ka[i] < kend)
                ra[set][i] = *reinterpret_cast<const uint4 *>(ga[i] + (A_KFAST ? (size_t)k0 : (size_t)k0 * p.lda));
        }
#pragma unroll
        for (int i = 0; i < B_CH; ++i) {
            rb[set][i] = make_uint4(0u, 0u, 0u, 0u);
            if (k0 + kb[i] < kend) rb[set][i] = *reinterpret_cast<const uint4 *>(gb[i] + (size_t)k0 * p.ldb);
        }
    };
    auto stage = [&](int set, unsigned char *s) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *reinterpret_cast<uint4 *>(s + sa_off[i]) = ra[set][i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) *reinterpret_cast<uint4 *>(s + sb_off[i]) = rb[set][i];
    };

    // ---- per-lane fragment offsets inside a stage
    const int li = lane & 31, kg = lane >> 5, grp = lane >> 4, i16 = lane & 15;
    int a_off[TM], b_off[TN];
#pragma unroll
    for (int mi = 0; mi < TM; ++mi) {
        if (A_KFAST)
            a_off[mi] = (wm * WM + mi * 32 + li) * SA + kg * 16;
        else
            a_off[mi] = (8 * (grp >> 1) + (i16 >> 2)) * SA +
                        (((wm * WM + mi * 32 + 16 * (grp & 1) + 4 * (i16 & 3)) * 2) ^ (S::A_SWZ ? (i16 >> 2) << 6 : 0));
    }
    // (every k-row a lane reads is its first one plus a multiple of 4, so its permutation is fixed)
#pragma unroll
    for (int ni = 0; ni < TN; ++ni)
        b_off[ni] = A_BYTES + (8 * (grp >> 1) + (i16 >> 2)) * SB +
                    (((wn * WN + ni * 32 + 16 * (grp & 1) + 4 * (i16 & 3)) * 2) ^ (S::B_SWZ ? (i16 >> 2) << 6 : 0));

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // One 16-deep sub-step of fragments: TM of A and TN of B, 8 reduction values per lane each.
    auto load_frags = [&](const unsigned char *s, int ks, bf16x8_t (&a)[TM], bf16x8_t (&b)[TN]) {
#pragma unroll
        for (int mi = 0; mi < TM; ++mi) {
            if (A_KFAST) {
                a[mi] = *reinterpret_cast<const bf16x8_t *>(s + a_off[mi] + ks * 32);
            } else {
                const unsigned char *q = s + a_off[mi] + ks * 16 * SA;
                i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, q));
                i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, q + 4 * SA));
                a[mi] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            }
        }
#pragma unroll
        for (int ni = 0; ni < TN; ++ni) {
            const unsigned char *q = s + b_off[ni] + ks * 16 * SB;
            i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, q));
            i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, q + 4 * SB));
            b[ni] = __builtin_bit_cast(bf16x8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    };
    // PIPELINED: the fragments of sub-step ks+1 are requested before the matrix instructions of
    // sub-step ks are issued, into a second register set, and the scheduler is told to spread those
    // LDS reads between the matrix instructions, so that a wavefront keeps the matrix cores and the
    // LDS pipe busy at the same time by itself.  That pays where a SIMD holds one wavefront of the
    // workgroup (4-wavefront tiles: +8 % on the 128 x 128 weight-gradient product) and on the 256-row
    // tiles with 64 x 64 wavefront tiles (+2-5 %); with two wavefronts per SIMD and small wavefront
    // tiles the other wavefront already fills the gaps and the second register set only costs
    // (128 x 128 and 64 x 128 with 8 wavefronts: -1 to -6 %), and 256 x 256 has no registers left for it.
    constexpr bool PIPELINED = (WGM * WGN == 4) || (BM == 256 && BN < 256);
    constexpr int DS_READS = TM * (A_KFAST ? 1 : 2) + TN * 2;       // LDS read instructions per sub-step
    constexpr int MFMAS = TM * TN;
    auto multiply = [&](const unsigned char *s) {
        if constexpr (PIPELINED) {
            bf16x8_t a[2][TM], b[2][TN];
            load_frags(s, 0, a[0], b[0]);
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                if (ks + 1 < BK / 16) load_frags(s, ks + 1, a[(ks + 1) & 1], b[(ks + 1) & 1]);
#pragma unroll
                for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                    for (int ni = 0; ni < TN; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][mi], b[ks & 1][ni], acc[mi][ni], 0, 0, 0);
                if (ks + 1 < BK / 16) interleave_mfma_with_lds_reads<0, MFMAS, DS_READS>();
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                bf16x8_t a[TM], b[TN];
                load_frags(s, ks, a, b);
#pragma unroll
                for (int mi = 0; mi < TM; ++mi)
#pragma unroll
                    for (int ni = 0; ni < TN; ++ni)
                        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[ni], acc[mi][ni], 0, 0, 0);
            }
        }
    };

    unsigned char *const bufs[2] = {smem, smem + STAGE};
    const int nfull = (kend - kbeg) / BK;           // whole steps; a partial one may follow
    if (nfull > 0) {
#pragma unroll
        for (int j = 0; j < PF; ++j)
            if (j < nfull) fetch_full(j, kbeg + j * BK);
        stage(0, bufs[0]);
        __syncthreads();
        // invariant at the top of step s (j = s mod PF): LDS stage s&1 holds step s, register
        // sets j+1 .. j+PF-1 are in flight for steps s+1 .. s+PF-1, set j is free
        int s = 0;
        for (; s + 2 * PF - 1 < nfull; s += PF) {
#pragma unroll
            for (int j = 0; j < PF; ++j) {
                fetch_full(j, kbeg + (s + j + PF) * BK);
                multiply(bufs[j & 1]);
                stage((j + 1) % PF, bufs[(j + 1) & 1]);
                __syncthreads();
            }
        }
        const int rem = nfull - s;                  // 1 .. 2*PF-1 steps left
#pragma unroll
        for (int j = 0; j < 2 * PF - 1; ++j) {
            if (j < rem) {
                if (s + j + PF < nfull) fetch_full(j % PF, kbeg + (s + j + PF) * BK);
                multiply(bufs[j & 1]);
                if (j + 1 < rem) stage((j + 1) % PF, bufs[(j + 1) & 1]);
                __syncthreads();
            }
        }
    }
    if (kbeg + nfull * BK < kend) {                 // the partial step, not pipelined
        fetch_tail(0, kbeg + nfull * BK);
        stage(0, bufs[0]);
        __syncthreads();
        multiply(bufs[0]);
        __syncthreads();
    }

    if constexpr (JOIN) {
        if (p.splits > 1) {
            __shared__ unsigned arrived;
            float *const tile_parts = p.parts + (size_t)tile_id * p.splits * (BM * BN);
            store_part<TM, TN>(tile_parts + (size_t)slice * (BM * BN), acc);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_s_waitcnt(0);        // every lane's part has arrived before the workgroup counts itself in
            __syncthreads();
            if (tid == 0)
                arrived = __hip_atomic_fetch_add(p.counters + tile_id, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            if (arrived != (unsigned)(p.splits - 1)) return;      // the same for every lane of the workgroup
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
            for (int z = 0; z < p.splits; ++z) add_part<TM, TN>(tile_parts + (size_t)z * (BM * BN), acc);
            if (tid == 0) __hip_atomic_store(p.counters + tile_id, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // accumulator element 4*g4 + e of a 32x32 tile: row 8*g4 + 4*(lane/32) + e, column lane%32
    if constexpr (EPI == EPI_UNPROJECT_MFMA) {
        // Eq. 7 for selections that cannot be pooled (patch 8): per patch, tokens[64][BN] =
        // (1/64) * S[64][r] * coefficients[r][BN] with S the +-1 matrix, on the matrix cores.
        // The tile's rows (patch, basis) go to LDS as bf16 in the layout of a reduction-slow
        // operand; the sign operand is built in registers from the bases' natural indices;
        // token rows are staged in LDS so that global stores are 16 bytes per lane.
        static_assert(BN == 128 && LP == 3, "matrix-core epilogue: 128 channels per tile, patch 8");
        constexpr int S_CO = BN * 2 + 64;       // pitch of the coefficient rows (transposing LDS reads)
        constexpr int S_TK = BN * 2 + 16;       // pitch of the staged token rows
        constexpr int MTW = NT == 256 ? 2 : 1;  // 32-token tiles per wavefront (4 wavefronts: both; 8: one each)
        static_assert(NT == 256 || NT == 512, "4 or 8 wavefronts");
        static_assert((BM + 16) * S_CO + 64 * S_TK <= S::TOTAL, "epilogue does not fit in LDS");
        __shared__ unsigned char lds_nat[64];
        unsigned char *cot = smem, *stg = smem + (BM + 16) * S_CO;
        if (tid < 64) lds_nat[tid] = p.nat[tid];
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int row = wm * WM + mi * 32 + g4 * 8 + kg * 4 + e;
                        int col = wn * WN + ni * 32 + li;
                        *reinterpret_cast<unsigned short *>(cot + row * S_CO + col * 2) =
                            (unsigned short)f32_to_bf16_bits(acc[mi][ni][g4 * 4 + e]);
                    }
        // the last sub-step of the last patch reads up to 15 rows past the tile: zeros
        for (int c = tid; c < 16 * (S_CO / 16); c += NT)
            *reinterpret_cast<uint4 *>(cot + BM * S_CO + c * 16) = make_uint4(0u, 0u, 0u, 0u);
        __syncthreads();
        const int ch = wave & 3, mt0 = NT == 256 ? 0 : wave >> 2;
        const int ksteps = (p.r + 15) >> 4;
        bf16x8_t sgn[MTW][4];
#pragma unroll
        for (int m = 0; m < MTW; ++m)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const unsigned tk = (unsigned)((mt0 + m) * 32 + li);
                i16x8_t v;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int k = ks * 16 + kg * 8 + e;
                    const unsigned nk = lds_nat[k < p.r ? k : 0];
                    v[e] = k < p.r ? (short)((__popc(nk & tk) & 1) ? 0xBF80 - 0x10000 : 0x3F80) : (short)0;     // bf16 -1, +1, 0
                }
                sgn[m][ks] = __builtin_bit_cast(bf16x8_t, v);
            }
        const int patches = p.bm_step / p.r;
        const float inv = 1.0f / 64.0f;
        for (int pt = 0; pt < patches; ++pt) {
            const long q = (long)(m0 / p.r) + pt;
            if (q >= p.Q) break;                    // the same for every lane of the workgroup
            f32x16_t o[MTW];
#pragma unroll
            for (int m = 0; m < MTW; ++m)
#pragma unroll
                for (int e = 0; e < 16; ++e) o[m][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < ksteps) {
                    const unsigned char *qd = cot + (pt * p.r + ks * 16 + 8 * (grp >> 1) + (i16 >> 2)) * S_CO +
                                              (ch * 32 + 16 * (grp & 1) + 4 * (i16 & 3)) * 2;
                    i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, qd));
                    i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LBP_LDS_PTR(i16x4_t, qd + 4 * S_CO));
                    i16x8_t bv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    // a last step that is not full reads rows of the next patch (or the zero rows behind
                    // the tile): they must not reach the product even times a zero sign, or a coefficient
                    // that is not finite there would turn this patch's tokens into NaN
                    if ((ks + 1) * 16 > p.r) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (ks * 16 + kg * 8 + e >= p.r) bv[e] = 0;
                    }
                    bf16x8_t b = __builtin_bit_cast(bf16x8_t, bv);
#pragma unroll
                    for (int m = 0; m < MTW; ++m)      // rows of the product = channels, columns = tokens
                        o[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, sgn[m][ks], o[m], 0, 0, 0);
                }
            }
            // element 4*g4+e of o: channel ch*32 + 8*g4 + 4*kg + e, token (mt0+m)*32 + li
#pragma unroll
            for (int m = 0; m < MTW; ++m) {
                const int tk = (mt0 + m) * 32 + li;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
                    *reinterpret_cast<uint2 *>(stg + tk * S_TK + (ch * 32 + g4 * 8 + kg * 4) * 2) =
                        make_uint2(pack_bf16x2(o[m][g4 * 4] * inv, o[m][g4 * 4 + 1] * inv),
                                   pack_bf16x2(o[m][g4 * 4 + 2] * inv, o[m][g4 * 4 + 3] * inv));
            }
            __syncthreads();
            long img;
            int a0, b0;
            p.geom.origin(q, img, a0, b0);
            unsigned short *dst = reinterpret_cast<unsigned short *>(p.C) +
                                  p.geom.token(img, a0, b0) * p.N + n0;
            const int hv = p.geom.Ht - a0, wv = p.geom.Wt - b0;     // tokens of the patch inside the grid
            for (int c = tid; c < 64 * (BN / 8); c += NT) {
                const int tk = c >> 4, cc = c & 15, h = tk >> 3, w = tk & 7;
                if (n0 + cc * 8 < p.N && h < hv && w < wv) {
                    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
                    u32x4_t v = *reinterpret_cast<const u32x4_t *>(stg + tk * S_TK + cc * 16);
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(dst + ((size_t)h * p.geom.Wt + w) * p.N + cc * 8));
                }
            }
            __syncthreads();                        // the staging rows are free again
        }
        if (p.extra_rows > 0) {       // tokens outside the grid: bf16 rows of the product times 1/64 (exact)
            int lo, hi;
            extra_row_range(p, m0, lo, hi);
            for (int it = tid; it < (hi - lo) * (BN / 8); it += NT) {
                const int lr = lo + it / (BN / 8), cc = it % (BN / 8);
                const int col = n0 + cc * 8;
                if (col >= p.N) continue;
                const long j = (long)m0 + lr - p.Q * p.r;
                const long img = j / p.extra;
                const int e = (int)(j - img * p.extra);
                uint4 v = *reinterpret_cast<const uint4 *>(cot + lr * S_CO + cc * 16);
                v.x = pack_bf16x2(bf16_lo_to_f32(v.x) * inv, bf16_hi_to_f32(v.x) * inv);
                v.y = pack_bf16x2(bf16_lo_to_f32(v.y) * inv, bf16_hi_to_f32(v.y) * inv);
                v.z = pack_bf16x2(bf16_lo_to_f32(v.z) * inv, bf16_hi_to_f32(v.z) * inv);
                v.w = pack_bf16x2(bf16_lo_to_f32(v.w) * inv, bf16_hi_to_f32(v.w) * inv);
                *reinterpret_cast<uint4 *>(reinterpret_cast<unsigned short *>(p.C) + ((size_t)img * p.geom.img + e) * p.N + col) = v;
            }
        }
    } else if constexpr (EPI == EPI_UNPROJECT) {
        constexpr int CTS = BN + 8;
        static_assert(BM * CTS * 4 <= S::TOTAL, "tile does not fit in LDS");
        float *ct = reinterpret_cast<float *>(smem);
        // the loop above ended with a barrier: nobody reads operands any more
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int row = wm * WM + mi * 32 + g4 * 8 + kg * 4 + e;
                        int col = wn * WN + ni * 32 + li;
                        ct[row * CTS + col] = acc[mi][ni][g4 * 4 + e];
                    }
        __syncthreads();
        switch (p.mh * 4 + p.mw) {
#define LBP_CASE(MH, MW)                                                                         \
    case MH * 4 + MW:                                                                            \
        if constexpr (MH <= LP && MW <= LP && ((1 << LP) >> MH) * ((1 << LP) >> MW) <= 16)      \
            unproject_tile<LP, MH, MW, BN, NT>(ct, CTS, p, m0, n0, tid);                         \
        break;
            LBP_CASE(0, 0) LBP_CASE(0, 1) LBP_CASE(0, 2) LBP_CASE(0, 3)
            LBP_CASE(1, 0) LBP_CASE(1, 1) LBP_CASE(1, 2) LBP_CASE(1, 3)
            LBP_CASE(2, 0) LBP_CASE(2, 1) LBP_CASE(2, 2) LBP_CASE(2, 3)
            LBP_CASE(3, 0) LBP_CASE(3, 1) LBP_CASE(3, 2) LBP_CASE(3, 3)
#undef LBP_CASE
            default: break;
        }
        if (p.extra_rows > 0) {       // tokens outside the grid: their rows are the gradient itself, scaled
            int lo, hi;
            extra_row_range(p, m0, lo, hi);
            constexpr float inv = 1.0f / (float)((1 << LP) * (1 << LP));
            constexpr int HALF = BN / 2;
            for (int it = tid; it < (hi - lo) * HALF; it += NT) {
                const int lr = lo + it / HALF, cp = it % HALF;
                const int col = n0 + 2 * cp;
                if (col >= p.N) continue;
                const long j = (long)m0 + lr - p.Q * p.r;
                const long img = j / p.extra;
                const int e = (int)(j - img * p.extra);
                uint32_t *dst = reinterpret_cast<uint32_t *>(p.C) + (((size_t)img * p.geom.img + e) * p.N + col) / 2;
                *dst = pack_bf16x2(ct[lr * CTS + 2 * cp] * inv, ct[lr * CTS + 2 * cp + 1] * inv);
            }
        }
    } else {
#pragma unroll
        for (int mi = 0; mi < TM; ++mi)
#pragma unroll
            for (int ni = 0; ni < TN; ++ni) {
                int col = n0 + wn * WN + ni * 32 + li;
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int row = m0 + wm * WM + mi * 32 + g4 * 8 + kg * 4 + e;
                        if (row < p.M && col < p.N) {
                            float v = acc[mi][ni][g4 * 4 + e] * p.scale;
                            if (EPI == EPI_F32 || (EPI == EPI_PLAIN && !p.store_bf16)) {
                                float *Cz = reinterpret_cast<float *>(p.C) + (size_t)slice * p.M * p.N;
                                Cz[(size_t)row * p.N + col] = v;
                            } else {
                                reinterpret_cast<unsigned short *>(p.C)[(size_t)row * p.N + col] =
                                    (unsigned short)f32_to_bf16_bits(v);
                            }
                        }
                    }
            }
    }
}

template <int BM, int BN, int WGM, int WGN, int PF, bool A_KFAST, int EPI, int LP, bool JOIN = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(Params p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    gemm_body<BM, BN, WGM, WGN, PF, A_KFAST, EPI, LP, JOIN>(p, blockIdx.x, blockIdx.y, smem);
}

// A kernel that uses more than 64 KB of dynamic LDS has to be allowed to, once per device (the
// attribute belongs to the current device's copy of the kernel).  `configured` has one flag per
// device; racing threads set the same value.
constexpr int kMaxLaunchDevices = 64;
inline hipError_t allow_dynamic_lds(const void *kern, int bytes, bool *configured)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxLaunchDevices) return hipErrorInvalidDevice;
    if (!configured[dev]) {
        e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        configured[dev] = true;
    }
    return hipSuccess;
}

template <int BM, int BN, int WGM, int WGN, int PF, bool A_KFAST, int EPI, int LP, bool JOIN = false>
hipError_t launch_one(const Params &p, int splits, hipStream_t stream)
{
    constexpr int LDS = Smem<BM, BN, A_KFAST>::TOTAL;
    auto kern = gemm_kernel<BM, BN, WGM, WGN, PF, A_KFAST, EPI, LP, JOIN>;
    static bool configured[kMaxLaunchDevices] = {};     // per instantiation
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), LDS, configured);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)splits);
    hipLaunchKernelGGL(kern, grid, dim3(64 * WGM * WGN), LDS, stream, p);
    return hipGetLastError();
}

// Two independent products in one launch: workgroups [0, blocks_first) run `first`, the rest run
// `second`; inside each range the index is tile + tiles * slice.  A low-rank product alone leaves
// compute units idle (a hundred-odd tiles on 256 units); launched together the two products of
// Algorithm 1 (the weight gradient and the input gradient only share the read-only g^y) fill them
// and save one launch gap.  Both bodies are the ones of the single-product kernels, so results are
// bit-identical to separate launches.
struct PairParams {
    Params first, second;
    int blocks_first, blocks_second;
    int second_leads;     // 1: the workgroups of `second` have the lower indices (are dispatched first)
};

template <int WGM, int WGN, int PF, int BM1, int BN1, bool KF1, int EPI1, int LP1, int BM2, int BN2, bool KF2,
          int EPI2, int LP2, bool JOIN1 = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_pair_kernel(PairParams pp)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // (both orders keep a tile's workgroup index modulo 8, hence its XCD, a function of its tile id only)
    const int b = pp.second_leads ? (blockIdx.x < (unsigned)pp.blocks_second ? (int)blockIdx.x + pp.blocks_first
                                                                             : (int)blockIdx.x - pp.blocks_second)
                                  : (int)blockIdx.x;
    if (b < pp.blocks_first) {
        const int T = pp.first.tiles_m * pp.first.tiles_n;
        const int z = b / T;
        gemm_body<BM1, BN1, WGM, WGN, PF, KF1, EPI1, LP1, JOIN1>(pp.first, b - z * T, z, smem);
    } else {
        const int c = b - pp.blocks_first;
        const int T = pp.second.tiles_m * pp.second.tiles_n;
        const int z = c / T;
        gemm_body<BM2, BN2, WGM, WGN, PF, KF2, EPI2, LP2>(pp.second, c - z * T, z, smem);
    }
}

template <int WGM, int WGN, int PF, int BM1, int BN1, bool KF1, int EPI1, int LP1, int BM2, int BN2, bool KF2,
          int EPI2, int LP2, bool JOIN1 = false>
hipError_t launch_pair(const Params &first, int splits_first, const Params &second, int splits_second,
                       hipStream_t stream, bool second_leads = false)
{
    constexpr int L1 = Smem<BM1, BN1, KF1>::TOTAL, L2 = Smem<BM2, BN2, KF2>::TOTAL;
    constexpr int LDS = L1 > L2 ? L1 : L2;
    auto kern = gemm_pair_kernel<WGM, WGN, PF, BM1, BN1, KF1, EPI1, LP1, BM2, BN2, KF2, EPI2, LP2, JOIN1>;
    static bool configured[kMaxLaunchDevices] = {};
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), LDS, configured);
    if (e != hipSuccess) return e;
    PairParams pp;
    pp.first = first;
    pp.second = second;
    pp.blocks_first = first.tiles_m * first.tiles_n * splits_first;
    pp.blocks_second = second.tiles_m * second.tiles_n * splits_second;
    pp.second_leads = second_leads ? 1 : 0;
    const unsigned blocks = (unsigned)(pp.blocks_first + pp.blocks_second);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(64 * WGM * WGN), LDS, stream, pp);
    return hipGetLastError();
}

// All instantiations of one tile shape and prefetch depth: output kind x operand layout; lp is
// log2(patch) for the fused reverse projection.
template <int BM, int BN, int WGM, int WGN, int PF, bool FUSED>
hipError_t launch_tile(const Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s)
{
    if (out == GemmOut::kUnproject) {
        if constexpr (FUSED) {
            if (p.splits > 1) {      // slices that join inside the launch: the 8-wavefront 128-wide tiles, patch 8
                if constexpr (BN == 128 && WGM * WGN == 8) {
                    if (lp != 3) return hipErrorInvalidValue;
                    if (p.mfma_epilogue) return launch_one<BM, BN, WGM, WGN, PF, true, EPI_UNPROJECT_MFMA, 3, true>(p, p.splits, s);
                    return launch_one<BM, BN, WGM, WGN, PF, true, EPI_UNPROJECT, 3, true>(p, p.splits, s);
                }
                return hipErrorInvalidValue;
            }
            if (p.mfma_epilogue) {
                if constexpr (BN == 128) {
                    if (lp == 3) return launch_one<BM, BN, WGM, WGN, PF, true, EPI_UNPROJECT_MFMA, 3>(p, 1, s);
                }
                return hipErrorInvalidValue;
            }
            if (lp == 3) return launch_one<BM, BN, WGM, WGN, PF, true, EPI_UNPROJECT, 3>(p, 1, s);
            if (lp == 2) return launch_one<BM, BN, WGM, WGN, PF, true, EPI_UNPROJECT, 2>(p, 1, s);
        }
        return hipErrorInvalidValue;
    }
    if (out == GemmOut::kF32) {
        if (a_kfast) return launch_one<BM, BN, WGM, WGN, PF, true, EPI_F32, 0>(p, splits, s);
        return launch_one<BM, BN, WGM, WGN, PF, false, EPI_F32, 0>(p, splits, s);
    }
    if (a_kfast) return launch_one<BM, BN, WGM, WGN, PF, true, EPI_BF16, 0>(p, 1, s);
    return launch_one<BM, BN, WGM, WGN, PF, false, EPI_BF16, 0>(p, 1, s);
}

}  // namespace mfma

// One entry per tile shape, defined in gemm_mfma_<shape>.hip.
hipError_t mfma_tile_128x128(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);
hipError_t mfma_tile_64x128(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);
hipError_t mfma_tile_256x128(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);
hipError_t mfma_tile_256x256(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);
hipError_t mfma_tile_128x128w8(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);
hipError_t mfma_tile_64x128w8(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);
hipError_t mfma_tile_64x64(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);
hipError_t mfma_tile_256x192(const mfma::Params &p, bool a_kfast, GemmOut out, int lp, int splits, hipStream_t s);

// Grouped launch of the input-gradient product `x` (A reduction-fast; tile 128x128 or 64x128 with 8
// wavefronts: bm_x = 128 or 64; out_x as in launch_gemm, kUnproject needs patch 8) and the
// weight-gradient product `w` (A reduction-slow, 128x128 tile with 8 wavefronts, fp32 or bf16 store
// by w.store_bf16).  hipErrorInvalidValue for a combination that is not instantiated.
hipError_t mfma_pair_w8(const mfma::Params &x, int bm_x, GemmOut out_x, int splits_x, const mfma::Params &w,
                        int splits_w, hipStream_t s, bool w_leads = false);
// The same for 64 x 64 tiles with 4 wavefronts on both products (pooled fused epilogue only).
hipError_t mfma_pair_64x64(const mfma::Params &x, GemmOut out_x, int splits_x, const mfma::Params &w, int splits_w,
                           hipStream_t s, bool w_leads = false);

}  // namespace lbp
