/*
 * lbp_wht.h -- C ABI of the MI355X (gfx950) library for low-rank backpropagation through one
 * linear layer with Walsh-Hadamard projections (LBP-WHT).
 *
 * The call shape follows the problem statement of Algorithm 1 (Section 3.1):
 *     input  x, w, g_y and the set I of selected WHT bases;
 *     output the approximated gradients g~_x and g~_w.
 *
 * Conventions shared by every entry point
 *   Layout   token-major, channel innermost, row-major, densely packed:
 *              x  [N][H][W][Cin]      gy [N][H][W][Cout]     W  [Cout][Cin]
 *              gx [N][H][W][Cin]      gW [Cout][Cin]
 *            (Section 2 writes w in R^{Cy x Cx}; y = x w^T per token.)
 *   Patches  the H x W token grid of every image is tiled into non-overlapping patch x patch
 *            blocks; the order-`patch` 2-D WHT of Section 3 is applied inside each block, and the
 *            weight gradient sums over blocks and images.  A grid whose H or W is not a multiple
 *            of patch (the 7 x 7 = 49-token maps of Section 3.3) is treated as zero-padded at
 *            its bottom and right edges up to the next multiple: there are
 *            P = N * ceil(H/patch) * ceil(W/patch) blocks, padding tokens are never read or
 *            written, and the 1/patch^2 factors are unchanged.  Low-rank buffers have P*r rows.
 *   Bases    basis_idx[k] = u*patch + v, with (u, v) the 0-based SEQUENCY indices along the grid's
 *            H axis (u) and W axis (v): index 0 is the constant basis and a larger index is a
 *            higher frequency (Section 3.2).  Entries must be distinct and in [0, patch^2).
 *   Scaling  the forward projection (Eq. 6) is applied unnormalised; gx and gW each carry one factor
 *            1/patch^2, so that keeping all patch^2 bases reproduces exact backpropagation (Eq. 2).
 *   Memory   x, gy, W, gx, gW and workspaces are DEVICE pointers owned by the caller, 16-byte
 *            aligned; `shape` and `basis_idx` are HOST pointers read only during the call.
 *            Outputs are overwritten (never accumulated into) and must not overlap any input.
 *   Stream   `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *            enqueued on it; no entry point synchronises the device unless it says so.
 *   Errors   every function returning int gives LBP_OK (0) or a negative lbp_status_t.  Argument
 *            errors are detected on the host before any HIP call is made, so they can be provoked
 *            and tested on a machine without a GPU.  There is no CPU fallback: without a usable
 *            gfx950 device the compute entry points return LBP_ERR_HIP.
 *   Threads  entry points may be called from several host threads, but backward calls on one
 *            device are ordered by the caller's stream order only: they share that device's
 *            workspace (the internal one or the one set with lbp_set_workspace, which is per
 *            process) and a small array of tile counters inside the library, so two backward
 *            calls must not overlap in time on one device (different streams need an event
 *            between them).
 */
#ifndef LBP_WHT_H
#define LBP_WHT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LBP_F32 = 0,   /* IEEE binary32 tensors, fp32 arithmetic                                  */
    LBP_BF16 = 1   /* bfloat16 tensors, bf16 matrix-core products with fp32 accumulation      */
} lbp_dtype_t;

typedef enum {
    LBP_ORDER_L1 = 0,   /* LP_L1  low-pass order (Eq. 8): shells of constant u+v              */
    LBP_ORDER_LINF = 1  /* LP_Linf low-pass order (Eq. 9): shells of constant max(u,v)        */
} lbp_order_t;

typedef enum {
    LBP_OK = 0,
    LBP_ERR_NULL = -1,     /* a required pointer is NULL                                       */
    LBP_ERR_SHAPE = -2,    /* non-positive dimension, or a size beyond what 32-bit row indices
                              address (N*H*W >= 2^31)                                          */
    LBP_ERR_PATCH = -3,    /* patch not in {2, 4, 8, 16}                                       */
    LBP_ERR_RANK = -4,     /* r < 1 or r > patch^2                                             */
    LBP_ERR_BASIS = -5,    /* a basis index out of [0, patch^2) or listed twice                */
    LBP_ERR_DTYPE = -6,    /* unknown dtype / gw_dtype, or an unsupported combination          */
    LBP_ERR_ALIAS = -7,    /* an output buffer overlaps an input or the other output           */
    LBP_ERR_ALIGN = -8,    /* a device pointer is not 16-byte aligned, or a channel count is not
                              a multiple of the vector width the kernels need (8 for bf16, 4 for
                              fp32)                                                            */
    LBP_ERR_ORDER = -9,    /* order is neither LBP_ORDER_L1 nor LBP_ORDER_LINF                 */
    LBP_ERR_WORKSPACE = -10, /* caller-provided workspace too small                            */
    LBP_ERR_HIP = -11,     /* a HIP call failed (no device, allocation, launch); the HIP error
                              code is kept and returned by lbp_last_hip_error()                */
    LBP_ERR_OPTION = -12   /* lbp_set_option: unknown name or a value it does not take         */
} lbp_status_t;

typedef struct {
    int32_t N, H, W;     /* batch size and token grid of one image                             */
    int32_t Cin, Cout;   /* C_x and C_y of Section 2                                           */
    int32_t dtype;       /* lbp_dtype_t of x, gy, W and gx                                     */
    int32_t gw_dtype;    /* lbp_dtype_t of gW: LBP_F32, or the same as dtype                   */
} lbp_shape_t;

/*
 * Low-pass basis selection, Section 3.2 (Eq. 8 for LP_L1, Eq. 9 for LP_Linf).
 * Writes the first r sequency pairs of the chosen order into basis_idx (host, r ints).
 * Inside a shell the order is: LP_L1 by (u+v, max(u,v), u); LP_Linf by (max(u,v), u+v, u), so for
 * r = k(k+1)/2 (LP_L1) or r = k^2 (LP_Linf) the set is exactly the paper's LP-k selection.
 * Pure host integer code; never touches the GPU.
 */
int lbp_wht_select_bases(int patch, int r, int order, int32_t *basis_idx);

/*
 * Low-heuristic-error (LHE) selection, Section 3.2: the r bases with the largest profiled energy.
 * `energy` is a HOST array of patch^2 doubles indexed u*patch + v (what lbp_wht_energy accumulates,
 * copied back by the caller).  Writes the r indices by decreasing energy; bases of equal energy keep
 * their LP_L1 order (the paper leaves ties open).  Pure host code.
 */
int lbp_wht_select_lhe(const double *energy, int patch, int r, int32_t *basis_idx);

/*
 * Profiling step of the LHE selection (Section 3.2; the spectrum shown in Section 4.5): adds to
 * energy[u*patch + v] (DEVICE, patch^2 doubles, caller zeroes it before the first call) the sum over
 * all patches and channels of the squared unnormalised WHT coefficient (Eq. 6) of basis (u, v) of
 * `in` [N][H][W][C].  Call it on gy for a few training steps, copy `energy` back, then call
 * lbp_wht_select_lhe.  Needs lbp_wht_energy_workspace_bytes of workspace (all coefficients are
 * materialised once; this is a profiling call, not part of the per-step path).  bf16 tensors: the
 * coefficients are rounded to bf16 before they are squared.  Sums run in a fixed order.
 */
int lbp_wht_energy(const void *in, int N, int H, int W, int C, int dtype, int patch, double *energy,
                   void *stream);
size_t lbp_wht_energy_workspace_bytes(int N, int H, int W, int C, int dtype, int patch);

/*
 * Algorithm 1 (Section 3.1): x^ = WHT(x; I), g^y = WHT(gy; I), g^w = g^y^T x^, g^x = g^y w,
 * g~x = WHT^-1(g^x; I), g~w = g^w, with Eq. 6 / Eq. 7 per token patch.
 *   x, gy, W   inputs (device);  gx, gW outputs (device), either may be NULL to skip it.
 *   basis_idx  host array of r indices (see "Bases" above); r in [1, patch^2].
 * Uses the workspace set by lbp_set_workspace, else an internal per-device buffer that grows on
 * demand (the first call at a new size allocates device memory; later calls do not).
 * The two products depend only on the projections, not on each other: when both gradients are
 * requested they may run as one kernel launch.
 */
int lbp_wht_backward(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                     int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream);

/*
 * lbp_wht_backward for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same bits
 * as lbp_wht_backward, but the projected tensors, split-K partial sums and unfused coefficients
 * live in a fixed array of LBP_STATIC_SCRATCH_BYTES that is part of the library's device image
 * (every GPU the library runs on holds its own copy until the process ends) instead of the
 * workspace.  The call makes no hipMalloc / hipFree and ignores lbp_set_workspace.
 *   LBP_ERR_WORKSPACE  the call would need more scratch than the array holds (the need is what
 *                      lbp_wht_workspace_bytes reports at most; ViT-B fc1, N = 64, r = 8 needs
 *                      15.7 MB); nothing is launched.
 * All calls on one GPU share that GPU's array, whatever their streams: two calls that overlap in
 * time on one GPU race.  Calls ordered by one stream are safe; nothing in the array has to
 * start at zero (every region is written before it is read within a call).
 */
#define LBP_STATIC_SCRATCH_BYTES (32u << 20)
int lbp_wht_backward_static(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                            int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream);

/*
 * Algorithm 1 with its first statement hoisted out: x^ = WHT(x; I) depends only on the layer's input
 * and the index set, so the forward pass can compute it once (lbp_wht_project on x) and keep it
 * instead of x, which is patch^2/r times larger.  x_r is that tensor, [P*r][Cin] of shape->dtype,
 * projected with the SAME basis_idx; everything else as lbp_wht_backward.  The backward then never
 * reads x.  Results are bit-identical to lbp_wht_backward on the same x.
 */
int lbp_wht_backward_preprojected(const void *x_r, const void *gy, const void *W,
                                  const lbp_shape_t *shape, int patch, const int32_t *basis_idx, int r,
                                  void *gx, void *gW, void *stream);

/*
 * Statements 3 to 6 of Algorithm 1 alone, from tensors that are already projected: x_r = x^ [P*r][Cin]
 * and gy_r = g^y [P*r][Cout] (both of shape->dtype, made with the SAME basis_idx by lbp_wht_project_pair
 * or lbp_wht_project), W [Cout][Cin].  g~w = (1/patch^2) g^y^T x^ and g~x = (1/patch^2) WHT^-1(g^y W; I)
 * as in lbp_wht_backward, with bit-identical results.  For callers that project elsewhere (or time
 * the products by themselves).
 */
int lbp_wht_products(const void *x_r, const void *gy_r, const void *W, const lbp_shape_t *shape, int patch,
                     const int32_t *basis_idx, int r, void *gx, void *gW, void *stream);

/*
 * Token sequences with tokens that are not on the grid.  A ViT layer sees, per image, `extra` tokens
 * (a class token, a distillation token) followed by the H*W patch tokens: x, gy and gx are
 * [N][extra + H*W][C] here.  Algorithm 1 is stated for the H x W map; the paper does not say what
 * happens to the others.  This library keeps them exact: a token outside the grid belongs to no
 * patch, its row of gx is g_y,row W and its outer product g_y,row^T x_row is added to gW (its share of
 * Eq. 2); the grid tokens go through Algorithm 1 as in lbp_wht_backward.  extra = 0 is
 * lbp_wht_backward itself.  shape->H, shape->W describe the grid only.
 *
 * lbp_wht_project_tokens is the forward-pass half for x: out is [P*r + N*extra][C], the projected grid
 * (as lbp_wht_project) followed by the extra tokens unchanged, image-major; that tensor is the x_r of
 * lbp_wht_backward_tokens_preprojected.  LBP_ERR_SHAPE for a negative `extra`.
 */
int lbp_wht_backward_tokens(const void *x, const void *gy, const void *W, const lbp_shape_t *shape, int extra,
                            int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream);
int lbp_wht_project_tokens(const void *in, int N, int H, int W, int extra, int C, int dtype, int patch,
                           const int32_t *basis_idx, int r, void *out, void *stream);
int lbp_wht_backward_tokens_preprojected(const void *x_r, const void *gy, const void *W, const lbp_shape_t *shape,
                                         int extra, int patch, const int32_t *basis_idx, int r, void *gx, void *gW,
                                         void *stream);
/* lbp_wht_energy on such sequences: the spectrum of the grid tokens; the extra tokens have no
 * coefficients and are skipped.  Same workspace as lbp_wht_energy. */
/*
 * The first two statements of Algorithm 1 for token sequences, both tensors in ONE launch, and
 * statements 3-6 from their results (lbp_wht_project_pair / lbp_wht_products with `extra` tokens
 * per image in front of the grid).  x_r is [P*r + N*extra][Cin], gy_r [P*r + N*extra][Cout]: the
 * coefficient rows, then the tokens outside the grid image by image -- x's as they are, g_y's
 * multiplied by patch^2 (exact; the 1/patch^2 of both products removes it), which is the form
 * lbp_wht_products_tokens expects.  lbp_wht_products_tokens on these gives the bits of
 * lbp_wht_backward_tokens.
 */
int lbp_wht_project_pair_tokens(const void *x, const void *gy, const lbp_shape_t *shape, int extra, int patch,
                                const int32_t *basis_idx, int r, void *x_r, void *gy_r, void *stream);
int lbp_wht_products_tokens(const void *x_r, const void *gy_r, const void *W, const lbp_shape_t *shape, int extra,
                            int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream);
int lbp_wht_energy_tokens(const void *in, int N, int H, int W, int extra, int C, int dtype, int patch,
                          double *energy, void *stream);
/* Workspace of the backward calls above (lbp_wht_workspace_bytes with `extra` tokens per image). */
size_t lbp_wht_workspace_bytes_tokens(const lbp_shape_t *shape, int extra, int patch, int r);

/*
 * What a backward call with these arguments would launch, as one line of text (host logic only, no
 * device work, usable without a GPU): the projection kernel, whether the two products share a
 * launch, tile shape and split-K factor of each product, fused or separate reverse projection, and
 * the workspace size.  num_cus <= 0 takes the current device's compute-unit count (256 if there
 * is no device).  Writes at most len - 1 characters and a NUL to buf.  For logs and tests; the
 * wording is not a stable interface.
 */
int lbp_wht_describe_plan(const lbp_shape_t *shape, int extra, int patch, const int32_t *basis_idx, int r,
                          int want_gx, int want_gw, int num_cus, char *buf, size_t len);

/*
 * For measurement, not part of the method: the same call as lbp_wht_backward, bracketed by HIP
 * events on `stream`.  It WAITS for the work to finish and returns the elapsed milliseconds of the
 * three stages in stage_ms (host, 3 floats): [0] projection of gy and x, [1] weight-gradient
 * product, [2] input-gradient product with the reverse projection; here the two products are
 * always launched one after the other (each with the tiles that suit it alone).  Callers:
 * benchmarks that report where the time of a call goes.
 */
int lbp_wht_backward_profile(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                             int patch, const int32_t *basis_idx, int r, void *gx, void *gW,
                             void *stream, float *stage_ms);

/*
 * Exact backward of Eq. 2 (Section 2), the full-rank comparison point built from the same
 * kernels: gx = gy W (per token), gW = gy^T x (summed over all tokens).  Same argument rules.
 */
int full_bp_backward(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                     void *gx, void *gW, void *stream);

/*
 * The projection p(.) of Eq. 6 alone (first two statements of Algorithm 1), for one tensor:
 *   in  [N][H][W][C] (device, dtype)  ->  out [(N*H*W/patch^2) * r][C] (device, same dtype),
 * row (q*r + k) holding coefficient k of patch q = (n*ceil(H/patch) + a)*ceil(W/patch) + b, unnormalised.
 * It is what the backward runs internally on x and gy; exported so that the projection can be
 * measured and checked by itself.
 */
int lbp_wht_project(const void *in, int N, int H, int W, int C, int dtype, int patch,
                    const int32_t *basis_idx, int r, void *out, void *stream);

/*
 * The first two statements of Algorithm 1 exactly as lbp_wht_backward runs them: x^ = WHT(x; I) and
 * g^y = WHT(gy; I) in ONE kernel launch (gy's workgroups first, x's filling the tail).
 *   x [N][H][W][Cin], gy [N][H][W][Cout]  ->  x_r [P*r][Cin], gy_r [P*r][Cout], all of shape->dtype
 * (shape->gw_dtype is ignored).  Exported so that the dominant kernel of the backward can be timed
 * by itself, and for callers that keep x^ from the forward pass.
 */
int lbp_wht_project_pair(const void *x, const void *gy, const lbp_shape_t *shape, int patch,
                         const int32_t *basis_idx, int r, void *x_r, void *gy_r, void *stream);

/*
 * The reverse projection p^-1(.) of Eq. 7 alone, with the 1/patch^2 factor:
 *   in  [(N*H*W/patch^2) * r][C] (device, ALWAYS fp32: it is the accumulator of g^y w)
 *   out [N][H][W][C] (device, dtype).
 */
int lbp_wht_unproject(const void *in, int N, int H, int W, int C, int dtype, int patch,
                      const int32_t *basis_idx, int r, void *out, void *stream);

/* Bytes of device workspace lbp_wht_backward / full_bp_backward need for this problem
 * (r = 0 and patch = 0 ask for full_bp_backward).  0 on invalid arguments. */
size_t lbp_wht_workspace_bytes(const lbp_shape_t *shape, int patch, int r);

/* Hands the library a caller-owned device buffer to use as workspace on the current device for all
 * later calls of this process (dev_ptr = NULL returns to the internal buffer).  The caller keeps
 * ownership and must keep it alive while calls are in flight.  Calls whose need exceeds `bytes`
 * return LBP_ERR_WORKSPACE. */
int lbp_set_workspace(void *dev_ptr, size_t bytes);

/* Frees the internal workspaces of all devices (synchronises each device first). */
int lbp_release_workspace(void);

/*
 * Kernel-choice switches, for tests and measurement only (normal use never needs them: the
 * planner chooses).  Process-wide; the value NULL puts a switch back to its default.  The first
 * use of the switches also reads environment variables of the same names, once per process.
 *   "LBP_WHT_PATH"        "generic" | "register" | "mfma"   projection kernels (default: chosen per selection)
 *   "LBP_GEMM_PATH"       "simple"                          plain cross-check products
 *   "LBP_GEMM_TILE"       "0" .. "7"                        one tile shape for every product
 *   "LBP_FUSE_UNPROJECT"  "0" | "1"                         reverse projection never / always fused where possible
 *   "LBP_GEMM_GROUP"      "0" | "1" | "2"                   the two products in separate launches / grouped where possible /
 *                                                           grouped with the weight-gradient workgroups always first
 *   "LBP_GX_COEF"         "f32" | "bf16"                    coefficients handed to an unfused reverse projection
 *   "LBP_GX_JOIN"         "1" .. "8"                        slices of the fused input-gradient product's reduction that
 *                                                           combine inside the grouped launch (default: chosen per shape)
 * Returns LBP_ERR_NULL (name is NULL) or LBP_ERR_OPTION (unknown name or value).  No HIP call.
 */
int lbp_set_option(const char *name, const char *value);

/* Static description of a status code. */
const char *lbp_strerror(int code);

/* HIP error code (hipError_t as int) of the most recent LBP_ERR_HIP on this thread, else 0. */
int lbp_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int lbp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LBP_WHT_H */
