// C-ABI entry points (include/lbp_wht.h): host-side validation first, then kernel launches on
// the caller's stream.  No torch types, no CPU fallback: without a usable device every compute
// entry point returns LBP_ERR_HIP.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "kernels.h"
#include "lbp_host.h"

namespace {

thread_local int t_last_hip_error = 0;

int hip_fail(hipError_t e)
{
    t_last_hip_error = (int)e;
    (void)hipGetLastError();   // clear the sticky launch error, it has been recorded
    return LBP_ERR_HIP;
}

constexpr int kMaxDevices = 64;

// Scratch of lbp_wht_backward_static, the entry point that allocates nothing.  Part of the device
// image: every GPU holds its own copy at its own address.  On the host this name is only a handle
// for hipGetSymbolAddress; the address kernels get is DeviceState::static_ws.
constexpr size_t kStaticScratchBytes = LBP_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

struct DeviceState {
    void *internal_ws = nullptr;
    size_t internal_bytes = 0;
    void *user_ws = nullptr;
    size_t user_bytes = 0;
    int num_cus = 0;
    char *static_ws = nullptr;      // device address of `scratch` on this device
};

std::mutex g_mutex;
DeviceState g_dev[kMaxDevices];

// Current device and its state; LBP_ERR_HIP if there is none.
int current_device(int *dev, DeviceState **st)
{
    int d = -1;
    hipError_t e = hipGetDevice(&d);
    if (e != hipSuccess) return hip_fail(e);
    if (d < 0 || d >= kMaxDevices) return hip_fail(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(g_mutex);
    if (g_dev[d].num_cus == 0) {
        int cus = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, d);
        if (e != hipSuccess) return hip_fail(e);
        // first call on this device, which is current: its copy of the static scratch array
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u)) return hip_fail(hipErrorInvalidSymbol);
        g_dev[d].static_ws = static_cast<char *>(ptr);
        g_dev[d].num_cus = cus > 0 ? cus : 256;
    }
    *dev = d;
    *st = &g_dev[d];
    return LBP_OK;
}

// Workspace of at least `bytes` on the current device: the caller's if one was set, else the
// internal grow-only buffer.
int get_workspace(DeviceState *st, size_t bytes, char **out)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    if (st->user_ws) {
        if (st->user_bytes < bytes) return LBP_ERR_WORKSPACE;
        *out = (char *)st->user_ws;
        return LBP_OK;
    }
    if (st->internal_bytes < bytes) {
        if (st->internal_ws) {
            // earlier calls may still be reading the old buffer on some stream
            hipError_t e = hipDeviceSynchronize();
            if (e != hipSuccess) return hip_fail(e);
            e = hipFree(st->internal_ws);
            st->internal_ws = nullptr;
            st->internal_bytes = 0;
            if (e != hipSuccess) return hip_fail(e);
        }
        size_t want = bytes + bytes / 4;
        hipError_t e = hipMalloc(&st->internal_ws, want);
        if (e != hipSuccess) {
            st->internal_ws = nullptr;
            return hip_fail(e);
        }
        st->internal_bytes = want;
    }
    *out = (char *)st->internal_ws;
    return LBP_OK;
}

// The kernel-choice switches (lbp_set_option) in the kernels' own types.
lbp::GemmPath gemm_path_option() { return lbp::options().gemm_simple ? lbp::GemmPath::kSimple : lbp::GemmPath::kAuto; }
lbp::WhtPath wht_path_option() { return static_cast<lbp::WhtPath>(lbp::options().wht_path); }

// Pointer, alias and alignment rules common to both backward entry points.
int validate_buffers(const void *x, const void *gy, const void *W, const lbp_shape_t *s, void *gx,
                     void *gW, size_t x_rows = 0, int extra = 0, size_t gy_rows = 0)
{
    if (!x || !gy || !W) return LBP_ERR_NULL;
    if (!gx && !gW) return LBP_ERR_NULL;
    const void *ptrs[5] = {x, gy, W, gx, gW};
    int rc = lbp::validate_alignment(ptrs, 5);
    if (rc) return rc;
    size_t esz = lbp::dtype_size(s->dtype);
    size_t M = (size_t)s->N * ((size_t)s->H * s->W + extra);
    size_t nx = (x_rows ? x_rows : M) * s->Cin * esz, ngy = (gy_rows ? gy_rows : M) * s->Cout * esz;
    size_t nw = (size_t)s->Cout * s->Cin * esz;
    size_t ngx = M * s->Cin * esz, ngw = (size_t)s->Cout * s->Cin * lbp::dtype_size(s->gw_dtype);
    const void *ins[3] = {x, gy, W};
    size_t in_bytes[3] = {nx, ngy, nw};
    for (int i = 0; i < 3; ++i) {
        if (lbp::ranges_overlap(gx, ngx, ins[i], in_bytes[i])) return LBP_ERR_ALIAS;
        if (lbp::ranges_overlap(gW, ngw, ins[i], in_bytes[i])) return LBP_ERR_ALIAS;
    }
    if (lbp::ranges_overlap(gx, ngx, gW, ngw)) return LBP_ERR_ALIAS;
    return LBP_OK;
}

#define LBP_HIP(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return hip_fail(e_);     \
    } while (0)

// `extra` tokens per image in front of the grid: non-negative, and all tokens still count in 31 bits.
bool tokens_ok(const lbp_shape_t *s, int extra)
{
    return extra >= 0 && (long)s->N * ((long)s->H * s->W + extra) <= 0x7fffffffL;
}

// The launch plan of one low-rank backward call: tiles, split-K factors, fused or separate
// reverse projection, grouped or separate products, workspace layout (host logic only).
int plan_call(const lbp_shape_t *shape, int extra, int patch, int r, const lbp::BasisPlan &plan, int num_cus,
              bool both_outputs, lbp::WorkspacePlan *ws)
{
    const lbp::Options opt = lbp::options();
    const lbp::GemmPath gpath = opt.gemm_simple ? lbp::GemmPath::kSimple : lbp::GemmPath::kAuto;
    const int fuse_env = opt.fuse_unproject;
    const bool can_fuse = fuse_env != 0 && lbp::gemm_can_fuse_unproject(plan, shape->dtype, gpath);
    const bool allow_group = both_outputs && gpath != lbp::GemmPath::kSimple && opt.gemm_group != 0;
    // a product that stores bf16 coefficients for the reverse projection: matrix-core products and
    // the matrix-core form of the reverse projection only
    int coef16 = opt.gx_coef;
    if (gpath == lbp::GemmPath::kSimple || shape->dtype != LBP_BF16 ||
        !lbp::unproject_bf16_supported(plan, static_cast<lbp::WhtPath>(opt.wht_path), shape->dtype, shape->Cin))
        coef16 = 0;
    return lbp::plan_workspace(shape, patch, r, num_cus, can_fuse, fuse_env == 1, ws,
                               !lbp::gemm_unproject_pooled(plan), allow_group, extra, coef16, opt.gx_join);
}

// Describes the weight-gradient product; returns true when it leaves fp32 partial sums in `part`
// that launch_splitk_reduce still has to combine (scaled) into gW.
bool weight_gradient_args(const void *A, const void *B, int Cout, int Cin, long K, int dtype, int gw_dtype,
                          const lbp::GemmPlan &plan, float scale, float *part, void *gW, lbp::GemmPath gpath,
                          lbp::GemmArgs *out)
{
    lbp::GemmArgs g;
    g.tile = plan.tile;
    g.A = A; g.B = B;
    g.M = Cout; g.N = Cin; g.K = (int)K;
    g.lda = Cout; g.ldb = Cin;
    g.a_kfast = false;
    g.dtype = dtype;
    const bool mfma = dtype == LBP_BF16 && gpath != lbp::GemmPath::kSimple;
    const bool direct = plan.splits == 1 && (gw_dtype == LBP_F32 || mfma);
    if (direct) {
        g.splits = 1;
        g.out = gw_dtype == LBP_F32 ? lbp::GemmOut::kF32 : lbp::GemmOut::kBF16;
        g.C = gW;
        g.scale = scale;
    } else {
        g.splits = plan.splits;
        g.out = lbp::GemmOut::kF32;
        g.C = part;
        g.scale = 1.0f;
    }
    *out = g;
    return !direct;
}

int weight_gradient(const void *A, const void *B, int Cout, int Cin, long K, int dtype, int gw_dtype,
                    const lbp::GemmPlan &plan, float scale, float *part, void *gW, lbp::GemmPath gpath,
                    hipStream_t s)
{
    lbp::GemmArgs g;
    const bool reduce = weight_gradient_args(A, B, Cout, Cin, K, dtype, gw_dtype, plan, scale, part, gW, gpath, &g);
    LBP_HIP(lbp::launch_gemm(g, gpath, s));
    if (reduce) LBP_HIP(lbp::launch_splitk_reduce(part, plan.splits, (long)Cout * Cin, scale, gW, gw_dtype, s));
    return LBP_OK;
}

}  // namespace

extern "C" {

int lbp_version(void) { return 200; }

const char *lbp_strerror(int code) { return lbp::status_string(code); }

int lbp_last_hip_error(void) { return t_last_hip_error; }

int lbp_set_option(const char *name, const char *value) { return lbp::set_option(name, value); }

int lbp_wht_select_bases(int patch, int r, int order, int32_t *basis_idx)
{
    return lbp::select_bases(patch, r, order, basis_idx);
}

size_t lbp_wht_workspace_bytes(const lbp_shape_t *shape, int patch, int r)
{
    return lbp_wht_workspace_bytes_tokens(shape, 0, patch, r);
}

size_t lbp_wht_workspace_bytes_tokens(const lbp_shape_t *shape, int extra, int patch, int r)
{
    if (lbp::validate_shape(shape, patch) != LBP_OK || !tokens_ok(shape, extra)) return 0;
    if (patch != 0 && (r < 1 || r > patch * patch)) return 0;
    // the split-K factors, hence the size, depend on the device's compute-unit count: use the
    // current device's if there is one, else that of an MI355X
    int cus = 256, dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        cus = v;
    else
        (void)hipGetLastError();
    // the plan of a call depends on the selection (fusable or not, pooled or not) and on whether
    // both gradients are requested: report the largest
    size_t total = 0;
    for (int v = 0; v < 24; ++v) {
        for (int join = 0; join <= 8; ++join) {      // (0: the planner's choice; 1..8: what LBP_GX_JOIN can force)
            lbp::WorkspacePlan ws;
            if (lbp::plan_workspace(shape, patch, r, cus, (v & 1) != 0, false, &ws, (v & 2) != 0, (v & 4) != 0, extra,
                                    v >> 3, join) != LBP_OK)
                return 0;
            if (ws.total > total) total = ws.total;
            if (patch == 0) break;
        }
        if (patch == 0) break;
    }
    if (patch == 0 && shape->dtype == LBP_BF16)   // staging of gx for the plain cross-check kernels
        total += ((size_t)shape->N * ((size_t)shape->H * shape->W + extra) * shape->Cin * 4 + 255) / 256 * 256;
    return total;
}

int lbp_set_workspace(void *dev_ptr, size_t bytes)
{
    if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255u)) return LBP_ERR_ALIGN;
    int dev;
    DeviceState *st;
    int rc = current_device(&dev, &st);
    if (rc) return rc;
    std::lock_guard<std::mutex> lock(g_mutex);
    st->user_ws = dev_ptr;
    st->user_bytes = dev_ptr ? bytes : 0;
    return LBP_OK;
}

int lbp_release_workspace(void)
{
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess) {
        (void)hipGetLastError();
        return LBP_OK;   // no device: nothing was ever allocated
    }
    int prev = 0;
    LBP_HIP(hipGetDevice(&prev));
    std::lock_guard<std::mutex> lock(g_mutex);
    for (int d = 0; d < count && d < kMaxDevices; ++d) {
        if (!g_dev[d].internal_ws) continue;
        LBP_HIP(hipSetDevice(d));
        LBP_HIP(hipDeviceSynchronize());
        LBP_HIP(hipFree(g_dev[d].internal_ws));
        g_dev[d].internal_ws = nullptr;
        g_dev[d].internal_bytes = 0;
    }
    LBP_HIP(hipSetDevice(prev));
    return LBP_OK;
}

int lbp_wht_project(const void *in, int N, int H, int W, int C, int dtype, int patch,
                    const int32_t *basis_idx, int r, void *out, void *stream)
{
    return lbp_wht_project_tokens(in, N, H, W, 0, C, dtype, patch, basis_idx, r, out, stream);
}

int lbp_wht_project_tokens(const void *in, int N, int H, int W, int extra, int C, int dtype, int patch,
                           const int32_t *basis_idx, int r, void *out, void *stream)
{
    if (!in || !out || !basis_idx) return LBP_ERR_NULL;
    int rc = lbp::validate_grid(N, H, W, C, dtype, patch);
    if (rc) return rc;
    if (extra < 0 || (long)N * ((long)H * W + extra) > 0x7fffffffL) return LBP_ERR_SHAPE;
    lbp::BasisPlan plan;
    rc = lbp::make_basis_plan(patch, basis_idx, r, &plan);
    if (rc) return rc;
    const void *ptrs[2] = {in, out};
    rc = lbp::validate_alignment(ptrs, 2);
    if (rc) return rc;
    size_t esz = lbp::dtype_size(dtype);
    size_t M = (size_t)N * ((size_t)H * W + extra);
    const size_t Mq = (size_t)lbp::patch_count(N, H, W, patch) * r;
    if (lbp::ranges_overlap(in, M * C * esz, out, (Mq + (size_t)N * extra) * C * esz)) return LBP_ERR_ALIAS;
    int dev;
    DeviceState *st;
    rc = current_device(&dev, &st);
    if (rc) return rc;
    LBP_HIP(lbp::launch_project(in, out, N, H, W, C, dtype, plan, wht_path_option(), (hipStream_t)stream, extra,
                                1.0f));
    return LBP_OK;
}

int lbp_wht_project_pair(const void *x, const void *gy, const lbp_shape_t *shape, int patch,
                         const int32_t *basis_idx, int r, void *x_r, void *gy_r, void *stream)
{
    return lbp_wht_project_pair_tokens(x, gy, shape, 0, patch, basis_idx, r, x_r, gy_r, stream);
}

int lbp_wht_project_pair_tokens(const void *x, const void *gy, const lbp_shape_t *shape, int extra, int patch,
                                const int32_t *basis_idx, int r, void *x_r, void *gy_r, void *stream)
{
    if (!x || !gy || !x_r || !gy_r || !basis_idx || !shape) return LBP_ERR_NULL;
    int rc = lbp::validate_shape(shape, patch);
    if (rc) return rc;
    if (lbp::patch_log2(patch) < 0) return LBP_ERR_PATCH;
    if (!tokens_ok(shape, extra)) return LBP_ERR_SHAPE;
    lbp::BasisPlan plan;
    rc = lbp::make_basis_plan(patch, basis_idx, r, &plan);
    if (rc) return rc;
    const void *ptrs[4] = {x, gy, x_r, gy_r};
    rc = lbp::validate_alignment(ptrs, 4);
    if (rc) return rc;
    const size_t esz = lbp::dtype_size(shape->dtype);
    const size_t M = (size_t)shape->N * ((size_t)shape->H * shape->W + extra);
    const size_t Mr = (size_t)lbp::patch_count(shape->N, shape->H, shape->W, patch) * r + (size_t)shape->N * extra;
    const void *bufs[4] = {x, gy, x_r, gy_r};
    const size_t bytes[4] = {M * shape->Cin * esz, M * shape->Cout * esz, Mr * shape->Cin * esz,
                             Mr * shape->Cout * esz};
    for (int i = 2; i < 4; ++i)
        for (int j = 0; j < i; ++j)
            if (lbp::ranges_overlap(bufs[i], bytes[i], bufs[j], bytes[j])) return LBP_ERR_ALIAS;
    int dev;
    DeviceState *st;
    rc = current_device(&dev, &st);
    if (rc) return rc;
    // tokens outside the grid follow the coefficient rows: x's as they are, g_y's times patch^2 (exact),
    // which the 1/patch^2 of both products takes away again
    LBP_HIP(lbp::launch_project_pair(gy, gy_r, shape->Cout, x, x_r, shape->Cin, shape->N, shape->H, shape->W,
                                     shape->dtype, plan, wht_path_option(), (hipStream_t)stream, extra,
                                     (float)(patch * patch), 1.0f));
    return LBP_OK;
}

int lbp_wht_select_lhe(const double *energy, int patch, int r, int32_t *basis_idx)
{
    return lbp::select_lhe(energy, patch, r, basis_idx);
}

size_t lbp_wht_energy_workspace_bytes(int N, int H, int W, int C, int dtype, int patch)
{
    if (lbp::validate_grid(N, H, W, C, dtype, patch) != LBP_OK || patch == 0) return 0;
    const long Q = lbp::patch_count(N, H, W, patch);
    size_t coef = ((size_t)Q * patch * patch * C * lbp::dtype_size(dtype) + 255) / 256 * 256;
    return coef + (size_t)patch * patch * lbp::energy_chunks(Q) * sizeof(double);
}

int lbp_wht_energy(const void *in, int N, int H, int W, int C, int dtype, int patch, double *energy,
                   void *stream)
{
    return lbp_wht_energy_tokens(in, N, H, W, 0, C, dtype, patch, energy, stream);
}

int lbp_wht_energy_tokens(const void *in, int N, int H, int W, int extra, int C, int dtype, int patch,
                          double *energy, void *stream)
{
    if (!in || !energy) return LBP_ERR_NULL;
    if (lbp::patch_log2(patch) < 0) return LBP_ERR_PATCH;
    int rc = lbp::validate_grid(N, H, W, C, dtype, patch);
    if (rc) return rc;
    if (extra < 0 || (long)N * ((long)H * W + extra) > 0x7fffffffL) return LBP_ERR_SHAPE;
    const void *ptrs[2] = {in, energy};
    rc = lbp::validate_alignment(ptrs, 2);
    if (rc) return rc;
    const int pp = patch * patch;
    int32_t all[lbp::kMaxBases];
    for (int j = 0; j < pp; ++j) all[j] = j;
    lbp::BasisPlan plan;
    rc = lbp::make_basis_plan(patch, all, pp, &plan);
    if (rc) return rc;
    int dev;
    DeviceState *st;
    rc = current_device(&dev, &st);
    if (rc) return rc;
    char *base = nullptr;
    rc = get_workspace(st, lbp_wht_energy_workspace_bytes(N, H, W, C, dtype, patch), &base);
    if (rc) return rc;
    const long Q = lbp::patch_count(N, H, W, patch);
    const size_t coef_bytes = ((size_t)Q * pp * C * lbp::dtype_size(dtype) + 255) / 256 * 256;
    hipStream_t s = (hipStream_t)stream;
    // all p^2 coefficients of every patch (row q*p^2 + j = basis j in sequency order), then their squares
    // (tokens outside the grid have no coefficients: they are skipped)
    LBP_HIP(lbp::launch_project(in, base, N, H, W, C, dtype, plan, wht_path_option(), s, extra, 0.0f));
    LBP_HIP(lbp::launch_energy(base, Q, pp, C, dtype, (double *)(base + coef_bytes), energy, s));
    return LBP_OK;
}

int lbp_wht_unproject(const void *in, int N, int H, int W, int C, int dtype, int patch,
                      const int32_t *basis_idx, int r, void *out, void *stream)
{
    if (!in || !out || !basis_idx) return LBP_ERR_NULL;
    int rc = lbp::validate_grid(N, H, W, C, dtype, patch);
    if (rc) return rc;
    lbp::BasisPlan plan;
    rc = lbp::make_basis_plan(patch, basis_idx, r, &plan);
    if (rc) return rc;
    const void *ptrs[2] = {in, out};
    rc = lbp::validate_alignment(ptrs, 2);
    if (rc) return rc;
    size_t M = (size_t)N * H * W;
    if (lbp::ranges_overlap(in, (size_t)lbp::patch_count(N, H, W, patch) * r * C * 4, out, M * C * lbp::dtype_size(dtype)))
        return LBP_ERR_ALIAS;
    int dev;
    DeviceState *st;
    rc = current_device(&dev, &st);
    if (rc) return rc;
    LBP_HIP(lbp::launch_unproject((const float *)in, 1, out, N, H, W, C, dtype, plan, wht_path_option(),
                                  (hipStream_t)stream));
    return LBP_OK;
}

}  // extern "C"

namespace {

// Algorithm 1.  `ev`, when not NULL, holds 4 events recorded on the stream before the projection,
// after it, after the weight-gradient product and after the input-gradient product.
// x_projected: `x` already is x^ = WHT(x; I), [P*r][Cin], kept from the forward pass.
// gy_projected: `gy` already is g^y = WHT(gy; I) too (only with x_projected): the products alone.
int backward_impl(const void *x, const void *gy, const void *W, const lbp_shape_t *shape, int patch,
                  const int32_t *basis_idx, int r, void *gx, void *gW, void *stream, hipEvent_t *ev,
                  bool x_projected = false, int extra = 0, bool gy_projected = false, bool static_scratch = false)
{
    if (!shape || !basis_idx) return LBP_ERR_NULL;
    if (lbp::patch_log2(patch) < 0) return LBP_ERR_PATCH;
    int rc = lbp::validate_shape(shape, patch);
    if (rc) return rc;
    if (!tokens_ok(shape, extra)) return LBP_ERR_SHAPE;
    lbp::BasisPlan plan;
    rc = lbp::make_basis_plan(patch, basis_idx, r, &plan);
    if (rc) return rc;
    // rows of the projected tensors: (patch, basis) pairs first, then the tokens outside the grid
    const long Mq = lbp::patch_count(shape->N, shape->H, shape->W, patch) * r;
    const long Mr = Mq + (long)shape->N * extra;
    if (gy_projected && !x_projected) return LBP_ERR_SHAPE;
    rc = validate_buffers(x, gy, W, shape, gx, gW, x_projected ? (size_t)Mr : 0, extra, gy_projected ? (size_t)Mr : 0);
    if (rc) return rc;

    int dev;
    DeviceState *st;
    rc = current_device(&dev, &st);
    if (rc) return rc;
    const lbp::GemmPath gpath = gemm_path_option();
    lbp::WorkspacePlan ws;
    // both gradients wanted: the two products may share one launch (not when timed stage by stage)
    rc = plan_call(shape, extra, patch, r, plan, st->num_cus, gx && gW && !ev, &ws);
    if (rc) return rc;
    char *base = nullptr;
    if (static_scratch) {       // no allocation on this path: the fixed array or an error
        if (ws.total > kStaticScratchBytes) return LBP_ERR_WORKSPACE;
        base = st->static_ws;
    } else {
        rc = get_workspace(st, ws.total, &base);
        if (rc) return rc;
    }

    hipStream_t s = (hipStream_t)stream;
    const lbp::WhtPath path = wht_path_option();
    const int N = shape->N, H = shape->H, Wd = shape->W, Cin = shape->Cin, Cout = shape->Cout;
    const int dt = shape->dtype;
    const long img_tokens = (long)H * Wd + extra;
    const float inv_pp = 1.0f / (float)(patch * patch);
    const void *gy_r = gy_projected ? gy : base + ws.gy_r;
    const void *x_r = x_projected ? x : base + ws.x_r;
    float *gx_r = (float *)(base + ws.gx_r);
    float *part = (float *)(base + ws.splitk);

    if (ev) LBP_HIP(hipEventRecord(ev[0], s));
    // g^y = WHT(gy; I) is needed by both products; x^ = WHT(x; I) only by the weight gradient
    // (first two statements of Algorithm 1).  One launch covers both tensors.
    // Tokens outside the grid join the projected tensors as they are (Eq. 2 stays exact for them);
    // their g_y rows carry patch^2, a power of two, which the 1/patch^2 of both products takes away.
    const float pp = (float)(patch * patch);
    if (gy_projected)
        ;   // both projections were done by the caller
    else if (gW && !x_projected)
        LBP_HIP(lbp::launch_project_pair(gy, base + ws.gy_r, Cout, x, base + ws.x_r, Cin, N, H, Wd, dt, plan, path, s,
                                         extra, pp, 1.0f));
    else
        LBP_HIP(lbp::launch_project(gy, base + ws.gy_r, N, H, Wd, Cout, dt, plan, path, s, extra, pp));
    if (ev) LBP_HIP(hipEventRecord(ev[1], s));
    // g~w = g^w = g^y^T x^  (with the 1/p^2 of the normalisation)
    lbp::GemmArgs gw_args, g;
    bool gw_reduce = false;
    if (gW)
        gw_reduce = weight_gradient_args(gy_r, x_r, Cout, Cin, Mr, dt, shape->gw_dtype, ws.gw, inv_pp, part, gW,
                                         gpath, &gw_args);
    if (gx) {
        // g^x = g^y w, then g~x = WHT^-1(g^x; I): fused into the product's epilogue when the
        // kernel supports the selection, else through an fp32 buffer and a kernel of its own
        g.A = gy_r; g.B = W;
        g.M = (int)Mr; g.N = Cin; g.K = Cout;
        g.lda = Cout; g.ldb = Cin;
        g.a_kfast = true;
        g.dtype = dt;
        g.tile = ws.gx.tile;
        if (ws.gx_fused) {
            g.splits = 1;
            g.out = lbp::GemmOut::kUnproject;
            g.C = gx;
            g.grid_h = H; g.grid_w = Wd;
            g.plan = &plan;
            g.extra = extra;
            g.extra_rows = N * extra;
            if (ws.gx_join > 1) {       // slices that combine inside the launch
                g.splits = ws.gx_join;
                g.join_parts = gx_r;
                g.join_bytes = ws.gx_join_bytes;
                const bool ok = ws.grouped && gW ? lbp::gemm_pair_supported(g, gw_args, gpath) : lbp::gemm_join_supported(g, gpath);
                if (!ok) {     // (the planner only asks where the kernels exist)
                    g.splits = 1;
                    g.join_parts = nullptr;
                    g.join_bytes = 0;
                }
            }
        } else if (ws.gx_coef16) {
            g.splits = 1;
            g.out = lbp::GemmOut::kBF16;
            g.C = gx_r;
        } else {
            g.splits = ws.gx.splits;
            g.out = lbp::GemmOut::kF32;
            g.C = gx_r;
        }
    }
    // The two products are independent: one launch for both where a grouped kernel exists (not
    // when the stages are timed one by one).
    const bool grouped = ws.grouped && gW && gx && lbp::gemm_pair_supported(g, gw_args, gpath);
    if (grouped)
        LBP_HIP(lbp::launch_gemm_pair(g, gw_args, s));
    else if (gW)
        LBP_HIP(lbp::launch_gemm(gw_args, gpath, s));
    if (gW && gw_reduce)
        LBP_HIP(lbp::launch_splitk_reduce(part, ws.gw.splits, (long)Cout * Cin, inv_pp, gW, shape->gw_dtype, s));
    if (ev) LBP_HIP(hipEventRecord(ev[2], s));
    if (gx) {
        if (!grouped) LBP_HIP(lbp::launch_gemm(g, gpath, s));
        if (!ws.gx_fused && ws.gx_coef16) {
            LBP_HIP(lbp::launch_unproject_bf16(gx_r, gx, N, H, Wd, Cin, plan, s, extra));
        } else if (!ws.gx_fused) {
            LBP_HIP(lbp::launch_unproject(gx_r, ws.gx.splits, gx, N, H, Wd, Cin, dt, plan, path, s, extra, Mr));
            LBP_HIP(lbp::launch_scatter_extra(gx_r + (size_t)Mq * Cin, ws.gx.splits, (size_t)Mr * Cin, gx, N, extra,
                                              img_tokens, Cin, dt, inv_pp, s));
        }
    }
    if (ev) LBP_HIP(hipEventRecord(ev[3], s));
    return LBP_OK;
}

}  // namespace

extern "C" {

int lbp_wht_backward(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                     int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream)
{
    return backward_impl(x, gy, W, shape, patch, basis_idx, r, gx, gW, stream, nullptr);
}

int lbp_wht_backward_static(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                            int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream)
{
    return backward_impl(x, gy, W, shape, patch, basis_idx, r, gx, gW, stream, nullptr, false, 0, false, true);
}

int lbp_wht_backward_preprojected(const void *x_r, const void *gy, const void *W,
                                  const lbp_shape_t *shape, int patch, const int32_t *basis_idx, int r,
                                  void *gx, void *gW, void *stream)
{
    return backward_impl(x_r, gy, W, shape, patch, basis_idx, r, gx, gW, stream, nullptr, true);
}

int lbp_wht_describe_plan(const lbp_shape_t *shape, int extra, int patch, const int32_t *basis_idx, int r,
                          int want_gx, int want_gw, int num_cus, char *buf, size_t len)
{
    if (!shape || !basis_idx || !buf || len == 0) return LBP_ERR_NULL;
    buf[0] = 0;
    if (lbp::patch_log2(patch) < 0) return LBP_ERR_PATCH;
    int rc = lbp::validate_shape(shape, patch);
    if (rc) return rc;
    if (!tokens_ok(shape, extra)) return LBP_ERR_SHAPE;
    if (!want_gx && !want_gw) return LBP_ERR_NULL;
    lbp::BasisPlan plan;
    rc = lbp::make_basis_plan(patch, basis_idx, r, &plan);
    if (rc) return rc;
    if (num_cus <= 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            num_cus = v;
        else
            (void)hipGetLastError();
        if (num_cus <= 0) num_cus = 256;
    }
    lbp::WorkspacePlan ws;
    rc = plan_call(shape, extra, patch, r, plan, num_cus, want_gx && want_gw, &ws);
    if (rc) return rc;
    const bool mfma = shape->dtype == LBP_BF16 && gemm_path_option() != lbp::GemmPath::kSimple;
    const lbp::WhtPath path = wht_path_option();
    const int pooled = (patch >> plan.mh) * (patch >> plan.mw);
    char gw[160] = "", gxs[200] = "";
    if (want_gw)
        std::snprintf(gw, sizeof gw, "gW: tile %s, split-K %d%s; ", mfma ? lbp::kGemmTiles[ws.gw.tile].name : "fp32 64x64",
                      ws.gw.splits, ws.gw.splits > 1 ? " + reduction kernel" : "");
    if (want_gx) {
        if (ws.gx_fused)
            std::snprintf(gxs, sizeof gxs, "gx: tile %s, reverse projection fused (%s epilogue)%s%.0d%s; ",
                          lbp::kGemmTiles[ws.gx.tile].name, lbp::gemm_unproject_pooled(plan) ? "pooled" : "matrix-core",
                          ws.gx_join > 1 ? ", reduction in " : "", ws.gx_join > 1 ? ws.gx_join : 0,
                          ws.gx_join > 1 ? " slices joined in the launch" : "");
        else if (ws.gx_coef16)
            std::snprintf(gxs, sizeof gxs, "gx: tile %s, bf16 coefficients + %s reverse-projection kernel; ",
                          lbp::kGemmTiles[ws.gx.tile].name,
                          lbp::projection_kernel_name(plan, path, shape->dtype, shape->Cin));
        else
            std::snprintf(gxs, sizeof gxs, "gx: tile %s, split-K %d + %s reverse-projection kernel; ",
                          mfma ? lbp::kGemmTiles[ws.gx.tile].name : "fp32 64x64", ws.gx.splits,
                          lbp::projection_kernel_name(plan, path, shape->dtype, shape->Cin));
    }
    std::snprintf(buf, len, "projection: %s kernel (%d of %d coefficients per patch after pooling); products: %s; %s%sworkspace %zu bytes",
                  lbp::projection_kernel_name(plan, path, shape->dtype, shape->Cout), pooled, patch * patch,
                  ws.grouped ? "one grouped launch" : "separate launches", gw, gxs, ws.total);
    return LBP_OK;
}

int lbp_wht_products(const void *x_r, const void *gy_r, const void *W, const lbp_shape_t *shape, int patch,
                     const int32_t *basis_idx, int r, void *gx, void *gW, void *stream)
{
    return backward_impl(x_r, gy_r, W, shape, patch, basis_idx, r, gx, gW, stream, nullptr, true, 0, true);
}

int lbp_wht_products_tokens(const void *x_r, const void *gy_r, const void *W, const lbp_shape_t *shape, int extra,
                            int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream)
{
    return backward_impl(x_r, gy_r, W, shape, patch, basis_idx, r, gx, gW, stream, nullptr, true, extra, true);
}

int lbp_wht_backward_tokens(const void *x, const void *gy, const void *W, const lbp_shape_t *shape, int extra,
                            int patch, const int32_t *basis_idx, int r, void *gx, void *gW, void *stream)
{
    return backward_impl(x, gy, W, shape, patch, basis_idx, r, gx, gW, stream, nullptr, false, extra);
}

int lbp_wht_backward_tokens_preprojected(const void *x_r, const void *gy, const void *W, const lbp_shape_t *shape,
                                         int extra, int patch, const int32_t *basis_idx, int r, void *gx, void *gW,
                                         void *stream)
{
    return backward_impl(x_r, gy, W, shape, patch, basis_idx, r, gx, gW, stream, nullptr, true, extra);
}

int lbp_wht_backward_profile(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                             int patch, const int32_t *basis_idx, int r, void *gx, void *gW,
                             void *stream, float *stage_ms)
{
    if (!stage_ms) return LBP_ERR_NULL;
    hipEvent_t ev[4] = {nullptr, nullptr, nullptr, nullptr};
    int rc = LBP_OK;
    for (int i = 0; i < 4 && rc == LBP_OK; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) rc = hip_fail(hipGetLastError());
    if (rc == LBP_OK) rc = backward_impl(x, gy, W, shape, patch, basis_idx, r, gx, gW, stream, ev);
    if (rc == LBP_OK) {
        hipError_t e = hipEventSynchronize(ev[3]);
        for (int i = 0; i < 3 && e == hipSuccess; ++i) e = hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]);
        if (e != hipSuccess) rc = hip_fail(e);
    }
    for (int i = 0; i < 4; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    return rc;
}

int full_bp_backward(const void *x, const void *gy, const void *W, const lbp_shape_t *shape,
                     void *gx, void *gW, void *stream)
{
    if (!shape) return LBP_ERR_NULL;
    int rc = lbp::validate_shape(shape, 0);
    if (rc) return rc;
    rc = validate_buffers(x, gy, W, shape, gx, gW);
    if (rc) return rc;
    int dev;
    DeviceState *st;
    rc = current_device(&dev, &st);
    if (rc) return rc;
    const int Cin = shape->Cin, Cout = shape->Cout, dt = shape->dtype;
    const long M = (long)shape->N * shape->H * shape->W;
    lbp::WorkspacePlan ws;
    rc = lbp::plan_workspace(shape, 0, 0, st->num_cus, false, false, &ws);
    if (rc) return rc;
    // the plain bf16 kernel needs an fp32 staging buffer of M x Cin for gx
    size_t gx_stage = gx && dt == LBP_BF16 && gemm_path_option() == lbp::GemmPath::kSimple
                          ? ((size_t)M * Cin * 4 + 255) / 256 * 256 : 0;
    char *base = nullptr;
    rc = get_workspace(st, ws.total + gx_stage, &base);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    float *part = (float *)(base + ws.splitk);

    const lbp::GemmPath gpath = gemm_path_option();
    if (gW) {   // gW = gy^T x  (Eq. 2)
        rc = weight_gradient(gy, x, Cout, Cin, M, dt, shape->gw_dtype, ws.gw, 1.0f, part, gW, gpath, s);
        if (rc) return rc;
    }
    if (gx) {   // gx = gy W  (Eq. 2)
        lbp::GemmArgs g;
        g.A = gy; g.B = W;
        g.M = (int)M; g.N = Cin; g.K = Cout;
        g.lda = Cout; g.ldb = Cin;
        g.a_kfast = true;
        g.dtype = dt;
        g.splits = 1;
        if (dt == LBP_F32) {
            g.out = lbp::GemmOut::kF32;
            g.C = gx;
            LBP_HIP(lbp::launch_gemm(g, gpath, s));
        } else if (gpath != lbp::GemmPath::kSimple) {
            g.tile = ws.gx.tile;
            g.out = lbp::GemmOut::kBF16;
            g.C = gx;
            LBP_HIP(lbp::launch_gemm(g, gpath, s));
        } else {
            // the plain bf16 kernel only stores fp32: stage and convert
            float *stage = (float *)(base + ws.total);
            g.out = lbp::GemmOut::kF32;
            g.C = stage;
            LBP_HIP(lbp::launch_gemm(g, gpath, s));
            LBP_HIP(lbp::launch_splitk_reduce(stage, 1, M * Cin, 1.0f, gx, LBP_BF16, s));
        }
    }
    return LBP_OK;
}

}  // extern "C"
