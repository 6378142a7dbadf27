/*
 * CPU oracle for LBP-WHT (low-rank backpropagation through one linear layer with
 * Walsh-Hadamard projections).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what the
 * method computes, used only to check the GPU library and as the timed CPU
 * baseline of the benchmark.  It shares no code with the GPU library and the GPU
 * library never calls it.
 *
 * Everything is double precision, explicit matrices and plain loops:
 *   - Sylvester construction of the Hadamard matrix, rows re-ordered by their
 *     number of sign changes (sequency), because the paper indexes bases so
 *     that a smaller index is a lower frequency (Section 3.2, Figure 2c caption).
 *   - Low-pass selection LP_L1 / LP_Linf (Section 3.2, Eq. 8 and 9).
 *   - Projection p(.) and reverse projection p^-1(.) in the matrix form of
 *     Eq. 6 and Eq. 7, applied per p x p patch of the token grid.
 *   - Algorithm 1: x^ = p(x), g^y = p(gy), g^w = g^y^T x^, g^x = g^y w,
 *     g~x = p^-1(g^x), g~w = g^w.
 *   - Exact backward of Eq. 2 for comparison.
 *
 * Readings of the paper taken here (the paper is silent or inconsistent):
 *   - token-major matrices: X[M][Cin], GY[M][Cout], W[Cout][Cin];
 *     gx = GY W, gW = GY^T X  (Eq. 1-2 as printed do not type-check).
 *   - B^T B = p^2 I, so Eq. 6 followed by Eq. 7 scales by p^2.  The forward
 *     projection is left unnormalised and 1/p^2 is applied once to gW and once
 *     to gx, which makes "all bases kept" reproduce exact backpropagation.
 *   - indices are 0-based sequency pairs (u along the grid's H axis, v along its
 *     W axis), basis_idx = u*p + v; LP_L1-k keeps u+v <= k-1 (this gives the
 *     k(k+1)/2 bases the paper's tables list), LP_Linf-k keeps max(u,v) <= k-1.
 *   - ranks between two shells: total orders
 *        LP_L1   sort key (u+v, max(u,v), u)
 *        LP_Linf sort key (max(u,v), u+v, u)
 *     and the first r pairs are kept (not fixed by the paper: parity unpinned
 *     for non-triangular / non-square r beyond the lists printed in the tests).
 *   - the H x W token grid of every image is tiled into non-overlapping p x p
 *     patches; the paper's formulas hold per patch; gW sums over patches and
 *     over the batch.
 *
 * All functions return 0 on success and a negative number on a bad argument.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

static int is_pow2(int p) { return p > 0 && (p & (p - 1)) == 0; }

/* Sylvester construction: H_1 = [1], H_2m = [[H_m, H_m], [H_m, -H_m]].  Had is p x p. */
int oracle_sylvester(int p, int8_t *Had)
{
    if (!is_pow2(p) || !Had) return -1;
    Had[0] = 1;
    for (int m = 1; m < p; m *= 2) {
        /* grow the m x m block in the top-left corner to 2m x 2m, in place (stride p) */
        for (int i = 0; i < m; ++i)
            for (int j = 0; j < m; ++j) {
                int8_t v = Had[i * p + j];
                Had[i * p + (j + m)] = v;
                Had[(i + m) * p + j] = v;
                Had[(i + m) * p + (j + m)] = (int8_t)-v;
            }
    }
    return 0;
}

/* Walsh (sequency) ordering: Wal[s] is the Sylvester row with exactly s sign changes. */
int oracle_walsh(int p, int8_t *Wal)
{
    if (!is_pow2(p) || !Wal) return -1;
    int8_t *Had = (int8_t *)malloc((size_t)p * p);
    int *seen = (int *)calloc((size_t)p, sizeof(int));
    if (!Had || !seen) { free(Had); free(seen); return -2; }
    oracle_sylvester(p, Had);
    int rc = 0;
    for (int i = 0; i < p; ++i) {
        int changes = 0;
        for (int j = 1; j < p; ++j)
            if (Had[i * p + j] != Had[i * p + j - 1]) ++changes;
        if (seen[changes]) rc = -3;          /* must be a permutation of 0..p-1 */
        seen[changes] = 1;
        memcpy(Wal + (size_t)changes * p, Had + (size_t)i * p, (size_t)p);
    }
    free(Had);
    free(seen);
    return rc;
}

/* Low-pass selection (Section 3.2).  order 0 = LP_L1, 1 = LP_Linf.  idx[k] = u*p + v. */
int oracle_select_bases(int p, int r, int order, int32_t *idx)
{
    if (!is_pow2(p) || r < 1 || r > p * p || (order != 0 && order != 1) || !idx) return -1;
    int n = p * p;
    int (*key)[4] = (int (*)[4])malloc((size_t)n * sizeof(int[4]));
    if (!key) return -2;
    for (int u = 0; u < p; ++u)
        for (int v = 0; v < p; ++v) {
            int l1 = u + v, linf = u > v ? u : v;
            int *e = key[u * p + v];
            e[0] = order == 0 ? l1 : linf;
            e[1] = order == 0 ? linf : l1;
            e[2] = u;
            e[3] = u * p + v;
        }
    /* insertion sort, lexicographic on the three key fields */
    for (int i = 1; i < n; ++i) {
        int cur[4];
        memcpy(cur, key[i], sizeof cur);
        int j = i - 1;
        while (j >= 0) {
            int *e = key[j];
            int gt = e[0] != cur[0] ? e[0] > cur[0] : e[1] != cur[1] ? e[1] > cur[1] : e[2] > cur[2];
            if (!gt) break;
            memcpy(key[j + 1], key[j], sizeof cur);
            --j;
        }
        memcpy(key[j + 1], cur, sizeof cur);
    }
    for (int k = 0; k < r; ++k) idx[k] = key[k][3];
    free(key);
    return 0;
}

static int check_idx(int p, int r, const int32_t *idx)
{
    if (!is_pow2(p) || r < 1 || r > p * p || !idx) return -1;
    for (int k = 0; k < r; ++k) {
        if (idx[k] < 0 || idx[k] >= p * p) return -1;
        for (int j = 0; j < k; ++j)
            if (idx[j] == idx[k]) return -1;
    }
    return 0;
}

/* Flattened 2-D bases as the columns of B (p^2 x r, row-major):
 * B[(h*p + w)*r + k] = Wal[u_k][h] * Wal[v_k][w]   (Eq. 6, the matrix (B_i1j1 ... B_irjr)). */
int oracle_basis_matrix(int p, int r, const int32_t *idx, int8_t *B)
{
    if (check_idx(p, r, idx) || !B) return -1;
    int8_t *Wal = (int8_t *)malloc((size_t)p * p);
    if (!Wal) return -2;
    int rc = oracle_walsh(p, Wal);
    for (int h = 0; h < p && !rc; ++h)
        for (int w = 0; w < p; ++w)
            for (int k = 0; k < r; ++k) {
                int u = idx[k] / p, v = idx[k] % p;
                B[(size_t)(h * p + w) * r + k] = (int8_t)(Wal[u * p + h] * Wal[v * p + w]);
            }
    free(Wal);
    return rc;
}

static int check_grid(int N, int H, int W, int C, int p)
{
    if (N < 1 || H < 1 || W < 1 || C < 1 || !is_pow2(p)) return -1;
    if (H % p || W % p) return -1;
    return 0;
}

/* token index (row of the M x C matrix) of position (h, w) inside patch (n, a, b) */
static inline size_t token_of(int n, int a, int b, int h, int w, int H, int W, int p)
{
    return ((size_t)n * H + (size_t)a * p + h) * W + (size_t)b * p + w;
}

/* p(.) of Eq. 6 per patch: Xr[(q*r + k)*C + c] = sum_t B[t][k] * X[token(q,t)][c],
 * q = (n*(H/p) + a)*(W/p) + b.  No normalisation. */
int oracle_project(const double *X, int N, int H, int W, int C, int p, int r,
                   const int32_t *idx, double *Xr)
{
    if (!X || !Xr || check_grid(N, H, W, C, p) || check_idx(p, r, idx)) return -1;
    int pp = p * p, PH = H / p, PW = W / p;
    int8_t *B = (int8_t *)malloc((size_t)pp * r);
    if (!B) return -2;
    oracle_basis_matrix(p, r, idx, B);
    long Q = (long)N * PH * PW;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < Q; ++q) {
        int b = (int)(q % PW), a = (int)((q / PW) % PH), n = (int)(q / ((long)PW * PH));
        for (int k = 0; k < r; ++k) {
            double *out = Xr + ((size_t)q * r + k) * C;
            for (int c = 0; c < C; ++c) out[c] = 0.0;
            for (int h = 0; h < p; ++h)
                for (int w = 0; w < p; ++w) {
                    const double *in = X + token_of(n, a, b, h, w, H, W, p) * C;
                    double s = (double)B[(size_t)(h * p + w) * r + k];
                    for (int c = 0; c < C; ++c) out[c] += s * in[c];
                }
        }
    }
    free(B);
    return 0;
}

/* p^-1(.) of Eq. 7 per patch with the 1/p^2 that makes it invert p(.) on span(B):
 * X[token(q,t)][c] = (1/p^2) * sum_k B[t][k] * Xr[(q*r + k)*C + c]. */
int oracle_unproject(const double *Xr, int N, int H, int W, int C, int p, int r,
                     const int32_t *idx, double *X)
{
    if (!X || !Xr || check_grid(N, H, W, C, p) || check_idx(p, r, idx)) return -1;
    int pp = p * p, PH = H / p, PW = W / p;
    int8_t *B = (int8_t *)malloc((size_t)pp * r);
    if (!B) return -2;
    oracle_basis_matrix(p, r, idx, B);
    long Q = (long)N * PH * PW;
    double scale = 1.0 / (double)pp;
#pragma omp parallel for schedule(static)
    for (long q = 0; q < Q; ++q) {
        int b = (int)(q % PW), a = (int)((q / PW) % PH), n = (int)(q / ((long)PW * PH));
        for (int h = 0; h < p; ++h)
            for (int w = 0; w < p; ++w) {
                double *out = X + token_of(n, a, b, h, w, H, W, p) * C;
                for (int c = 0; c < C; ++c) out[c] = 0.0;
                for (int k = 0; k < r; ++k) {
                    const double *in = Xr + ((size_t)q * r + k) * C;
                    double s = (double)B[(size_t)(h * p + w) * r + k];
                    for (int c = 0; c < C; ++c) out[c] += s * in[c];
                }
                for (int c = 0; c < C; ++c) out[c] *= scale;
            }
    }
    free(B);
    return 0;
}

/* C[m][n] = sum_k A[m][k] * Bm[k][n]   (A is Mr x K, Bm is K x Nc, all row-major) */
static void matmul_nn(const double *A, const double *Bm, double *Cm, long Mr, long K, long Nc)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < Mr; ++m) {
        double *c = Cm + m * Nc;
        for (long n = 0; n < Nc; ++n) c[n] = 0.0;
        for (long k = 0; k < K; ++k) {
            double a = A[m * K + k];
            const double *brow = Bm + k * Nc;
            for (long n = 0; n < Nc; ++n) c[n] += a * brow[n];
        }
    }
}

/* C[m][n] = scale * sum_k A[k][m] * Bm[k][n]   (A is K x Mc, Bm is K x Nc) */
static void matmul_tn(const double *A, const double *Bm, double *Cm, long K, long Mc, long Nc,
                      double scale)
{
#pragma omp parallel for schedule(static)
    for (long m = 0; m < Mc; ++m) {
        double *c = Cm + m * Nc;
        for (long n = 0; n < Nc; ++n) c[n] = 0.0;
        for (long k = 0; k < K; ++k) {
            double a = A[k * Mc + m];
            const double *brow = Bm + k * Nc;
            for (long n = 0; n < Nc; ++n) c[n] += a * brow[n];
        }
        for (long n = 0; n < Nc; ++n) c[n] *= scale;
    }
}

/* Exact backward, Eq. 2 (token-major reading): gx = GY W, gW = GY^T X. */
int oracle_full_bp_backward(const double *x, const double *gy, const double *w,
                            int N, int H, int W, int Cin, int Cout, double *gx, double *gW)
{
    if (!x || !gy || !w || N < 1 || H < 1 || W < 1 || Cin < 1 || Cout < 1) return -1;
    long M = (long)N * H * W;
    if (gx) matmul_nn(gy, w, gx, M, Cout, Cin);
    if (gW) matmul_tn(gy, x, gW, M, Cout, Cin, 1.0);
    return 0;
}

/* Algorithm 1.  x, gy: [N][H][W][C] token-major; w: [Cout][Cin]; gx: [N][H][W][Cin];
 * gW: [Cout][Cin].  Either output may be NULL. */
int oracle_lbp_wht_backward(const double *x, const double *gy, const double *w,
                            int N, int H, int W, int Cin, int Cout, int p,
                            const int32_t *idx, int r, double *gx, double *gW)
{
    if (!x || !gy || !w || check_grid(N, H, W, Cin, p) || Cout < 1 || check_idx(p, r, idx))
        return -1;
    long Q = (long)N * (H / p) * (W / p), Mr = Q * r;
    double *xr = (double *)malloc((size_t)Mr * Cin * sizeof(double));
    double *gyr = (double *)malloc((size_t)Mr * Cout * sizeof(double));
    double *gxr = gx ? (double *)malloc((size_t)Mr * Cin * sizeof(double)) : NULL;
    int rc = (!xr || !gyr || (gx && !gxr)) ? -2 : 0;
    if (!rc) rc = oracle_project(x, N, H, W, Cin, p, r, idx, xr);          /* x^  = p(x)      */
    if (!rc) rc = oracle_project(gy, N, H, W, Cout, p, r, idx, gyr);       /* g^y = p(gy)     */
    if (!rc && gW) matmul_tn(gyr, xr, gW, Mr, Cout, Cin, 1.0 / (p * p));   /* g^w = g^y^T x^  */
    if (!rc && gx) {
        matmul_nn(gyr, w, gxr, Mr, Cout, Cin);                             /* g^x = g^y w     */
        rc = oracle_unproject(gxr, N, H, W, Cin, p, r, idx, gx);           /* g~x = p^-1(g^x) */
    }
    free(xr);
    free(gyr);
    free(gxr);
    return rc;
}

/* ---- the same results one output at a time, for spot checks at sizes where the whole
 * oracle would take too long.  Same formulas, evaluated only where asked. ---- */

/* rows of g~x for the listed tokens (token = (n*H + h)*W + w): out[i][0..Cin) */
int oracle_lbp_gx_tokens(const double *gy, const double *w, int N, int H, int W, int Cin,
                         int Cout, int p, const int32_t *idx, int r,
                         const int64_t *tokens, int ntok, double *out)
{
    if (!gy || !w || !tokens || !out || ntok < 0 || check_grid(N, H, W, Cin, p) || Cout < 1 ||
        check_idx(p, r, idx))
        return -1;
    int pp = p * p;
    int8_t *B = (int8_t *)malloc((size_t)pp * r);
    if (!B) return -2;
    oracle_basis_matrix(p, r, idx, B);
    long M = (long)N * H * W;
    for (int i = 0; i < ntok; ++i)
        if (tokens[i] < 0 || tokens[i] >= M) { free(B); return -1; }
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < ntok; ++i) {
        long tok = (long)tokens[i];
        int wq = (int)(tok % W), hq = (int)((tok / W) % H), n = (int)(tok / ((long)W * H));
        int a = hq / p, b = wq / p, t = (hq % p) * p + (wq % p);
        double *gyr = (double *)calloc((size_t)r * Cout, sizeof(double));
        double *gxr = (double *)calloc((size_t)r * Cin, sizeof(double));
        for (int k = 0; k < r; ++k)
            for (int h = 0; h < p; ++h)
                for (int ww = 0; ww < p; ++ww) {
                    const double *in = gy + token_of(n, a, b, h, ww, H, W, p) * Cout;
                    double s = (double)B[(size_t)(h * p + ww) * r + k];
                    for (int c = 0; c < Cout; ++c) gyr[(size_t)k * Cout + c] += s * in[c];
                }
        for (int k = 0; k < r; ++k)
            for (int co = 0; co < Cout; ++co) {
                double g = gyr[(size_t)k * Cout + co];
                for (int ci = 0; ci < Cin; ++ci) gxr[(size_t)k * Cin + ci] += g * w[(size_t)co * Cin + ci];
            }
        for (int ci = 0; ci < Cin; ++ci) {
            double acc = 0.0;
            for (int k = 0; k < r; ++k) acc += (double)B[(size_t)t * r + k] * gxr[(size_t)k * Cin + ci];
            out[(size_t)i * Cin + ci] = acc / (double)pp;
        }
        free(gyr);
        free(gxr);
    }
    free(B);
    return 0;
}

/* entries g~w[co[i]][ci[i]] */
int oracle_lbp_gw_entries(const double *x, const double *gy, int N, int H, int W, int Cin,
                          int Cout, int p, const int32_t *idx, int r,
                          const int32_t *co, const int32_t *ci, int n_entries, double *out)
{
    if (!x || !gy || !co || !ci || !out || n_entries < 0 || check_grid(N, H, W, Cin, p) ||
        Cout < 1 || check_idx(p, r, idx))
        return -1;
    int pp = p * p, PH = H / p, PW = W / p;
    int8_t *B = (int8_t *)malloc((size_t)pp * r);
    if (!B) return -2;
    oracle_basis_matrix(p, r, idx, B);
    long Q = (long)N * PH * PW;
    for (int i = 0; i < n_entries; ++i)
        if (co[i] < 0 || co[i] >= Cout || ci[i] < 0 || ci[i] >= Cin) { free(B); return -1; }
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < n_entries; ++i) {
        double acc = 0.0;
        for (long q = 0; q < Q; ++q) {
            int b = (int)(q % PW), a = (int)((q / PW) % PH), n = (int)(q / ((long)PW * PH));
            for (int k = 0; k < r; ++k) {
                double g = 0.0, xv = 0.0;
                for (int h = 0; h < p; ++h)
                    for (int ww = 0; ww < p; ++ww) {
                        size_t tok = token_of(n, a, b, h, ww, H, W, p);
                        double s = (double)B[(size_t)(h * p + ww) * r + k];
                        g += s * gy[tok * Cout + co[i]];
                        xv += s * x[tok * Cin + ci[i]];
                    }
                acc += g * xv;
            }
        }
        out[i] = acc / (double)pp;
    }
    free(B);
    return 0;
}

/* rows of the exact gx (Eq. 2) for the listed tokens */
int oracle_full_gx_tokens(const double *gy, const double *w, long M, int Cin, int Cout,
                          const int64_t *tokens, int ntok, double *out)
{
    if (!gy || !w || !tokens || !out || ntok < 0 || M < 1 || Cin < 1 || Cout < 1) return -1;
    for (int i = 0; i < ntok; ++i)
        if (tokens[i] < 0 || tokens[i] >= M) return -1;
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < ntok; ++i) {
        long tok = (long)tokens[i];
        double *o = out + (size_t)i * Cin;
        for (int c = 0; c < Cin; ++c) o[c] = 0.0;
        for (int co = 0; co < Cout; ++co) {
            double g = gy[(size_t)tok * Cout + co];
            for (int c = 0; c < Cin; ++c) o[c] += g * w[(size_t)co * Cin + c];
        }
    }
    return 0;
}

/* entries of the exact gW (Eq. 2) */
int oracle_full_gw_entries(const double *x, const double *gy, long M, int Cin, int Cout,
                           const int32_t *co, const int32_t *ci, int n_entries, double *out)
{
    if (!x || !gy || !co || !ci || !out || n_entries < 0 || M < 1 || Cin < 1 || Cout < 1) return -1;
    for (int i = 0; i < n_entries; ++i)
        if (co[i] < 0 || co[i] >= Cout || ci[i] < 0 || ci[i] >= Cin) return -1;
#pragma omp parallel for schedule(dynamic)
    for (int i = 0; i < n_entries; ++i) {
        double acc = 0.0;
        for (long m = 0; m < M; ++m) acc += gy[(size_t)m * Cout + co[i]] * x[(size_t)m * Cin + ci[i]];
        out[i] = acc;
    }
    return 0;
}

/* Energy of every basis (Section 3.2, low-heuristic-error selection; the spectrum of Section 4.5):
 * E[u*p + v] = sum over patches and channels of (coefficient of basis (u,v))^2, unnormalised
 * coefficients of Eq. 6.  By Parseval sum_j E[j] = p^2 * ||X||^2. */
int oracle_wht_energy(const double *X, int N, int H, int W, int C, int p, double *E)
{
    if (!X || !E || check_grid(N, H, W, C, p)) return -1;
    int pp = p * p;
    int32_t *all = (int32_t *)malloc((size_t)pp * sizeof(int32_t));
    if (!all) return -2;
    for (int j = 0; j < pp; ++j) all[j] = j;
    long Q = (long)N * (H / p) * (W / p);
    double *coef = (double *)malloc((size_t)Q * pp * C * sizeof(double));
    if (!coef) { free(all); return -2; }
    int rc = oracle_project(X, N, H, W, C, p, pp, all, coef);
    for (int j = 0; j < pp && !rc; ++j) {
        double e = 0.0;
        for (long q = 0; q < Q; ++q)
            for (int c = 0; c < C; ++c) {
                double v = coef[((size_t)q * pp + j) * C + c];
                e += v * v;
            }
        E[j] = e;
    }
    free(coef);
    free(all);
    return rc;
}

/* Low-heuristic-error selection (Section 3.2): the r bases with the largest profiled energy, listed
 * by decreasing energy.  The paper leaves ties open; here equal energies keep the LP_L1 order
 * (reading of this build: parity unpinned for ties). */
int oracle_select_lhe(const double *E, int p, int r, int32_t *idx)
{
    if (!E || !idx || !is_pow2(p) || r < 1 || r > p * p) return -1;
    int pp = p * p;
    int32_t *order = (int32_t *)malloc((size_t)pp * sizeof(int32_t));
    if (!order) return -2;
    int rc = oracle_select_bases(p, pp, 0, order);     /* LP_L1 order as the tie-break */
    /* stable insertion sort by decreasing energy */
    for (int i = 1; i < pp && !rc; ++i) {
        int32_t cur = order[i];
        int j = i - 1;
        while (j >= 0 && E[order[j]] < E[cur]) { order[j + 1] = order[j]; --j; }
        order[j + 1] = cur;
    }
    for (int k = 0; k < r && !rc; ++k) idx[k] = order[k];
    free(order);
    return rc;
}

/* Cost model of Table 1 (Section 3.3), FLOPs for one map of L tokens and rank r:
 * out[0] vanilla BP 4 Cx Cy L, out[1] projection (Cx+Cy) L r, out[2] low-rank matmuls
 * 4 Cx Cy r, out[3] reverse projection Cx L r. */
int oracle_flop_model(long Cx, long Cy, long L, long r, double out[4])
{
    if (Cx < 1 || Cy < 1 || L < 1 || r < 1 || !out) return -1;
    out[0] = 4.0 * (double)Cx * (double)Cy * (double)L;
    out[1] = (double)(Cx + Cy) * (double)L * (double)r;
    out[2] = 4.0 * (double)Cx * (double)Cy * (double)r;
    out[3] = (double)Cx * (double)L * (double)r;
    return 0;
}
