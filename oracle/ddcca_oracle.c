/*
 * CPU fp64 oracle for the two-stage DDCCANet feature extractor -- TEST INFRASTRUCTURE ONLY.
 *
 * This file is the plain, slow definition of what the GPU path computes.  It is used
 * by the test-suite, by the smoke check and by the benchmark's CPU-baseline leg and by
 * nothing else; the product library never links or calls it, and it shares no code
 * with the HIP sources.  Every routine follows the paper's definitions directly
 * (Section II for the model, Section III for the batch identity); there is no
 * blocking, fusion or algebraic shortcut.  The only concession to run time is an
 * OpenMP loop over images whose per-thread sums are added in thread order.
 *
 * Conventions (the paper leaves them open; these are the readings used everywhere):
 *   - one patch per pixel, zero padding by r=(k-1)/2, k odd        (Eq. 1: M*p*q columns)
 *   - patch element a = dy*k + dx, row-major                       (Eq. 4-5, res_{l1,l2})
 *   - every patch has its own mean removed (mean over its k*k entries, zeros included)
 *   - the stage "convolution" is a cross-correlation (no flip)     (Eq. 6)
 *   - S(x) = 1 iff x > 0                                           (Eq. 8)
 *   - filter l (1-based) owns bit l-1 of the hash code             (Eq. 9)
 * All images are double precision, row-major [n][h][w].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. 1 with the padding / mean-removal reading above: the mean-removed k*k patch
 * centred on pixel (y,x) of one h*w image. */
void orc_patch(const double *img, int h, int w, int k, int y, int x, double *out)
{
    const int r = (k - 1) / 2;
    const int D = k * k;
    double sum = 0.0;
    for (int dy = 0; dy < k; ++dy)
        for (int dx = 0; dx < k; ++dx) {
            const int yy = y + dy - r, xx = x + dx - r;
            double v = 0.0;
            if (yy >= 0 && yy < h && xx >= 0 && xx < w)
                v = img[(size_t)yy * w + xx];
            out[dy * k + dx] = v;
            sum += v;
        }
    const double mean = sum / D;
    for (int a = 0; a < D; ++a)
        out[a] -= mean;
}

/* Un-normalised sums over all patches of all n image pairs (Section II-A, and the
 * batch identity Eq. 15: calling this on consecutive batches ADDS into S11/S22/S12):
 *   S11 += sum x1 x1^T,  S22 += sum x2 x2^T,  S12 += sum x1 x2^T      (each D*D)   */
void orc_corr_sums(const double *V1, const double *V2, int64_t n, int h, int w, int k,
                   double *S11, double *S22, double *S12)
{
    const int D = k * k;
    const size_t P = (size_t)h * w;
    int nt = orc_num_threads();
    double *acc = (double *)calloc((size_t)nt * 3 * D * D, sizeof(double));
#pragma omp parallel num_threads(nt)
    {
        int t = 0;
#ifdef _OPENMP
        t = omp_get_thread_num();
#endif
        double *a11 = acc + (size_t)t * 3 * D * D, *a22 = a11 + D * D, *a12 = a22 + D * D;
        double *x1 = (double *)malloc(sizeof(double) * D), *x2 = (double *)malloc(sizeof(double) * D);
#pragma omp for schedule(static)
        for (int64_t m = 0; m < n; ++m)
            for (int y = 0; y < h; ++y)
                for (int x = 0; x < w; ++x) {
                    orc_patch(V1 + m * P, h, w, k, y, x, x1);
                    orc_patch(V2 + m * P, h, w, k, y, x, x2);
                    for (int a = 0; a < D; ++a) {
                        const double p1 = x1[a], p2 = x2[a];
                        for (int b = 0; b < D; ++b) {
                            a11[a * D + b] += p1 * x1[b];
                            a22[a * D + b] += p2 * x2[b];
                            a12[a * D + b] += p1 * x2[b];
                        }
                    }
                }
        free(x1);
        free(x2);
    }
    for (int t = 0; t < nt; ++t) {
        const double *a = acc + (size_t)t * 3 * D * D;
        for (int i = 0; i < D * D; ++i) {
            S11[i] += a[i];
            S22[i] += a[i + D * D];
            S12[i] += a[i + 2 * D * D];
        }
    }
    free(acc);
}

/* Class-conditioned cross-view sums (Section II-A: C_w, C_b "within-class and
 * between-class correlation matrices between I1 and I2").  A sample is an image; the
 * patches of two samples pair up when they sit at the same pixel u and belong to the
 * same map group g.  For every cell (c,g) and pixel u the patches of the cell's
 * members are summed per view and the two sums multiplied:
 *   Sw = sum_{c,g} sum_u (sum_{m in (c,g)} x1_{m,u}) (sum_{m in (c,g)} x2_{m,u})^T
 *   ST = sum_{g}   sum_u (sum_{m in g}     x1_{m,u}) (sum_{m in g}     x2_{m,u})^T
 * so that Sw holds all same-class pairs, ST all pairs and ST-Sw the different-class
 * pairs.  cls[m] in [0,n_cls), grp[m] in [0,n_grp).  Outputs are overwritten. */
void orc_class_sums(const double *V1, const double *V2, const int32_t *cls, const int32_t *grp,
                    int64_t n, int n_cls, int n_grp, int h, int w, int k, double *Sw, double *ST)
{
    const int D = k * k;
    const size_t P = (size_t)h * w;
    memset(Sw, 0, sizeof(double) * D * D);
    memset(ST, 0, sizeof(double) * D * D);
    const int n_pix = h * w;
    /* members of each cell (c,g), in image order */
    const int n_cell = n_cls * n_grp;
    int64_t *start = (int64_t *)calloc((size_t)n_cell + 1, sizeof(int64_t));
    int64_t *fill = (int64_t *)calloc((size_t)n_cell, sizeof(int64_t));
    int64_t *member = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    for (int64_t m = 0; m < n; ++m) start[cls[m] * n_grp + grp[m] + 1] += 1;
    for (int e = 0; e < n_cell; ++e) start[e + 1] += start[e];
    for (int64_t m = 0; m < n; ++m) {
        const int e = cls[m] * n_grp + grp[m];
        member[start[e] + fill[e]++] = m;
    }
    int nt = orc_num_threads();
    double *acc = (double *)calloc((size_t)nt * 2 * D * D, sizeof(double));
#pragma omp parallel num_threads(nt)
    {
        int t = 0;
#ifdef _OPENMP
        t = omp_get_thread_num();
#endif
        double *aw = acc + (size_t)t * 2 * D * D, *aT = aw + D * D;
        double *x = (double *)malloc(sizeof(double) * D);
        double *s1 = (double *)malloc(sizeof(double) * D), *s2 = (double *)malloc(sizeof(double) * D);
        double *t1 = (double *)malloc(sizeof(double) * D), *t2 = (double *)malloc(sizeof(double) * D);
#pragma omp for schedule(static)
        for (int u = 0; u < n_pix; ++u) {
            const int y = u / w, xq = u % w;
            for (int g = 0; g < n_grp; ++g) {
                for (int a = 0; a < D; ++a) t1[a] = t2[a] = 0.0;
                for (int c = 0; c < n_cls; ++c) {
                    const int e = c * n_grp + g;
                    for (int a = 0; a < D; ++a) s1[a] = s2[a] = 0.0;
                    for (int64_t i = start[e]; i < start[e + 1]; ++i) {
                        const int64_t m = member[i];
                        orc_patch(V1 + m * P, h, w, k, y, xq, x);
                        for (int a = 0; a < D; ++a) s1[a] += x[a];
                        orc_patch(V2 + m * P, h, w, k, y, xq, x);
                        for (int a = 0; a < D; ++a) s2[a] += x[a];
                    }
                    for (int a = 0; a < D; ++a)
                        for (int b = 0; b < D; ++b)
                            aw[a * D + b] += s1[a] * s2[b];
                    for (int a = 0; a < D; ++a) { t1[a] += s1[a]; t2[a] += s2[a]; }
                }
                for (int a = 0; a < D; ++a)
                    for (int b = 0; b < D; ++b)
                        aT[a * D + b] += t1[a] * t2[b];
            }
        }
        free(x); free(s1); free(s2); free(t1); free(t2);
    }
    for (int t = 0; t < nt; ++t) {
        const double *a = acc + (size_t)t * 2 * D * D;
        for (int i = 0; i < D * D; ++i) { Sw[i] += a[i]; ST[i] += a[i + D * D]; }
    }
    free(acc); free(start); free(fill); free(member);
}

/* A handful of entries of the un-normalised sums, for spot checks at sizes where the
 * full D*D accumulation is too slow on a CPU: entry e is
 *   sum over all patches of  x^{va[e]}[a[e]] * x^{vb[e]}[b[e]]   (va,vb in {1,2}). */
void orc_corr_entries(const double *V1, const double *V2, int64_t n, int h, int w, int k,
                      int n_entries, const int32_t *va, const int32_t *a, const int32_t *vb,
                      const int32_t *b, double *out)
{
    const int D = k * k;
    const size_t P = (size_t)h * w;
    int nt = orc_num_threads();
    double *acc = (double *)calloc((size_t)nt * n_entries, sizeof(double));
#pragma omp parallel num_threads(nt)
    {
        int t = 0;
#ifdef _OPENMP
        t = omp_get_thread_num();
#endif
        double *x1 = (double *)malloc(sizeof(double) * D), *x2 = (double *)malloc(sizeof(double) * D);
#pragma omp for schedule(static)
        for (int64_t m = 0; m < n; ++m)
            for (int y = 0; y < h; ++y)
                for (int x = 0; x < w; ++x) {
                    orc_patch(V1 + m * P, h, w, k, y, x, x1);
                    orc_patch(V2 + m * P, h, w, k, y, x, x2);
                    for (int e = 0; e < n_entries; ++e) {
                        const double p = (va[e] == 1 ? x1 : x2)[a[e]];
                        const double q = (vb[e] == 1 ? x1 : x2)[b[e]];
                        acc[(size_t)t * n_entries + e] += p * q;
                    }
                }
        free(x1); free(x2);
    }
    for (int e = 0; e < n_entries; ++e) {
        out[e] = 0.0;
        for (int t = 0; t < nt; ++t) out[e] += acc[(size_t)t * n_entries + e];
    }
    free(acc);
}

/* Cyclic (row-by-row) Jacobi eigenvalue iteration for a real symmetric n*n matrix A
 * (row-major, overwritten; on return its diagonal holds the eigenvalues) with the
 * rotations accumulated in V (n*n, columns = eigenvectors).  Stops when the
 * off-diagonal Frobenius norm is <= tol * ||A||_F or after max_sweeps sweeps.
 * Returns the number of sweeps done.  Used by the DCCA solve (Eq. 2-3). */
int orc_jacobi_sym(double *A, int n, double *V, double tol, int max_sweeps)
{
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j)
            V[i * n + j] = (i == j) ? 1.0 : 0.0;
    double fro = 0.0;
    for (int i = 0; i < n * n; ++i) fro += A[i] * A[i];
    fro = sqrt(fro);
    int sweep = 0;
    for (; sweep < max_sweeps; ++sweep) {
        double off = 0.0;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                if (i != j) off += A[i * n + j] * A[i * n + j];
        if (sqrt(off) <= tol * fro) break;
        for (int p = 0; p < n - 1; ++p)
            for (int q = p + 1; q < n; ++q) {
                const double apq = A[p * n + q];
                if (apq == 0.0) continue;
                const double theta = (A[q * n + q] - A[p * n + p]) / (2.0 * apq);
                const double tt = (theta >= 0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                const double c = 1.0 / sqrt(tt * tt + 1.0), s = tt * c;
                for (int i = 0; i < n; ++i) {           /* A <- A J  (columns p,q) */
                    const double aip = A[i * n + p], aiq = A[i * n + q];
                    A[i * n + p] = c * aip - s * aiq;
                    A[i * n + q] = s * aip + c * aiq;
                }
                for (int j = 0; j < n; ++j) {           /* A <- J^T A (rows p,q) */
                    const double apj = A[p * n + j], aqj = A[q * n + j];
                    A[p * n + j] = c * apj - s * aqj;
                    A[q * n + j] = s * apj + c * aqj;
                }
                for (int i = 0; i < n; ++i) {           /* V <- V J */
                    const double vip = V[i * n + p], viq = V[i * n + q];
                    V[i * n + p] = c * vip - s * viq;
                    V[i * n + q] = s * vip + c * viq;
                }
            }
    }
    return sweep;
}

/* Eq. 6: every image correlated with each of the L k*k filters, zero padding, same
 * size: out[m][g][y][x] = sum_{dy,dx} W[g][dy][dx] * Vpad[m][y+dy-r][x+dx-r]. */
void orc_conv(const double *V, int64_t n, int h, int w, const double *W, int L, int k, double *out)
{
    const int r = (k - 1) / 2;
    const size_t P = (size_t)h * w;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < n; ++m)
        for (int g = 0; g < L; ++g)
            for (int y = 0; y < h; ++y)
                for (int x = 0; x < w; ++x) {
                    double s = 0.0;
                    for (int dy = 0; dy < k; ++dy)
                        for (int dx = 0; dx < k; ++dx) {
                            const int yy = y + dy - r, xx = x + dx - r;
                            if (yy >= 0 && yy < h && xx >= 0 && xx < w)
                                s += W[(g * k + dy) * k + dx] * V[m * P + (size_t)yy * w + xx];
                        }
                    out[(m * L + g) * P + (size_t)y * w + x] = s;
                }
}

/* Eq. 7-9: Q[m][y][x] = sum_{l=1..L2} 2^{l-1} * [ Z[m][l-1][y][x] > 0 ]. */
void orc_hash(const double *Z, int64_t n, int L2, int h, int w, int32_t *Q)
{
    const size_t P = (size_t)h * w;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < n; ++m)
        for (size_t u = 0; u < P; ++u) {
            int32_t code = 0;
            for (int l = 0; l < L2; ++l)
                if (Z[(m * L2 + l) * P + u] > 0.0) code += (int32_t)1 << l;
            Q[m * P + u] = code;
        }
}

/* Section II-C: the code map is cut into b_h*b_w blocks whose top-left corners sit at
 * (i*s_y, j*s_x) for every i,j with the block fully inside the map; hist[m][i][j][t]
 * counts the pixels of block (i,j) whose code is t, t = 0..bins-1. */
void orc_block_hist(const int32_t *Q, int64_t n, int h, int w, int bh, int bw, int sy, int sx,
                    int bins, int64_t *hist)
{
    const int nby = (h - bh) / sy + 1, nbx = (w - bw) / sx + 1;
    const size_t P = (size_t)h * w;
    memset(hist, 0, sizeof(int64_t) * (size_t)n * nby * nbx * bins);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < n; ++m)
        for (int i = 0; i < nby; ++i)
            for (int j = 0; j < nbx; ++j) {
                int64_t *hb = hist + (((size_t)m * nby + i) * nbx + j) * bins;
                for (int y = i * sy; y < i * sy + bh; ++y)
                    for (int x = j * sx; x < j * sx + bw; ++x)
                        hb[Q[m * P + (size_t)y * w + x]] += 1;
            }
}
