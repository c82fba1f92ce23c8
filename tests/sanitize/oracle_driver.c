/* Runs every routine of the CPU oracle once on small inputs (including an image smaller than the patch and a
 * one-pixel image) so that a build with -fsanitize=address,undefined sees each loop's first and last access.
 * Prints "oracle sanitize ok" when nothing aborted; checks a few values so that the calls cannot be elided. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_num_threads(void);
void orc_patch(const double *img, int h, int w, int k, int y, int x, double *out);
void orc_corr_sums(const double *V1, const double *V2, int64_t n, int h, int w, int k, double *S11, double *S22,
                   double *S12);
void orc_class_sums(const double *V1, const double *V2, const int32_t *cls, const int32_t *grp, int64_t n, int n_cls,
                    int n_grp, int h, int w, int k, double *Sw, double *ST);
void orc_corr_entries(const double *V1, const double *V2, int64_t n, int h, int w, int k, int n_entries,
                      const int32_t *va, const int32_t *a, const int32_t *vb, const int32_t *b, double *out);
int orc_jacobi_sym(double *A, int n, double *V, double tol, int max_sweeps);
void orc_conv(const double *V, int64_t n, int h, int w, const double *W, int L, int k, double *out);
void orc_hash(const double *Z, int64_t n, int L2, int h, int w, int32_t *Q);
void orc_block_hist(const int32_t *Q, int64_t n, int h, int w, int bh, int bw, int sy, int sx, int bins,
                    int64_t *hist);

static double *filled(size_t n, unsigned seed)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    for (size_t i = 0; i < n; ++i) {
        seed = seed * 1664525u + 1013904223u;
        p[i] = (double)(seed >> 8) / 16777216.0 - 0.5;
    }
    return p;
}

static int one_geometry(int n, int h, int w, int k, int L, int L2, int bh, int bw, int sy, int sx)
{
    const int D = k * k;
    const size_t P = (size_t)h * w;
    double *V1 = filled(n * P, 1u + h), *V2 = filled(n * P, 7u + w);
    double *S = (double *)calloc((size_t)5 * D * D, sizeof(double));
    int32_t *cls = (int32_t *)malloc(sizeof(int32_t) * n), *grp = (int32_t *)malloc(sizeof(int32_t) * n);
    for (int i = 0; i < n; ++i) { cls[i] = i % 3; grp[i] = (i / 3) % 2; }
    double *patch = (double *)malloc(sizeof(double) * D);
    orc_patch(V1, h, w, k, 0, 0, patch);
    orc_patch(V1, h, w, k, h - 1, w - 1, patch);
    double sum = 0.0;
    for (int a = 0; a < D; ++a) sum += patch[a];
    orc_corr_sums(V1, V2, n, h, w, k, S, S + D * D, S + 2 * D * D);
    orc_class_sums(V1, V2, cls, grp, n, 3, 2, h, w, k, S + 3 * D * D, S + 4 * D * D);
    int32_t va[2] = {1, 2}, a[2] = {0, D - 1}, vb[2] = {2, 2}, b[2] = {D - 1, 0};
    double ent[2];
    orc_corr_entries(V1, V2, n, h, w, k, 2, va, a, vb, b, ent);
    int bad = !(sum < 1e-9 && sum > -1e-9);
    bad |= !(ent[0] - S[2 * D * D + D - 1] < 1e-9 && S[2 * D * D + D - 1] - ent[0] < 1e-9);
    double *E = (double *)malloc(sizeof(double) * D * D);
    for (int i = 0; i < D; ++i)                               /* symmetric input for the eigen routine */
        for (int j = 0; j < D; ++j) S[i * D + j] = 0.5 * (S[i * D + j] + S[j * D + i]);
    orc_jacobi_sym(S, D, E, 1e-15, 60);
    double *W = filled((size_t)L * D, 3u), *Y = (double *)malloc(sizeof(double) * n * L * P);
    orc_conv(V1, n, h, w, W, L, k, Y);
    double *W2 = filled((size_t)L2 * D, 5u), *Z = (double *)malloc(sizeof(double) * (size_t)n * L * L2 * P);
    orc_conv(Y, (int64_t)n * L, h, w, W2, L2, k, Z);
    int32_t *Q = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * L * P);
    orc_hash(Z, (int64_t)n * L, L2, h, w, Q);
    if (bh <= h && bw <= w) {
        const int nby = (h - bh) / sy + 1, nbx = (w - bw) / sx + 1;
        int64_t *H = (int64_t *)malloc(sizeof(int64_t) * (size_t)n * L * nby * nbx * ((size_t)1 << L2));
        orc_block_hist(Q, (int64_t)n * L, h, w, bh, bw, sy, sx, 1 << L2, H);
        int64_t tot = 0;
        for (int t = 0; t < (1 << L2); ++t) tot += H[t];
        bad |= tot != (int64_t)bh * bw;
        free(H);
    }
    free(V1); free(V2); free(S); free(cls); free(grp); free(patch); free(E); free(W); free(Y); free(W2); free(Z);
    free(Q);
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= one_geometry(7, 9, 11, 3, 2, 3, 4, 4, 2, 2);
    bad |= one_geometry(6, 8, 6, 5, 3, 2, 8, 6, 4, 3);        /* block = whole map */
    bad |= one_geometry(6, 2, 3, 5, 2, 2, 2, 2, 1, 1);        /* image smaller than the patch */
    bad |= one_geometry(6, 1, 1, 3, 1, 1, 1, 1, 1, 1);        /* one pixel */
    bad |= one_geometry(6, 10, 7, 7, 2, 4, 7, 7, 4, 4);       /* trailing rows dropped by the block grid */
    if (bad) { printf("oracle sanitize: value check failed\n"); return 1; }
    printf("oracle sanitize ok (%d threads)\n", orc_num_threads());
    return 0;
}
