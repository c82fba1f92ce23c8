// Class-conditioned part of the correlation step (Section II-A: within-class and
// between-class correlation between the two views).  Patch extraction and mean removal
// are linear in the image, so the per-pixel sum of a cell's patches is the patch of the
// cell's SUM IMAGE.  These kernels build, per view, the sum image of every
// (class, g) cell and of every g over all classes; the patch-Gram kernel then runs on
// those few images and its cross-view block gives C_w and C_T.
#include "ddcca_internal.h"

namespace ddcca {

// Clears the sum images.  A kernel rather than a memset so that a caller may capture the learning calls into a
// HIP graph (memset nodes are avoided).
__global__ void zero_f64_kernel(double2 *__restrict__ p, int64_t n2)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += stride) p[i] = make_double2(0.0, 0.0);
}

__global__ void label_check_kernel(const int32_t *__restrict__ cls, int64_t n_img, int n_cls, int *flag)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_img) {
        const int c = cls[i];
        if (c < 0 || c >= n_cls) atomicOr(flag, 1);
    }
}

// grid (pixel chunks, n_cls*G, sample segments).  A workgroup owns 1024 pixels of one cell and one
// contiguous segment of the samples: it scans the segment's labels 64 at a time, and for every
// member sample (in ascending order, so the sum is reproducible) adds that sample's map g to fp64
// accumulators, both views.  Segment s adds into its own copy sums[s] of the sum images (the
// copies are added in order when the images are finalised): with few cells the sample segments
// are what fills the chip.
__global__ __launch_bounds__(256) void class_sum_kernel(const float *__restrict__ v1, const float *__restrict__ v2,
                                                        const int32_t *__restrict__ cls, int64_t n_img, int G,
                                                        int64_t P, double *__restrict__ sums, int64_t n_cell)
{
    const int cell = blockIdx.y;
    // label windows of this segment
    const int64_t n_win = (n_img + 63) / 64;
    const int64_t win0 = n_win * blockIdx.z / gridDim.z, win1 = n_win * (blockIdx.z + 1) / gridDim.z;
    sums += (int64_t)blockIdx.z * 2 * n_cell * P;
    const int c = cell / G, g = cell - c * G;
    const int lane = threadIdx.x & 63;
    const int64_t p0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    double a1[4] = {0, 0, 0, 0}, a2[4] = {0, 0, 0, 0};
    const bool vec = (P & 3) == 0 && ((((uintptr_t)v1) | ((uintptr_t)v2)) & 15) == 0;
    for (int64_t base = win0 * 64; base < win1 * 64; base += 64) {
        const int64_t idx = base + lane;
        const int lab = idx < n_img ? cls[idx] : -1;
        unsigned long long mask = __ballot(lab == c);
        while (mask) {
            if (vec && p0 + 3 < P) {
                // up to four members at a time: their loads are all requested before the first is added (the
                // additions stay in ascending sample order)
                float4 x[4], y[4];
                int cnt = 0;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (mask) {
                        const int j = __ffsll((long long)mask) - 1;
                        mask &= mask - 1;
                        const int64_t o = ((base + j) * G + g) * P + p0;
                        x[u] = *reinterpret_cast<const float4 *>(v1 + o);
                        y[u] = *reinterpret_cast<const float4 *>(v2 + o);
                        cnt = u + 1;
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (u < cnt) {
                        a1[0] += x[u].x; a1[1] += x[u].y; a1[2] += x[u].z; a1[3] += x[u].w;
                        a2[0] += y[u].x; a2[1] += y[u].y; a2[2] += y[u].z; a2[3] += y[u].w;
                    }
                }
                continue;
            }
            const int j = __ffsll((long long)mask) - 1;
            mask &= mask - 1;
            const int64_t o = ((base + j) * G + g) * P + p0;
            {
                for (int e = 0; e < 4; ++e)
                    if (p0 + e < P) {
                        a1[e] += v1[o + e];
                        a2[e] += v2[o + e];
                    }
            }
        }
    }
    double *s1 = sums + (int64_t)cell * P, *s2 = sums + (n_cell + cell) * P;
    for (int e = 0; e < 4; ++e)
        if (p0 + e < P) {
            s1[p0 + e] += a1[e];
            s2[p0 + e] += a2[e];
        }
}

// img[view][cell][p] = (float) sum over segments of sums[seg][view][cell][p];
// img[view][n_cell + g][p] = (float) sum over classes.
// A workgroup owns 16 pixels of one (g, view): 16 lanes of classes x 16 pixels; lane j takes classes
// j, j+16, ...; the 16 partial totals are added in lane order.
__global__ __launch_bounds__(256) void class_finalize_kernel(const double *__restrict__ sums, int n_cls, int G,
                                                             int64_t P, float *__restrict__ img, int n_seg)
{
    __shared__ double part[16][17];
    const int px = threadIdx.x & 15, cl = threadIdx.x >> 4;
    const int64_t p = (int64_t)blockIdx.x * 16 + px;
    const int g = blockIdx.y, view = blockIdx.z;
    const int64_t n_cell = (int64_t)n_cls * G;
    const double *s = sums + view * n_cell * P;
    float *o = img + view * (n_cell + G) * P;
    double tot = 0.0;
    if (p < P)
        for (int c = cl; c < n_cls; c += 16) {
            double v = 0.0;
            for (int sg = 0; sg < n_seg; ++sg) v += s[(int64_t)sg * 2 * n_cell * P + ((int64_t)c * G + g) * P + p];
            o[((int64_t)c * G + g) * P + p] = (float)v;
            tot += v;
        }
    part[cl][px] = tot;
    __syncthreads();
    if (cl == 0 && p < P) {
        double t = 0.0;
        for (int j = 0; j < 16; ++j) t += part[j][px];
        o[(n_cell + g) * P + p] = (float)t;
    }
}

int launch_zero_sums(ddcca_ctx *ctx, double *sums, size_t n)
{
    ProfScope prof(ctx, DDCCA_K_CLASS_SUM);
    // n is even (two views) and the buffer comes from hipMalloc: double2 stores are aligned
    const int64_t n2 = (int64_t)(n / 2);
    const unsigned grid = (unsigned)std::min<int64_t>(4096, std::max<int64_t>(1, (n2 + 255) / 256));
    hipLaunchKernelGGL(zero_f64_kernel, dim3(grid), dim3(256), 0, ctx->stream, reinterpret_cast<double2 *>(sums), n2);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int launch_label_check(ddcca_ctx *ctx, const int32_t *cls, int64_t n_img, int n_cls, int *flag)
{
    ProfScope prof(ctx, DDCCA_K_CLASS_SUM);
    hipLaunchKernelGGL(label_check_kernel, dim3((unsigned)((n_img + 255) / 256)), dim3(256), 0, ctx->stream, cls, n_img,
                       n_cls, flag);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int class_sum_segments(int64_t n_cell, int64_t P)
{
    const int64_t wgs = ((P + 1023) / 1024) * n_cell;
    // few cells: up to 16 segments towards 2048 workgroups; otherwise only what it takes to reach 1024
    int64_t s = std::min<int64_t>(16, std::max<int64_t>(1, (wgs < 256 ? 2048 : 1024) / wgs));
    // the copies of the sum images stay below 1 GiB
    while (s > 1 && s * 2 * n_cell * P * (int64_t)sizeof(double) > ((int64_t)1 << 30)) --s;
    return (int)s;
}

int launch_class_sum(ddcca_ctx *ctx, const float *v1, const float *v2, const int32_t *cls, int64_t n_img, int G,
                     int n_cls, int64_t P, double *sums, int n_seg)
{
    ProfScope prof(ctx, DDCCA_K_CLASS_SUM);
    const int64_t n_cell = (int64_t)n_cls * G;
    const unsigned chunks = (unsigned)((P + 1023) / 1024);
    if (n_cell > 65535) return fail(ctx, DDCCA_EINVAL, "n_cls * G must not exceed 65535");
    hipLaunchKernelGGL(class_sum_kernel, dim3(chunks, (unsigned)n_cell, (unsigned)n_seg), dim3(256), 0, ctx->stream, v1,
                       v2, cls, n_img, G, P, sums, n_cell);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int launch_class_finalize(ddcca_ctx *ctx, const double *sums, int n_cls, int G, int64_t P, float *img, int n_seg)
{
    ProfScope prof(ctx, DDCCA_K_CLASS_SUM);
    hipLaunchKernelGGL(class_finalize_kernel, dim3((unsigned)((P + 15) / 16), G, 2), dim3(256), 0, ctx->stream, sums,
                       n_cls, G, P, img, n_seg);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
