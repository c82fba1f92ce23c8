// Output layer: hashing of the L2 maps of one input into a code map (Eq. 7-9) fused
// with the per-block code histogram (Section II-C).  Integer work only; HBM-bound.
#include "ddcca_internal.h"

namespace ddcca {

// General kernel: one workgroup owns one block row (i) of one map and a chunk of block
// columns.  Its LDS holds the chunk's histograms as 32-bit counters; every pixel of the
// block row's bh image rows is hashed once by this workgroup and added to each block
// column of the chunk that contains it.
template <int L2>
__global__ __launch_bounds__(256) void hash_hist_rows_kernel(const float *__restrict__ maps, int h, int w, int bh,
                                                             int bw, int sy, int sx, int nby, int nbx,
                                                             int cols_per_wg, uint16_t *__restrict__ hist,
                                                             int64_t group, int64_t group_stride)
{
    extern __shared__ unsigned int lds_hist[];
    constexpr int BINS = 1 << L2;
    const int64_t n = blockIdx.z;
    const int i = blockIdx.y;
    const int j0 = blockIdx.x * cols_per_wg;
    const int j1 = min(j0 + cols_per_wg, nbx);
    const int ncol = j1 - j0;
    for (int e = threadIdx.x; e < ncol * BINS; e += blockDim.x) lds_hist[e] = 0u;
    __syncthreads();

    const int64_t P = (int64_t)h * w;
    const float *base = maps + n * L2 * P;
    const int x_lo = j0 * sx;
    const int x_hi = (j1 - 1) * sx + bw;          // exclusive
    const int span = x_hi - x_lo;
    const int y0 = i * sy;
    for (int e = threadIdx.x; e < bh * span; e += blockDim.x) {
        const int yy = e / span, x = x_lo + (e - yy * span);
        const int64_t u = (int64_t)(y0 + yy) * w + x;
        unsigned int code = 0;
#pragma unroll
        for (int l = 0; l < L2; ++l) code |= (base[l * P + u] > 0.0f ? 1u : 0u) << l;
        // block columns j with j*sx <= x < j*sx + bw
        int jlo = (x - bw + sx) / sx;             // ceil((x - bw + 1) / sx) for x-bw+1 >= 0
        if (x - bw + 1 < 0) jlo = 0;
        int jhi = x / sx;
        jlo = max(jlo, j0);
        jhi = min(jhi, j1 - 1);
        for (int j = jlo; j <= jhi; ++j) atomicAdd(&lds_hist[(j - j0) * BINS + code], 1u);
    }
    __syncthreads();
    const int64_t A = (int64_t)nby * nbx;
    uint16_t *out = hist + (n / group) * group_stride + (n % group) * A * BINS + ((int64_t)i * nbx + j0) * BINS;
    for (int e = threadIdx.x; e < ncol * BINS; e += blockDim.x) out[e] = (uint16_t)lds_hist[e];
}

template <int L2>
static void launch_rows(ddcca_ctx *ctx, const float *maps, int64_t n, int h, int w, int bh, int bw, int sy, int sx,
                        uint16_t *hist, int64_t group, int64_t group_stride)
{
    const int nby = (h - bh) / sy + 1, nbx = (w - bw) / sx + 1;
    constexpr int BINS = 1 << L2;
    int cols = std::max(1, (48 * 1024) / (BINS * 4));
    cols = std::min(cols, nbx);
    const int chunks = (nbx + cols - 1) / cols;
    const size_t lds = (size_t)cols * BINS * sizeof(unsigned int);
    dim3 grid(chunks, nby, (unsigned)n);      // caller keeps n <= 65535 (grid.z limit)
    hipLaunchKernelGGL(hash_hist_rows_kernel<L2>, grid, dim3(256), lds, ctx->stream, maps, h, w, bh, bw, sy, sx, nby,
                       nbx, cols, hist, group, group_stride);
}

int launch_hash_hist(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w, int bh, int bw, int sy,
                     int sx, uint16_t *hist, int64_t group, int64_t group_stride)
{
    ProfScope prof(ctx, DDCCA_K_HASH_HIST);
    // grid.z carries the map index and is limited to 65535; sub-launches start at
    // multiples of `group` so that the output addressing stays (n / group, n % group)
    const int64_t step = std::max<int64_t>(group, (65535 / group) * group);
    for (int64_t n0 = 0; n0 < n; n0 += step) {
        const int64_t nb = std::min(step, n - n0);
        const float *m = maps + n0 * L2 * (int64_t)h * w;
        uint16_t *o = hist + (n0 / group) * group_stride;
        switch (L2) {
#define CASE(v) case v: launch_rows<v>(ctx, m, nb, h, w, bh, bw, sy, sx, o, group, group_stride); break;
            CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12)
#undef CASE
            default: return fail(ctx, DDCCA_EINVAL, "L2 out of range");
        }
    }
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
