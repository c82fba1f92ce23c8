// Stage convolution (Eq. 6) on the bf16 matrix pipeline with three-piece operands (see conv_split.h):
// same interface, tiling and output stores as the fp32 kernel of conv_multi.hip, fp32-grade accuracy.
//
// One workgroup: a 32-row x (32*NBX)-column output tile of one image, all L filters.  The input tile with
// its halo is split once, while it is staged, into three planes of packed bf16 pairs in LDS; the filter
// pieces live in registers.  Wavefront w owns tile rows w, w+4, ...
#include "conv_split.h"

namespace ddcca {

constexpr int CSPLIT_THREADS = 256;
constexpr int CSPLIT_TH = 32;
constexpr int CSPLIT_XB = 32;
constexpr int CSPLIT_MAX_NBX = 4;

template <int KS, int NBX>
__global__ __launch_bounds__(CSPLIT_THREADS) void conv_split_kernel(const float *__restrict__ in, int h, int w,
                                                                   const float *__restrict__ W, int L,
                                                                   float *__restrict__ out, int tiles_x, int tiles_y)
{
    typedef SplitGeom<KS, NBX, CSPLIT_TH> G;
    constexpr int R = G::R, TW = G::TW, STEPS = G::STEPS;
    __shared__ unsigned int planes[3 * G::PLANE];
    const int tiles = tiles_x * tiles_y;
    const int64_t n = blockIdx.x / tiles;
    const int t = blockIdx.x - (int)n * tiles;
    const int tx = t % tiles_x, ty = t / tiles_x;
    const int64_t P = (int64_t)h * w;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c = lane & 15;
    // staged columns [gxa, gxa + COLS): gxa = the multiple of 4 at or below the first halo column; pairs are
    // packed starting at the first halo column's parity so that every window of a lane starts on a word
    const int gy0 = ty * CSPLIT_TH - R, gx0 = tx * TW - R;
    const int gxa = gx0 & ~3, shx = gx0 - gxa, po = shx & 1;
    {
        const float *src = in + n * P;
        const bool vec4 = (w & 3) == 0 && (((uintptr_t)src) & 15) == 0;
        for (int e = threadIdx.x; e < G::PH * G::V4; e += CSPLIT_THREADS) {
            const int yy = e / G::V4, xv = e - yy * G::V4;
            const int gy = gy0 + yy, gx = gxa + 4 * xv;
            float v0 = 0.f, v1 = 0.f, v2 = 0.f, v3 = 0.f, v4 = 0.f;
            if (gy >= 0 && gy < h) {
                const float *row = src + (int64_t)gy * w;
                if (vec4 && gx >= 0 && gx + 3 < w) {
                    const float4 v = *reinterpret_cast<const float4 *>(row + gx);
                    v0 = v.x; v1 = v.y; v2 = v.z; v3 = v.w;
                } else {
                    if (gx >= 0 && gx < w) v0 = row[gx];
                    if (gx + 1 >= 0 && gx + 1 < w) v1 = row[gx + 1];
                    if (gx + 2 >= 0 && gx + 2 < w) v2 = row[gx + 2];
                    if (gx + 3 >= 0 && gx + 3 < w) v3 = row[gx + 3];
                }
                if (po && gx + 4 >= 0 && gx + 4 < w) v4 = row[gx + 4];
            }
            // word i of a plane row holds pixels (2i + po, 2i + 1 + po) of the staged row
            const int idx = yy * G::PWORDS + 2 * xv;
            if (po) {
                split_store_pair(planes, G::PLANE, idx, v1, v2);
                split_store_pair(planes, G::PLANE, idx + 1, v3, v4);
            } else {
                split_store_pair(planes, G::PLANE, idx, v0, v1);
                split_store_pair(planes, G::PLANE, idx + 1, v2, v3);
            }
        }
    }
    int toff[STEPS][4];
    split_offsets<G>(q, toff);
    SplitOperand wa[STEPS][3];
    split_weights<G, KS, true>(W, L, 0, q, c, wa);
    __syncthreads();

    const int rows = min(CSPLIT_TH, h - ty * CSPLIT_TH);
    const int gx_lane = tx * TW + 2 * c;
    // first pixel of the lane's windows: staged column shx + 2c  ->  word (shx - po) / 2 + c
    const unsigned int *lane_base = planes + (shx - po) / 2 + c;

    for (int g0 = 0; g0 < L; g0 += 8) {
        if (g0 > 0) split_weights<G, KS, true>(W, L, g0, q, c, wa);
        // uniform per workgroup: every store of this pass is an aligned float2 (w even: pairs never straddle the edge)
        const bool fast = (w & 1) == 0 && (((uintptr_t)out) & 7) == 0 && g0 + 8 <= L;
        const int nfull = min(NBX, (w - tx * TW) / CSPLIT_XB);   // column blocks of this tile fully inside the image
        // lane (q,c) ends with planes g0+2q (acc[0..1]) and g0+2q+1 (acc[2..3]) at columns x, x+1
        const int ga = g0 + 2 * q;
        for (int r = wave; r < rows; r += 4) {
            floatx4 acc[1][NBX];
            split_rows<G, NBX, 1>(lane_base + r * G::PWORDS, 0, G::PLANE, toff, wa, acc);
            const int gy = ty * CSPLIT_TH + r;
            float *dst = out + (n * L + ga) * P + (int64_t)gy * w + gx_lane;
            if (fast) {
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int b = 0; b < NBX; ++b)
                        if (b < nfull || gx_lane + b * CSPLIT_XB < w)
                            *reinterpret_cast<float2 *>(dst + e * P + b * CSPLIT_XB) =
                                make_float2(acc[0][b][2 * e], acc[0][b][2 * e + 1]);
            } else {
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    if (ga + e >= L) continue;
#pragma unroll
                    for (int b = 0; b < NBX; ++b) {
                        const int gx = gx_lane + b * CSPLIT_XB;
                        if (gx < w) dst[e * P + b * CSPLIT_XB] = acc[0][b][2 * e];
                        if (gx + 1 < w) dst[e * P + b * CSPLIT_XB + 1] = acc[0][b][2 * e + 1];
                    }
                }
            }
        }
    }
}

template <int KS, int NBX>
static void conv_split_launch_nbx(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L,
                                  float *out)
{
    const int tiles_x = (w + NBX * CSPLIT_XB - 1) / (NBX * CSPLIT_XB);
    const int tiles_y = (h + CSPLIT_TH - 1) / CSPLIT_TH;
    const int64_t tiles = (int64_t)tiles_x * tiles_y;
    const int64_t per_launch = std::max<int64_t>(1, ((int64_t)1 << 30) / tiles);   // grid.x stays below 2^31
    for (int64_t n0 = 0; n0 < n; n0 += per_launch) {
        const int64_t nb = std::min(per_launch, n - n0);
        hipLaunchKernelGGL((conv_split_kernel<KS, NBX>), dim3((unsigned)(nb * tiles)), dim3(CSPLIT_THREADS), 0,
                           ctx->stream, in + n0 * (int64_t)h * w, h, w, W, L, out + n0 * L * (int64_t)h * w, tiles_x,
                           tiles_y);
    }
}

template <int KS>
static int conv_split_launch(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L,
                             float *out)
{
    // equal-width tiles of at most CSPLIT_MAX_NBX column blocks
    const int xblocks = (w + CSPLIT_XB - 1) / CSPLIT_XB;
    const int tiles_x = (xblocks + CSPLIT_MAX_NBX - 1) / CSPLIT_MAX_NBX;
    const int nbx = (xblocks + tiles_x - 1) / tiles_x;
    switch (nbx) {
        case 1: conv_split_launch_nbx<KS, 1>(ctx, in, n, h, w, W, L, out); break;
        case 2: conv_split_launch_nbx<KS, 2>(ctx, in, n, h, w, W, L, out); break;
        case 3: conv_split_launch_nbx<KS, 3>(ctx, in, n, h, w, W, L, out); break;
        default: conv_split_launch_nbx<KS, 4>(ctx, in, n, h, w, W, L, out); break;
    }
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int launch_conv_split(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L,
                      float *out)
{
    ProfScope prof(ctx, DDCCA_K_CONV);
    switch (k) {
        case 3: return conv_split_launch<3>(ctx, in, n, h, w, W, L, out);
        case 5: return conv_split_launch<5>(ctx, in, n, h, w, W, L, out);
        case 7: return conv_split_launch<7>(ctx, in, n, h, w, W, L, out);
        case 9: return conv_split_launch<9>(ctx, in, n, h, w, W, L, out);
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
}

}  // namespace ddcca
