// Stage convolution (Eq. 6): every input image correlated with the L k*k filters of the
// stage, zero padding, same size.  One workgroup stages an input tile with its halo in
// LDS once and produces all L output planes from it, so the input is read once and the
// L outputs leave as full rows of the tile.
#include "ddcca_internal.h"

namespace ddcca {

constexpr int CONV_TH = 16;   // tile rows
constexpr int CONV_TW = 64;   // tile columns (one wavefront per tile row group)

// Thread t of the 256: column x = t % 64, rows y = t / 64 + 4*j (j = 0..3).
template <int KS, int LG>   // LG: filters handled per pass (accumulators per pixel)
__global__ __launch_bounds__(256) void conv_direct_kernel(const float *__restrict__ in, int h, int w,
                                                          const float *__restrict__ W, int L,
                                                          float *__restrict__ out, int tiles_x, int tiles_y)
{
    constexpr int R = (KS - 1) / 2;
    constexpr int PH = CONV_TH + 2 * R, PW = CONV_TW + 2 * R;
    constexpr int PITCH = PW + 1;
    __shared__ float tile[PH * PITCH];
    const int tiles = tiles_x * tiles_y;
    const int64_t n = blockIdx.x / tiles;
    const int t = blockIdx.x - (int)n * tiles;
    const int tx = t % tiles_x, ty = t / tiles_x;
    const int64_t P = (int64_t)h * w;
    const float *src = in + n * P;
    const int gy0 = ty * CONV_TH - R, gx0 = tx * CONV_TW - R;
    for (int e = threadIdx.x; e < PH * PW; e += 256) {
        const int yy = e / PW, xx = e - yy * PW;
        const int gy = gy0 + yy, gx = gx0 + xx;
        float v = 0.f;
        if (gy >= 0 && gy < h && gx >= 0 && gx < w) v = src[(int64_t)gy * w + gx];
        tile[yy * PITCH + xx] = v;
    }
    __syncthreads();
    const int lx = threadIdx.x & 63, ly = threadIdx.x >> 6;
    const int gx = tx * CONV_TW + lx;
    for (int g0 = 0; g0 < L; g0 += LG) {
        float acc[4][LG];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int g = 0; g < LG; ++g) acc[j][g] = 0.f;
#pragma unroll
        for (int dy = 0; dy < KS; ++dy)
#pragma unroll
            for (int dx = 0; dx < KS; ++dx) {
                float wv[LG];
#pragma unroll
                for (int g = 0; g < LG; ++g) wv[g] = (g0 + g < L) ? W[((g0 + g) * KS + dy) * KS + dx] : 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p = tile[(ly + 4 * j + dy) * PITCH + lx + dx];
#pragma unroll
                    for (int g = 0; g < LG; ++g) acc[j][g] = fmaf(wv[g], p, acc[j][g]);
                }
            }
        if (gx < w) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int gy = ty * CONV_TH + ly + 4 * j;
                if (gy < h) {
#pragma unroll
                    for (int g = 0; g < LG; ++g)
                        if (g0 + g < L) out[(n * L + g0 + g) * P + (int64_t)gy * w + gx] = acc[j][g];
                }
            }
        }
    }
}

template <int KS>
static void conv_launch(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L, float *out)
{
    const int tiles_x = (w + CONV_TW - 1) / CONV_TW, tiles_y = (h + CONV_TH - 1) / CONV_TH;
    const int64_t tiles = (int64_t)tiles_x * tiles_y;
    const int64_t per_launch = std::max<int64_t>(1, ((int64_t)1 << 30) / tiles);   // grid.x stays below 2^31
    for (int64_t n0 = 0; n0 < n; n0 += per_launch) {
        const int64_t nb = std::min(per_launch, n - n0);
        hipLaunchKernelGGL((conv_direct_kernel<KS, 8>), dim3((unsigned)(nb * tiles)), dim3(256), 0, ctx->stream,
                           in + n0 * (int64_t)h * w, h, w, W, L, out + n0 * L * (int64_t)h * w, tiles_x, tiles_y);
    }
}

int launch_conv(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L, float *out)
{
    ProfScope prof(ctx, DDCCA_K_CONV);
    switch (k) {
        case 3: conv_launch<3>(ctx, in, n, h, w, W, L, out); break;
        case 5: conv_launch<5>(ctx, in, n, h, w, W, L, out); break;
        case 7: conv_launch<7>(ctx, in, n, h, w, W, L, out); break;
        case 9: conv_launch<9>(ctx, in, n, h, w, W, L, out); break;
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
