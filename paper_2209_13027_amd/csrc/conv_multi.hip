// Stage convolution (Eq. 6): every input image correlated with the L k*k filters of the
// stage, zero padding, same size.  out[n][g][y][x] = sum W[g][dy][dx] in[n][y+dy-r][x+dx-r].
//
// The contraction over the k*k taps for 8 filters at once is dense, so it runs on
// v_mfma_f32_16x16x4_f32 as an implicit GEMM without an im2col buffer:
//   rows (A operand)  : (filter g, x-shift s), g < 8, s in {0,1}      -> 16 rows
//   cols (B operand)  : 16 pixel positions x = x0 + 2c of one image row
//   K                 : taps (dy, dx'), dx' in 0..k  (k+1 columns: both shifts fit)
//   A[(g,s)][(dy,dx')] = W[g][dy][dx'-s]  (0 when dx'-s is outside 0..k-1)
//   B[(dy,dx')][c]     = in[y+dy-r][x0+2c+dx'-r]
//   => D[(g,s)][c]     = out[g][y][x0+2c+s]
// Packing two x-shifts of 8 filters into the 16 rows keeps the matrix unit k/(k+1) busy
// (a plain 8-wide filter dimension would leave half of it idle).  The A operand depends
// only on the filters, so it lives in registers for the whole kernel; the B operand is one
// LDS read per MFMA from the staged input tile.  Each lane ends up with (x, x+1) pairs of
// one output plane, written as 8-byte stores that form 128-byte row segments.
#include "ddcca_internal.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int CONV_THREADS = 256;
constexpr int CONV_TH = 32;        // tile rows per workgroup
constexpr int CONV_XB = 32;        // pixels per MFMA column block (16 columns x 2 shifts)
constexpr int CONV_MAX_NBX = 4;    // column blocks per tile (tile width <= 128)

template <int KS>
__global__ __launch_bounds__(CONV_THREADS) void conv_mfma_kernel(const float *__restrict__ in, int h, int w,
                                                                 const float *__restrict__ W, int L,
                                                                 float *__restrict__ out, int tiles_x, int tiles_y,
                                                                 int nbx, int pitch)
{
    constexpr int R = (KS - 1) / 2;
    constexpr int KW = KS + 1;                    // tap columns incl. the shift
    constexpr int TAPS = KS * KW;
    constexpr int KK = (TAPS + 3) / 4;            // MFMA steps
    constexpr int PH = CONV_TH + 2 * R;
    extern __shared__ float tile[];               // [PH][pitch]
    const int tiles = tiles_x * tiles_y;
    const int64_t n = blockIdx.x / tiles;
    const int t = blockIdx.x - (int)n * tiles;
    const int tx = t % tiles_x, ty = t / tiles_x;
    const int tw = nbx * CONV_XB;
    const int pw = tw + 2 * R + 1;                // +1: the odd shift reads one more column
    const int64_t P = (int64_t)h * w;
    const float *src = in + n * P;
    const int gy0 = ty * CONV_TH - R, gx0 = tx * tw - R;
    for (int e = threadIdx.x; e < PH * pw; e += CONV_THREADS) {
        const int yy = e / pw, xx = e - yy * pw;
        const int gy = gy0 + yy, gx = gx0 + xx;
        float v = 0.f;
        if (gy >= 0 && gy < h && gx >= 0 && gx < w) v = src[(int64_t)gy * w + gx];
        tile[yy * pitch + xx] = v;
    }

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c = lane & 15;
    // B-operand window offsets of this lane's tap (4*kk + q) for every step
    int toff[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int tap = 4 * kk + q;
        const int dy = tap / KW, dx = tap - dy * KW;
        toff[kk] = tap < TAPS ? dy * pitch + dx : 0;
    }
    __syncthreads();

    const int rows = min(CONV_TH, h - ty * CONV_TH);
    const int units = rows * nbx;                 // (row, column block) pairs of this tile
    const bool out_al8 = (((uintptr_t)out) & 7) == 0;

    for (int g0 = 0; g0 < L; g0 += 8) {
        // A operand: row (g,s) = lane%16, tap 4*kk + lane/16
        float wa[KK];
        {
            const int g = g0 + (c >> 1), s = c & 1;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const int tap = 4 * kk + q;
                const int dy = tap / KW, dxw = tap - dy * KW - s;
                float v = 0.f;
                if (tap < TAPS && dxw >= 0 && dxw < KS && g < L) v = W[(g * KS + dy) * KS + dxw];
                wa[kk] = v;
            }
        }
        for (int u = wave; u < units; u += 8) {
            // two independent units per iteration: u and u+4
            const int u1 = u + 4;
            const bool has1 = u1 < units;
            const int r0 = u / nbx, b0 = u - r0 * nbx;
            const int r1 = has1 ? u1 / nbx : r0, b1 = has1 ? u1 - r1 * nbx : b0;
            const float *p0 = tile + r0 * pitch + b0 * CONV_XB + 2 * c;
            const float *p1 = tile + r1 * pitch + b1 * CONV_XB + 2 * c;
            floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const float x0 = p0[toff[kk]];
                const float x1 = p1[toff[kk]];
                acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[kk], x0, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[kk], x1, acc1, 0, 0, 0);
            }
            // lane (q,c) holds filter g0+2q (acc[0..1]) and g0+2q+1 (acc[2..3]) at x, x+1
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const floatx4 acc = half ? acc1 : acc0;
                if (half && !has1) break;
                const int rr = half ? r1 : r0, bb = half ? b1 : b0;
                const int gy = ty * CONV_TH + rr;
                const int gx = tx * tw + bb * CONV_XB + 2 * c;
                if (gx >= w) continue;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    const int g = g0 + 2 * q + e;
                    if (g >= L) continue;
                    const int64_t o = (n * L + g) * P + (int64_t)gy * w + gx;
                    const float a = acc[2 * e], b = acc[2 * e + 1];
                    if (gx + 1 < w && out_al8 && (o & 1) == 0) {
                        *reinterpret_cast<float2 *>(out + o) = make_float2(a, b);
                    } else {
                        out[o] = a;
                        if (gx + 1 < w) out[o + 1] = b;
                    }
                }
            }
        }
    }
}

template <int KS>
static int conv_launch(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L, float *out)
{
    constexpr int R = (KS - 1) / 2;
    const int xblocks = (w + CONV_XB - 1) / CONV_XB;
    const int tiles_x = (xblocks + CONV_MAX_NBX - 1) / CONV_MAX_NBX;
    const int nbx = (xblocks + tiles_x - 1) / tiles_x;          // equal-width tiles
    const int tiles_y = (h + CONV_TH - 1) / CONV_TH;
    int pitch = nbx * CONV_XB + 2 * R + 1;
    pitch += (pitch & 1) ? 0 : 1;                                // odd pitch: rows start in different banks
    const size_t lds = (size_t)(CONV_TH + 2 * R) * pitch * sizeof(float);
    const int64_t tiles = (int64_t)tiles_x * tiles_y;
    const int64_t per_launch = std::max<int64_t>(1, ((int64_t)1 << 30) / tiles);   // grid.x stays below 2^31
    for (int64_t n0 = 0; n0 < n; n0 += per_launch) {
        const int64_t nb = std::min(per_launch, n - n0);
        hipLaunchKernelGGL(conv_mfma_kernel<KS>, dim3((unsigned)(nb * tiles)), dim3(CONV_THREADS), lds, ctx->stream,
                           in + n0 * (int64_t)h * w, h, w, W, L, out + n0 * L * (int64_t)h * w, tiles_x, tiles_y, nbx,
                           pitch);
    }
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int launch_conv(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L, float *out)
{
    ProfScope prof(ctx, DDCCA_K_CONV);
    switch (k) {
        case 3: return conv_launch<3>(ctx, in, n, h, w, W, L, out);
        case 5: return conv_launch<5>(ctx, in, n, h, w, W, L, out);
        case 7: return conv_launch<7>(ctx, in, n, h, w, W, L, out);
        case 9: return conv_launch<9>(ctx, in, n, h, w, W, L, out);
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
}

}  // namespace ddcca
