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
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int CONV_THREADS = 256;
constexpr int CONV_TH = 32;        // tile rows per workgroup
constexpr int CONV_XB = 32;        // pixels per MFMA column block (16 columns x 2 shifts)
constexpr int CONV_MAX_NBX = 4;    // column blocks per tile (tile width <= 128)

// One workgroup: a 32-row x (32*NBX)-column output tile of one image, all L filters.
// Wavefront w owns tile rows w, w+4, ...; for one row it runs NBX independent accumulator
// chains (one per 32-pixel column block), so one window-offset add serves NBX LDS reads and
// NBX MFMAs.
template <int KS, int NBX>
__global__ __launch_bounds__(CONV_THREADS) void conv_mfma_kernel(const float *__restrict__ in, int h, int w,
                                                                 const float *__restrict__ W, int L,
                                                                 float *__restrict__ out, int tiles_x, int tiles_y)
{
    constexpr int R = (KS - 1) / 2;
    constexpr int KW = KS + 1;                    // tap columns incl. the shift
    constexpr int TAPS = KS * KW;
    constexpr int KK = (TAPS + 3) / 4;            // MFMA steps
    constexpr int PH = CONV_TH + 2 * R;
    constexpr int TW = NBX * CONV_XB;
    constexpr int PW = TW + 2 * R + 1;            // +1: the odd shift reads one more column
    constexpr int PITCH = PW | 1;                 // odd pitch: rows start in different banks
    __shared__ float tile[PH * PITCH];
    const int tiles = tiles_x * tiles_y;
    const int64_t n = blockIdx.x / tiles;
    const int t = blockIdx.x - (int)n * tiles;
    const int tx = t % tiles_x, ty = t / tiles_x;
    const int64_t P = (int64_t)h * w;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    {
        // stage the input tile with its halo (PW is a compile-time constant: cheap index split)
        const float *src = in + n * P;
        const int gy0 = ty * CONV_TH - R, gx0 = tx * TW - R;
#pragma unroll 4
        for (int e = threadIdx.x; e < PH * PW; e += CONV_THREADS) {
            const int yy = e / PW, xx = e - yy * PW;
            const int gy = gy0 + yy, gx = gx0 + xx;
            float v = 0.f;
            if (gy >= 0 && gy < h && gx >= 0 && gx < w) v = src[(int64_t)gy * w + gx];
            tile[yy * PITCH + xx] = v;
        }
    }
    const int q = lane >> 4, c = lane & 15;
    // B-operand window offsets of this lane's tap (4*kk + q) for every step
    int toff[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int tap = 4 * kk + q;
        const int dy = tap / KW, dx = tap - dy * KW;
        toff[kk] = tap < TAPS ? dy * PITCH + dx : 0;
    }
    // A operand: row (g,s) = lane%16, tap 4*kk + lane/16; fetched for the first filter group while
    // the tile loads are still in flight
    float wa[KK];
    auto load_weights = [&](int g0) {
        const int g = g0 + (c >> 1), s = c & 1;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int tap = 4 * kk + q;
            const int dy = tap / KW, dxw = tap - dy * KW - s;
            float v = 0.f;
            if (tap < TAPS && dxw >= 0 && dxw < KS && g < L) v = W[(g * KS + dy) * KS + dxw];
            wa[kk] = v;
        }
    };
    load_weights(0);
    __syncthreads();

    const int rows = min(CONV_TH, h - ty * CONV_TH);
    const int gx_lane = tx * TW + 2 * c;

    for (int g0 = 0; g0 < L; g0 += 8) {
        if (g0 > 0) load_weights(g0);             // the first group was fetched before the barrier
        // uniform per workgroup: every store of this pass is an aligned float2 (w even: pairs never straddle the edge)
        const bool fast = (w & 1) == 0 && (((uintptr_t)out) & 7) == 0 && g0 + 8 <= L;
        // uniform: rows of a multiple of 32 pixels on a 128-byte aligned base (rows that split cache lines lose by the hint)
        const bool streaming = (w & 31) == 0 && (((uintptr_t)out) & 127) == 0;
        const int nfull = min(NBX, (w - tx * TW) / CONV_XB);   // column blocks of this tile fully inside the image
        // lane (q,c) ends with planes g0+2q (acc[0..1]) and g0+2q+1 (acc[2..3]) at columns x, x+1
        const int ga = g0 + 2 * q;
        for (int r = wave; r < rows; r += 4) {
            const float *prow = tile + r * PITCH + 2 * c;
            floatx4 acc[NBX];
#pragma unroll
            for (int b = 0; b < NBX; ++b) acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const float *pk = prow + toff[kk];
#pragma unroll
                for (int b = 0; b < NBX; ++b)
                    acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[kk], pk[b * CONV_XB], acc[b], 0, 0, 0);
            }
            const int gy = ty * CONV_TH + r;
            float *dst = out + (n * L + ga) * P + (int64_t)gy * w + gx_lane;
            if (fast && streaming) {
                // the same stores with the non-temporal hint: the 128-byte segments are whole, aligned cache lines
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int b = 0; b < NBX; ++b)
                        if (b < nfull || gx_lane + b * CONV_XB < w)
                            __builtin_nontemporal_store(floatx2{acc[b][2 * e], acc[b][2 * e + 1]},
                                                        reinterpret_cast<floatx2 *>(dst + e * P + b * CONV_XB));
            } else if (fast) {
                // 8-byte aligned rows, all 8 planes exist: column blocks fully inside the image are
                // stored unconditionally, the ragged one (if any) per pixel pair
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int b = 0; b < NBX; ++b)
                        if (b < nfull || gx_lane + b * CONV_XB < w)
                            *reinterpret_cast<float2 *>(dst + e * P + b * CONV_XB) =
                                make_float2(acc[b][2 * e], acc[b][2 * e + 1]);
            } else {
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    if (ga + e >= L) continue;
#pragma unroll
                    for (int b = 0; b < NBX; ++b) {
                        const int gx = gx_lane + b * CONV_XB;
                        if (gx < w) dst[e * P + b * CONV_XB] = acc[b][2 * e];
                        if (gx + 1 < w) dst[e * P + b * CONV_XB + 1] = acc[b][2 * e + 1];
                    }
                }
            }
        }
    }
}

template <int KS, int NBX>
static void conv_launch_nbx(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L, float *out)
{
    const int tiles_x = (w + NBX * CONV_XB - 1) / (NBX * CONV_XB);
    const int tiles_y = (h + CONV_TH - 1) / CONV_TH;
    const int64_t tiles = (int64_t)tiles_x * tiles_y;
    const int64_t per_launch = std::max<int64_t>(1, ((int64_t)1 << 30) / tiles);   // grid.x stays below 2^31
    for (int64_t n0 = 0; n0 < n; n0 += per_launch) {
        const int64_t nb = std::min(per_launch, n - n0);
        hipLaunchKernelGGL((conv_mfma_kernel<KS, NBX>), dim3((unsigned)(nb * tiles)), dim3(CONV_THREADS), 0,
                           ctx->stream, in + n0 * (int64_t)h * w, h, w, W, L, out + n0 * L * (int64_t)h * w, tiles_x,
                           tiles_y);
    }
}

template <int KS>
static int conv_launch(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L, float *out)
{
    // equal-width tiles of at most CONV_MAX_NBX column blocks
    const int xblocks = (w + CONV_XB - 1) / CONV_XB;
    const int tiles_x = (xblocks + CONV_MAX_NBX - 1) / CONV_MAX_NBX;
    const int nbx = (xblocks + tiles_x - 1) / tiles_x;
    switch (nbx) {
        case 1: conv_launch_nbx<KS, 1>(ctx, in, n, h, w, W, L, out); break;
        case 2: conv_launch_nbx<KS, 2>(ctx, in, n, h, w, W, L, out); break;
        case 3: conv_launch_nbx<KS, 3>(ctx, in, n, h, w, W, L, out); break;
        default: conv_launch_nbx<KS, 4>(ctx, in, n, h, w, W, L, out); break;
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
