// Lag-structured accumulation of the patch Gram (Section II-A matrices; an algebraic shortcut the paper does not
// use).  With the images extended by zeros, entry (a, b) of the raw patch Gram summed over ALL patch centres of
// the plane depends only on the lag between the two taps:
//     sum_p X[p + s_a] X'[p + s_b] = R_{s_b - s_a},    R_d = sum_u X[u] X'[u + d],
// (2k-1)^2 lag correlations per view pair instead of k^4 entries.  The sum wanted runs over the patch centres
// inside the image only; the centres outside it whose window still touches the image lie in a frame of width
// r, a few per cent of all patches, and their Gram is accumulated by the dense kernel (ring mode) and
// subtracted.  Everything else downstream (centre-pixel form, H M H export, solve) is unchanged:
// lag_to_stacked_kernel writes  sum y y^T  for y = x - x_centre in the layout of the dense kernel's slots from
//     S_y[a][b] = R(s_b - s_a) - R(s_c - s_a) - R(s_b - s_c) + R(0)          (c = the centre tap).
//
// The lag correlations run on v_mfma_f32_16x16x4_f32, one image row at a time: rows of the matrix instruction =
// horizontal lag, columns = vertical lag, K = 4 consecutive pixels x' of the row:
//     A[dx][x'] = X[y][x' - dx],   B[x'][dy] = X'[y + dy][x'],   D[dx][dy] += sum_x' A B.
// Three products per step (view 1 x view 1, 2 x 2, 1 x 2) against 21 / 6 tiles of the dense kernel at k = 7 / 5.
// The raw products carry the DC level of the images, which the differences to the centre pixel of the dense
// kernel do not, so the fp32 accumulators are added to fp64 registers after every image row.
// k <= 7 only: 2k-1 lags per axis have to fit the 16 rows of the instruction.
#include "ddcca_internal.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int LAG_THREADS = 256;
constexpr int LAG_TH = 16;                 // image rows per tile
constexpr int LAG_TW_MAX = 128;            // image columns per tile (multiple of 4)
constexpr int LAG_E = 3 * 256;             // doubles per slot: three 16 x 16 tiles (11, 22, 12) in accumulator layout

struct LagParams {
    const float *v1, *v2;                  // [n_maps][h][w]
    int h, w, tiles_x, tiles_y, tw;
    int pitch, view_stride;                // LDS floats per tile row / per view
    int64_t n_items;                       // n_maps * tiles_y * tiles_x
    double *slots;                         // [grid][LAG_E]
    int slots_valid;                       // slots below this hold earlier sums
};

// One workgroup walks a contiguous range of (map, tile) items.  A tile is LAG_TH image rows x tw columns with a
// halo of K = k-1 on every side (zeros outside the image), both views.  Wavefront w owns tile rows w, w+4, ...
template <int KS, bool CROSS>
__global__ __launch_bounds__(LAG_THREADS) void lag_gram_kernel(LagParams p)
{
    constexpr int K = KS - 1;              // largest lag
    constexpr int NL = 2 * K + 1;          // lags per axis
    static_assert(NL <= 16, "the lags of one axis must fit the 16 rows of the matrix instruction");
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = min(lane & 15, NL - 1);  // lag index of this lane's row / column (rows past NL repeat the last)
    const int kk = lane >> 4;
    const int PH = LAG_TH + 2 * K, PW = p.tw + 2 * K;
    const int64_t per = p.n_items / gridDim.x, extra = p.n_items % gridDim.x;
    const int64_t first = blockIdx.x * per + min((int64_t)blockIdx.x, extra);
    const int64_t count = per + (blockIdx.x < extra ? 1 : 0);
    const int tiles = p.tiles_x * p.tiles_y;
    const int64_t P = (int64_t)p.h * p.w;
    double accd[3][4];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) accd[t][v] = 0.0;
    // A operand: image row y = tile row y + K, column x' - dx = tile column x' + K - (m - K)
    // B operand: image row y + dy = tile row y + m, column x' = tile column x' + K
    const int a_off = K * p.pitch + kk - m + 2 * K;
    const int b_off = m * p.pitch + kk + K;
    for (int64_t it = 0; it < count; ++it) {
        const int64_t item = first + it;
        const int64_t mp = item / tiles;
        const int t = (int)(item - mp * tiles);
        const int ty = t / p.tiles_x, tx = t - ty * p.tiles_x;
        const int gy0 = ty * LAG_TH - K, gx0 = tx * p.tw - K;
        __syncthreads();                              // the previous tile is no longer read
        const float *s1 = p.v1 + mp * P, *s2 = p.v2 + mp * P;
        // wavefront w stages tile rows w, w+4, ...; lane l the columns l, l+64, ...
        for (int yy = wave; yy < PH; yy += 4) {
            const int gy = gy0 + yy;
            const bool yok = gy >= 0 && gy < p.h;
            const int64_t ro = (int64_t)gy * p.w;
            for (int xx = lane; xx < PW; xx += 64) {
                const int gx = gx0 + xx;
                float a = 0.f, b = 0.f;
                if (yok && gx >= 0 && gx < p.w) {
                    a = s1[ro + gx];
                    b = s2[ro + gx];
                }
                lds[yy * p.pitch + xx] = a;
                lds[p.view_stride + yy * p.pitch + xx] = b;
            }
        }
        __syncthreads();
        const int rows = min(LAG_TH, p.h - ty * LAG_TH);
        const int cols = min(p.tw, p.w - tx * p.tw);
        const int steps = (cols + 3) >> 2;            // tw is a multiple of 4: columns past the image hold zeros
        for (int y = wave; y < rows; y += 4) {
            const float *ra1 = lds + y * p.pitch + a_off, *rb1 = lds + y * p.pitch + b_off;
            const float *ra2 = ra1 + p.view_stride, *rb2 = rb1 + p.view_stride;
            floatx4 c11 = {0.f, 0.f, 0.f, 0.f}, c22 = {0.f, 0.f, 0.f, 0.f}, c12 = {0.f, 0.f, 0.f, 0.f};
            // two steps per iteration: their operands pair up in two-address LDS reads
            int s = 0;
            for (; s + 1 < steps; s += 2) {
                const float a1 = ra1[4 * s], a1n = ra1[4 * s + 4], b2 = rb2[4 * s], b2n = rb2[4 * s + 4];
                if (!CROSS) {
                    const float a2 = ra2[4 * s], a2n = ra2[4 * s + 4], b1 = rb1[4 * s], b1n = rb1[4 * s + 4];
                    c11 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, c11, 0, 0, 0);
                    c22 = __builtin_amdgcn_mfma_f32_16x16x4f32(a2, b2, c22, 0, 0, 0);
                    c12 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b2, c12, 0, 0, 0);
                    c11 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1n, b1n, c11, 0, 0, 0);
                    c22 = __builtin_amdgcn_mfma_f32_16x16x4f32(a2n, b2n, c22, 0, 0, 0);
                    c12 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1n, b2n, c12, 0, 0, 0);
                } else {
                    c12 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b2, c12, 0, 0, 0);
                    c12 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1n, b2n, c12, 0, 0, 0);
                }
            }
            if (s < steps) {
                const float a1 = ra1[4 * s], b2 = rb2[4 * s];
                if (!CROSS) {
                    const float a2 = ra2[4 * s], b1 = rb1[4 * s];
                    c11 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, c11, 0, 0, 0);
                    c22 = __builtin_amdgcn_mfma_f32_16x16x4f32(a2, b2, c22, 0, 0, 0);
                }
                c12 = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b2, c12, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (!CROSS) {
                    accd[0][v] += (double)c11[v];
                    accd[1][v] += (double)c22[v];
                }
                accd[2][v] += (double)c12[v];
            }
        }
    }
    // workgroup total in fp64: the wavefronts add in order, then the slot takes it
    __syncthreads();
    double *st = reinterpret_cast<double *>(lds);
    for (int wv = 0; wv < 4; ++wv) {
        if (wave == wv) {
#pragma unroll
            for (int t = 0; t < 3; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int e = (t * 4 + v) * 64 + lane;
                    st[e] = (wv == 0 ? 0.0 : st[e]) + accd[t][v];
                }
        }
        __syncthreads();
    }
    double *slot = p.slots + (size_t)blockIdx.x * LAG_E;
    const bool rmw = (int)blockIdx.x < p.slots_valid;
    for (int e = threadIdx.x; e < LAG_E; e += LAG_THREADS) slot[e] = (rmw ? slot[e] : 0.0) + st[e];
}

// R_d of one view pair from a reduced slot: accumulator layout, row = horizontal lag index, column = vertical.
__device__ __forceinline__ double lag_value(const double *R, int type, int dy, int dx, int K)
{
    const int ix = dx + K, iy = dy + K;
    return R[(type * 4 + (ix & 3)) * 64 + 16 * (ix >> 2) + iy];
}

// S_x[(d,a)][(d',b)] = sum over all patch centres of X_d[p + s_a] X_d'[p + s_b] = R^{dd'}(s_b - s_a);
// R^{21}(d) = R^{12}(-d).
__device__ __forceinline__ double lag_raw(const double *R, int d, int a, int d2, int b, int ks, int K, bool cross)
{
    const int ay = a / ks, ax = a - ay * ks, by = b / ks, bx = b - by * ks;
    if (d == d2) return cross ? 0.0 : lag_value(R, d, by - ay, bx - ax, K);
    return d == 0 ? lag_value(R, 2, by - ay, bx - ax, K) : lag_value(R, 2, ay - by, ax - bx, K);
}

// stacked[e] = (Gram of y = x - x_centre over all patch centres of the plane, from the lag correlations R)
//              - stacked[e] (the same Gram over the frame outside the image, from the dense kernel's ring mode),
// element e in the slot layout of the dense kernel: tile (bi, bj) number t, register v, lane l hold entry
// (16 bi + 4 (l / 16) + v, 16 bj + l % 16) of the stacked 2(D-1) x 2(D-1) matrix.
__global__ void lag_to_stacked_kernel(const double *__restrict__ R, double *__restrict__ stacked, int ks, int cross)
{
    const int D = ks * ks, DR = D - 1, CEN = (D - 1) / 2, K = ks - 1;
    const int NB = (2 * DR) / 16, NT = NB * (NB + 1) / 2;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= NT * 256) return;
    const int t = e >> 8, v = (e >> 6) & 3, l = e & 63;
    int bi = 0, rem = t;
    while (rem >= NB - bi) {
        rem -= NB - bi;
        ++bi;
    }
    const int bj = bi + rem;
    const int row = 16 * bi + 4 * (l >> 4) + v, col = 16 * bj + (l & 15);
    const int d = row >= DR ? 1 : 0, d2 = col >= DR ? 1 : 0;
    const int ar = row - d * DR, br = col - d2 * DR;
    const int a = ar >= CEN ? ar + 1 : ar, b = br >= CEN ? br + 1 : br;
    const bool cr = cross != 0;
    const double s = lag_raw(R, d, a, d2, b, ks, K, cr) - lag_raw(R, d, a, d2, CEN, ks, K, cr) -
                     lag_raw(R, d, CEN, d2, b, ks, K, cr) + lag_raw(R, d, CEN, d2, CEN, ks, K, cr);
    stacked[e] = s - stacked[e];
}

bool lag_supported(int k) { return 2 * (k - 1) + 1 <= 16; }
int max_lag_slots(ddcca_ctx *ctx) { return ctx->n_cu * 6; }

template <int KS>
static void lag_launch(ddcca_ctx *ctx, const LagParams &p, int grid, size_t lds, bool cross)
{
    if (cross) hipLaunchKernelGGL((lag_gram_kernel<KS, true>), dim3(grid), dim3(LAG_THREADS), lds, ctx->stream, p);
    else hipLaunchKernelGGL((lag_gram_kernel<KS, false>), dim3(grid), dim3(LAG_THREADS), lds, ctx->stream, p);
}

int launch_lag_gram(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t n_maps, int h, int w, int k,
                    bool cross_only, double *slots, int max_slots, int *slots_valid)
{
    ProfScope prof(ctx, cross_only ? DDCCA_K_GRAM_CROSS : DDCCA_K_GRAM);
    if (!lag_supported(k)) return fail(ctx, DDCCA_EINVAL, "the lag-structured Gram needs k <= 7");
    LagParams p;
    p.v1 = v1; p.v2 = v2; p.h = h; p.w = w;
    const int K = k - 1;
    const int w4 = (w + 3) & ~3;
    const int ntx = (w4 + LAG_TW_MAX - 1) / LAG_TW_MAX;
    p.tw = (((w4 + ntx - 1) / ntx) + 3) & ~3;
    p.tiles_x = (w + p.tw - 1) / p.tw;
    p.tiles_y = (h + LAG_TH - 1) / LAG_TH;
    p.n_items = n_maps * p.tiles_x * p.tiles_y;
    // row pitch: tile width + halo, congruent to 17 mod 32 so that the rows y .. y + 2K a B operand reads fall
    // into different banks
    int pitch = p.tw + 2 * K + 4;
    while (pitch % 32 != 17) ++pitch;
    p.pitch = pitch;
    p.view_stride = (LAG_TH + 2 * K) * pitch + 8;
    const size_t lds = std::max<size_t>((size_t)2 * p.view_stride * sizeof(float), (size_t)LAG_E * sizeof(double));
    p.slots = slots;
    p.slots_valid = *slots_valid;
    const int grid = (int)std::min<int64_t>(max_slots, std::max<int64_t>(p.n_items, 1));
    switch (k) {
        case 3: lag_launch<3>(ctx, p, grid, lds, cross_only); break;
        case 5: lag_launch<5>(ctx, p, grid, lds, cross_only); break;
        case 7: lag_launch<7>(ctx, p, grid, lds, cross_only); break;
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
    DDCCA_HIP(ctx, hipGetLastError());
    *slots_valid = std::max(*slots_valid, grid);
    return DDCCA_OK;
}

int launch_lag_to_stacked(ddcca_ctx *ctx, const double *R, double *stacked, int k, bool cross_only)
{
    ProfScope prof(ctx, DDCCA_K_REDUCE);
    const int E = gram_tiles(k) * 256;
    hipLaunchKernelGGL(lag_to_stacked_kernel, dim3((E + 255) / 256), dim3(256), 0, ctx->stream, R, stacked, k,
                       cross_only ? 1 : 0);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
