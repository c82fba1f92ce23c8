// Patch Gram accumulation (Section II-A matrices, Section III Eq. 15 batching):
//   for every pixel of every map pair, z = [x1; x2] (the two mean-removed k*k patches,
//   2D entries) and  G += z z^T.
// The patch matrix of Eq. 1 is never formed: an image tile with its halo is staged in
// LDS, the per-patch means are computed once per tile, and the MFMA operands are read
// straight from the tile with a per-lane window offset.  The contraction runs on
// v_mfma_f32_16x16x4_f32 (K = 4 consecutive patches of a tile row per instruction).
// For a Gram the A operand of row block bi and the B operand of column block bj have
// the same register layout (lane l: stacked row 16*b + l%16, patch l/16), so one LDS
// read per block feeds every tile of that block row and block column.
#include "ddcca_internal.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int GRAM_THREADS = 256;          // 4 wavefronts; each owns every 4th patch row of the tile
constexpr int GRAM_TH = 16;                // patch rows per tile
constexpr int GRAM_TW_MAX = 128;           // patch columns per tile (multiple of 4)

struct GramParams {
    const float *v1, *v2;                  // [n_maps][h][w]
    int64_t n_items;                       // n_maps * tiles_y * tiles_x
    int h, w, tiles_x, tiles_y, tw;        // tw: tile width in patches
    int pitch;                             // LDS row pitch of the pixel tile (floats)
    int view_stride;                       // LDS floats per view's pixel tile
    int flush_items;                       // items between fp64 flushes
    double *slots;                         // [n_slots][NT*256]
    int slots_valid;                       // slots below this hold earlier partial sums
};

template <int KS>
struct GramGeom {
    static constexpr int D = KS * KS;
    static constexpr int R = (KS - 1) / 2;
    static constexpr int NB = (2 * D + 15) / 16;
    static constexpr int NT = NB * (NB + 1) / 2;
};

template <int KS>
__global__ __launch_bounds__(GRAM_THREADS) void patch_gram_kernel(GramParams p)
{
    using G = GramGeom<KS>;
    constexpr int D = G::D, R = G::R, NB = G::NB, NT = G::NT;
    extern __shared__ float lds[];
    float *pix = lds;                                     // [2][GRAM_TH + 2R][pitch]
    float *mean = lds + 2 * p.view_stride;                // [2][GRAM_TH][tw]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, i = lane & 15;
    const int mean_view_stride = GRAM_TH * p.tw;

    // per-lane operand offsets for each 16-row block of the stacked vector
    int pix_off[NB], mean_off[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        int row = 16 * b + i;
        if (row >= 2 * D) row = 0;                        // padding rows: any valid address; results unused
        const int view = row >= D ? 1 : 0;
        const int a = row - view * D;
        const int dy = a / KS, dx = a - dy * KS;
        pix_off[b] = view * p.view_stride + dy * p.pitch + dx + q;
        mean_off[b] = view * mean_view_stride + q;
    }

    floatx4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};

    // contiguous range of work items for this workgroup
    const int64_t per = p.n_items / gridDim.x, extra = p.n_items % gridDim.x;
    const int64_t first = blockIdx.x * per + min((int64_t)blockIdx.x, extra);
    const int64_t count = per + (blockIdx.x < extra ? 1 : 0);
    const int tiles = p.tiles_x * p.tiles_y;
    const int64_t P = (int64_t)p.h * p.w;
    const int slot = blockIdx.x * 4 + wave;
    double *my_slot = p.slots + (size_t)slot * NT * 256;
    bool rmw = slot < p.slots_valid;
    int since_flush = 0;
    constexpr int PH = GRAM_TH + 2 * R;
    const int pw = p.tw + 2 * R;

    for (int64_t it = 0; it < count; ++it) {
        const int64_t item = first + it;
        const int64_t m = item / tiles;
        const int t = (int)(item - m * tiles);
        const int ty = t / p.tiles_x, tx = t - ty * p.tiles_x;
        const int gy0 = ty * GRAM_TH - R, gx0 = tx * p.tw - R;
        __syncthreads();                                  // previous item's reads are done
        for (int e = threadIdx.x; e < PH * pw; e += GRAM_THREADS) {
            const int yy = e / pw, xx = e - yy * pw;
            const int gy = gy0 + yy, gx = gx0 + xx;
            float a = 0.f, b = 0.f;
            if (gy >= 0 && gy < p.h && gx >= 0 && gx < p.w) {
                const int64_t o = m * P + (int64_t)gy * p.w + gx;
                a = p.v1[o];
                b = p.v2[o];
            }
            pix[yy * p.pitch + xx] = a;
            pix[p.view_stride + yy * p.pitch + xx] = b;
        }
        __syncthreads();
        // per-patch means (zero padding counts as zeros)
        for (int e = threadIdx.x; e < 2 * GRAM_TH * p.tw; e += GRAM_THREADS) {
            const int view = e / (GRAM_TH * p.tw);
            const int r = e - view * GRAM_TH * p.tw;
            const int py = r / p.tw, px = r - py * p.tw;
            const float *src = pix + view * p.view_stride + py * p.pitch + px;
            float s = 0.f;
#pragma unroll
            for (int dy = 0; dy < KS; ++dy)
#pragma unroll
                for (int dx = 0; dx < KS; ++dx) s += src[dy * p.pitch + dx];
            mean[view * mean_view_stride + r] = s * (1.0f / D);
        }
        __syncthreads();

        const int rows = min(GRAM_TH, p.h - ty * GRAM_TH);
        const int cols = min(p.tw, p.w - tx * p.tw);
        const int full = cols >> 2, tail = cols & 3;
        for (int py = wave; py < rows; py += 4) {
            const float *prow = pix + py * p.pitch;
            const float *mrow = mean + py * p.tw;
            for (int kx = 0; kx < full; ++kx) {
                float z[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b) z[b] = prow[pix_off[b] + 4 * kx] - mrow[mean_off[b] + 4 * kx];
                int t2 = 0;
#pragma unroll
                for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                    for (int bj = bi; bj < NB; ++bj, ++t2)
                        acc[t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[bi], z[bj], acc[t2], 0, 0, 0);
            }
            if (tail) {                                   // ragged end of the row: patches past the image add 0
                const bool ok = q < tail;
                float z[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const float v = prow[pix_off[b] + 4 * full] - mrow[mean_off[b] + 4 * full];
                    z[b] = ok ? v : 0.f;
                }
                int t2 = 0;
#pragma unroll
                for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                    for (int bj = bi; bj < NB; ++bj, ++t2)
                        acc[t2] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[bi], z[bj], acc[t2], 0, 0, 0);
            }
        }
        if (++since_flush >= p.flush_items || it == count - 1) {
            // fold the fp32 tile accumulators into this wavefront's fp64 slot
#pragma unroll
            for (int t3 = 0; t3 < NT; ++t3)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    double *dst = my_slot + (t3 * 4 + v) * 64 + lane;
                    const double add = (double)acc[t3][v];
                    *dst = rmw ? *dst + add : add;
                }
#pragma unroll
            for (int t3 = 0; t3 < NT; ++t3) acc[t3] = floatx4{0.f, 0.f, 0.f, 0.f};
            rmw = true;
            since_flush = 0;
        }
    }
    if (count == 0 && !rmw) {                             // idle workgroup: its slots must still read as zero
        for (int e = lane; e < NT * 256; e += 64) my_slot[e] = 0.0;
    }
}

// Sum the per-wavefront slots in a fixed order: grid (elements/256, segments); segment s
// adds slots s, s+S, s+2S, ... into seg[s][e].
__global__ void gram_reduce_seg_kernel(const double *__restrict__ slots, int n_slots, int E, double *__restrict__ seg)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    const int S = gridDim.y, s = blockIdx.y;
    double sum = 0.0;
    for (int j = s; j < n_slots; j += S) sum += slots[(size_t)j * E + e];
    seg[(size_t)s * E + e] = sum;
}

__global__ void gram_reduce_final_kernel(const double *__restrict__ seg, int S, int E, double *__restrict__ stacked)
{
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= E) return;
    double sum = 0.0;
    for (int s = 0; s < S; ++s) sum += seg[(size_t)s * E + e];
    stacked[e] = sum;
}

// Entry (r,c) of the stacked 2D x 2D Gram from its tile storage (upper block triangle).
__device__ inline double stacked_entry(const double *st, int NB, int r, int c)
{
    int bi = r >> 4, bj = c >> 4;
    if (bi > bj) {
        int t = r; r = c; c = t;
        t = bi; bi = bj; bj = t;
    }
    const int tile = bi * NB - bi * (bi - 1) / 2 + (bj - bi);
    const int i = r & 15, j = c & 15;
    return st[(size_t)(tile * 4 + (i & 3)) * 64 + (i >> 2) * 16 + j];
}

// mats = [C11 | C22 | C12 | Cw | CT], each D*D, divided by the patch count; one workgroup
// per matrix.  Every patch is mean-free, so each exact matrix M satisfies M = H M H with
// H = I - 11^T/D.  The fp32 products leave a residue of order 1e-7 on the constant
// direction, which the ridge of the solve (eigenvalue eps on that direction) would
// amplify by 1/ridge; the projection H M H, done here in fp64, removes exactly that
// residue and nothing else.
__global__ __launch_bounds__(256) void gram_export_kernel(const double *__restrict__ st_main,
                                                          const double *__restrict__ st_cls,
                                                          const double *__restrict__ st_tot, int D, int NB,
                                                          double inv_n, double *__restrict__ mats)
{
    extern __shared__ double ex[];
    double *M = ex, *rsum = ex + D * D, *csum = rsum + D, *tot = csum + D;
    const int which = blockIdx.x;
    for (int e = threadIdx.x; e < D * D; e += blockDim.x) {
        const int a = e / D, b = e - a * D;
        double v;
        switch (which) {
            case 0:   // within-view blocks: mirrored entries are equal up to rounding order
                v = 0.5 * (stacked_entry(st_main, NB, a, b) + stacked_entry(st_main, NB, b, a)); break;
            case 1:
                v = 0.5 * (stacked_entry(st_main, NB, D + a, D + b) + stacked_entry(st_main, NB, D + b, D + a)); break;
            case 2: v = stacked_entry(st_main, NB, a, D + b); break;
            case 3: v = stacked_entry(st_cls, NB, a, D + b); break;
            default: v = stacked_entry(st_tot, NB, a, D + b); break;
        }
        M[e] = v * inv_n;
    }
    __syncthreads();
    if (threadIdx.x < D) {
        double r = 0.0, c = 0.0;
        for (int j = 0; j < D; ++j) {
            r += M[threadIdx.x * D + j];
            c += M[j * D + threadIdx.x];
        }
        rsum[threadIdx.x] = r / D;
        csum[threadIdx.x] = c / D;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int j = 0; j < D; ++j) t += rsum[j];
        tot[0] = t / D;
    }
    __syncthreads();
    double *out = mats + (size_t)which * D * D;
    for (int e = threadIdx.x; e < D * D; e += blockDim.x) {
        const int a = e / D, b = e - a * D;
        out[e] = M[e] - rsum[a] - csum[b] + tot[0];
    }
}

static int gram_occupancy(int k)
{
    // workgroups per compute unit the register budget allows (accumulators: tiles*4 per lane)
    return k <= 5 ? 4 : (k == 7 ? 2 : 1);
}

int max_gram_slots(ddcca_ctx *ctx, int k) { return ctx->n_cu * gram_occupancy(k) * 4; }

template <int KS>
static int gram_launch(ddcca_ctx *ctx, GramParams p, int grid, size_t lds)
{
    static bool attr_set = false;
    if (!attr_set) {
        DDCCA_HIP(ctx, hipFuncSetAttribute((const void *)patch_gram_kernel<KS>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set = true;
    }
    hipLaunchKernelGGL(patch_gram_kernel<KS>, dim3(grid), dim3(GRAM_THREADS), lds, ctx->stream, p);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int launch_patch_gram(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t n_maps, int h, int w, int k,
                      double *slots, int max_slots, int *slots_valid)
{
    ProfScope prof(ctx, DDCCA_K_GRAM);
    GramParams p;
    p.v1 = v1; p.v2 = v2; p.h = h; p.w = w;
    const int w4 = (w + 3) & ~3;
    // split wide images into equal column tiles of at most GRAM_TW_MAX patches
    const int ntx = (w4 + GRAM_TW_MAX - 1) / GRAM_TW_MAX;
    p.tw = (((w4 + ntx - 1) / ntx) + 3) & ~3;
    p.tiles_x = (w + p.tw - 1) / p.tw;
    p.tiles_y = (h + GRAM_TH - 1) / GRAM_TH;
    p.n_items = n_maps * p.tiles_x * p.tiles_y;
    const int r = (k - 1) / 2;
    // row pitch: >= tile width + halo, and congruent to k+3 mod 32 so that the window
    // rows a lane group touches fall into distinct LDS banks
    int pitch = p.tw + 2 * r;
    while (pitch % 32 != (k + 3) % 32) ++pitch;
    p.pitch = pitch;
    p.view_stride = (GRAM_TH + 2 * r) * pitch + 16;      // +16: shift view 2 by half the banks
    const size_t lds = (size_t)(2 * p.view_stride + 2 * GRAM_TH * p.tw + 8) * sizeof(float);
    // about 16k patches between fp64 flushes per wavefront
    const int patches_per_wave_item = (GRAM_TH / 4) * p.tw;
    p.flush_items = std::max(1, 16384 / patches_per_wave_item);
    p.slots = slots;
    p.slots_valid = *slots_valid;
    const int max_grid = max_slots / 4;
    int grid = (int)std::min<int64_t>(max_grid, std::max<int64_t>(p.n_items, 1));
    // slots that already hold data must all be revisited or kept: a smaller grid leaves
    // the upper ones untouched (still valid), a larger one initialises new ones
    int rc;
    switch (k) {
        case 3: rc = gram_launch<3>(ctx, p, grid, lds); break;
        case 5: rc = gram_launch<5>(ctx, p, grid, lds); break;
        case 7: rc = gram_launch<7>(ctx, p, grid, lds); break;
        case 9: rc = gram_launch<9>(ctx, p, grid, lds); break;
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
    if (rc) return rc;
    *slots_valid = std::max(*slots_valid, grid * 4);
    return DDCCA_OK;
}

int launch_gram_reduce(ddcca_ctx *ctx, const double *slots, int n_slots, int k, double *stacked)
{
    ProfScope prof(ctx, DDCCA_K_REDUCE);
    const int E = gram_tiles(k) * 256;
    const int S = std::max(1, std::min(64, n_slots / 8));
    int rc;
    if ((rc = ensure(ctx, ctx->seg, (size_t)64 * E * sizeof(double)))) return rc;
    double *seg = (double *)ctx->seg.ptr;
    hipLaunchKernelGGL(gram_reduce_seg_kernel, dim3((E + 255) / 256, S), dim3(256), 0, ctx->stream, slots, n_slots, E,
                       seg);
    hipLaunchKernelGGL(gram_reduce_final_kernel, dim3((E + 255) / 256), dim3(256), 0, ctx->stream, seg, S, E, stacked);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int launch_export(ddcca_ctx *ctx, const double *stacked_main, const double *stacked_cls, const double *stacked_tot,
                  int k, double n_patches, double *mats)
{
    ProfScope prof(ctx, DDCCA_K_REDUCE);
    const int D = k * k;
    const size_t lds = (size_t)(D * D + 2 * D + 2) * sizeof(double);
    hipLaunchKernelGGL(gram_export_kernel, dim3(5), dim3(256), lds, ctx->stream, stacked_main, stacked_cls,
                       stacked_tot, D, gram_blocks(k), 1.0 / n_patches, mats);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
