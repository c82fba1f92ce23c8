// Last stage convolution (Eq. 6) fused with the output layer (Eq. 7-12): the L2 maps of an
// input map are computed tile by tile on the matrix unit, reduced to their sign bits, combined
// into the hash code of every pixel and counted into the block histograms in LDS.  The L2 maps
// never reach memory: per input map the kernel reads h*w floats (plus halos) and writes the
// histograms (or their information-quality values).
//
// The contraction is the implicit GEMM of the stand-alone stage convolution, instruction for
// instruction (rows = (filter, x-shift), columns = 16 pixel positions, K = taps, ascending),
// so every map value, and with it every code and count, is bit-identical to running the
// convolution and the hash+histogram kernels one after the other.
//
// One workgroup owns RB block rows x a chunk of block columns of one input map (their packed
// 16-bit histograms stay in LDS, as in the unfused kernel) and walks the pixel rectangle those
// blocks cover in 32-row x (32*NBX)-column tiles: stage tile + halo in LDS, one wavefront per
// tile row runs NBX accumulator chains, takes the signs, ORs the partial codes of the four
// 16-lane groups together (each holds two filters) and adds the 32 pixels of a column block
// to the histograms of the blocks that contain them.
#include "hist_common.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int FUSED_THREADS = 256;
constexpr int FUSED_TH = 32;              // tile rows
constexpr int FUSED_XB = 32;              // pixels per MFMA column block (16 columns x 2 shifts)
constexpr int FUSED_MAX_NBX = 4;
constexpr int FUSED_LDS_BYTES = 80 * 1024;   // per workgroup: two workgroups share a compute unit's 160 KB

struct FusedParams {
    const float *in;      // [n][h][w]
    const float *W;       // [L2][k][k]
    void *out;
    const float *lut;
    int lut_n;
    double log_total;
    int out_type;
    int L2;
    int h, w, bh, bw, sy, sx, nby, nbx;
    int rb, cols, row_groups, col_chunks;
    int64_t group, group_stride;
    unsigned magic_sy, magic_sx;
    int hist_words;       // LDS words of the histograms (padded to 4)
    int lut_words;        // LDS words reserved for the table (padded to 4)
};

template <int KS, int NBX>
__host__ __device__ constexpr int fused_tile_floats()
{
    return (FUSED_TH + KS - 1) * ((NBX * FUSED_XB + KS) | 1);
}

template <int KS, int NBX, int NG>
__global__ __launch_bounds__(FUSED_THREADS) void conv_hash_hist_kernel(FusedParams p)
{
    constexpr int R = (KS - 1) / 2;
    constexpr int KW = KS + 1;                    // tap columns incl. the shift
    constexpr int TAPS = KS * KW;
    constexpr int KK = (TAPS + 3) / 4;            // MFMA steps
    constexpr int TW = NBX * FUSED_XB;
    constexpr int PW = TW + 2 * R + 1;            // +1: the odd shift reads one more column
    constexpr int PITCH = PW | 1;
    extern __shared__ unsigned int lds[];
    unsigned int *lds_hist = lds;
    float *lds_lut = reinterpret_cast<float *>(lds + p.hist_words);
    float *tile = lds_lut + p.lut_words;

    const int bins = 1 << p.L2;
    const int words = bins > 1 ? bins / 2 : 1;    // 32-bit words per packed histogram
    const int per_map = p.row_groups * p.col_chunks;
    const int64_t n = blockIdx.x / per_map;
    const int rr = (int)(blockIdx.x - n * per_map);
    const int rg = rr / p.col_chunks, cc = rr - rg * p.col_chunks;
    const int i0 = rg * p.rb, i1 = min(i0 + p.rb, p.nby);
    const int j0 = cc * p.cols, j1 = min(j0 + p.cols, p.nbx);
    const int nrow = i1 - i0, ncol = j1 - j0;
    const int n_words = nrow * ncol * words;
    for (int e = threadIdx.x; e < n_words; e += FUSED_THREADS) lds_hist[e] = 0u;
    if (p.out_type != DDCCA_FEAT_COUNT_U16)
        for (int e = threadIdx.x; e < p.lut_n; e += FUSED_THREADS) lds_lut[e] = p.lut[e];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c = lane & 15;
    // B-operand window offsets of this lane's tap (4*kk + q) for every step
    int toff[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int tap = 4 * kk + q;
        const int dy = tap / KW, dx = tap - dy * KW;
        toff[kk] = tap < TAPS ? dy * PITCH + dx : 0;
    }
    // A operand: row (g,s) = lane%16, tap 4*kk + lane/16, for every group of 8 filters
    float wa[NG][KK];
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int g = 8 * gi + (c >> 1), s = c & 1;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int tap = 4 * kk + q;
            const int dy = tap / KW, dxw = tap - dy * KW - s;
            float v = 0.f;
            if (tap < TAPS && dxw >= 0 && dxw < KS && g < p.L2) v = p.W[(g * KS + dy) * KS + dxw];
            wa[gi][kk] = v;
        }
    }

    const int64_t P = (int64_t)p.h * p.w;
    const float *src = p.in + n * P;
    const int y_lo = i0 * p.sy, y_hi = (i1 - 1) * p.sy + p.bh;       // pixel rows [y_lo, y_hi)
    const int x_lo = j0 * p.sx, x_hi = (j1 - 1) * p.sx + p.bw;       // pixel columns [x_lo, x_hi)
    const int my_s = q & 1, my_ioff = q >> 1;                        // this lane's pixel of a pair / block-row parity

    for (int ty0 = y_lo; ty0 < y_hi; ty0 += FUSED_TH) {
        const int rows = min(FUSED_TH, y_hi - ty0);
        for (int tx0 = x_lo; tx0 < x_hi; tx0 += TW) {
            __syncthreads();                      // the previous tile has been consumed (first pass: LDS initialised)
            {
                const int gy0 = ty0 - R, gx0 = tx0 - R;
                const int n_el = (rows + 2 * R) * PW;
#pragma unroll 4
                for (int e = threadIdx.x; e < n_el; e += FUSED_THREADS) {
                    const int yy = e / PW, xx = e - yy * PW;
                    const int gy = gy0 + yy, gx = gx0 + xx;
                    float v = 0.f;
                    if (gy >= 0 && gy < p.h && gx >= 0 && gx < p.w) v = src[(int64_t)gy * p.w + gx];
                    tile[yy * PITCH + xx] = v;
                }
            }
            __syncthreads();
            for (int r = wave; r < rows; r += 4) {
                const float *prow = tile + r * PITCH + 2 * c;
                unsigned pc[NBX];
#pragma unroll
                for (int b = 0; b < NBX; ++b) pc[b] = 0u;
#pragma unroll
                for (int gi = 0; gi < NG; ++gi) {
                    floatx4 acc[NBX];
#pragma unroll
                    for (int b = 0; b < NBX; ++b) acc[b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int kk = 0; kk < KK; ++kk) {
                        const float *pk = prow + toff[kk];
#pragma unroll
                        for (int b = 0; b < NBX; ++b)
                            acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[gi][kk], pk[b * FUSED_XB], acc[b], 0, 0, 0);
                    }
                    // lane (q,c): acc[0], acc[1] = filter 8gi+2q at pixels x, x+1; acc[2], acc[3] = filter 8gi+2q+1
                    const int sh = 8 * gi + 2 * q;
#pragma unroll
                    for (int b = 0; b < NBX; ++b)
                        pc[b] |= ((acc[b][0] > 0.0f ? 1u : 0u) << sh) | ((acc[b][2] > 0.0f ? 1u : 0u) << (sh + 1)) |
                                 ((acc[b][1] > 0.0f ? 1u : 0u) << (sh + 16)) | ((acc[b][3] > 0.0f ? 1u : 0u) << (sh + 17));
                }
                const int y = ty0 + r;
                int ilo, ihi;
                block_range(y, p.bh, p.sy, p.magic_sy, i0, i1, ilo, ihi);
#pragma unroll
                for (int b = 0; b < NBX; ++b) {
                    unsigned v = pc[b];
                    v |= (unsigned)__shfl_xor((int)v, 16);
                    v |= (unsigned)__shfl_xor((int)v, 32);
                    // 64 lanes, 32 pixels: lane (q,c) takes pixel x0 + 2c + (q&1) and the block rows ilo + (q>>1), +2, ...
                    const unsigned code = (v >> (16 * my_s)) & 0xffffu;
                    const int x = tx0 + b * FUSED_XB + 2 * c + my_s;
                    if (x < x_hi) {
                        int jlo, jhi;
                        block_range(x, p.bw, p.sx, p.magic_sx, j0, j1, jlo, jhi);
                        const unsigned inc = 1u << (16 * (code & 1));
                        const unsigned word = code >> 1;
                        for (int i = ilo + my_ioff; i <= ihi; i += 2)
                            for (int j = jlo; j <= jhi; ++j)
                                atomicAdd(&lds_hist[((i - i0) * ncol + (j - j0)) * words + word], inc);
                    }
                }
            }
        }
    }
    __syncthreads();

    // copy out: block row i of the chunk is ncol*bins contiguous elements in the output
    const int64_t A = (int64_t)p.nby * p.nbx;
    const int esz = p.out_type == DDCCA_FEAT_IQ_F32 ? 4 : 2;
    const int64_t map_off = (n / p.group) * p.group_stride + (n % p.group) * A * bins;
    char *out_map = reinterpret_cast<char *>(p.out) + map_off * esz;
    const int vw = 8 / esz;                                          // packed words per 16-byte store
    if (bins >= 2 * vw && ((((uintptr_t)out_map) | (uintptr_t)(A * bins * esz) | (uintptr_t)(p.group_stride * esz)) & 15) == 0) {
        const int row_vec = ncol * words / vw;
        for (int e = threadIdx.x; e < nrow * row_vec; e += FUSED_THREADS) {
            const int ir = e / row_vec, v = e - ir * row_vec;
            const unsigned *sp = lds_hist + (ir * ncol * words) + vw * v;
            char *dst = out_map + (((int64_t)(i0 + ir) * p.nbx + j0) * bins + 2 * vw * v) * esz;
            uint4 val;
            if (p.out_type == DDCCA_FEAT_COUNT_U16) {
                val = *reinterpret_cast<const uint4 *>(sp);
            } else if (p.out_type == DDCCA_FEAT_IQ_F32) {
                const unsigned w0 = sp[0], w1 = sp[1];
                val.x = __float_as_uint(iq_value(w0 & 0xffffu, lds_lut, p.lut_n, p.log_total));
                val.y = __float_as_uint(iq_value(w0 >> 16, lds_lut, p.lut_n, p.log_total));
                val.z = __float_as_uint(iq_value(w1 & 0xffffu, lds_lut, p.lut_n, p.log_total));
                val.w = __float_as_uint(iq_value(w1 >> 16, lds_lut, p.lut_n, p.log_total));
            } else {
                unsigned o[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const unsigned wv = sp[t];
                    const __half lo = __float2half_rn(iq_value(wv & 0xffffu, lds_lut, p.lut_n, p.log_total));
                    const __half hi = __float2half_rn(iq_value(wv >> 16, lds_lut, p.lut_n, p.log_total));
                    o[t] = (unsigned)__half_as_ushort(lo) | ((unsigned)__half_as_ushort(hi) << 16);
                }
                val = make_uint4(o[0], o[1], o[2], o[3]);
            }
            *reinterpret_cast<uint4 *>(dst) = val;
        }
    } else {
        for (int e = threadIdx.x; e < nrow * ncol * bins; e += FUSED_THREADS) {
            const int ir = e / (ncol * bins), rest = e - ir * ncol * bins;
            const unsigned wv = lds_hist[ir * ncol * words + (rest >> 1)];
            const unsigned cnt = (bins > 1 ? (wv >> (16 * (rest & 1))) : wv) & 0xffffu;
            char *dst = out_map + (((int64_t)(i0 + ir) * p.nbx + j0) * bins + rest) * esz;
            if (p.out_type == DDCCA_FEAT_COUNT_U16)
                *reinterpret_cast<uint16_t *>(dst) = (uint16_t)cnt;
            else if (p.out_type == DDCCA_FEAT_IQ_F32)
                *reinterpret_cast<float *>(dst) = iq_value(cnt, lds_lut, p.lut_n, p.log_total);
            else
                *reinterpret_cast<__half *>(dst) = __float2half_rn(iq_value(cnt, lds_lut, p.lut_n, p.log_total));
        }
    }
}

template <int KS, int NBX, int NG>
static int fused_launch(ddcca_ctx *ctx, FusedParams p, int64_t n)
{
    static bool attr_set = false;
    if (!attr_set) {
        DDCCA_HIP(ctx, hipFuncSetAttribute((const void *)conv_hash_hist_kernel<KS, NBX, NG>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, FUSED_LDS_BYTES));
        attr_set = true;
    }
    const size_t lds = ((size_t)p.hist_words + p.lut_words + fused_tile_floats<KS, NBX>()) * 4;
    if (lds > (size_t)FUSED_LDS_BYTES) return fail(ctx, DDCCA_EINVAL, "internal: fused kernel LDS budget exceeded");
    const int64_t per_map = (int64_t)p.row_groups * p.col_chunks;
    const int64_t esz = p.out_type == DDCCA_FEAT_IQ_F32 ? 4 : 2;
    const int64_t maps_per_launch = std::max<int64_t>(p.group, (((int64_t)1 << 30) / per_map) / p.group * p.group);
    for (int64_t n0 = 0; n0 < n; n0 += maps_per_launch) {
        const int64_t nb = std::min(maps_per_launch, n - n0);
        FusedParams q = p;
        q.in = p.in + n0 * (int64_t)p.h * p.w;
        q.out = reinterpret_cast<char *>(p.out) + (n0 / p.group) * p.group_stride * esz;
        hipLaunchKernelGGL((conv_hash_hist_kernel<KS, NBX, NG>), dim3((unsigned)(nb * per_map)), dim3(FUSED_THREADS),
                           lds, ctx->stream, q);
    }
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

template <int KS, int NG>
static int fused_pick_nbx(ddcca_ctx *ctx, FusedParams &p, int64_t n)
{
    // Geometry.  Histogram budget: what the largest tile leaves of the workgroup's LDS.  Block columns and
    // block rows are spread evenly over the chunks / groups so that the workgroups of a map do equal work.
    const int bins = 1 << p.L2;
    const int hist_bytes = (bins > 1 ? bins / 2 : 1) * 4;
    p.lut_words = p.out_type != DDCCA_FEAT_COUNT_U16 ? (p.lut_n + 3) / 4 * 4 : 0;
    const int budget = FUSED_LDS_BYTES - fused_tile_floats<KS, FUSED_MAX_NBX>() * 4 - p.lut_words * 4 - 16;
    const int max_blocks = std::max(1, budget / hist_bytes);
    p.col_chunks = (p.nbx + max_blocks - 1) / max_blocks;
    p.cols = (p.nbx + p.col_chunks - 1) / p.col_chunks;
    const int rb_max = std::max(1, max_blocks / p.cols);
    p.row_groups = (p.nby + rb_max - 1) / rb_max;
    p.rb = (p.nby + p.row_groups - 1) / p.row_groups;
    p.row_groups = (p.nby + p.rb - 1) / p.rb;
    p.hist_words = (p.rb * p.cols * (hist_bytes / 4) + 3) / 4 * 4;
    // equal-width tiles of at most FUSED_MAX_NBX column blocks across the widest pixel rectangle
    const int width = (p.cols - 1) * p.sx + p.bw;
    const int xblocks = (width + FUSED_XB - 1) / FUSED_XB;
    const int tiles_x = (xblocks + FUSED_MAX_NBX - 1) / FUSED_MAX_NBX;
    const int nbx_tile = (xblocks + tiles_x - 1) / tiles_x;
    switch (nbx_tile) {
        case 1: return fused_launch<KS, 1, NG>(ctx, p, n);
        case 2: return fused_launch<KS, 2, NG>(ctx, p, n);
        case 3: return fused_launch<KS, 3, NG>(ctx, p, n);
        default: return fused_launch<KS, 4, NG>(ctx, p, n);
    }
}

template <int KS>
static int fused_pick_groups(ddcca_ctx *ctx, FusedParams &p, int64_t n)
{
    return p.L2 <= 8 ? fused_pick_nbx<KS, 1>(ctx, p, n) : fused_pick_nbx<KS, 2>(ctx, p, n);
}

int launch_conv_hash_hist(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L2,
                          int bh, int bw, int sy, int sx, void *out, int out_type, int64_t group,
                          int64_t group_stride)
{
    FusedParams p;
    p.in = in; p.W = W; p.out = out; p.out_type = out_type; p.L2 = L2;
    p.h = h; p.w = w; p.bh = bh; p.bw = bw; p.sy = sy; p.sx = sx;
    p.nby = (h - bh) / sy + 1;
    p.nbx = (w - bw) / sx + 1;
    p.group = group; p.group_stride = group_stride;
    const bool small = h < 65536 && w < 65536;
    p.magic_sy = small ? (unsigned)((((uint64_t)1 << 32) + sy - 1) / sy) : 0u;
    p.magic_sx = small ? (unsigned)((((uint64_t)1 << 32) + sx - 1) / sx) : 0u;
    int rc;
    if ((rc = prepare_iq_table(ctx, out_type, bh, bw, L2, &p.lut, &p.lut_n, &p.log_total))) return rc;
    ProfScope prof(ctx, DDCCA_K_CONV_HASH_HIST);
    switch (k) {
        case 3: return fused_pick_groups<3>(ctx, p, n);
        case 5: return fused_pick_groups<5>(ctx, p, n);
        case 7: return fused_pick_groups<7>(ctx, p, n);
        case 9: return fused_pick_groups<9>(ctx, p, n);
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
}

}  // namespace ddcca
