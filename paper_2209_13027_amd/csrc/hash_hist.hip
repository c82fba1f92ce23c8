// Output layer: hashing of the L2 maps of one input into a code map (Eq. 7-9) fused with the
// per-block code histogram (Section II-C).  Integer work only; HBM-bound: every map pixel is
// read (ideally once) and every uint16 count is written once.
//
// One workgroup owns RB consecutive block rows of one map and a chunk of block columns.  Its
// LDS holds their histograms as packed 16-bit counters (two bins per 32-bit word, which is
// also the memory layout of the output, so the counts leave LDS as a plain vector copy).
// Every pixel of the rows the block rows cover is hashed once per workgroup (L2 coalesced
// plane reads, strict "> 0") and added with an LDS atomic to each block that contains it.
// A count never exceeds the block area (<= 65535, checked on the host), so the two halves
// of a word cannot overflow into each other.
#include "ddcca_internal.h"

namespace ddcca {

constexpr int HIST_THREADS = 256;
constexpr int HIST_LDS_BYTES = 32 * 1024;   // histogram bytes per workgroup (occupancy 4-5 per CU)

struct HistParams {
    const float *maps;
    uint16_t *hist;
    int h, w, bh, bw, sy, sx, nby, nbx;
    int rb;             // block rows per workgroup
    int cols;           // block columns per workgroup
    int row_groups;     // ceil(nby / rb)
    int col_chunks;     // ceil(nbx / cols)
    int64_t group, group_stride;
    int vec4;           // rows may be read as aligned float4
    unsigned magic_sy, magic_sx;   // ceil(2^32 / stride) when h, w < 65536 (exact division by mul-hi), else 0
};

// x / d for 0 <= x < 65536 with magic = ceil(2^32 / d) (exact), plain division otherwise.
__device__ __forceinline__ int fast_div(int x, int d, unsigned magic)
{
    return magic ? (int)__umulhi((unsigned)x, magic) : x / d;
}

// Block rows [ilo, ihi] (clipped to the workgroup's [i0, i1)) that contain image row y.
__device__ __forceinline__ void block_range(int y, int b, int s, unsigned magic, int lo, int hi, int &first, int &last)
{
    first = y - b + 1 < 0 ? 0 : fast_div(y - b + s, s, magic);     // ceil((y - b + 1) / s)
    last = fast_div(y, s, magic);
    first = max(first, lo);
    last = min(last, hi - 1);
}

template <int L2>
__device__ __forceinline__ void hist_add(unsigned int *lds_hist, const HistParams &p, int x, unsigned code, int ilo,
                                         int ihi, int i0, int j0, int j1, int ncol)
{
    constexpr int WORDS = (1 << L2) > 1 ? (1 << L2) / 2 : 1;   // 32-bit words per histogram
    int jlo, jhi;
    block_range(x, p.bw, p.sx, p.magic_sx, j0, j1, jlo, jhi);
    const unsigned inc = 1u << (16 * (code & 1));
    const unsigned word = code >> 1;
    for (int i = ilo; i <= ihi; ++i)
        for (int j = jlo; j <= jhi; ++j)
            atomicAdd(&lds_hist[((i - i0) * ncol + (j - j0)) * WORDS + word], inc);
}

template <int L2>
__global__ __launch_bounds__(HIST_THREADS) void hash_hist_kernel(HistParams p)
{
    extern __shared__ unsigned int lds_hist[];
    constexpr int BINS = 1 << L2;
    constexpr int WORDS = BINS > 1 ? BINS / 2 : 1;
    const int per_map = p.row_groups * p.col_chunks;
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2.  Renumber them so
    // that consecutive work items (neighbouring block-row groups of one map, which share
    // image rows) run on the same XCD and find the shared rows in its L2.
    const unsigned nwg = gridDim.x, xcd = blockIdx.x & 7u, pos = blockIdx.x >> 3;
    const unsigned per = nwg >> 3, rem = nwg & 7u;
    const unsigned item = (xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per) + pos;
    const int64_t n = item / per_map;
    const int r = (int)(item - n * per_map);
    const int rg = r / p.col_chunks, cc = r - rg * p.col_chunks;
    const int i0 = rg * p.rb, i1 = min(i0 + p.rb, p.nby);
    const int j0 = cc * p.cols, j1 = min(j0 + p.cols, p.nbx);
    const int nrow = i1 - i0, ncol = j1 - j0;
    const int n_words = nrow * ncol * WORDS;
    for (int e = threadIdx.x; e < n_words; e += HIST_THREADS) lds_hist[e] = 0u;
    __syncthreads();

    const int64_t P = (int64_t)p.h * p.w;
    const float *base = p.maps + n * L2 * P;
    const int y_lo = i0 * p.sy, y_hi = (i1 - 1) * p.sy + p.bh;       // rows [y_lo, y_hi)
    const int x_lo = j0 * p.sx, x_hi = (j1 - 1) * p.sx + p.bw;       // columns [x_lo, x_hi)
    // threads as TROWS rows x TCOLS columns of work items (no per-item index division); a
    // wavefront reads whole contiguous row pieces: 32 quads (512 B) suffice for narrow maps,
    // 64 quads (1 KB) for wide ones
    const int wide = (x_hi - x_lo) > 128 ? 1 : 0;
    const int TCOLS = wide ? 64 : 32, TROWS = HIST_THREADS / TCOLS;
    const int tcol = threadIdx.x & (TCOLS - 1), trow = threadIdx.x / TCOLS;
    if (p.vec4) {
        // aligned quads of 4 pixels; the quad range covers [x_lo, x_hi) and is clipped per pixel
        const int q_lo = x_lo >> 2, q_hi = (x_hi + 3) >> 2;
        for (int y = y_lo + trow; y < y_hi; y += TROWS) {
            int ilo, ihi;
            block_range(y, p.bh, p.sy, p.magic_sy, i0, i1, ilo, ihi);
            const float *row = base + (int64_t)y * p.w;
            for (int xq = q_lo + tcol; xq < q_hi; xq += TCOLS) {
                const float *src = row + 4 * xq;
                unsigned c0 = 0, c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
                for (int l = 0; l < L2; ++l) {
                    const float4 v = *reinterpret_cast<const float4 *>(src + l * P);
                    c0 |= (v.x > 0.0f ? 1u : 0u) << l;
                    c1 |= (v.y > 0.0f ? 1u : 0u) << l;
                    c2 |= (v.z > 0.0f ? 1u : 0u) << l;
                    c3 |= (v.w > 0.0f ? 1u : 0u) << l;
                }
                const int x = 4 * xq;
                if (x >= x_lo && x < x_hi) hist_add<L2>(lds_hist, p, x, c0, ilo, ihi, i0, j0, j1, ncol);
                if (x + 1 >= x_lo && x + 1 < x_hi) hist_add<L2>(lds_hist, p, x + 1, c1, ilo, ihi, i0, j0, j1, ncol);
                if (x + 2 >= x_lo && x + 2 < x_hi) hist_add<L2>(lds_hist, p, x + 2, c2, ilo, ihi, i0, j0, j1, ncol);
                if (x + 3 >= x_lo && x + 3 < x_hi) hist_add<L2>(lds_hist, p, x + 3, c3, ilo, ihi, i0, j0, j1, ncol);
            }
        }
    } else {
        for (int y = y_lo + trow; y < y_hi; y += TROWS) {
            int ilo, ihi;
            block_range(y, p.bh, p.sy, p.magic_sy, i0, i1, ilo, ihi);
            const float *row = base + (int64_t)y * p.w;
            for (int x = x_lo + tcol; x < x_hi; x += TCOLS) {
                unsigned code = 0;
#pragma unroll
                for (int l = 0; l < L2; ++l) code |= (row[l * P + x] > 0.0f ? 1u : 0u) << l;
                hist_add<L2>(lds_hist, p, x, code, ilo, ihi, i0, j0, j1, ncol);
            }
        }
    }
    __syncthreads();

    // copy out: block row i of the chunk is ncol*BINS contiguous uint16 in the output
    const int64_t A = (int64_t)p.nby * p.nbx;
    uint16_t *out_map = p.hist + (n / p.group) * p.group_stride + (n % p.group) * A * BINS;
    if (BINS >= 8 && ((((uintptr_t)out_map) | (uintptr_t)(A * BINS * 2) | (uintptr_t)(p.group_stride * 2)) & 15) == 0) {
        const int row_vec = ncol * WORDS / 4;                        // uint4 per block row of the chunk
        for (int e = threadIdx.x; e < nrow * row_vec; e += HIST_THREADS) {
            const int ir = e / row_vec, v = e - ir * row_vec;
            const uint4 val = *reinterpret_cast<const uint4 *>(lds_hist + (ir * ncol * WORDS) + 4 * v);
            uint16_t *dst = out_map + ((int64_t)(i0 + ir) * p.nbx + j0) * BINS;
            *reinterpret_cast<uint4 *>(dst + 8 * v) = val;
        }
    } else {
        for (int e = threadIdx.x; e < nrow * ncol * BINS; e += HIST_THREADS) {
            const int ir = e / (ncol * BINS), rest = e - ir * ncol * BINS;
            const unsigned wv = lds_hist[ir * ncol * WORDS + (rest >> 1)];
            uint16_t *dst = out_map + ((int64_t)(i0 + ir) * p.nbx + j0) * BINS;
            dst[rest] = (uint16_t)((BINS > 1 ? (wv >> (16 * (rest & 1))) : wv) & 0xffffu);
        }
    }
}

template <int L2>
static void hist_launch(ddcca_ctx *ctx, HistParams p, int64_t n)
{
    constexpr int BINS = 1 << L2;
    constexpr int HIST_BYTES = (BINS > 1 ? BINS / 2 : 1) * 4;         // packed histogram of one block
    const int max_blocks = std::max(1, HIST_LDS_BYTES / HIST_BYTES);
    p.cols = std::min(p.nbx, max_blocks);
    p.col_chunks = (p.nbx + p.cols - 1) / p.cols;
    // several block rows per workgroup cut the re-reading of the rows that overlapping blocks share
    p.rb = std::max(1, std::min(p.nby, max_blocks / p.cols));
    p.row_groups = (p.nby + p.rb - 1) / p.rb;
    const size_t lds = (size_t)p.rb * p.cols * HIST_BYTES;
    const int64_t per_map = (int64_t)p.row_groups * p.col_chunks;
    const int64_t maps_per_launch = std::max<int64_t>(p.group, (((int64_t)1 << 30) / per_map) / p.group * p.group);
    for (int64_t n0 = 0; n0 < n; n0 += maps_per_launch) {
        const int64_t nb = std::min(maps_per_launch, n - n0);
        HistParams q = p;
        q.maps = p.maps + n0 * L2 * (int64_t)p.h * p.w;
        q.hist = p.hist + (n0 / p.group) * p.group_stride;
        hipLaunchKernelGGL(hash_hist_kernel<L2>, dim3((unsigned)(nb * per_map)), dim3(HIST_THREADS), lds, ctx->stream,
                           q);
    }
}

int launch_hash_hist(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w, int bh, int bw, int sy,
                     int sx, uint16_t *hist, int64_t group, int64_t group_stride)
{
    ProfScope prof(ctx, DDCCA_K_HASH_HIST);
    HistParams p;
    p.maps = maps; p.hist = hist;
    p.h = h; p.w = w; p.bh = bh; p.bw = bw; p.sy = sy; p.sx = sx;
    p.nby = (h - bh) / sy + 1;
    p.nbx = (w - bw) / sx + 1;
    p.group = group; p.group_stride = group_stride;
    p.vec4 = ((w & 3) == 0 && (((uintptr_t)maps) & 15) == 0) ? 1 : 0;
    const bool small = h < 65536 && w < 65536;
    p.magic_sy = small ? (unsigned)((((uint64_t)1 << 32) + sy - 1) / sy) : 0u;
    p.magic_sx = small ? (unsigned)((((uint64_t)1 << 32) + sx - 1) / sx) : 0u;
    switch (L2) {
#define CASE(v) case v: hist_launch<v>(ctx, p, n); break;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12)
#undef CASE
        default: return fail(ctx, DDCCA_EINVAL, "L2 out of range");
    }
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
