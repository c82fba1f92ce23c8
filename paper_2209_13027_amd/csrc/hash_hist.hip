// Output layer: hashing of the L2 maps of one input into a code map (Eq. 7-9) fused with the
// per-block code histogram (Section II-C).  Integer work only; HBM-bound: every map pixel is
// read (ideally once) and every uint16 count is written once.
//
// LDS holds block histograms as packed 16-bit counters (two bins per 32-bit word, which is
// also the memory layout of the output, so the counts leave LDS as a plain vector copy).
// A pixel is hashed (L2 coalesced plane reads, strict "> 0") and added with an LDS atomic to
// each block that contains it.  A count never exceeds the block area (<= 65535, checked on
// the host), so the two halves of a word cannot overflow into each other.
//
// Two kernels.  hash_hist_kernel (any geometry): one workgroup owns RB consecutive block rows
// of one map and a chunk of block columns; with overlapping blocks the pixel rows that two
// groups of block rows share are read by both -- neighbouring groups walk their rows in
// opposite directions, so that they want the shared rows at the same time and the second
// read is served by the L2 of the XCD they share.  hash_hist_sweep_kernel (maps wider than 256
// columns whose rows are readable as aligned float4, a ring of block rows fits in LDS): one
// workgroup sweeps a whole map top to bottom in phases of a few block strides; only the block
// rows that overlap the rows swept so far and are not yet complete are live, in a ring of LDS
// slots, and a block row is written out and its slot cleared as soon as the sweep has passed
// its last pixel row, so every pixel is read exactly once.  Measured: the LDS atomics bound
// neither kernel (with them removed the time stays the same); the sweep kernels level off at
// 5.0 TB/s whatever their schedule, the first kernel's many small independent workgroups reach
// 5.6 TB/s of algorithmic bytes on maps of 128 columns and 5.07 on 256 (sweep: 4.95).
//
// The same kernel also writes the information-quality form of the output (Eq. 10):
// o = -log p(t), p(t) = (count + 1) / (block area + bins), as fp32 or fp16.  The values for
// the possible counts come from a table (built in fp64 by a one-workgroup kernel, rounded
// once to fp32) that every workgroup copies into LDS, so the epilogue is one LDS gather per
// output element and the kernel stays bound by its HBM writes.
#include "hist_common.h"

namespace ddcca {

constexpr int HIST_THREADS = 256;
// LDS per workgroup of the row-group kernel, histograms plus the information-quality table: 40 KB (four workgroups
// per compute unit; 15 block rows of 15 x 256 bins: three groups of 5), and 60 KB for maps wider than 128 columns read
// as floats (two groups of 8 and 7, two workgroups per compute unit).  Measured, 60 against 40 KB: 256-column maps 5.21
// -> 5.43 TB/s (7.0 -> 6.5 ms per step of the 256 x 256 workload), 128-column maps 5.94 -> 5.98, 112 x 92 maps with 7 x 7
// blocks 5.9 -> 4.5 (slower), and the kernel that counts from code maps, bound by its own instructions, 17 % slower;
// 52 KB (groups of 6, 6 and 3) is slower than either, so the block rows are dealt evenly over the fewest groups the
// budget allows.
constexpr int HIST_LDS_BYTES = 40 * 1024;
constexpr int HIST_LDS_BYTES_WIDE = 60 * 1024;
constexpr int SWEEP_LDS_BYTES = 40 * 1024;  // the same for the ring of the sweep kernel
constexpr int CODE_ROWS = 8;                // code-map rows a thread has in flight

struct HistParams {
    const float *maps;
    const unsigned char *codes;   // CODES kernels: [n][ceil(L2/8)][h][w] hash code bytes (the maps are not read)
    void *hist;         // uint16 counts, or fp32 / fp16 information quality
    const float *lut;   // information-quality table, lut[c] = log(total) - log(c + 1)
    int lut_n;
    double log_total;
    int h, w, bh, bw, sy, sx, nby, nbx;
    int ring;           // sweep kernel: block rows held in LDS
    int phase_rows;     // sweep kernel: pixel rows per phase (a multiple of the block stride)
    int rb;             // block rows per workgroup
    int cols;           // block columns per workgroup
    int row_groups;     // ceil(nby / rb)
    int col_chunks;     // ceil(nbx / cols)
    int64_t group, group_stride;
    int vec4;           // rows may be read as aligned float4
    unsigned magic_sy, magic_sx;   // ceil(2^32 / stride) when h, w < 65536 (exact division by mul-hi), else 0
};

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

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));
typedef float floatx4_nt __attribute__((ext_vector_type(4)));

// Four pixels of a plane that nothing reads again soon: a 16-byte load with the non-temporal hint.
__device__ __forceinline__ float4 load_streamed4(const float *src)
{
    const floatx4_nt t = __builtin_nontemporal_load(reinterpret_cast<const floatx4_nt *>(src));
    return make_float4(t.x, t.y, t.z, t.w);
}

// Whether block rows of this output can leave as aligned 16-byte vectors.
template <int OUT>
__device__ __forceinline__ bool out_vec_ok(const void *out_map, int64_t map_elems, int64_t group_stride)
{
    constexpr int ESZ = (int)sizeof(typename HistOut<OUT>::type);
    return ((((uintptr_t)out_map) | (uintptr_t)(map_elems * ESZ) | (uintptr_t)(group_stride * ESZ)) & 15) == 0;
}

// Write nrow block rows of ncol packed histograms each (src: LDS, rows ncol*WORDS words apart) to dst (rows
// dst_row_stride elements apart) in the output type; CLEAR: zero the LDS words afterwards.
template <int L2, int OUT, bool CLEAR>
__device__ __forceinline__ void copy_out_rows(unsigned int *src_rows, int nrow, int ncol,
                                              typename HistOut<OUT>::type *dst, int64_t dst_row_stride, bool vec_ok,
                                              const float *lds_lut, const HistParams &p)
{
    typedef typename HistOut<OUT>::type OutT;
    constexpr int BINS = 1 << L2;
    constexpr int WORDS = BINS > 1 ? BINS / 2 : 1;
    constexpr int ESZ = (int)sizeof(OutT);
    constexpr int VW = 8 / ESZ;                                      // packed words per 16-byte store: 4, 2 or 1
    if (BINS >= 2 * VW && vec_ok) {
        const int row_vec = ncol * WORDS / VW;                       // 16-byte vectors per block row
        // uniform: every block row is a run of whole, aligned 128-byte lines: the histograms leave with the
        // non-temporal hint (nothing reads them again soon; measured 3 % on the 128-column workloads, 0.5 % at 256
        // columns -- the same hint on the plane READS costs 3-7 %: it takes the rows two neighbouring row groups
        // share out of the L2 they meet in).  Rows that split lines keep ordinary stores.
        const bool streaming = ((ncol * BINS * ESZ) & 127) == 0 && ((dst_row_stride * ESZ) & 127) == 0 &&
                               (((uintptr_t)dst) & 127) == 0;
        for (int e = threadIdx.x; e < nrow * row_vec; e += HIST_THREADS) {
            const int ir = e / row_vec, v = e - ir * row_vec;
            unsigned *src = src_rows + (ir * ncol * WORDS) + VW * v;
            OutT *d = dst + ir * dst_row_stride + 2 * VW * v;
            if (OUT == DDCCA_FEAT_COUNT_U16) {
                if (streaming)
                    __builtin_nontemporal_store(*reinterpret_cast<const uintx4 *>(src), reinterpret_cast<uintx4 *>(d));
                else
                    *reinterpret_cast<uint4 *>(d) = *reinterpret_cast<const uint4 *>(src);
            } else {
                alignas(16) OutT vals[2 * VW];
#pragma unroll
                for (int q = 0; q < VW; ++q) {
                    const unsigned wv = src[q];
                    vals[2 * q] = hist_convert<OUT>(wv & 0xffffu, lds_lut, p.lut_n, p.log_total);
                    vals[2 * q + 1] = hist_convert<OUT>(wv >> 16, lds_lut, p.lut_n, p.log_total);
                }
                if (streaming)
                    __builtin_nontemporal_store(*reinterpret_cast<const uintx4 *>(vals), reinterpret_cast<uintx4 *>(d));
                else
                    *reinterpret_cast<uint4 *>(d) = *reinterpret_cast<const uint4 *>(vals);
            }
            if (CLEAR) {
#pragma unroll
                for (int q = 0; q < VW; ++q) src[q] = 0u;
            }
        }
    } else {
        for (int e = threadIdx.x; e < nrow * ncol * BINS; e += HIST_THREADS) {
            const int ir = e / (ncol * BINS), rest = e - ir * ncol * BINS;
            const unsigned wv = src_rows[ir * ncol * WORDS + (rest >> 1)];
            const unsigned c = (BINS > 1 ? (wv >> (16 * (rest & 1))) : wv) & 0xffffu;
            dst[ir * dst_row_stride + rest] = hist_convert<OUT>(c, lds_lut, p.lut_n, p.log_total);
        }
        if (CLEAR) {
            __syncthreads();                                         // two bins share a word: clear after all reads
            for (int e = threadIdx.x; e < nrow * ncol * WORDS; e += HIST_THREADS) src_rows[e] = 0u;
        }
    }
}

__global__ void iq_lut_kernel(double total, int n, float *lut)
{
    const double log_total = log(total);
    for (int c = threadIdx.x; c < n; c += blockDim.x) lut[c] = (float)(log_total - log((double)(c + 1)));
}

// CODES: the input is the hash code itself, one byte plane per 8 filters (written by the convolution that would
// have written the maps), instead of L2 planes of floats.
// PIPE: a thread's next row is requested before its current one is counted (twice the registers for the planes in
// flight: chosen by the launcher when a thread has rows enough for it to pay).
template <int L2, int OUT, bool CODES = false, bool PIPE = false>
__global__ __launch_bounds__(HIST_THREADS) void hash_hist_kernel(HistParams p, int lds_hist_words)
{
    extern __shared__ unsigned int lds_hist[];
    typedef typename HistOut<OUT>::type OutT;
    constexpr int BINS = 1 << L2;
    constexpr int WORDS = BINS > 1 ? BINS / 2 : 1;
    float *lds_lut = reinterpret_cast<float *>(lds_hist + lds_hist_words);
    if (OUT != DDCCA_FEAT_COUNT_U16)
        for (int e = threadIdx.x; e < p.lut_n; e += HIST_THREADS) lds_lut[e] = p.lut[e];
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
    const float *base = CODES ? nullptr : p.maps + n * L2 * P;
    constexpr int CP = (L2 + 7) / 8;                                 // code byte planes
    const unsigned char *cbase = CODES ? p.codes + n * CP * P : nullptr;
    const int y_lo = i0 * p.sy, y_hi = (i1 - 1) * p.sy + p.bh;       // rows [y_lo, y_hi)
    const int x_lo = j0 * p.sx, x_hi = (j1 - 1) * p.sx + p.bw;       // columns [x_lo, x_hi)
    // threads as TROWS rows x TCOLS columns of work items (no per-item index division); a
    // wavefront reads whole contiguous row pieces: 32 quads (512 B) suffice for narrow maps,
    // 64 quads (1 KB) for wide ones
    const int wide = (x_hi - x_lo) > 128 ? 1 : 0;
    const int TCOLS = wide ? 64 : 32, TROWS = HIST_THREADS / TCOLS;
    const int tcol = threadIdx.x & (TCOLS - 1), trow = threadIdx.x / TCOLS;
    if (CODES && p.vec4) {
        // Code maps: no load latency to hide the bookkeeping behind, so the loops are turned inside out: a thread
        // keeps its group of four columns, whose block columns are found once, and walks down the rows.
        const int q_lo = x_lo >> 2, q_hi = (x_hi + 3) >> 2;
        for (int xq = q_lo + tcol; xq < q_hi; xq += TCOLS) {
            int jlo[4], jhi[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int x = 4 * xq + k;
                block_range(x, p.bw, p.sx, p.magic_sx, j0, j1, jlo[k], jhi[k]);
                if (x < x_lo || x >= x_hi) jhi[k] = jlo[k] - 1;          // not a column of this workgroup: no block
            }
            // the code words of the thread's next CODE_ROWS rows are all requested before the first is used: one
            // small load per row and thread, waited for one by one, would leave the workgroup idle for a memory
            // round trip per row
            for (int yb = y_lo + trow; yb < y_hi; yb += CODE_ROWS * TROWS) {
                unsigned int v[CODE_ROWS][CP];
#pragma unroll
                for (int r = 0; r < CODE_ROWS; ++r) {
                    const int y = min(yb + r * TROWS, y_hi - 1);                 // (a row past the end: reloaded, unused)
#pragma unroll
                    for (int i = 0; i < CP; ++i)
                        v[r][i] = *reinterpret_cast<const unsigned int *>(cbase + i * P + (int64_t)y * p.w + 4 * xq);
                }
#pragma unroll
                for (int r = 0; r < CODE_ROWS; ++r) {
                    const int y = yb + r * TROWS;
                    if (y >= y_hi) break;
                    int ilo, ihi;
                    block_range(y, p.bh, p.sy, p.magic_sy, i0, i1, ilo, ihi);
                    unsigned c[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int i = 0; i < CP; ++i) {
                        c[0] |= (v[r][i] & 0xffu) << (8 * i);
                        c[1] |= ((v[r][i] >> 8) & 0xffu) << (8 * i);
                        c[2] |= ((v[r][i] >> 16) & 0xffu) << (8 * i);
                        c[3] |= (v[r][i] >> 24) << (8 * i);
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const unsigned inc = 1u << (16 * (c[k] & 1));
                        unsigned int *cell = lds_hist + (c[k] >> 1) - j0 * WORDS;
                        for (int i = ilo; i <= ihi; ++i)
                            for (int j = jlo[k]; j <= jhi[k]; ++j) atomicAdd(cell + ((i - i0) * ncol + j) * WORDS, inc);
                    }
                }
            }
        }
    } else if (p.vec4) {
        // aligned quads of 4 pixels; the quad range covers [x_lo, x_hi) and is clipped per pixel
        const int q_lo = x_lo >> 2, q_hi = (x_hi + 3) >> 2;
        // Neighbouring groups of block rows share the pixel rows where their blocks overlap, and they run side by
        // side on one XCD.  Even groups walk their rows bottom-up and odd ones top-down, so that a group and its
        // lower neighbour want the shared rows at the same time (both at the start, or both at the end) and the
        // second request finds them in that XCD's L2.
        const bool upward = (rg & 1) == 0 && p.row_groups > 1;
        // Rows that no other workgroup reads are requested with the non-temporal hint (they are read once: measured
        // 4 % on 128-column maps, 11 % on 256-column ones); the rows shared with a neighbouring row group keep
        // ordinary loads, which is what lets the second reader find them in the L2 (the hint on every row costs 3-7 %),
        // and so does everything when the block columns are split over workgroups.
        const int overlap = max(p.bh - p.sy, 0);
        const int own_lo = p.col_chunks > 1 ? y_hi : rg > 0 ? y_lo + overlap : y_lo;
        const int own_hi = rg + 1 < p.row_groups ? y_hi - overlap : y_hi;
        if (PIPE && q_hi - q_lo <= TCOLS) {
            // one group of four columns per thread (the usual case): the planes of the thread's next row are
            // requested before the pixels of the current one are counted
            const int xq = q_lo + tcol, nrows = y_hi - y_lo;
            auto row_of = [&](int r) { return upward ? y_hi - 1 - r : y_lo + r; };
            auto request = [&](int r, float4 (&v)[L2]) {
                const int y = row_of(r);
                const float *src = base + (int64_t)y * p.w + 4 * xq;
                if (y >= own_lo && y < own_hi) {
#pragma unroll
                    for (int l = 0; l < L2; ++l) v[l] = load_streamed4(src + l * P);
                } else {
#pragma unroll
                    for (int l = 0; l < L2; ++l) v[l] = *reinterpret_cast<const float4 *>(src + l * P);
                }
            };
            auto count = [&](int r, const float4 (&v)[L2]) {
                int ilo, ihi;
                block_range(row_of(r), p.bh, p.sy, p.magic_sy, i0, i1, ilo, ihi);
                unsigned c0 = 0, c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
                for (int l = 0; l < L2; ++l) {
                    c0 |= (v[l].x > 0.0f ? 1u : 0u) << l;
                    c1 |= (v[l].y > 0.0f ? 1u : 0u) << l;
                    c2 |= (v[l].z > 0.0f ? 1u : 0u) << l;
                    c3 |= (v[l].w > 0.0f ? 1u : 0u) << l;
                }
                const int x = 4 * xq;
                if (x >= x_lo && x < x_hi) hist_add<L2>(lds_hist, p, x, c0, ilo, ihi, i0, j0, j1, ncol);
                if (x + 1 >= x_lo && x + 1 < x_hi) hist_add<L2>(lds_hist, p, x + 1, c1, ilo, ihi, i0, j0, j1, ncol);
                if (x + 2 >= x_lo && x + 2 < x_hi) hist_add<L2>(lds_hist, p, x + 2, c2, ilo, ihi, i0, j0, j1, ncol);
                if (x + 3 >= x_lo && x + 3 < x_hi) hist_add<L2>(lds_hist, p, x + 3, c3, ilo, ihi, i0, j0, j1, ncol);
            };
            if (!CODES && xq < q_hi && trow < nrows) {
                float4 va[L2], vb[L2];
                int r = trow;
                request(r, va);
                while (true) {
                    const int r2 = r + TROWS;
                    if (r2 < nrows) request(r2, vb);
                    count(r, va);
                    if (r2 >= nrows) break;
                    r = r2 + TROWS;
                    if (r < nrows) request(r, va);
                    count(r2, vb);
                    if (r >= nrows) break;
                }
            }
        } else
        for (int r = trow; r < y_hi - y_lo; r += TROWS) {
            const int y = upward ? y_hi - 1 - r : y_lo + r;
            int ilo, ihi;
            block_range(y, p.bh, p.sy, p.magic_sy, i0, i1, ilo, ihi);
            const float *row = CODES ? nullptr : base + (int64_t)y * p.w;
            for (int xq = q_lo + tcol; xq < q_hi; xq += TCOLS) {
                unsigned c0 = 0, c1 = 0, c2 = 0, c3 = 0;
                const float *src = row + 4 * xq;
                float4 v[L2];
                if (y >= own_lo && y < own_hi) {
#pragma unroll
                    for (int l = 0; l < L2; ++l) v[l] = load_streamed4(src + l * P);
                } else {
#pragma unroll
                    for (int l = 0; l < L2; ++l) v[l] = *reinterpret_cast<const float4 *>(src + l * P);
                }
#pragma unroll
                for (int l = 0; l < L2; ++l) {
                    c0 |= (v[l].x > 0.0f ? 1u : 0u) << l;
                    c1 |= (v[l].y > 0.0f ? 1u : 0u) << l;
                    c2 |= (v[l].z > 0.0f ? 1u : 0u) << l;
                    c3 |= (v[l].w > 0.0f ? 1u : 0u) << l;
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
            const float *row = CODES ? nullptr : base + (int64_t)y * p.w;
            for (int x = x_lo + tcol; x < x_hi; x += TCOLS) {
                unsigned code = 0;
                if constexpr (CODES) {
#pragma unroll
                    for (int i = 0; i < CP; ++i) code |= (unsigned)cbase[i * P + (int64_t)y * p.w + x] << (8 * i);
                } else {
#pragma unroll
                    for (int l = 0; l < L2; ++l) code |= (row[l * P + x] > 0.0f ? 1u : 0u) << l;
                }
                hist_add<L2>(lds_hist, p, x, code, ilo, ihi, i0, j0, j1, ncol);
            }
        }
    }
    __syncthreads();

    // copy out: block row i of the chunk is ncol*BINS contiguous elements in the output
    const int64_t A = (int64_t)p.nby * p.nbx;
    OutT *out_map = reinterpret_cast<OutT *>(p.hist) + (n / p.group) * p.group_stride + (n % p.group) * A * BINS;
    copy_out_rows<L2, OUT, false>(lds_hist, nrow, ncol, out_map + ((int64_t)i0 * p.nbx + j0) * BINS,
                                  (int64_t)p.nbx * BINS, out_vec_ok<OUT>(out_map, A * BINS, p.group_stride), lds_lut, p);
}

template <int L2, int OUT>
__global__ __launch_bounds__(HIST_THREADS) void hash_hist_sweep_kernel(HistParams p, int lds_hist_words)
{
    extern __shared__ unsigned int lds_hist[];
    typedef typename HistOut<OUT>::type OutT;
    constexpr int BINS = 1 << L2;
    constexpr int WORDS = BINS > 1 ? BINS / 2 : 1;
    float *lds_lut = reinterpret_cast<float *>(lds_hist + lds_hist_words);
    if (OUT != DDCCA_FEAT_COUNT_U16)
        for (int e = threadIdx.x; e < p.lut_n; e += HIST_THREADS) lds_lut[e] = p.lut[e];
    const int64_t n = blockIdx.x;
    const int row_words = p.nbx * WORDS;                 // one block row of histograms
    for (int e = threadIdx.x; e < p.ring * row_words; e += HIST_THREADS) lds_hist[e] = 0u;
    __syncthreads();

    const int64_t P = (int64_t)p.h * p.w;
    const float *base = p.maps + n * L2 * P;
    const int64_t A = (int64_t)p.nby * p.nbx;
    OutT *out_map = reinterpret_cast<OutT *>(p.hist) + (n / p.group) * p.group_stride + (n % p.group) * A * BINS;
    const bool vec_out = out_vec_ok<OUT>(out_map, A * BINS, p.group_stride);
    const int y_all = (p.nby - 1) * p.sy + p.bh;         // rows below belong to no block
    const int x_hi = (p.nbx - 1) * p.sx + p.bw;          // columns to the right belong to no block
    const int q_hi = (x_hi + 3) >> 2;
    const int wide = x_hi > 128 ? 1 : 0;
    const int TCOLS = wide ? 64 : 32, TROWS = HIST_THREADS / TCOLS;
    const int tcol = threadIdx.x & (TCOLS - 1), trow = threadIdx.x / TCOLS;
    int next_flush = 0;                                  // first block row not yet written out
    for (int y0 = 0; y0 < y_all; y0 += p.phase_rows) {
        const int y1 = min(y0 + p.phase_rows, y_all);
        for (int y = y0 + trow; y < y1; y += TROWS) {
            int ilo, ihi;
            block_range(y, p.bh, p.sy, p.magic_sy, 0, p.nby, ilo, ihi);
            const int slot_lo = ilo % p.ring;
            const float *row = base + (int64_t)y * p.w;
            for (int xq = tcol; xq < q_hi; xq += TCOLS) {
                const float *src = row + 4 * xq;
                unsigned code[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int l = 0; l < L2; ++l) {
                    const float4 v = load_streamed4(src + l * P);        // every pixel is read once
                    code[0] |= (v.x > 0.0f ? 1u : 0u) << l;
                    code[1] |= (v.y > 0.0f ? 1u : 0u) << l;
                    code[2] |= (v.z > 0.0f ? 1u : 0u) << l;
                    code[3] |= (v.w > 0.0f ? 1u : 0u) << l;
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int x = 4 * xq + k;
                    if (x >= x_hi) break;
                    int jlo, jhi;
                    block_range(x, p.bw, p.sx, p.magic_sx, 0, p.nbx, jlo, jhi);
                    const unsigned inc = 1u << (16 * (code[k] & 1));
                    const unsigned word = code[k] >> 1;
                    int slot = slot_lo;
                    for (int i = ilo; i <= ihi; ++i) {
                        for (int j = jlo; j <= jhi; ++j) atomicAdd(&lds_hist[slot * row_words + j * WORDS + word], inc);
                        slot = slot + 1 == p.ring ? 0 : slot + 1;
                    }
                }
            }
        }
        __syncthreads();
        // block rows whose last pixel row lies inside the rows swept so far are complete: write them, clear their slots
        const int i_end = y1 < p.bh ? 0 : min(p.nby, fast_div(y1 - p.bh, p.sy, p.magic_sy) + 1);
        for (int i = next_flush; i < i_end; ++i)
            copy_out_rows<L2, OUT, true>(lds_hist + (i % p.ring) * row_words, 1, p.nbx, out_map + (int64_t)i * p.nbx * BINS,
                                         (int64_t)p.nbx * BINS, vec_out, lds_lut, p);
        next_flush = max(next_flush, i_end);
        __syncthreads();
    }
}

template <int L2, int OUT, bool CODES = false>
static void hist_launch(ddcca_ctx *ctx, HistParams p, int64_t n)
{
    constexpr int BINS = 1 << L2;
    constexpr int HIST_BYTES = (BINS > 1 ? BINS / 2 : 1) * 4;         // packed histogram of one block
    constexpr int ESZ = (int)sizeof(typename HistOut<OUT>::type);
    // sweep kernel: aligned float4 rows and a ring of block rows within the LDS budget.  A phase covers m block
    // strides (enough rows for about two 4-pixel groups per thread); during it the block rows from the oldest
    // incomplete one to the newest one touched are live: ceil(bh / sy) + m - 1 of them.
    if (!CODES && p.vec4 && (p.nbx - 1) * p.sx + p.bw > 256) {
        const int row_bytes = p.nbx * HIST_BYTES;
        const int live = (p.bh + p.sy - 1) / p.sy;
        const int quads_per_stride = (((p.nbx - 1) * p.sx + p.bw + 3) / 4) * p.sy;
        int m = std::max(1, (2 * HIST_THREADS + quads_per_stride - 1) / quads_per_stride);
        m = std::min(m, std::max(1, SWEEP_LDS_BYTES / row_bytes - live + 1));
        m = std::min(m, p.nby);
        const int ring = live + m - 1;
        if ((int64_t)ring * row_bytes <= SWEEP_LDS_BYTES) {
            p.ring = ring;
            p.phase_rows = m * p.sy;
            const int hist_words = ring * (row_bytes / 4);
            const size_t lds = (size_t)hist_words * 4 + (OUT != DDCCA_FEAT_COUNT_U16 ? (size_t)p.lut_n * 4 : 0);
            const int64_t maps_per_launch = std::max<int64_t>(p.group, ((int64_t)1 << 30) / p.group * p.group);
            for (int64_t n0 = 0; n0 < n; n0 += maps_per_launch) {
                const int64_t nb = std::min(maps_per_launch, n - n0);
                HistParams q = p;
                q.maps = p.maps + n0 * L2 * (int64_t)p.h * p.w;
                q.hist = reinterpret_cast<char *>(p.hist) + (n0 / p.group) * p.group_stride * ESZ;
                hipLaunchKernelGGL((hash_hist_sweep_kernel<L2, OUT>), dim3((unsigned)nb), dim3(HIST_THREADS), lds,
                                   ctx->stream, q, hist_words);
            }
            return;
        }
    }
    const int lut_bytes = OUT != DDCCA_FEAT_COUNT_U16 ? p.lut_n * 4 : 0;
    const bool wide = !CODES && p.w > 128;
    const int max_blocks = std::max(1, ((wide ? HIST_LDS_BYTES_WIDE : HIST_LDS_BYTES) - lut_bytes) / HIST_BYTES);
    p.cols = std::min(p.nbx, max_blocks);
    p.col_chunks = (p.nbx + p.cols - 1) / p.cols;
    // several block rows per workgroup cut the re-reading of the rows that overlapping blocks share; the fewest row
    // groups the budget allows, equally high
    const int rb_max = std::max(1, std::min(p.nby, max_blocks / p.cols));
    p.row_groups = (p.nby + rb_max - 1) / rb_max;
    p.rb = (p.nby + p.row_groups - 1) / p.row_groups;
    p.row_groups = (p.nby + p.rb - 1) / p.rb;
    const int hist_words = p.rb * p.cols * (HIST_BYTES / 4);
    const size_t lds = (size_t)hist_words * 4 + (OUT != DDCCA_FEAT_COUNT_U16 ? (size_t)p.lut_n * 4 : 0);
    const int64_t per_map = (int64_t)p.row_groups * p.col_chunks;
    // the pipelined form when a thread has one group of four columns and at least three rows of a row group
    const int span = (p.cols - 1) * p.sx + p.bw, group_rows = (p.rb - 1) * p.sy + p.bh;
    const int tcols = span > 128 ? 64 : 32;
    // (groups of four columns a chunk spans: its first column is a multiple of cols * sx)
    const int quads = (span + 3) / 4 + ((p.col_chunks > 1 && (p.cols * p.sx) % 4 != 0) ? 1 : 0);
    const bool pipe = !CODES && p.vec4 && quads <= tcols && group_rows >= 3 * (HIST_THREADS / tcols);
    const int64_t maps_per_launch = std::max<int64_t>(p.group, (((int64_t)1 << 30) / per_map) / p.group * p.group);
    for (int64_t n0 = 0; n0 < n; n0 += maps_per_launch) {
        const int64_t nb = std::min(maps_per_launch, n - n0);
        HistParams q = p;
        if (CODES) q.codes = p.codes + n0 * ((L2 + 7) / 8) * (int64_t)p.h * p.w;
        else q.maps = p.maps + n0 * L2 * (int64_t)p.h * p.w;
        q.hist = reinterpret_cast<char *>(p.hist) + (n0 / p.group) * p.group_stride * ESZ;
        if (pipe)
            hipLaunchKernelGGL((hash_hist_kernel<L2, OUT, false, true>), dim3((unsigned)(nb * per_map)),
                               dim3(HIST_THREADS), lds, ctx->stream, q, hist_words);
        else
            hipLaunchKernelGGL((hash_hist_kernel<L2, OUT, CODES>), dim3((unsigned)(nb * per_map)), dim3(HIST_THREADS),
                               lds, ctx->stream, q, hist_words);
    }
}

template <int OUT>
static int hist_dispatch(ddcca_ctx *ctx, const HistParams &p, int64_t n, int L2)
{
    if (p.codes) {
        switch (L2) {
#define CASE(v) case v: hist_launch<v, OUT, true>(ctx, p, n); break;
            CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12)
#undef CASE
            default: return fail(ctx, DDCCA_EINVAL, "L2 out of range");
        }
        return DDCCA_OK;
    }
    switch (L2) {
#define CASE(v) case v: hist_launch<v, OUT>(ctx, p, n); break;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8) CASE(9) CASE(10) CASE(11) CASE(12)
#undef CASE
        default: return fail(ctx, DDCCA_EINVAL, "L2 out of range");
    }
    return DDCCA_OK;
}

int prepare_iq_table(ddcca_ctx *ctx, int out_type, int bh, int bw, int L2, const float **lut, int *lut_n,
                     double *log_total)
{
    *lut = nullptr;
    *lut_n = 0;
    *log_total = 0.0;
    if (out_type == DDCCA_FEAT_COUNT_U16) return DDCCA_OK;
    // values for counts 0 .. min(area, IQ_LUT_MAX - 1), rebuilt when the block area or bin count changes
    const int64_t total = (int64_t)bh * bw + ((int64_t)1 << L2);
    const int n = (int)std::min<int64_t>((int64_t)bh * bw + 1, IQ_LUT_MAX);
    int rc;
    if ((rc = ensure(ctx, ctx->iq_lut, IQ_LUT_MAX * sizeof(float)))) return rc;
    if (ctx->iq_lut_total != total || ctx->iq_lut_n != n) {
        hipLaunchKernelGGL(iq_lut_kernel, dim3(1), dim3(256), 0, ctx->stream, (double)total, n,
                           (float *)ctx->iq_lut.ptr);
        DDCCA_HIP(ctx, hipGetLastError());
        ctx->iq_lut_total = total;
        ctx->iq_lut_n = n;
    }
    *lut = (const float *)ctx->iq_lut.ptr;
    *lut_n = n;
    *log_total = std::log((double)total);
    return DDCCA_OK;
}

static int hist_run(ddcca_ctx *ctx, const float *maps, const unsigned char *codes, int64_t n, int L2, int h, int w,
                    int bh, int bw, int sy, int sx, void *out, int out_type, int64_t group, int64_t group_stride,
                    int kernel_id)
{
    HistParams p;
    p.maps = maps; p.codes = codes; p.hist = out;
    p.h = h; p.w = w; p.bh = bh; p.bw = bw; p.sy = sy; p.sx = sx;
    p.nby = (h - bh) / sy + 1;
    p.nbx = (w - bw) / sx + 1;
    p.group = group; p.group_stride = group_stride;
    // rows readable as aligned groups of four pixels: 16 bytes of floats, or 4 bytes of codes
    p.vec4 = codes ? (((w & 3) == 0 && (((uintptr_t)codes) & 3) == 0) ? 1 : 0)
                   : (((w & 3) == 0 && (((uintptr_t)maps) & 15) == 0) ? 1 : 0);
    const bool small = h < 65536 && w < 65536;
    p.magic_sy = small ? (unsigned)((((uint64_t)1 << 32) + sy - 1) / sy) : 0u;
    p.magic_sx = small ? (unsigned)((((uint64_t)1 << 32) + sx - 1) / sx) : 0u;
    int rc;
    if ((rc = prepare_iq_table(ctx, out_type, bh, bw, L2, &p.lut, &p.lut_n, &p.log_total))) return rc;
    ProfScope prof(ctx, kernel_id);
    switch (out_type) {
        case DDCCA_FEAT_COUNT_U16: rc = hist_dispatch<DDCCA_FEAT_COUNT_U16>(ctx, p, n, L2); break;
        case DDCCA_FEAT_IQ_F32: rc = hist_dispatch<DDCCA_FEAT_IQ_F32>(ctx, p, n, L2); break;
        case DDCCA_FEAT_IQ_F16: rc = hist_dispatch<DDCCA_FEAT_IQ_F16>(ctx, p, n, L2); break;
        default: return fail(ctx, DDCCA_EINVAL, "unknown feature type");
    }
    if (rc) return rc;
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

int launch_hash_hist(ddcca_ctx *ctx, const float *maps, int64_t n, int L2, int h, int w, int bh, int bw, int sy,
                     int sx, void *out, int out_type, int64_t group, int64_t group_stride)
{
    return hist_run(ctx, maps, nullptr, n, L2, h, w, bh, bw, sy, sx, out, out_type, group, group_stride,
                    DDCCA_K_HASH_HIST);
}

// The same histograms from code maps (one byte per pixel and 8 filters, launch_conv_split_codes): the second half of the fused
// last stage when the convolution runs on three-piece operands.
int launch_code_hist(ddcca_ctx *ctx, const unsigned char *codes, int64_t n, int L2, int h, int w, int bh, int bw,
                     int sy, int sx, void *out, int out_type, int64_t group, int64_t group_stride)
{
    return hist_run(ctx, nullptr, codes, n, L2, h, w, bh, bw, sy, sx, out, out_type, group, group_stride,
                    DDCCA_K_CONV_HASH_HIST);
}

}  // namespace ddcca
