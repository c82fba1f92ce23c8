// Lag-structured accumulation of the patch Gram (Section II-A matrices; an algebraic shortcut the paper does not
// use).  With the images extended by zeros, entry (a, b) of the raw patch Gram summed over ALL patch centres of
// the plane depends only on the lag between the two taps:
//     sum_p X[p + s_a] X'[p + s_b] = R_{s_b - s_a},    R_d = sum_u X[u] X'[u + d],
// (2k-1)^2 lag correlations per view pair instead of k^4 entries.  The sum wanted runs over the patch centres
// inside the image only: with u = p + s_a that is the same sum over u with up to r rows at the top or bottom and
// up to r columns at the left or right of the image left out (which ones depends on the first tap a), so next to
// R_d the kernels keep the contributions of the r first and last image rows (lag_gram_kernel, per row group)
// and of the r first and last columns and the corners (lag_cols_kernel).  Everything downstream (centre-pixel
// form, H M H export, solve) is unchanged: lag_to_stacked_kernel writes  sum y y^T  for y = x - x_centre in the
// layout of the dense kernel's slots from
//     S_y[a][b] = S_x[a][b] - S_x[a][c] - S_x[c][b] + S_x[c][c]          (c = the centre tap).
//
// The lag correlations run on v_mfma_f32_16x16x4_f32 along image rows, K = 4 consecutive pixels x' of a row per
// instruction.  All four ORDERED view pairs (1,1) (2,2) (1,2) (2,1) are kept, so a horizontal lag dx < 0 is read
// as the exchanged pair at the negated lag and the rows of the instruction only hold dx = 0 .. k-1; RG = 2 / 3 /
// 5 image rows (k = 7 / 5 / 3) then share one instruction (geometry: LagGeom below):
//     A[(rho,dx)][x'] = X[y0 + rho][x' - dx],   B[x'][c] = X'[y0 + c - (k-1)][x'],
//     D[(rho,dx)][rho + dy + k-1] += sum_x' A B   = lag (dy, dx) of image row y0 + rho.
// The raw products carry the DC level of the images, which the differences to the centre pixel of the dense
// kernel do not, so the fp32 accumulators (each a sum along one image row) are added to fp64 registers after
// every row group.
// k = 9 has 17 vertical lags, one more than the instruction has columns: there an instruction holds one image
// row and the lags -8 .. 7 on both axes, an entry whose lag has a component +8 is taken as the transposed entry
// (S_x[a][b] of the pair (d,d') = S_x[b][a] of (d',d), lag negated), and the single tap pair whose lag is
// (+8,-8) -- opposite corners of the patch -- is summed directly by lag_special_kernel.
#include "ddcca_internal.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int LAG_THREADS = 256;
constexpr int LAG_TW_MAX = 128;            // image columns per tile (multiple of 4)

// Geometry of the lag statistics for patch side KS.  The four ORDERED pair types (1,1) (2,2) (1,2) (2,1) are kept
// for every k, so that a horizontal lag dx < 0 can be read as the exchanged pair at the negated lag and the rows
// of the matrix instruction only have to hold dx = 0 .. K: RG consecutive image rows then share one instruction
// (rows (rho, dx), rho = image row inside the group; columns = vertical offset from the group's first row,
// c = rho + dy + K).  k = 9 keeps dx = -K .. K-1 in its sixteen rows, one image row at a time.
template <int KS>
struct LagGeom {
    static constexpr int K = KS - 1;                   // largest lag
    static constexpr int RR = (KS - 1) / 2;            // patch radius = border rows / columns kept apart
    static constexpr bool WIDE = 2 * K + 1 > 16;       // k = 9
    static constexpr int NL = WIDE ? 16 : 2 * K + 1;   // lags per axis in the border-column statistics: -K .. NL-1-K
    static constexpr int NLL = NL * NL;
    static constexpr int NTY = 4;                      // pair types (1,1) (2,2) (1,2) (2,1)
    static constexpr int E = NTY * 256;                // doubles per row set: one 16 x 16 tile per type
    static constexpr int NJ = WIDE ? 16 : K + 1;       // horizontal lags held per image row
    static constexpr int DX0 = WIDE ? -K : 0;          // the first of them
    static constexpr int RG = 16 / NJ;                 // image rows per matrix instruction
    static constexpr int CMAX = WIDE ? 15 : RG - 1 + 2 * K;   // last column in use
    static constexpr int TH = KS == 7 ? 24 : KS == 5 ? 24 : KS == 3 ? 20 : 16;   // image rows per tile: a multiple of 4 RG
    static constexpr int NTG = (RR + RG - 1) / RG;     // row groups that hold one of the RR top rows
    static constexpr int NBG = (RR - 1 + RG - 1) / RG + 1;   // ... bottom rows (whatever the image height)
    static constexpr int SETS = 1 + NTG + NBG;         // all rows; top groups; bottom groups
    static constexpr int SLOT = SETS * E + (WIDE ? 8 : 0);   // lag_gram_kernel slot (+ lag_special_kernel's)
    static_assert(CMAX <= 15 && RG * NJ <= 16 && TH % (4 * RG) == 0 && NTG <= 4 && NBG <= 4, "lag geometry");
};
// view (0 / 1) of the first and of the second factor of a pair type
__host__ __device__ constexpr int lag_view_a(int t) { return (t == 1 || t == 3) ? 1 : 0; }
__host__ __device__ constexpr int lag_view_b(int t) { return (t == 1 || t == 2) ? 1 : 0; }

struct LagParams {
    const float *v1, *v2;                  // [n_maps][h][w]
    int h, w, tiles_x, tiles_y, tw;
    int pitch, view_stride;                // LDS floats per tile row / per view
    int64_t n_items;                       // n_maps * tiles_y * tiles_x
    double *slots;                         // [grid][SLOT]
    int slots_valid;                       // slots below this hold earlier sums
};

// One workgroup walks a contiguous range of (map, tile) items.  A tile is TH image rows x tw columns with a halo
// of K = k-1 on every side (zeros outside the image), both views.  Wavefront w owns the row groups w, w+4, ... of
// a tile; tiles start at multiples of 4 RG rows, so row group gi of the IMAGE always belongs to wavefront gi % 4.
template <int KS>
__global__ __launch_bounds__(LAG_THREADS) void lag_gram_kernel(LagParams p)
{
    using G = LagGeom<KS>;
    constexpr int K = G::K, RR = G::RR, NTY = G::NTY, RG = G::RG, TH = G::TH, NTG = G::NTG, NBG = G::NBG;
    constexpr int NMF = 4;                         // matrix instructions per step
    extern __shared__ float lds[];
    typedef __attribute__((address_space(3))) float lds_float;
    typedef __attribute__((address_space(3))) char lds_char;
    const lds_char *const lds_base = (const lds_char *)lds;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: what depends on it stays on the scalar unit
    // this lane's row (rho, dx) of the A operand and column c of the B operand (rows / columns past the ones in
    // use repeat the last)
    const int irow = min(lane & 15, RG * G::NJ - 1);
    const int rho = irow / G::NJ, dx = irow - rho * G::NJ + G::DX0;
    const int ccol = min(lane & 15, G::CMAX);
    const int kk = lane >> 4;
    const int PH = TH + 2 * K, PW = p.tw + 2 * K;
    const int64_t per = p.n_items / gridDim.x, extra = p.n_items % gridDim.x;
    const int64_t first = blockIdx.x * per + min((int64_t)blockIdx.x, extra);
    const int64_t count = per + (blockIdx.x < extra ? 1 : 0);
    const int tiles = p.tiles_x * p.tiles_y;
    const int64_t P = (int64_t)p.h * p.w;
    double accd[NTY][4], acct[NTY][4], accb[NTY][4];     // all rows; this wavefront's top / bottom row group
#pragma unroll
    for (int t = 0; t < NTY; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) accd[t][v] = acct[t][v] = accb[t][v] = 0.0;
    // Row groups that hold border rows: the top ones are groups 0 .. NTG-1 (owners: wavefronts 0 .. NTG-1), the
    // bottom ones the groups gb0 .. glast of the rows h-RR .. h-1 (at most NBG <= 4 consecutive groups: one owner
    // each).  A wavefront keeps the sums of its top group and of its bottom group in register sets of their own.
    const int gb0 = max(0, p.h - RR) / RG, glast = (p.h - 1) / RG;
    const int my_top = (wave < NTG && wave * RG < p.h) ? wave : -1;
    const int cand = gb0 + ((wave - gb0 % 4) + 4) % 4;
    const int my_bot = cand <= glast ? cand : -1;
    // A operand: image row y0 + rho = tile row y + rho + K, column x' - dx = tile column x' + K - dx
    // B operand: image row y0 + c - K = tile row y + c, column x' = tile column x' + K
    const int a_off = (rho + K) * p.pitch + kk - dx + K;
    const int b_off = ccol * p.pitch + kk + K;
    // Tile staging: thread (wave w, lane l) owns tile elements (row w + 4 jy, column l + 64 jx).  The loads of the
    // next tile are issued before the current one is contracted and written to LDS afterwards, so their latency
    // hides behind the matrix work.
    constexpr int NJY = (TH + 2 * K + 3) / 4, NJX = (LAG_TW_MAX + 2 * K + 63) / 64;
    float fa[NJY][NJX], fb[NJY][NJX];
    auto fetch = [&](int64_t item) {
        const int64_t mp = item / tiles;
        const int t = (int)(item - mp * tiles);
        const int ty = t / p.tiles_x, tx = t - ty * p.tiles_x;
        const int gy0 = ty * TH - K + wave, gx0 = tx * p.tw - K + lane;
        const float *s1 = p.v1 + mp * P, *s2 = p.v2 + mp * P;
#pragma unroll
        for (int jy = 0; jy < NJY; ++jy) {
            const int gy = gy0 + 4 * jy;
            const bool yok = gy >= 0 && gy < p.h && wave + 4 * jy < PH;
#pragma unroll
            for (int jx = 0; jx < NJX; ++jx) {
                const int gx = gx0 + 64 * jx;
                float a = 0.f, b = 0.f;
                if (yok && gx >= 0 && gx < p.w && lane + 64 * jx < PW) {
                    const int64_t o = (int64_t)gy * p.w + gx;
                    a = s1[o];
                    b = s2[o];
                }
                fa[jy][jx] = a;
                fb[jy][jx] = b;
            }
        }
    };
    auto store = [&]() {
#pragma unroll
        for (int jy = 0; jy < NJY; ++jy) {
            const int yy = wave + 4 * jy;
#pragma unroll
            for (int jx = 0; jx < NJX; ++jx) {
                const int xx = lane + 64 * jx;
                if (yy < PH && xx < PW) {
                    lds[yy * p.pitch + xx] = fa[jy][jx];
                    lds[p.view_stride + yy * p.pitch + xx] = fb[jy][jx];
                }
            }
        }
    };
    if (count > 0) {
        fetch(first);
        store();
    }
    __syncthreads();
    for (int64_t it = 0; it < count; ++it) {
        const int64_t item = first + it;
        const int64_t mp = item / tiles;
        const int t = (int)(item - mp * tiles);
        const int ty = t / p.tiles_x, tx = t - ty * p.tiles_x;
        const bool more = it + 1 < count;
        if (more) fetch(item + 1);
        const int rows = min(TH, p.h - ty * TH);
        const int cols = min(p.tw, p.w - tx * p.tw);
        const int steps = (cols + 3) >> 2;            // tw is a multiple of 4: columns past the image hold zeros
        // The fp32 accumulators are added to the fp64 registers after every row group (a sum along ONE image row
        // per accumulator row): the raw products carry the DC level of the images, and sums over several rows of
        // a view with a large DC level already cost a digit (measured 3e-6 instead of 1e-6 relative on C22 when
        // four rows were summed in fp32).
        floatx4 c[NTY];
#pragma unroll
        for (int t2 = 0; t2 < NTY; ++t2) c[t2] = floatx4{0.f, 0.f, 0.f, 0.f};
        // (is_top / is_bot are the same for the whole wavefront.  The empty asm statements keep the compiler from
        // turning the rare border-group additions into unconditional ones with selects, and from holding the
        // converted values of the common path in registers for them.)
        auto flush = [&](bool is_top, bool is_bot) {
            auto border = [&](double (&acc)[NTY][4]) {
#pragma unroll
                for (int t2 = 0; t2 < NTY; ++t2) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float x = c[t2][v];
                        asm volatile("" : "+v"(x));
                        acc[t2][v] += (double)x;
                    }
                }
            };
            if (is_top) border(acct);
            if (is_bot) border(accb);
#pragma unroll
            for (int t2 = 0; t2 < NTY; ++t2) {
#pragma unroll
                for (int v = 0; v < 4; ++v) accd[t2][v] += (double)c[t2][v];
                c[t2] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
        };
        // one step: a1 x b1 -> (1,1), a2 x b2 -> (2,2), a1 x b2 -> (1,2), a2 x b1 -> (2,1)
        auto step = [&](float a1, float b2, float a2, float b1) {
            c[0] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b1, c[0], 0, 0, 0);
            c[1] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2, b2, c[1], 0, 0, 0);
            c[2] = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, b2, c[2], 0, 0, 0);
            c[3] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2, b1, c[3], 0, 0, 0);
        };
        const int g_tile = ty * (TH / RG);            // image row group of the tile's first
        for (int g = wave; g * RG < rows; g += 4) {
            const int y = g * RG;                     // first tile row of the group
            const float *ra1 = lds + y * p.pitch + a_off, *rb1 = lds + y * p.pitch + b_off;
            const float *ra2 = ra1 + p.view_stride, *rb2 = rb1 + p.view_stride;
            const int gi = g_tile + g;
            const bool is_top = gi == my_top, is_bot = gi == my_bot;
            // Two steps form a pair whose operands come in two-address LDS reads; the pairs alternate between
            // two operand sets so that the reads of the next pair are in flight during the MFMAs of this one.
            // The four operand streams advance through one running pointer each, every read at a constant
            // offset from it.  o[] = a1, a1', b2, b2', a2, a2', b1, b1'
            // (byte addresses inside LDS, made opaque so that each stays ONE register that the reads offset)
            unsigned qa1 = (unsigned)((y * p.pitch + a_off) * 4), qb2 = (unsigned)((p.view_stride + y * p.pitch + b_off) * 4);
            unsigned qa2 = qa1 + (unsigned)p.view_stride * 4, qb1 = qb2 - (unsigned)p.view_stride * 4;
            asm volatile("" : "+v"(qa1), "+v"(qb2), "+v"(qa2), "+v"(qb1));
            auto at = [&](unsigned q, int off) { return *(const lds_float *)(lds_base + q + 4 * off); };
            auto load_pair = [&](float (&o)[8], int off) {
                o[0] = at(qa1, off); o[1] = at(qa1, off + 4);
                o[2] = at(qb2, off); o[3] = at(qb2, off + 4);
                o[4] = at(qa2, off); o[5] = at(qa2, off + 4);
                o[6] = at(qb1, off); o[7] = at(qb1, off + 4);
                __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);                 // LDS reads first
            };
            auto mfma_pair = [&](const float (&o)[8]) {
                step(o[0], o[2], o[4], o[6]);
                step(o[1], o[3], o[5], o[7]);
                __builtin_amdgcn_sched_group_barrier(0x008, 2 * NMF, 0);           // then the MFMAs of the pair
            };
            const int np = steps >> 1;
            float oa[8], ob[8];
            if (np > 0) load_pair(oa, 0);
            int ip = 0;
            for (; ip + 1 < np; ip += 2) {
                load_pair(ob, 8);
                mfma_pair(oa);
                // (after the last pair of an even count this reads one pair further, at most tw + 2K + 7 floats
                // into the tile row: inside the row pitch or, in a view's last row, the pad behind it; unused)
                load_pair(oa, 16);
                mfma_pair(ob);
                qa1 += 64; qb2 += 64; qa2 += 64; qb1 += 64;
            }
            if (ip < np) mfma_pair(oa);
            if (steps & 1) {
                const int s = steps - 1;
                step(ra1[4 * s], rb2[4 * s], ra2[4 * s], rb1[4 * s]);
            }
            flush(is_top, is_bot);
        }
        __syncthreads();                              // every wavefront is done with the tile
        if (more) {
            store();
            __syncthreads();
        }
    }
    // workgroup total in fp64: the wavefronts add in order, then the slot takes it
    __syncthreads();
    double *st = reinterpret_cast<double *>(lds);
    for (int wv = 0; wv < 4; ++wv) {
        if (wave == wv) {
#pragma unroll
            for (int t = 0; t < NTY; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int e = (t * 4 + v) * 64 + lane;
                    st[e] = (wv == 0 ? 0.0 : st[e]) + accd[t][v];
                }
        }
        __syncthreads();
    }
    // slot: [SETS][E]: all rows, top row groups 0 .. NTG-1, bottom row groups gb0 .. gb0 + NBG-1
    double *slot = p.slots + (size_t)blockIdx.x * G::SLOT;
    const bool rmw = (int)blockIdx.x < p.slots_valid;
    for (int e = threadIdx.x; e < G::E; e += LAG_THREADS) slot[e] = (rmw ? slot[e] : 0.0) + st[e];
    // border groups: the owner writes its registers; sets of groups the image does not have are cleared
    if (!rmw) {
        for (int set = 0; set < NTG + NBG; ++set) {
            const bool owned = set < NTG ? set * RG < p.h : gb0 + (set - NTG) <= glast;
            if (!owned)
                for (int e = threadIdx.x; e < G::E; e += LAG_THREADS) slot[(size_t)(1 + set) * G::E + e] = 0.0;
        }
    }
    if (my_top >= 0) {
        double *d = slot + (size_t)(1 + my_top) * G::E;
#pragma unroll
        for (int t = 0; t < NTY; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int e = (t * 4 + v) * 64 + lane;
                d[e] = (rmw ? d[e] : 0.0) + acct[t][v];
            }
    }
    if (my_bot >= 0) {
        double *d = slot + (size_t)(1 + NTG + my_bot - gb0) * G::E;
#pragma unroll
        for (int t = 0; t < NTY; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int e = (t * 4 + v) * 64 + lane;
                d[e] = (rmw ? d[e] : 0.0) + accb[t][v];
            }
    }
}

// ---- border columns ------------------------------------------------------------------------------------
// What the lag correlations over-count is the part of  sum_u X[u] X'[u + d]  whose u lies in the first or last
// rows / columns of the image (which ones depends on the first tap, see lag_entry below).  The rows come out of
// lag_gram_kernel; this kernel adds up, per border column c (r on either side) and lag d,
//     colsum[c][d] = sum_y X[y][c] X'[y + dy][c + dx]
// and keeps the terms of the r top and r bottom rows apart (the corners, which rows and columns both cover).
// The column sums are the lag kernel's contraction turned by ninety degrees, one column at a time:
//     A[dy][y'] = X[y' - dy][c],   B[y'][dx] = X'[y'][c + dx],   D[dy][dx] += sum_y' A B     (y' = y + dy),
// on v_mfma_f32_16x16x4_f32 with K = 4 consecutive rows; the corner terms are single products on the vector ALU.
// grid (image ranges, side); a workgroup stages, per chunk of rows, the r + 2K columns next to its side of both
// views; the (column, pair type) chains are dealt to the wavefronts, the corner entries to the threads.
// Slot of a workgroup row: [type][side][column offset] x ( 256 doubles: the column sums in accumulator layout,
// row = vertical lag index; then [2r][NL^2]: the terms of top row o (index o) and bottom row h-1-o (r + o) ).
constexpr int LAGC_ROWS = 64;              // image rows per chunk (a multiple of 4)
// threads: 256, from k = 7 on 512 (twelve / sixteen chains and 2028 / 4096 corner triples to share out)
template <int KS>
constexpr int lagc_threads() { return KS >= 7 ? 512 : 256; }
// wavefronts per SIMD the register budget is cut for
template <int KS>
constexpr int lagc_waves() { return KS >= 9 ? 2 : KS >= 7 ? 4 : 3; }

struct LagColParams {
    const float *v1, *v2;
    int h, w;
    int64_t n_maps;
    double *slots;                         // [gridDim.x][NTY][2][r][256 + 2r*NL*NL]
    int slots_valid;
};

template <int KS>
__global__ __launch_bounds__(lagc_threads<KS>(), lagc_waves<KS>()) void lag_cols_kernel(LagColParams p)
{
    using G = LagGeom<KS>;
    constexpr int K = G::K, NL = G::NL, NLL = G::NLL, RR = G::RR, NTY = G::NTY;
    constexpr int LAGC_THREADS = lagc_threads<KS>(), NW = LAGC_THREADS / 64;
    constexpr int BW = RR + 2 * K;         // staged columns: the r border columns and K more on either side
    constexpr int BH = LAGC_ROWS + 2 * K;  // staged rows: the chunk and K more on either side
    constexpr int ENTRY = 256 + 2 * RR * NLL;                      // doubles per (type, side, column)
    constexpr int NCH = (NTY * RR + NW - 1) / NW;                  // chains per wavefront at most
    constexpr int NCE = (NTY * RR * NLL + LAGC_THREADS - 1) / LAGC_THREADS;   // (type, column, lag) triples per thread
    __shared__ float sb[2][BH * BW];       // view d: rows y0 - K .., columns cb0 .. (zeros outside the image)
    const int side = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: what depends on it stays on the scalar unit
    const int m = min(lane & 15, NL - 1), kk = lane >> 4;
    const int cb0 = side == 0 ? -K : p.w - RR - K;                 // image column of staged column 0
    constexpr int ntype = NTY, t0 = 0;                             // every pair type
    const int nchain = RR * ntype;
    const int64_t per = p.n_maps / gridDim.x, extra = p.n_maps % gridDim.x;
    const int64_t first = blockIdx.x * per + min((int64_t)blockIdx.x, extra);
    const int64_t count = per + (blockIdx.x < extra ? 1 : 0);
    const int64_t P = (int64_t)p.h * p.w;
    // (a workgroup adds few images' single products per corner entry: fp32 is enough there; fp64 from the slot on)
    double colsum[NCH][4];
    float corner[NCE][2 * RR];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v) colsum[c][v] = 0.0;
    // corner terms: thread-owned triples (pair type, column offset, lag), number tid + 256 j; per triple the 2r
    // border rows.  Decoded once: staged offsets of the two factors inside a staged row, and the views.
    int cor_a[NCE], cor_b[NCE];            // offset of X[.][ca] and of X'[. + dy][ca + dx] relative to the row start
    bool cor_on[NCE], cor_a2[NCE], cor_b2[NCE];
#pragma unroll
    for (int j = 0; j < NCE; ++j) {
        const int e = tid + LAGC_THREADS * j;
        const int li = e % NLL, rest = e / NLL;
        const int ox = rest % RR, ti = rest / RR;
        const int t = t0 + ti;
        const int ca = side == 0 ? ox : p.w - 1 - ox;
        cor_on[j] = e < ntype * RR * NLL && ca >= 0 && ca < p.w;
        cor_a[j] = ca - cb0;
        cor_b[j] = (li / NL - K) * BW + (ca - cb0) + li % NL - K;
        cor_a2[j] = lag_view_a(t) == 1;
        cor_b2[j] = lag_view_b(t) == 1;
#pragma unroll
        for (int q = 0; q < 2 * RR; ++q) corner[j][q] = 0.f;
    }
    // (image, chunk) pairs in one sequence; the loads of the next pair are issued before this one is worked on
    // and written to LDS afterwards
    constexpr int NST = (BH * BW + LAGC_THREADS - 1) / LAGC_THREADS;
    const int nchunk = (p.h + LAGC_ROWS - 1) / LAGC_ROWS;
    const int64_t total = count * nchunk;
    float f1[NST], f2[NST];
    auto fetch = [&](int64_t it) {
        const int64_t mp = first + it / nchunk;
        const int y0 = (int)(it % nchunk) * LAGC_ROWS;
        const int rows = min(LAGC_ROWS, p.h - y0);
        const float *i1 = p.v1 + mp * P, *i2 = p.v2 + mp * P;
#pragma unroll
        for (int j = 0; j < NST; ++j) {
            const int e = tid + LAGC_THREADS * j;
            const int yy = e / BW, xx = e - yy * BW;
            const int gy = y0 - K + yy, gx = cb0 + xx;
            // (all BH rows are written: the last steps of a ragged chunk read up to three rows past rows + 2K)
            const bool ok = e < BH * BW && yy < rows + 2 * K && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w;
            f1[j] = ok ? i1[(int64_t)gy * p.w + gx] : 0.f;
            f2[j] = ok ? i2[(int64_t)gy * p.w + gx] : 0.f;
        }
    };
    auto store = [&]() {
#pragma unroll
        for (int j = 0; j < NST; ++j) {
            const int e = tid + LAGC_THREADS * j;
            if (e < BH * BW) {
                sb[0][e] = f1[j];
                sb[1][e] = f2[j];
            }
        }
    };
    if (total > 0) {
        fetch(0);
        store();
    }
    __syncthreads();
    for (int64_t it = 0; it < total; ++it) {
        {
            const int y0 = (int)(it % nchunk) * LAGC_ROWS;
            const int rows = min(LAGC_ROWS, p.h - y0);
            const bool more = it + 1 < total;
            if (more) fetch(it + 1);
            // column sums: chain (column offset ox, pair type) number ox * ntype + t belongs to wavefront chain % NW;
            // the chains of a wavefront advance together, one step each at a time
            const int steps = (rows + 3) >> 2;                     // rows past the image hold zeros
            const float *pa[NCH], *pb[NCH];
            bool on[NCH];
            floatx4 d[NCH];
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const int chain = wave + NW * c;
                const int ox = chain / ntype, t = t0 + chain - ox * ntype;
                const int ca = side == 0 ? ox : p.w - 1 - ox;      // image column of the first operand
                on[c] = chain < nchain && ca >= 0 && ca < p.w;
                const int cx = on[c] ? ca - cb0 : K;
                // A: row y' - dy = staged row 4s + kk - m + 2K, column ca;  B: row y' = staged row 4s + kk + K,
                // column ca + dx = staged column (ca - cb0) + m - K
                pa[c] = sb[lag_view_a(t)] + (kk - m + 2 * K) * BW + cx;
                pb[c] = sb[lag_view_b(t)] + (kk + K) * BW + cx + m - K;
                d[c] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
            for (int s = 0; s < steps; ++s) {
#pragma unroll
                for (int c = 0; c < NCH; ++c)
                    if (on[c]) d[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(pa[c][4 * s * BW], pb[c][4 * s * BW], d[c], 0, 0, 0);
            }
#pragma unroll
            for (int c = 0; c < NCH; ++c)
                if (on[c])
#pragma unroll
                    for (int v = 0; v < 4; ++v) colsum[c][v] += (double)d[c][v];
            // corner terms of the border rows inside this chunk: q = o (top row o) or RR + o (bottom row h-1-o)
#pragma unroll
            for (int q = 0; q < 2 * RR; ++q) {
                const int o = q < RR ? q : q - RR;
                const int gy = q < RR ? o : p.h - 1 - o;
                if (o < p.h && gy >= y0 && gy < y0 + rows) {        // uniform over the workgroup
                    const int ro = (gy - y0 + K) * BW;
#pragma unroll
                    for (int j = 0; j < NCE; ++j)
                        if (cor_on[j])
                            corner[j][q] += sb[cor_a2[j] ? 1 : 0][ro + cor_a[j]] * sb[cor_b2[j] ? 1 : 0][ro + cor_b[j]];
                }
            }
            __syncthreads();                              // every wavefront is done with the staged block
            if (more) {
                store();
                __syncthreads();
            }
        }
    }
    // slot
    const bool rmw = (int)blockIdx.x < p.slots_valid;
    double *slot = p.slots + (size_t)blockIdx.x * NTY * 2 * RR * ENTRY;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int chain = wave + NW * c;
        if (chain < nchain) {
            const int ox = chain / ntype, t = t0 + chain - ox * ntype;
            double *d = slot + ((size_t)(t * 2 + side) * RR + ox) * ENTRY;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int e = v * 64 + lane;
                d[e] = (rmw ? d[e] : 0.0) + colsum[c][v];
            }
        }
    }
#pragma unroll
    for (int j = 0; j < NCE; ++j) {
        const int e = tid + LAGC_THREADS * j;
        if (e < ntype * RR * NLL) {
            const int li = e % NLL, rest = e / NLL;
            const int ox = rest % RR, ti = rest / RR;
            const int t = t0 + ti;
            double *d = slot + ((size_t)(t * 2 + side) * RR + ox) * ENTRY + 256 + li;
#pragma unroll
            for (int q = 0; q < 2 * RR; ++q) d[q * NLL] = (rmw ? d[q * NLL] : 0.0) + (double)corner[j][q];
        }
    }
}

// ---- the opposite-corner tap pair at k = 9 -----------------------------------------------------------------
// The one tap pair whose lag (+K, -K) no transposition brings into the range the matrix instruction holds:
// a* = top right tap, b* = bottom left tap.  Per ordered pair type (X, X')
//     V = sum over the patch centres p inside the image of  X[p + s_a*] X'[p + s_b*],
// summed directly, in fp64, into the eight doubles that follow a lag_gram_kernel slot (same grid, same slots).
struct LagSpecialParams {
    const float *v1, *v2;
    int h, w, r;
    int64_t n_maps;
    double *slots;                         // slot b: slots + b * slot_doubles + tail
    size_t slot_doubles, tail;
    int slots_valid;
};

__global__ __launch_bounds__(256) void lag_special_kernel(LagSpecialParams p)
{
    __shared__ double part[4][4];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: what depends on it stays on the scalar unit
    const int hp = p.h - 2 * p.r, wp = p.w - 2 * p.r;          // patch centres per column / row
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    if (hp > 0 && wp > 0) {
        const int64_t pp = (int64_t)hp * wp, total = p.n_maps * pp;
        const int64_t per = total / gridDim.x, extra = total % gridDim.x;
        const int64_t first = blockIdx.x * per + min((int64_t)blockIdx.x, extra);
        const int64_t end = first + per + (blockIdx.x < extra ? 1 : 0);
        const int64_t P = (int64_t)p.h * p.w;
        for (int64_t e = first + tid; e < end; e += 256) {
            const int64_t mp = e / pp;
            const int rem = (int)(e - mp * pp);
            const int py = rem / wp + p.r, px = rem % wp + p.r;
            const int64_t ua = mp * P + (int64_t)(py - p.r) * p.w + px + p.r;     // p + s_a*: r up, r to the right
            const int64_t ub = mp * P + (int64_t)(py + p.r) * p.w + px - p.r;     // p + s_b*: r down, r to the left
            const double a1 = p.v1[ua], a2 = p.v2[ua], b1 = p.v1[ub], b2 = p.v2[ub];
            s[0] += a1 * b1;
            s[1] += a2 * b2;
            s[2] += a1 * b2;
            s[3] += a2 * b1;
        }
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s[t] += __shfl_down(s[t], off, 64);
        if (lane == 0) part[wave][t] = s[t];
    }
    __syncthreads();
    if (tid < 4) {
        double *d = p.slots + (size_t)blockIdx.x * p.slot_doubles + p.tail + tid;
        const double v = part[0][tid] + part[1][tid] + part[2][tid] + part[3][tid];
        *d = ((int)blockIdx.x < p.slots_valid ? *d : 0.0) + v;
    }
}

// ---- from the statistics to the stacked Gram --------------------------------------------------------------
struct LagStats {
    const double *R;                       // [SETS][4][256] (+ 8 at k = 9): reduced lag_gram_kernel slots
    const double *C;                       // [4][2][r][256 + 2r*NL*NL]: reduced lag_cols_kernel slots
    int ks, h, w;
};

// the pair type with the two views exchanged
__device__ __forceinline__ int lag_type_swapped(int t) { return t == 2 ? 3 : t == 3 ? 2 : t; }

// host / device copy of the geometry for a run-time k
struct LagShape {
    int K, r, wide, NL, NJ, DX0, RG, NTG, NBG;
    __host__ __device__ explicit LagShape(int ks)
    {
        K = ks - 1;
        r = (ks - 1) / 2;
        wide = 2 * K + 1 > 16;
        NL = wide ? 16 : 2 * K + 1;
        NJ = wide ? 16 : K + 1;
        DX0 = wide ? -K : 0;
        RG = 16 / NJ;
        NTG = (r + RG - 1) / RG;
        NBG = (r - 1 + RG - 1) / RG + 1;
    }
};

// one element of a 16 x 16 row set in accumulator layout: row (rho, dx), column c
__device__ __forceinline__ double lag_set_value(const LagStats &st, const LagShape &g, int set, int type, int rho,
                                                int dx, int c)
{
    const int i = rho * g.NJ + dx - g.DX0;
    return st.R[(size_t)set * 1024 + (type * 4 + (i & 3)) * 64 + 16 * (i >> 2) + c];
}

// sum over the patch centres p INSIDE the image of X[p + s_a] X'[p + s_b] for the pair type (X, X'), a the tap
// of X: with u = p + s_a, u runs over the image minus the rows and columns that p + s_a can reach only from
// outside -- the first s rows if s = s_a.y > 0, the last -s if s < 0, the same for the columns -- so
//     = R(d) - (those rows of R) - (those columns) + (their corners),    d = s_b - s_a.
// The statistics hold the horizontal lags 0 .. K only (k = 9: -K .. K-1, vertical ones likewise): any other lag
// is looked up as the same sum with the factors exchanged (pair type swapped, taps swapped, lag negated), at
// k = 9 the lags (+K,-K) and (-K,+K) as the directly summed opposite-corner value.
__device__ double lag_entry(const LagStats &st, int type, int a, int b)
{
    const int ks = st.ks;
    const LagShape g(ks);
    const int r = g.r, K = g.K, NL = g.NL, NLL = NL * NL;
    int ay = a / ks, ax = a - ay * ks, by = b / ks, bx = b - by * ks;
    int dy = by - ay, dx = bx - ax;
    const bool out_of_range = g.wide ? (dy == K || dx == K) : dx < 0;
    if (out_of_range) {
        if (g.wide) {
            const double *special = st.R + (size_t)(1 + g.NTG + g.NBG) * 1024;
            if (dy == K && dx == -K) return special[type];
            if (dx == K && dy == -K) return special[lag_type_swapped(type)];
        }
        type = lag_type_swapped(type);
        int t = ay; ay = by; by = t;
        t = ax; ax = bx; bx = t;
        dy = -dy;
        dx = -dx;
    }
    const int sy = ay - r, sx = ax - r;
    const int ysd = sy > 0 ? 0 : 1, yn = min(sy > 0 ? sy : -sy, st.h);
    const int xsd = sx > 0 ? 0 : 1, xn = min(sx > 0 ? sx : -sx, st.w);
    // all rows: the image rows of a group sit in different accumulator rows
    double v = 0.0;
    for (int rho = 0; rho < g.RG; ++rho) v += lag_set_value(st, g, 0, type, rho, dx, rho + dy + K);
    // minus the yn first (ysd = 0) or last (ysd = 1) image rows
    const int gb0 = max(0, st.h - r) / g.RG;
    for (int o = 0; o < yn; ++o) {
        const int y = ysd == 0 ? o : st.h - 1 - o;
        const int set = ysd == 0 ? 1 + y / g.RG : 1 + g.NTG + (y / g.RG - gb0);
        v -= lag_set_value(st, g, set, type, y % g.RG, dx, y % g.RG + dy + K);
    }
    const int iy = dy + K, ix = dx + K;                 // lag indices of the border-column statistics
    const int entry = 256 + 2 * r * NLL;
    for (int o = 0; o < xn; ++o) {
        const double *c = st.C + ((size_t)(type * 2 + xsd) * r + o) * entry;
        v -= c[(iy & 3) * 64 + 16 * (iy >> 2) + ix];                 // column sum: row = vertical lag index
        for (int oy = 0; oy < yn; ++oy) v += c[256 + (ysd * r + oy) * NLL + iy * NL + ix];
    }
    return v;
}

// S_x[(d,a)][(d',b)] over the patch centres inside the image; the (2,1) pair is the (1,2) pair with the taps swapped
__device__ __forceinline__ double lag_raw(const LagStats &st, int d, int a, int d2, int b)
{
    if (d == d2) return lag_entry(st, d, a, b);
    return d == 0 ? lag_entry(st, 2, a, b) : lag_entry(st, 2, b, a);
}

// stacked[e] = Gram of y = x - x_centre over the patches of the image, element e in the slot layout of the dense
// kernel: tile (bi, bj) number t, register v, lane l hold entry (16 bi + 4 (l / 16) + v, 16 bj + l % 16) of the
// stacked 2(D-1) x 2(D-1) matrix;  S_y[a][b] = S_x[a][b] - S_x[a][c] - S_x[c][b] + S_x[c][c], c the centre tap.
__global__ void lag_to_stacked_kernel(LagStats st, double *__restrict__ stacked)
{
    const int ks = st.ks;
    const int D = ks * ks, DR = D - 1, CEN = (D - 1) / 2;
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
    stacked[e] = lag_raw(st, d, a, d2, b) - lag_raw(st, d, a, d2, CEN) - lag_raw(st, d, CEN, d2, b) +
                 lag_raw(st, d, CEN, d2, CEN);
}

bool lag_supported(int k) { return k == 3 || k == 5 || k == 7 || k == 9; }
int max_lag_slots(ddcca_ctx *ctx) { return ctx->n_cu * 6; }
int max_lag_col_slots(ddcca_ctx *ctx) { return ctx->n_cu * 3 / 2; }   // x 2 sides: three workgroups per CU
static bool lag_wide(int k) { return 2 * (k - 1) + 1 > 16; }
static int lag_tile_rows(int k)
{
    return k == 3 ? LagGeom<3>::TH : k == 5 ? LagGeom<5>::TH : k == 7 ? LagGeom<7>::TH : LagGeom<9>::TH;
}
size_t lag_slot_doubles(int k)
{
    const LagShape g(k);
    return (size_t)(1 + g.NTG + g.NBG) * 1024 + (lag_wide(k) ? 8 : 0);
}
size_t lag_col_slot_doubles(int k)
{
    const LagShape g(k);
    return (size_t)4 * 2 * g.r * (256 + 2 * g.r * g.NL * g.NL);
}

template <int KS>
static void lag_launch(ddcca_ctx *ctx, const LagParams &p, int grid, size_t lds, const LagColParams &c, dim3 cgrid)
{
    static_assert(LagGeom<KS>::SLOT == (1 + LagGeom<KS>::NTG + LagGeom<KS>::NBG) * 1024 + (LagGeom<KS>::WIDE ? 8 : 0), "slot layout");
    hipLaunchKernelGGL(lag_gram_kernel<KS>, dim3(grid), dim3(LAG_THREADS), lds, ctx->stream, p);
    hipLaunchKernelGGL(lag_cols_kernel<KS>, cgrid, dim3(lagc_threads<KS>()), 0, ctx->stream, c);
}

int launch_lag_gram(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t n_maps, int h, int w, int k,
                    double *slots, int max_slots, int *slots_valid, double *col_slots, int max_col_slots,
                    int *col_slots_valid)
{
    ProfScope prof(ctx, DDCCA_K_GRAM);
    if (!lag_supported(k)) return fail(ctx, DDCCA_EINVAL, "the lag-structured Gram needs k in {3, 5, 7, 9}");
    if (n_maps < 1 || h < 1 || w < 1) return fail(ctx, DDCCA_EINVAL, "lag-structured Gram: empty input");
    LagParams p;
    p.v1 = v1; p.v2 = v2; p.h = h; p.w = w;
    const int K = k - 1;
    const int w4 = (w + 3) & ~3;
    const int ntx = (w4 + LAG_TW_MAX - 1) / LAG_TW_MAX;
    p.tw = (((w4 + ntx - 1) / ntx) + 3) & ~3;
    p.tiles_x = (w + p.tw - 1) / p.tw;
    const int TH = lag_tile_rows(k);
    p.tiles_y = (h + TH - 1) / TH;
    p.n_items = n_maps * p.tiles_x * p.tiles_y;
    // row pitch: tile width + halo, congruent to 17 mod 32 so that the rows y .. y + 2K a B operand reads fall
    // into different banks
    int pitch = p.tw + 2 * K + 4;
    while (pitch % 32 != 17) ++pitch;
    p.pitch = pitch;
    p.view_stride = (TH + 2 * K) * pitch + 8;
    const size_t lds = std::max<size_t>((size_t)2 * p.view_stride * sizeof(float),
                                        (size_t)1024 * sizeof(double));
    if (p.tw > LAG_TW_MAX || lds > 64 * 1024) return fail(ctx, DDCCA_EINVAL, "lag-structured Gram: tile too large");
    p.slots = slots;
    p.slots_valid = *slots_valid;
    const int grid = (int)std::min<int64_t>(max_slots, std::max<int64_t>(p.n_items, 1));
    // the border columns and corners of the same maps
    LagColParams c;
    c.v1 = v1; c.v2 = v2; c.h = h; c.w = w; c.n_maps = n_maps;
    c.slots = col_slots;
    c.slots_valid = *col_slots_valid;
    const int cgrid = (int)std::min<int64_t>(max_col_slots, std::max<int64_t>(n_maps, 1));
    const dim3 cg(cgrid, 2);
    switch (k) {
        case 3: lag_launch<3>(ctx, p, grid, lds, c, cg); break;
        case 5: lag_launch<5>(ctx, p, grid, lds, c, cg); break;
        case 7: lag_launch<7>(ctx, p, grid, lds, c, cg); break;
        case 9: lag_launch<9>(ctx, p, grid, lds, c, cg); break;
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
    if (lag_wide(k)) {
        LagSpecialParams sp;
        sp.v1 = v1; sp.v2 = v2; sp.h = h; sp.w = w; sp.r = (k - 1) / 2; sp.n_maps = n_maps;
        sp.slots = slots;
        sp.slot_doubles = lag_slot_doubles(k);
        sp.tail = sp.slot_doubles - 8;
        sp.slots_valid = *slots_valid;
        hipLaunchKernelGGL(lag_special_kernel, dim3(grid), dim3(256), 0, ctx->stream, sp);
    }
    DDCCA_HIP(ctx, hipGetLastError());
    *slots_valid = std::max(*slots_valid, grid);
    *col_slots_valid = std::max(*col_slots_valid, cgrid);
    return DDCCA_OK;
}

int launch_lag_to_stacked(ddcca_ctx *ctx, const double *R, const double *C, double *stacked, int k, int h, int w)
{
    ProfScope prof(ctx, DDCCA_K_REDUCE);
    const int E = gram_tiles(k) * 256;
    LagStats st;
    st.R = R; st.C = C; st.ks = k; st.h = h; st.w = w;
    hipLaunchKernelGGL(lag_to_stacked_kernel, dim3((E + 255) / 256), dim3(256), 0, ctx->stream, st, stacked);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

}  // namespace ddcca
