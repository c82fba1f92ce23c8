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
// Main kernel ("ring"): one workgroup of 8 wavefronts sweeps one input map (or a chunk of its
// block columns) top to bottom in tiles of TH rows x (32*NBX) columns.  Only the block rows
// that overlap the current tile are live, so their packed 16-bit histograms sit in a ring of
// a few block rows in LDS; a block row is written out (and its slot cleared) as soon as the
// sweep has passed its last pixel row.  Every map value is therefore computed exactly once.
// Tiles are double-buffered: the next tile travels HBM -> registers while the current one is
// contracted, and is written to the other LDS buffer afterwards (one barrier per tile, one
// more when block rows are flushed).  A wavefront owns whole tile rows: NBX accumulator
// chains, signs, OR of the partial codes of the four 16-lane groups (each holds two filters),
// then the 32 pixels of a column block are added to the histograms of the blocks that
// contain them.
// Fallback kernel ("group"), for block geometries whose live block rows do not fit in LDS
// (very dense overlap, 4096 bins): a workgroup owns RB block rows x a chunk of block columns
// and recomputes the map rows that neighbouring groups share.
#include "hist_common.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int FUSED_XB = 32;              // pixels per MFMA column block (16 columns x 2 shifts)
constexpr int FUSED_MAX_NBX = 4;
constexpr int FUSED_LDS_BYTES = 80 * 1024;   // per workgroup: two workgroups share a compute unit's 160 KB
constexpr int RING_THREADS = 512;
constexpr int RING_MIN_WG = 4;            // wavefronts per SIMD the register budget must allow (two workgroups per compute unit)
constexpr int RING_WAVES = RING_THREADS / 64;
constexpr int RING_TH_MAX = 32;           // largest tile height of the ring kernel
constexpr int GROUP_THREADS = 256;
constexpr int GROUP_TH = 32;              // tile rows of the group kernel

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
    int cols, col_chunks; // block columns per workgroup, chunks per map
    int rb, row_groups;   // group kernel: block rows per workgroup, groups per map
    int th, ring;         // ring kernel: tile rows, block rows held in LDS
    int64_t group, group_stride;
    unsigned magic_sy, magic_sx, magic_ring;
    int hist_words;       // LDS words of the histograms (padded to 4)
    int lut_words;        // LDS words reserved for the table (padded to 4)
    int tile_floats;      // LDS floats of one tile buffer
};

template <int KS, int NBX>
struct FusedGeom {
    static constexpr int KSZ = KS;
    static constexpr int R = (KS - 1) / 2;
    static constexpr int KW = KS + 1;              // tap columns incl. the shift
    static constexpr int TAPS = KS * KW;
    static constexpr int KK = (TAPS + 3) / 4;      // MFMA steps
    static constexpr int TW = NBX * FUSED_XB;
    static constexpr int PW = TW + 2 * R + 1;      // +1: the odd shift reads one more column
    static constexpr int PITCH = PW | 1;           // odd pitch: rows start in different banks
    static constexpr int tile_floats(int th) { return (th + 2 * R) * PITCH; }
};

// Tile of the ring kernel: rows start at an image column that is a multiple of 4 (16-byte loads and
// LDS stores), which costs up to 3 columns of slack.
template <int KS, int NBX>
struct RingGeom {
    static constexpr int KSZ = KS;
    static constexpr int R = (KS - 1) / 2;
    static constexpr int KW = KS + 1;
    static constexpr int TAPS = KS * KW;
    static constexpr int KK = (TAPS + 3) / 4;
    static constexpr int TW = NBX * FUSED_XB;
    static constexpr int PITCH = (TW + 2 * R + 1 + 3 + 3) / 4 * 4;
    static constexpr int V4 = PITCH / 4;           // 16-byte vectors per tile row
    static constexpr int tile_floats(int th) { return (th + 2 * R) * PITCH; }
};

// Per-lane constants of the implicit GEMM: B-operand window offsets and the A operand (filters).
template <class G, int NG>
__device__ __forceinline__ void fused_operands(const float *W, int L2, int q, int c, int (&toff)[G::KK],
                                               float (&wa)[NG][G::KK])
{
    constexpr int KS = G::KSZ;
#pragma unroll
    for (int kk = 0; kk < G::KK; ++kk) {
        const int tap = 4 * kk + q;
        const int dy = tap / G::KW, dx = tap - dy * G::KW;
        toff[kk] = tap < G::TAPS ? dy * G::PITCH + dx : 0;
    }
    // A operand: row = lane%16 = 8*s + g (x-shift s, filter g of the group), tap 4*kk + lane/16, for every
    // group of 8 filters.  (The stand-alone convolution orders its rows (g,s); every output element is the
    // same dot product in the same order of taps either way.)
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        const int g = 8 * gi + (c & 7), s = c >> 3;
#pragma unroll
        for (int kk = 0; kk < G::KK; ++kk) {
            const int tap = 4 * kk + q;
            const int dy = tap / G::KW, dxw = tap - dy * G::KW - s;
            float v = 0.f;
            if (tap < G::TAPS && dxw >= 0 && dxw < KS && g < L2) v = W[(g * KS + dy) * KS + dxw];
            wa[gi][kk] = v;
        }
    }
}

// RU tile rows (RSTRIDE floats apart in LDS): the L2 map values of 32*NBX pixels per row on the matrix
// unit, then their hash codes.  Lane (q,c) receives, per row and column block, the code of pixel
// x0 + 2c + (q >> 1) (lanes q and q^1 hold the same value).
template <class G, int NBX, int NG, int RU, int RSTRIDE>
__device__ __forceinline__ void fused_row_codes(const float *prow, const int (&toff)[G::KK],
                                                const float (&wa)[NG][G::KK], int q, unsigned (&code)[RU][NBX])
{
#pragma unroll
    for (int u = 0; u < RU; ++u)
#pragma unroll
        for (int b = 0; b < NBX; ++b) code[u][b] = 0u;
    // output rows 4q..4q+3 of a lane: x-shift q>>1, filters 8gi + 4(q&1) + 0..3
    const unsigned m0 = 1u << (4 * (q & 1)), m1 = m0 << 1, m2 = m0 << 2, m3 = m0 << 3;
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
        floatx4 acc[RU][NBX];
#pragma unroll
        for (int kk = 0; kk < G::KK; ++kk) {
            const float *pk = prow + toff[kk];
#pragma unroll
            for (int u = 0; u < RU; ++u)
#pragma unroll
                for (int b = 0; b < NBX; ++b)
                    acc[u][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[gi][kk], pk[u * RSTRIDE + b * FUSED_XB],
                                                                     kk == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[u][b], 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < RU; ++u)
#pragma unroll
            for (int b = 0; b < NBX; ++b) {
                const unsigned bits = (acc[u][b][0] > 0.0f ? m0 : 0u) | (acc[u][b][1] > 0.0f ? m1 : 0u) |
                                      (acc[u][b][2] > 0.0f ? m2 : 0u) | (acc[u][b][3] > 0.0f ? m3 : 0u);
                code[u][b] |= bits << (8 * gi);
            }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u)
#pragma unroll
        for (int b = 0; b < NBX; ++b) code[u][b] |= (unsigned)__shfl_xor((int)code[u][b], 16);
}

// Convert `n_words` packed histogram words at `sp` (LDS) to the output element type at `dst`
// (both contiguous).  All threads of the workgroup take part; with `clear` every word is set
// to zero by the thread that read it.
__device__ __forceinline__ void fused_write_out(unsigned *sp, char *dst, int n_words, int bins, int out_type,
                                                const float *lds_lut, int lut_n, double log_total, bool aligned,
                                                bool clear, int tid, int n_threads)
{
    const int esz = out_type == DDCCA_FEAT_IQ_F32 ? 4 : 2;
    const int vw = 8 / esz;                                          // packed words per 16-byte store
    if (aligned && bins >= 2 * vw) {
        for (int e = tid; e < n_words / vw; e += n_threads) {
            unsigned *s = sp + vw * e;
            uint4 val;
            if (out_type == DDCCA_FEAT_COUNT_U16) {
                val = *reinterpret_cast<const uint4 *>(s);
                if (clear) *reinterpret_cast<uint4 *>(s) = make_uint4(0u, 0u, 0u, 0u);
            } else if (out_type == DDCCA_FEAT_IQ_F32) {
                const uint2 wv = *reinterpret_cast<const uint2 *>(s);
                if (clear) *reinterpret_cast<uint2 *>(s) = make_uint2(0u, 0u);
                val.x = __float_as_uint(iq_value(wv.x & 0xffffu, lds_lut, lut_n, log_total));
                val.y = __float_as_uint(iq_value(wv.x >> 16, lds_lut, lut_n, log_total));
                val.z = __float_as_uint(iq_value(wv.y & 0xffffu, lds_lut, lut_n, log_total));
                val.w = __float_as_uint(iq_value(wv.y >> 16, lds_lut, lut_n, log_total));
            } else {
                const uint4 wv = *reinterpret_cast<const uint4 *>(s);
                if (clear) *reinterpret_cast<uint4 *>(s) = make_uint4(0u, 0u, 0u, 0u);
                const unsigned in[4] = {wv.x, wv.y, wv.z, wv.w};
                unsigned o[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const __half lo = __float2half_rn(iq_value(in[t] & 0xffffu, lds_lut, lut_n, log_total));
                    const __half hi = __float2half_rn(iq_value(in[t] >> 16, lds_lut, lut_n, log_total));
                    o[t] = (unsigned)__half_as_ushort(lo) | ((unsigned)__half_as_ushort(hi) << 16);
                }
                val = make_uint4(o[0], o[1], o[2], o[3]);
            }
            *reinterpret_cast<uint4 *>(dst + (size_t)e * 16) = val;
        }
    } else {
        // one thread per word: its one (bins == 1) or two elements
        const int per_word = bins > 1 ? 2 : 1;
        for (int e = tid; e < n_words; e += n_threads) {
            const unsigned wv = sp[e];
            if (clear) sp[e] = 0u;
            for (int t = 0; t < per_word; ++t) {
                const unsigned cnt = (wv >> (16 * t)) & 0xffffu;
                char *d = dst + ((size_t)e * per_word + t) * esz;
                if (out_type == DDCCA_FEAT_COUNT_U16)
                    *reinterpret_cast<uint16_t *>(d) = (uint16_t)cnt;
                else if (out_type == DDCCA_FEAT_IQ_F32)
                    *reinterpret_cast<float *>(d) = iq_value(cnt, lds_lut, lut_n, log_total);
                else
                    *reinterpret_cast<__half *>(d) = __float2half_rn(iq_value(cnt, lds_lut, lut_n, log_total));
            }
        }
    }
}

// ------------------------------------------------------------------------------ ring kernel
template <int KS, int NBX, int NG, int RU>
__global__ __launch_bounds__(RING_THREADS, RING_MIN_WG) void conv_hash_hist_ring_kernel(FusedParams p)
{
    typedef RingGeom<KS, NBX> G;
    constexpr int R = G::R, KK = G::KK, TW = G::TW, PITCH = G::PITCH, V4 = G::V4;
    extern __shared__ unsigned int lds[];
    unsigned int *lds_hist = lds;
    float *lds_lut = reinterpret_cast<float *>(lds + p.hist_words);
    float *tile0 = lds_lut + p.lut_words;

    const int bins = 1 << p.L2;
    const int words = bins > 1 ? bins / 2 : 1;    // 32-bit words per packed histogram
    const int64_t n = blockIdx.x / p.col_chunks;
    const int cc = (int)(blockIdx.x - n * p.col_chunks);
    const int j0 = cc * p.cols, j1 = min(j0 + p.cols, p.nbx);
    const int ncol = j1 - j0;
    const int row_words = ncol * words;           // one block row of the chunk
    for (int e = threadIdx.x; e < p.ring * row_words; e += RING_THREADS) lds_hist[e] = 0u;
    if (p.out_type != DDCCA_FEAT_COUNT_U16)
        for (int e = threadIdx.x; e < p.lut_n; e += RING_THREADS) lds_lut[e] = p.lut[e];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: row indices stay on the scalar unit
    const int q = lane >> 4, c = lane & 15;
    int toff[KK];
    float wa[NG][KK];
    fused_operands<G, NG>(p.W, p.L2, q, c, toff, wa);

    const int64_t P = (int64_t)p.h * p.w;
    const float *src = p.in + n * P;
    const bool vec4 = (p.w & 3) == 0 && (((uintptr_t)src) & 15) == 0;
    const int y_hi = (p.nby - 1) * p.sy + p.bh;                      // pixel rows [0, y_hi)
    const int x_lo = j0 * p.sx, x_hi = (j1 - 1) * p.sx + p.bw;       // pixel columns [x_lo, x_hi)
    const int my_s = q >> 1, my_ioff = q & 1;                        // this lane's pixel of a pair / block-row parity
    const int tiles_x = (x_hi - x_lo + TW - 1) / TW;
    const int tiles_y = (y_hi + p.th - 1) / p.th;
    const int n_tiles = tiles_x * tiles_y;

    const int64_t A = (int64_t)p.nby * p.nbx;
    const int esz = p.out_type == DDCCA_FEAT_IQ_F32 ? 4 : 2;
    char *out_map = reinterpret_cast<char *>(p.out) + ((n / p.group) * p.group_stride + (n % p.group) * A * bins) * esz;
    // a block row of the chunk starts on a 16-byte boundary in the output
    const bool aligned = ((((uintptr_t)out_map) | (uintptr_t)((int64_t)p.nbx * bins * esz) | (uintptr_t)((int64_t)j0 * bins * esz)) & 15) == 0;

    // tile t: rows [ty0 - R, ty0 + rows + R), columns [gxa, gxa + PITCH), gxa = the multiple of 4 at or
    // below the first halo column.  A thread always moves the same 16-byte column of RPP rows per pass.
    constexpr int RPP = RING_THREADS / V4;        // tile rows per pass of the workgroup
    constexpr int NPRE = (RING_TH_MAX + 2 * R + RPP - 1) / RPP;
    const int st_xv = threadIdx.x % V4, st_yy = threadIdx.x / V4;    // st_yy >= RPP: no part in staging
    float4 pre[NPRE];
    auto fetch = [&](int t) {
        const int tyi = t / tiles_x, txi = t - tyi * tiles_x;
        const int ty0 = tyi * p.th, rows = min(p.th, y_hi - ty0);
        const int gy0 = ty0 - R + st_yy;
        const int gx = ((x_lo + txi * TW - R) & ~3) + 4 * st_xv;
        const int n_rows = st_yy < RPP ? rows + 2 * R - st_yy : 0;   // tile rows at and below this thread's first
        const bool whole = vec4 && gx >= 0 && gx + 3 < p.w;
        const float *col = src + gx;
#pragma unroll
        for (int u = 0; u < NPRE; ++u) {
            const int gy = gy0 + u * RPP;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (u * RPP < n_rows && gy >= 0 && gy < p.h) {
                const float *row = col + (int64_t)gy * p.w;
                if (whole) {
                    v = *reinterpret_cast<const float4 *>(row);
                } else {
                    if (gx >= 0 && gx < p.w) v.x = row[0];
                    if (gx + 1 >= 0 && gx + 1 < p.w) v.y = row[1];
                    if (gx + 2 >= 0 && gx + 2 < p.w) v.z = row[2];
                    if (gx + 3 >= 0 && gx + 3 < p.w) v.w = row[3];
                }
            }
            pre[u] = v;
        }
    };
    auto stash = [&](float *tile, int t) {
        const int tyi = t / tiles_x;
        const int rows = min(p.th, y_hi - tyi * p.th);
        const int n_rows = st_yy < RPP ? rows + 2 * R - st_yy : 0;
        float *dst = tile + st_yy * PITCH + 4 * st_xv;
#pragma unroll
        for (int u = 0; u < NPRE; ++u)
            if (u * RPP < n_rows) *reinterpret_cast<float4 *>(dst + u * RPP * PITCH) = pre[u];
    };

    fetch(0);
    stash(tile0, 0);
    int next_flush = 0;                           // first block row not yet written out
    int cur_txi = -1;
    int jo[NBX], nj[NBX];                         // this lane's pixel column per block: first block column (word offset), count
    unsigned brk = 0u;                            // bit b: the lane to the left (c - 1) has another block-column set, or c == 0
    for (int t = 0; t < n_tiles; ++t) {
        __syncthreads();                          // tile t is in LDS; cleared slots are visible
        const float *tile = tile0 + (t & 1) * p.tile_floats;
        if (t + 1 < n_tiles) fetch(t + 1);
        const int tyi = t / tiles_x, txi = t - tyi * tiles_x;
        const int ty0 = tyi * p.th, rows = min(p.th, y_hi - ty0);
        const int tx0 = x_lo + txi * TW;
        const int shx = (tx0 - R) & 3;            // first halo column inside the aligned tile row
        if (txi != cur_txi) {
            cur_txi = txi;
#pragma unroll
            for (int b = 0; b < NBX; ++b) {
                const int x = tx0 + b * FUSED_XB + 2 * c + my_s;
                int jlo = 0, jhi = -1;
                if (x < x_hi) block_range(x, p.bw, p.sx, p.magic_sx, j0, j1, jlo, jhi);
                jo[b] = (jlo - j0) * words;
                nj[b] = jhi - jlo + 1;
            }
            brk = 0u;
#pragma unroll
            for (int b = 0; b < NBX; ++b) {
                const int pj = __builtin_amdgcn_update_dpp(-1, jo[b], 0x111, 0xf, 0xf, false);   // row_shr:1
                const int pn = __builtin_amdgcn_update_dpp(-1, nj[b], 0x111, 0xf, 0xf, false);
                if (c == 0 || pj != jo[b] || pn != nj[b]) brk |= 1u << b;
            }
        }
        for (int r0 = wave; r0 < rows; r0 += RU * RING_WAVES) {
            unsigned codes[RU][NBX];
            fused_row_codes<G, NBX, NG, RU, RING_WAVES * PITCH>(tile + r0 * PITCH + shx + 2 * c, toff, wa, q, codes);
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                const int r = r0 + u * RING_WAVES;
                if (r >= rows) break;
                int ilo, ihi;
                block_range(ty0 + r, p.bh, p.sy, p.magic_sy, 0, p.nby, ilo, ihi);
                // 64 lanes, 32 pixels: lane (q,c) takes pixel x0 + 2c + (q&1) and the block rows ilo + (q>>1), +2, ...
                // Neighbouring pixels mostly share their code, and equal codes going to the same word would
                // serialise in LDS: a run of lanes (within a 16-lane group) with equal code and equal block
                // columns is added once, by its first lane, with the run length.
                unsigned word[NBX], inc[NBX];
#pragma unroll
                for (int b = 0; b < NBX; ++b) {
                    const unsigned code = codes[u][b];
                    const unsigned prev = (unsigned)__builtin_amdgcn_update_dpp(-1, (int)code, 0x111, 0xf, 0xf, false);
                    const bool head = ((brk >> b) & 1u) != 0u || prev != code;
                    const unsigned long long heads = __ballot(head);
                    const unsigned grp = (unsigned)(heads >> (lane & 48)) & 0xffffu;     // this 16-lane group's heads
                    const unsigned len = (unsigned)__ffs((int)((grp | 0x10000u) >> (c + 1)));   // lanes up to the next head
                    word[b] = code >> 1;
                    inc[b] = head ? len << (16 * (code & 1)) : 0u;
                }
                for (int ib = ilo; ib <= ihi; ib += 2) {
                    const int ic = min(ib + 1, ihi);
                    const int so_a = (p.magic_ring ? ib - p.ring * (int)__umulhi((unsigned)ib, p.magic_ring) : ib % p.ring) * row_words;
                    const int so_c = (p.magic_ring ? ic - p.ring * (int)__umulhi((unsigned)ic, p.magic_ring) : ic % p.ring) * row_words;
                    const int so = my_ioff ? so_c : so_a;
                    if (ib + my_ioff <= ihi) {
#pragma unroll
                        for (int b = 0; b < NBX; ++b) {
                            if (inc[b] == 0u) continue;
                            unsigned int *dst = lds_hist + so + jo[b] + word[b];
                            for (int jj = 0; jj < nj[b]; ++jj) atomicAdd(dst + jj * words, inc[b]);
                        }
                    }
                }
            }
        }
        if (t + 1 < n_tiles) stash(tile0 + ((t + 1) & 1) * p.tile_floats, t + 1);
        if (txi == tiles_x - 1) {
            // block rows whose last pixel row lies inside the rows swept so far are complete
            const int done = ty0 + rows - p.bh;
            const int i_end = done < 0 ? 0 : min(p.nby, fast_div(done, p.sy, p.magic_sy) + 1);
            if (i_end > next_flush) {
                __syncthreads();                  // every count of these block rows has been added
                for (int i = next_flush; i < i_end; ++i) {
                    const int slot = i % p.ring;
                    fused_write_out(lds_hist + slot * row_words, out_map + ((int64_t)i * p.nbx + j0) * bins * esz,
                                    row_words, bins, p.out_type, lds_lut, p.lut_n, p.log_total, aligned, true,
                                    threadIdx.x, RING_THREADS);
                }
                next_flush = i_end;
            }
        }
    }
}

// ----------------------------------------------------------------------------- group kernel
template <int KS, int NBX, int NG>
__global__ __launch_bounds__(GROUP_THREADS) void conv_hash_hist_group_kernel(FusedParams p)
{
    typedef FusedGeom<KS, NBX> G;
    constexpr int R = G::R, KK = G::KK, TW = G::TW, PW = G::PW, PITCH = G::PITCH;
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
    const int row_words = ncol * words;
    for (int e = threadIdx.x; e < nrow * row_words; e += GROUP_THREADS) lds_hist[e] = 0u;
    if (p.out_type != DDCCA_FEAT_COUNT_U16)
        for (int e = threadIdx.x; e < p.lut_n; e += GROUP_THREADS) lds_lut[e] = p.lut[e];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, c = lane & 15;
    int toff[KK];
    float wa[NG][KK];
    fused_operands<G, NG>(p.W, p.L2, q, c, toff, wa);

    const int64_t P = (int64_t)p.h * p.w;
    const float *src = p.in + n * P;
    const int y_lo = i0 * p.sy, y_hi = (i1 - 1) * p.sy + p.bh;       // pixel rows [y_lo, y_hi)
    const int x_lo = j0 * p.sx, x_hi = (j1 - 1) * p.sx + p.bw;       // pixel columns [x_lo, x_hi)
    const int my_s = q >> 1, my_ioff = q & 1;

    for (int ty0 = y_lo; ty0 < y_hi; ty0 += GROUP_TH) {
        const int rows = min(GROUP_TH, y_hi - ty0);
        for (int tx0 = x_lo; tx0 < x_hi; tx0 += TW) {
            __syncthreads();                      // the previous tile has been consumed (first pass: LDS initialised)
            {
                const int gy0 = ty0 - R, gx0 = tx0 - R;
                const int n_el = (rows + 2 * R) * PW;
#pragma unroll 4
                for (int e = threadIdx.x; e < n_el; e += GROUP_THREADS) {
                    const int yy = e / PW, xx = e - yy * PW;
                    const int gy = gy0 + yy, gx = gx0 + xx;
                    float v = 0.f;
                    if (gy >= 0 && gy < p.h && gx >= 0 && gx < p.w) v = src[(int64_t)gy * p.w + gx];
                    tile[yy * PITCH + xx] = v;
                }
            }
            __syncthreads();
            for (int r = wave; r < rows; r += GROUP_THREADS / 64) {
                unsigned codes[1][NBX];
                fused_row_codes<G, NBX, NG, 1, 0>(tile + r * PITCH + 2 * c, toff, wa, q, codes);
                const int y = ty0 + r;
                int ilo, ihi;
                block_range(y, p.bh, p.sy, p.magic_sy, i0, i1, ilo, ihi);
#pragma unroll
                for (int b = 0; b < NBX; ++b) {
                    const unsigned code = codes[0][b];
                    const int x = tx0 + b * FUSED_XB + 2 * c + my_s;
                    if (x < x_hi) {
                        int jlo, jhi;
                        block_range(x, p.bw, p.sx, p.magic_sx, j0, j1, jlo, jhi);
                        const unsigned inc = 1u << (16 * (code & 1));
                        const unsigned word = code >> 1;
                        for (int i = ilo + my_ioff; i <= ihi; i += 2)
                            for (int j = jlo; j <= jhi; ++j)
                                atomicAdd(&lds_hist[(i - i0) * row_words + (j - j0) * words + word], inc);
                    }
                }
            }
        }
    }
    __syncthreads();

    const int64_t A = (int64_t)p.nby * p.nbx;
    const int esz = p.out_type == DDCCA_FEAT_IQ_F32 ? 4 : 2;
    char *out_map = reinterpret_cast<char *>(p.out) + ((n / p.group) * p.group_stride + (n % p.group) * A * bins) * esz;
    const bool aligned = ((((uintptr_t)out_map) | (uintptr_t)((int64_t)p.nbx * bins * esz) | (uintptr_t)((int64_t)j0 * bins * esz)) & 15) == 0;
    for (int ir = 0; ir < nrow; ++ir)
        fused_write_out(lds_hist + ir * row_words, out_map + ((int64_t)(i0 + ir) * p.nbx + j0) * bins * esz, row_words,
                        bins, p.out_type, lds_lut, p.lut_n, p.log_total, aligned, false, threadIdx.x, GROUP_THREADS);
}

// ------------------------------------------------------------------------------------ host
template <typename Kernel>
static int fused_set_lds(ddcca_ctx *ctx, Kernel kernel, bool *done)
{
    if (!done[ctx->device]) {          // per device: the attribute is set on that device's code object
        DDCCA_HIP(ctx, hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           FUSED_LDS_BYTES));
        done[ctx->device] = true;
    }
    return DDCCA_OK;
}

// Rows a wavefront of the ring kernel contracts together: two when the registers allow it (one filter
// group, k <= 7) and the tile has at least 16 rows.
template <int KS, int NG> constexpr int ring_rows_together() { return NG == 1 && KS <= 7 ? 2 : 1; }

template <int KS, int NBX, int NG>
static int fused_launch(ddcca_ctx *ctx, FusedParams p, int64_t n, bool ring)
{
    static bool ring2_attr[MAX_DEVICES] = {}, ring1_attr[MAX_DEVICES] = {}, group_attr[MAX_DEVICES] = {};
    constexpr int RU2 = ring_rows_together<KS, NG>();
    const bool two = ring && RU2 == 2 && p.th >= 2 * RING_WAVES;
    int rc;
    if ((rc = !ring ? fused_set_lds(ctx, conv_hash_hist_group_kernel<KS, NBX, NG>, group_attr)
              : two ? fused_set_lds(ctx, conv_hash_hist_ring_kernel<KS, NBX, NG, RU2>, ring2_attr)
                    : fused_set_lds(ctx, conv_hash_hist_ring_kernel<KS, NBX, NG, 1>, ring1_attr)))
        return rc;
    p.tile_floats = ring ? RingGeom<KS, NBX>::tile_floats(p.th) : FusedGeom<KS, NBX>::tile_floats(GROUP_TH);
    const size_t lds = ((size_t)p.hist_words + p.lut_words + (size_t)p.tile_floats * (ring ? 2 : 1)) * 4;
    if (lds > (size_t)FUSED_LDS_BYTES) return fail(ctx, DDCCA_EINVAL, "internal: fused kernel LDS budget exceeded");
    const int64_t per_map = (int64_t)p.col_chunks * (ring ? 1 : p.row_groups);
    const int64_t esz = p.out_type == DDCCA_FEAT_IQ_F32 ? 4 : 2;
    const int64_t maps_per_launch = std::max<int64_t>(p.group, (((int64_t)1 << 30) / per_map) / p.group * p.group);
    for (int64_t n0 = 0; n0 < n; n0 += maps_per_launch) {
        const int64_t nb = std::min(maps_per_launch, n - n0);
        FusedParams q = p;
        q.in = p.in + n0 * (int64_t)p.h * p.w;
        q.out = reinterpret_cast<char *>(p.out) + (n0 / p.group) * p.group_stride * esz;
        if (two)
            hipLaunchKernelGGL((conv_hash_hist_ring_kernel<KS, NBX, NG, RU2>),
                               dim3((unsigned)(nb * per_map)), dim3(RING_THREADS), lds, ctx->stream, q);
        else if (ring)
            hipLaunchKernelGGL((conv_hash_hist_ring_kernel<KS, NBX, NG, 1>), dim3((unsigned)(nb * per_map)),
                               dim3(RING_THREADS), lds, ctx->stream, q);
        else
            hipLaunchKernelGGL((conv_hash_hist_group_kernel<KS, NBX, NG>), dim3((unsigned)(nb * per_map)),
                               dim3(GROUP_THREADS), lds, ctx->stream, q);
    }
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

template <int KS, int NG>
static int fused_dispatch_nbx(ddcca_ctx *ctx, const FusedParams &p, int64_t n, int nbx_tile, bool ring)
{
    switch (nbx_tile) {
        case 1: return fused_launch<KS, 1, NG>(ctx, p, n, ring);
        case 2: return fused_launch<KS, 2, NG>(ctx, p, n, ring);
        case 3: return fused_launch<KS, 3, NG>(ctx, p, n, ring);
        default: return fused_launch<KS, 4, NG>(ctx, p, n, ring);
    }
}

// equal-width tiles of at most FUSED_MAX_NBX column blocks across a pixel rectangle of this width
static int fused_tile_blocks(int width)
{
    const int xblocks = (width + FUSED_XB - 1) / FUSED_XB;
    const int tiles_x = (xblocks + FUSED_MAX_NBX - 1) / FUSED_MAX_NBX;
    return (xblocks + tiles_x - 1) / tiles_x;
}

// Largest number of block rows that overlap one tile of th pixel rows.
static int fused_live_rows(int th, int bh, int sy, int nby)
{
    const int y_hi = (nby - 1) * sy + bh;
    int live = 1;
    for (int ty0 = 0; ty0 < y_hi; ty0 += th) {
        const int y_last = std::min(ty0 + th, y_hi) - 1;
        const int first = ty0 - bh + 1 <= 0 ? 0 : (ty0 - bh + sy) / sy;    // ceil((ty0 - bh + 1) / sy)
        const int last = std::min(nby - 1, y_last / sy);
        live = std::max(live, last - first + 1);
    }
    return live;
}

template <int KS, int NG>
static int fused_plan(ddcca_ctx *ctx, FusedParams &p, int64_t n)
{
    const int bins = 1 << p.L2;
    const int hist_bytes = (bins > 1 ? bins / 2 : 1) * 4;             // packed histogram of one block
    p.lut_words = p.out_type != DDCCA_FEAT_COUNT_U16 ? (p.lut_n + 3) / 4 * 4 : 0;
    const int fixed = p.lut_words * 4 + 16;
    constexpr int PITCH_MAX = ((FUSED_MAX_NBX * FUSED_XB + KS) | 1);
    // Ring kernel: the fewest column chunks, then the tallest tile, whose live block rows and two tile
    // buffers fit in the workgroup's LDS.
    for (int chunks = 1; chunks <= p.nbx; ++chunks) {
        const int cols = (p.nbx + chunks - 1) / chunks;
        if ((p.nbx + cols - 1) / cols != chunks) continue;            // same chunk count as a smaller one
        const int nbt = fused_tile_blocks((cols - 1) * p.sx + p.bw);
        const int pitch = (nbt * FUSED_XB + KS + 6) / 4 * 4;          // RingGeom<KS, nbt>::PITCH
        for (int th = RING_TH_MAX; th >= 8; th /= 2) {
            const int ring = fused_live_rows(th, p.bh, p.sy, p.nby);
            const int64_t need = (int64_t)ring * cols * hist_bytes + fixed + 2 * (int64_t)(th + KS - 1) * pitch * 4;
            if (need > FUSED_LDS_BYTES) continue;
            p.cols = cols; p.col_chunks = chunks; p.th = th; p.ring = ring;
            p.rb = 0; p.row_groups = 0;
            p.hist_words = (ring * cols * (hist_bytes / 4) + 3) / 4 * 4;
            p.magic_ring = p.nby < 65536 ? (unsigned)((((uint64_t)1 << 32) + ring - 1) / ring) : 0u;
            return fused_dispatch_nbx<KS, NG>(ctx, p, n, nbt, true);
        }
    }
    // Group kernel.  Histogram budget: what the largest tile leaves of the workgroup's LDS; block columns and
    // block rows are spread evenly over the chunks / groups.
    const int budget = FUSED_LDS_BYTES - (GROUP_TH + KS - 1) * PITCH_MAX * 4 - fixed;
    const int max_blocks = std::max(1, budget / hist_bytes);
    p.col_chunks = (p.nbx + max_blocks - 1) / max_blocks;
    p.cols = (p.nbx + p.col_chunks - 1) / p.col_chunks;
    p.col_chunks = (p.nbx + p.cols - 1) / p.cols;
    const int rb_max = std::max(1, max_blocks / p.cols);
    p.row_groups = (p.nby + rb_max - 1) / rb_max;
    p.rb = (p.nby + p.row_groups - 1) / p.row_groups;
    p.row_groups = (p.nby + p.rb - 1) / p.rb;
    p.th = GROUP_TH; p.ring = 0; p.magic_ring = 0;
    p.hist_words = (p.rb * p.cols * (hist_bytes / 4) + 3) / 4 * 4;
    return fused_dispatch_nbx<KS, NG>(ctx, p, n, fused_tile_blocks((p.cols - 1) * p.sx + p.bw), false);
}

template <int KS>
static int fused_pick_groups(ddcca_ctx *ctx, FusedParams &p, int64_t n)
{
    return p.L2 <= 8 ? fused_plan<KS, 1>(ctx, p, n) : fused_plan<KS, 2>(ctx, p, n);
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
