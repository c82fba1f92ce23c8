// Stage convolution (Eq. 6) on the bf16 matrix pipeline with three-piece operands (see conv_split.h):
// out[n][g][y][x] = sum W[g][dy][dx] in[n][y+dy-r][x+dx-r], zero padding, same size, fp32-grade accuracy.
//
// Implicit GEMM without an im2col buffer, on v_mfma_f32_16x16x32_bf16:
//   rows (A operand)  : (filter g, x-shift s), g < 8, s in {0,1}      -> 16 rows
//   cols (B operand)  : 16 pixel positions x = x0 + 2c of one image row
//   K                 : taps (dy, dx'), dx' in 0..k (both shifts: k+1 columns, an even number), taken as pairs
//                       (dx', dx'+1), dx' even.  A pair is one 32-bit word of a tile stored as packed bf16 pairs;
//                       a lane feeds an instruction with four pairs (a "group"), one instruction covers four
//                       groups (lane / 16): 1 / 1 / 2 / 3 instructions per piece product for k = 3 / 5 / 7 / 9.
//   => D[(g,s)][c]    = out[g][y][x0+2c+s]; each lane ends with (x, x+1) pairs of two output planes, written as
//                       8-byte stores that form 128-byte row segments.
// The kernel is persistent: a workgroup walks a contiguous range of (image, tile) items.  The filter pieces are
// built once and stay in registers.  The input tile with its halo is split once into three planes of packed pairs
// in LDS; there are two such buffers, and the next tile travels HBM -> registers while the current one is
// contracted and is split into the other buffer afterwards (one barrier per tile).
// LDS banks: the four groups of an instruction read four different tap rows (or row ends), two groups per half
// wavefront; the plane pitch is chosen so that the 16 consecutive words of one group and those of its partner
// fall into disjoint banks, and a group whose slot holds no tap reads its partner's words (a broadcast).
#include "conv_split.h"

namespace ddcca {

constexpr int CSPLIT_XB = 32;           // pixels per column block (16 columns x 2 shifts)
constexpr int CSPLIT_MAX_NBX = 4;       // column blocks per tile
constexpr int CSPLIT_TH_MAX = 32;       // tile rows
// Most rows of a tile and workgroups per compute unit, per patch size.  k = 9 contracts long enough per tile for its
// matrix pipeline to be idle a third of the time with two wavefronts per SIMD (one splits its next tile or waits at
// the tile barrier, the other has the SIMD to itself); with tiles of 16 rows two buffers take 46 KB, the kernel
// compiled for three wavefronts per SIMD keeps 160 registers without spilling, and three workgroups share a compute
// unit: 256 x 256 maps 1.19 -> 1.16 ms per launch of 2 048, the convolutions of that workload 12.3 -> 11.7 ms per step.
template <int KS> constexpr int CSPLIT_TH1 = KS == 9 ? 16 : CSPLIT_TH_MAX;
template <int KS> constexpr int CSPLIT_WG_PER_CU = KS == 9 ? 3 : 2;

// RU consecutive output rows share the pixel operands: the taps of output row y+u are the input rows
// y+u .. y+u+k-1, so RU rows together read the k+RU-1 input rows y .. y+k+RU-2; one set of operand registers
// (the pairs of those input rows, in slots that are the same for all RU rows) feeds RU accumulator sets, each with
// its own filter pieces (tap row = input row - u, zero where that is outside 0..k-1).  That divides the LDS
// traffic per output by RU, which is what bounds this kernel: an instruction's pixel operand is 1 KiB per
// wavefront, the six piece products reuse three such operands, and four SIMDs at full matrix rate would ask the
// LDS for exactly its 128 bytes per cycle.
template <int KS, int NBX, int RU>
struct SplitConv {
    static constexpr int R = (KS - 1) / 2;
    static constexpr int KW = KS + 1;              // tap columns incl. the shift (even)
    static constexpr int RP = KW / 2;              // pairs per tap row
    static constexpr int JROWS = KS + RU - 1;      // input rows under RU output rows
    static constexpr int PAIRS = JROWS * RP;
    static constexpr int KG = (PAIRS + 3) / 4;     // groups of four pairs
    static constexpr int STEPS = (KG + 3) / 4;     // matrix instructions per piece product and output row
    static constexpr int TW = NBX * CSPLIT_XB;
    static constexpr int PH_MAX = CSPLIT_TH1<KS> + 2 * R;
    static constexpr int COLS = (TW + KW + 6) / 4 * 4;   // staged pixels per tile row (row start a multiple of 4)
    static constexpr int V4 = COLS / 4;
    // staged columns start at the multiple of 4 at or below the first halo column tx*TW - R (TW is a multiple of
    // 4, so the distance SHX and the pair parity PO are the same for every tile)
    static constexpr int SHX = (4 - R % 4) % 4;
    static constexpr int PO = SHX & 1;
    // words per plane row: at least COLS/2, and congruent to RES modulo MOD (the bank rule above)
    static constexpr int MOD = KS == 3 ? 16 : 32;
    static constexpr int RES = KS == 3 ? 8 : 16;
    static constexpr bool PAIRED_READS = KS >= 7;
    static constexpr int MINP = COLS / 2;
    static constexpr int PWORDS = MINP + (RES - MINP % MOD + MOD) % MOD;
    static constexpr int PLANE = PH_MAX * PWORDS;  // words per plane
    static constexpr int BUF = 3 * PLANE;          // words per buffer (h, m, l planes)

    // The pair in slot i of group q of instruction t: input row j (relative to the first output row's first tap
    // row) and pair dxp, i.e. tap columns 2*dxp and 2*dxp + 1.  Row-major over the pairs, except k = 5 with one
    // output row (three pairs per tap row): there group q holds row q and the fourth slots of groups 0..2 hold the
    // pairs of row 4, so that partner groups again read words one plane row apart; and k = 9 with one output row
    // (five pairs per tap row): the first two instructions take pairs 0..3 of one tap row per group (rows 0..7),
    // the third takes pairs 0..3 of row 8 and the fifth pairs of the nine rows, three per group.  Where the four
    // words of a group lie at offsets from its first word that are the same in every group (a tap row: 0, 1, 2,
    // 3), one address register and two-word read instructions serve them (SlotDeltas below).
    __host__ __device__ static constexpr bool slot(int t, int q, int i, int &j, int &dxp)
    {
        if (KS == 5 && RU == 1) {
            if (t > 0) { j = 0; dxp = 0; return false; }
            if (i < 3) { j = q; dxp = i; return true; }
            j = 4; dxp = q;
            return q < 3;
        }
        if (KS == 9 && RU == 1) {
            if (t < 2 || q == 0) { j = 4 * t + q; dxp = i; return true; }
            j = 3 * (q - 1) + (i < 3 ? i : 2); dxp = 4;
            return i < 3;
        }
        const int pair = 4 * (4 * t + q) + i;
        j = pair / RP;
        dxp = pair - j * RP;
        return pair < PAIRS;
    }
};

struct ConvSplitParams {
    const float *in;
    const float *W;
    float *out;
    int h, w, L, tiles_x, tiles_y, th;
    long long n_items;          // images * tiles
    unsigned char *codes;       // CODES kernels: [n][ceil(L/8)][h][w] hash code bytes instead of `out`
};

// A operand of lane (q, c) for output row u of a row group: row c of the instruction is filter g0 + c/2, shift
// c%2; per instruction and piece the four pairs of group q, tap row = input row - u.
template <class G, int KS>
__device__ __forceinline__ void split_weights(const float *W, int L, int g0, int u, int q, int c,
                                              SplitOperand (&wa)[G::STEPS][3])
{
    const int g = g0 + (c >> 1), s = c & 1;
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int j, dxp;
            const bool valid = G::slot(t, q, i, j, dxp);
            const int dy = j - u, dx = 2 * dxp;
            float v0 = 0.f, v1 = 0.f;
            if (valid && dy >= 0 && dy < KS && g < L) {
                if (dx - s >= 0 && dx - s < KS) v0 = W[(g * KS + dy) * KS + dx - s];
                if (dx + 1 - s >= 0 && dx + 1 - s < KS) v1 = W[(g * KS + dy) * KS + dx + 1 - s];
            }
            split3_pair(v0, v1, wa[t][0].w[i], wa[t][1].w[i], wa[t][2].w[i]);
        }
    }
}

// Word offsets (inside a plane, relative to the lane's pixel pair of the tile row of the first output row) of the
// four pairs of this lane's group, per instruction.  A slot without a pair (its filter pieces are zero) reads what
// the partner group of the half wavefront reads, else what group 0 reads.
template <class G>
__device__ __forceinline__ void split_offsets(int q, int (&toff)[G::STEPS][4])
{
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int j, dxp;
            if (!G::slot(t, q, i, j, dxp) && !((q & 1) && G::slot(t, q - 1, i, j, dxp))) G::slot(t, 0, i, j, dxp);
            toff[t][i] = j * G::PWORDS + dxp;
        }
}

// The part of a tile a thread carries from HBM to LDS in one pass: NV chunks of four staged pixels (+ the fifth
// pixel when the pairs straddle the chunks).  A tile takes PASSES passes of THREADS * NV chunks.
template <class G, int THREADS>
struct TileRegs {
    static constexpr int CHUNKS = G::PH_MAX * G::V4;
    static constexpr int NV_ALL = (CHUNKS + THREADS - 1) / THREADS;
    static constexpr int NV = NV_ALL < 12 ? NV_ALL : 12;
    static constexpr int PASSES = (CHUNKS + THREADS * NV - 1) / (THREADS * NV);
    float v[NV][4 + G::PO];
};

// Where chunk j of thread `tid` sits: tile row yy, first staged column 4*xv; whether the tile row is inside the image.
template <class G, int THREADS>
__device__ __forceinline__ void chunk_pos(int e0, int tid, int j, int &yy, int &xv)
{
    const int e = e0 + tid + j * THREADS;
    yy = e / G::V4;
    xv = e - yy * G::V4;
}

// Issue the loads of a tile.  Every load reads a valid address (the first pixels of the image stand in for what
// lies outside it) and nothing uses the values here: store_tile replaces the stand-ins by zeros, so all loads of a
// thread are in flight together and no branch surrounds them.  VEC4: w and the image base allow 16-byte loads
// (w a multiple of 4; the first staged column is one too, so a chunk lies wholly inside the image or outside).
template <class G, int THREADS, bool VEC4>
__device__ __forceinline__ void load_tile(TileRegs<G, THREADS> &t, int e0, int tid, const float *src, int h, int w,
                                          int gy0, int gxa, int ph)
{
#pragma unroll
    for (int j = 0; j < TileRegs<G, THREADS>::NV; ++j) {
        int yy, xv;
        chunk_pos<G, THREADS>(e0, tid, j, yy, xv);
        const int gy = gy0 + yy, gx = gxa + 4 * xv;
        const bool rowok = yy < ph && gy >= 0 && gy < h;
        const float *row = src + (int64_t)(rowok ? gy : 0) * w;
        if (VEC4) {
            const bool ok = rowok && gx >= 0 && gx < w;
            const float4 v = *reinterpret_cast<const float4 *>(row + (ok ? gx : 0));
            t.v[j][0] = v.x; t.v[j][1] = v.y; t.v[j][2] = v.z; t.v[j][3] = v.w;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) t.v[j][i] = row[rowok && gx + i >= 0 && gx + i < w ? gx + i : 0];
        }
        if (G::PO) t.v[j][4 * G::PO] = row[rowok && gx + 4 >= 0 && gx + 4 < w ? gx + 4 : 0];
    }
}

// Split the carried pixels into the three planes of one buffer: word i of a plane row holds the pieces of the
// staged pixels (2i + PO, 2i + 1 + PO); pixels outside the image are zero.
template <class G, int THREADS>
__device__ __forceinline__ void store_tile(const TileRegs<G, THREADS> &t, int e0, int tid, unsigned int *planes, int h,
                                           int w, int gy0, int gxa, int ph)
{
#pragma unroll
    for (int j = 0; j < TileRegs<G, THREADS>::NV; ++j) {
        int yy, xv;
        chunk_pos<G, THREADS>(e0, tid, j, yy, xv);
        if (yy >= ph) continue;
        const int gy = gy0 + yy, gx = gxa + 4 * xv;
        const bool rowok = gy >= 0 && gy < h;
        float v[5];
#pragma unroll
        for (int i = 0; i < 4 + G::PO; ++i) v[i] = rowok && gx + i >= 0 && gx + i < w ? t.v[j][i] : 0.f;
        unsigned int *dst = planes + yy * G::PWORDS + 2 * xv;
        unsigned ha, ma, la, hb, mb, lb;
        split3_pair(v[G::PO], v[1 + G::PO], ha, ma, la);
        split3_pair(v[2 + G::PO], v[3 + G::PO], hb, mb, lb);
        dst[0] = ha; dst[1] = hb;
        dst[G::PLANE] = ma; dst[G::PLANE + 1] = mb;
        dst[2 * G::PLANE] = la; dst[2 * G::PLANE + 1] = lb;
    }
}

// The pixel operand of one instruction slot set: the h, m and l pieces of this lane's four pairs.
struct PixelOperand {
    SplitOperand h, m, l;
};

// Per instruction and slot: whether the slot's word lies at the same offset from the group's first word in every
// group, and that offset.  An LDS read instruction costs the LDS about 4.4 clocks per wavefront whether it returns
// one word or two (measured: one-word reads 58 B per clock and compute unit, two-word reads 96, 16-byte reads 143),
// and at k >= 7 these reads, not their bytes, are what the contraction waits for; a slot with a uniform offset is
// read from the first slot's address register plus a constant, which lets the compiler pair it with its neighbour.
// A group none of whose slots holds a pair mirrors another group's addresses (split_offsets) and fits any offset; a
// group that holds some pairs but not this one makes the slot non-uniform (its own address is used).
template <class G>
struct SlotDeltas {
    int delta[G::STEPS][4];
    bool uniform[G::STEPS][4];
    constexpr SlotDeltas() : delta{}, uniform{}
    {
        for (int t = 0; t < G::STEPS; ++t)
            for (int i = 0; i < 4; ++i) {
                bool ok = true, have = false;
                int d = 0;
                for (int q = 0; q < 4; ++q) {
                    int j0 = 0, x0 = 0, j = 0, x = 0;
                    bool any = false;
                    for (int e = 0; e < 4; ++e) any = any || G::slot(t, q, e, j, x);
                    if (!any) continue;
                    const bool v0 = G::slot(t, q, 0, j0, x0), v = G::slot(t, q, i, j, x);
                    if (!v0 || !v) { ok = false; break; }
                    const int dd = (j - j0) * G::PWORDS + (x - x0);
                    if (have && dd != d) { ok = false; break; }
                    d = dd;
                    have = true;
                }
                uniform[t][i] = ok && have;
                delta[t][i] = d;
            }
    }
};

template <class G>
__device__ __forceinline__ void read_operand(PixelOperand &o, const unsigned int *src, const int (&off)[4], int t)
{
    constexpr SlotDeltas<G> tab{};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // (k = 3 and 5 are bound by their stores and measured 0-2 % slower with paired reads: left as they were)
        const int w = G::PAIRED_READS && tab.uniform[t][i] ? off[0] + tab.delta[t][i] : off[i];
        o.h.w[i] = src[w];
        o.m.w[i] = src[G::PLANE + w];
        o.l.w[i] = src[2 * G::PLANE + w];
    }
}

// RU consecutive output rows x NBX column blocks: acc[u][b] = the 16 x 16 outputs of row u, block b.  prow: word of
// the lane's first pixel pair in the tile row of the first output row, plane of the h pieces.  The work goes in
// sets of one instruction slot set x CB column blocks; the operands of the next set are read while the products
// of the current one run, and inside a set consecutive instructions belong to different accumulators (RU rows, or
// two column blocks when there is a single row).
template <class G, int NBX, int RU>
__device__ __forceinline__ void split_rows(const unsigned int *prow, const int (&toff)[G::STEPS][4],
                                           const SplitOperand (&wa)[RU][G::STEPS][3], floatx4 (&acc)[RU][NBX])
{
#pragma unroll
    for (int u = 0; u < RU; ++u)
#pragma unroll
        for (int b = 0; b < NBX; ++b) acc[u][b] = floatx4{0.f, 0.f, 0.f, 0.f};
    constexpr int CB = 1;     // (two blocks per set for single-row kernels was tried: k = 9 runs out of registers)
    constexpr int NB = NBX / CB, N = G::STEPS * NB;
    PixelOperand op[2][CB];
#pragma unroll
    for (int k = 0; k < CB; ++k) read_operand<G>(op[0][k], prow + k * 16, toff[0], 0);
#pragma unroll
    for (int idx = 0; idx < N; ++idx) {
        const int t = idx / NB, b0 = (idx - t * NB) * CB;
        if (idx + 1 < N) {
            const int t2 = (idx + 1) / NB, b2 = (idx + 1 - t2 * NB) * CB;
#pragma unroll
            for (int k = 0; k < CB; ++k) read_operand<G>(op[(idx + 1) & 1][k], prow + (b2 + k) * 16, toff[t2], t2);
        }
        // the reads above are issued before the products below (the scheduler would otherwise sink them to their
        // use and expose the LDS latency to the matrix pipeline)
        __builtin_amdgcn_sched_barrier(0);
        // small terms first: (h,l') (l,h') (m,m') (h,m') (m,h') (h,h')
        constexpr int WP[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
        for (int pr = 0; pr < 6; ++pr)
#pragma unroll
            for (int k = 0; k < CB; ++k) {
                const PixelOperand &o = op[idx & 1][k];
                const bf16x8 pix = pr == 0 ? o.l.v : (pr == 2 || pr == 3) ? o.m.v : o.h.v;
#pragma unroll
                for (int u = 0; u < RU; ++u)
                    acc[u][b0 + k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[u][t][WP[pr]].v, pix, acc[u][b0 + k], 0, 0, 0);
            }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// CODES: the maps are not written.  The maps of an input are hashed on the spot (Eq. 7-9: bit g of the code =
// [map g > 0]) and one byte per pixel and group of 8 filters leaves the kernel; the block histograms are counted
// from the code maps by hash_hist_kernel<.., CODES>.  Same products and sums as the map-writing kernel, so the codes are those of its
// maps bit for bit.
template <int KS, int NBX, int RU, int WAVES, bool VEC4, bool CODES>
__global__ __launch_bounds__(WAVES * 64, CSPLIT_WG_PER_CU<KS> == 3 ? 3 : 1) void conv_split_kernel(ConvSplitParams p)
{
    typedef SplitConv<KS, NBX, RU> G;
    constexpr int R = G::R, TW = G::TW, STEPS = G::STEPS, THREADS = WAVES * 64;
    typedef TileRegs<G, THREADS> Regs;
    static_assert(Regs::PASSES == 1, "a tile is carried in one pass");
    extern __shared__ unsigned int planes[];                       // two buffers of G::BUF words
    // workgroup b takes items b, b + grid, b + 2 grid, ...: at any time the workgroups of the chip write one
    // moving window of neighbouring tiles
    const long long item0 = blockIdx.x, istep = gridDim.x, item1 = p.n_items;
    if (item0 >= item1) return;
    const int h = p.h, w = p.w, L = p.L, th = p.th;
    const int64_t P = (int64_t)h * w;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane >> 4, c = lane & 15;
    const int tiles = p.tiles_x * p.tiles_y;
    const int ph = th + 2 * R;

    int toff[STEPS][4];
    split_offsets<G>(q, toff);
    // first pixel of the lane's windows: staged column SHX + 2c  ->  word (SHX - PO) / 2 + c
    const int lane_word = (G::SHX - G::PO) / 2 + c;
    Regs regs;

    for (int g0 = 0; g0 < L; g0 += 8) {
        SplitOperand wa[RU][STEPS][3];
#pragma unroll
        for (int u = 0; u < RU; ++u) split_weights<G, KS>(p.W, L, g0, u, q, c, wa[u]);
        // position of the first item
        int64_t n = item0 / tiles;
        int t0 = (int)(item0 - n * tiles);
        int ty = t0 / p.tiles_x, tx = t0 - ty * p.tiles_x;
        // and the step to the next one, as images and tiles
        const int64_t dn = istep / tiles;
        const int dt = (int)(istep - dn * tiles);
        load_tile<G, THREADS, VEC4>(regs, 0, threadIdx.x, p.in + n * P, h, w, ty * th - R, tx * TW - R - G::SHX, ph);
        store_tile<G, THREADS>(regs, 0, threadIdx.x, planes, h, w, ty * th - R, tx * TW - R - G::SHX, ph);
        __syncthreads();
        int cur = 0;
        // uniform: every store of this pass is an aligned float2 (w even: pairs never straddle the edge)
        const bool fast = (w & 1) == 0 && (((uintptr_t)p.out) & 7) == 0 && g0 + 8 <= L;
        // uniform: the 128-byte segments the lane groups write are whole, aligned cache lines (rows of a multiple of
        // 32 pixels on a 128-byte aligned base): the maps leave with the non-temporal hint.  Measured on single
        // launches of 4 GiB: 2-3 % at k = 7 and 9, 1-2 % at k = 5.  In the whole path the hint matters beyond the
        // launch that carries it, because what a kernel leaves dirty in the caches is written back during the next
        // one: with the hint on every map the step gains 1.2 % at 128 x 128, k = 7 and 0.5 % at 256 x 256, k = 9
        // (the histogram kernel that follows gains more than the convolution itself); with the hint only on the
        // large launches, or only on the small ones, a third of that or nothing.  On rows that split cache lines
        // (112 x 92 maps) the hint HALVES the store rate: those keep ordinary stores.
        const bool streaming = (w & 31) == 0 && (((uintptr_t)p.out) & 127) == 0;
        // CODES: a lane's two codes (columns x, x+1) leave as one aligned 16-bit store
        const bool code_pairs = (w & 1) == 0 && (((uintptr_t)p.codes) & 1) == 0;
        // CODES: where the sign of accumulator entry 2e + j of an even / odd column block goes in the lane's packed
        // word: bit 2q + e (the filter) of byte j (the column) of the block's 16 bits
        unsigned int code_bit[2][4];
#pragma unroll
        for (int ob = 0; ob < 2; ++ob)
#pragma unroll
            for (int ej = 0; ej < 4; ++ej) code_bit[ob][ej] = 1u << (16 * ob + 8 * (ej & 1) + 2 * q + (ej >> 1));
        // lane (q,c) ends with planes g0+2q (acc[0..1]) and g0+2q+1 (acc[2..3]) at columns x, x+1
        const int ga = g0 + 2 * q;
        for (long long item = item0; item < item1; item += istep) {
            // the item after this one
            t0 += dt;
            int64_t n2 = n + dn;
            if (t0 >= tiles) { t0 -= tiles; ++n2; }
            const int ty2 = t0 / p.tiles_x, tx2 = t0 - ty2 * p.tiles_x;
            const bool more = item + istep < item1;
            if (more)
                load_tile<G, THREADS, VEC4>(regs, 0, threadIdx.x, p.in + n2 * P, h, w, ty2 * th - R,
                                            tx2 * TW - R - G::SHX, ph);

            const unsigned int *buf = planes + cur * G::BUF + lane_word;
            const int rows = min(th, h - ty * th);
            const int gx_lane = tx * TW + 2 * c;
            const int nfull = min(NBX, (w - tx * TW) / CSPLIT_XB);   // column blocks fully inside the image
            for (int r = RU * wave; r < rows; r += RU * WAVES) {
                // (a row group that runs past the tile's last row reads staged rows of the buffer all the same
                // and its surplus rows are not written)
                floatx4 acc[RU][NBX];
                split_rows<G, NBX, RU>(buf + r * G::PWORDS, toff, wa, acc);
                if constexpr (CODES) {
#pragma unroll
                    for (int u = 0; u < RU; ++u) {
                        // this lane's share of the codes of its column pair in every block: bits 2q, 2q+1 (its two
                        // filters), low byte = column x, high byte = column x + 1; 16 bits per block
                        unsigned int part[2] = {0u, 0u};
#pragma unroll
                        for (int b = 0; b < NBX; ++b) {
                            unsigned int v = 0u;
#pragma unroll
                            for (int ej = 0; ej < 4; ++ej) v |= acc[u][b][ej] > 0.0f ? code_bit[b & 1][ej] : 0u;
                            part[b >> 1] |= v;
                        }
                        // OR over the four lane groups q (lanes c, c+16, c+32, c+48): every lane ends with all 8 bits
#pragma unroll
                        for (int i = 0; i < (NBX + 1) / 2; ++i) {
                            part[i] |= (unsigned int)__shfl_xor((int)part[i], 16);
                            part[i] |= (unsigned int)__shfl_xor((int)part[i], 32);
                        }
                        // lane group q writes block q: 64 lanes x 2 bytes = the 128 codes of the tile row
                        const int x = tx * TW + q * CSPLIT_XB + 2 * c;
                        if (r + u < rows && q < NBX && x < w) {
                            const unsigned int two = (part[(q >> 1) & ((NBX + 1) / 2 - 1)] >> (16 * (q & 1))) & 0xffffu;
                            unsigned char *d = p.codes + (n * ((L + 7) >> 3) + (g0 >> 3)) * P +
                                               (int64_t)(ty * th + r + u) * w + x;
                            if (code_pairs) {
                                *reinterpret_cast<unsigned short *>(d) = (unsigned short)two;
                            } else {
                                d[0] = (unsigned char)(two & 0xffu);
                                if (x + 1 < w) d[1] = (unsigned char)(two >> 8);
                            }
                        }
                    }
                    continue;
                }
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    if (r + u >= rows) continue;
                    const int gy = ty * th + r + u;
                    float *dst = p.out + (n * L + ga) * P + (int64_t)gy * w + gx_lane;
                    if (fast && streaming) {
#pragma unroll
                        for (int e = 0; e < 2; ++e)
#pragma unroll
                            for (int b = 0; b < NBX; ++b)
                                if (b < nfull || gx_lane + b * CSPLIT_XB < w)
                                    __builtin_nontemporal_store(floatx2{acc[u][b][2 * e], acc[u][b][2 * e + 1]},
                                                                reinterpret_cast<floatx2 *>(dst + e * P + b * CSPLIT_XB));
                    } else if (fast) {
#pragma unroll
                        for (int e = 0; e < 2; ++e)
#pragma unroll
                            for (int b = 0; b < NBX; ++b)
                                if (b < nfull || gx_lane + b * CSPLIT_XB < w)
                                    *reinterpret_cast<float2 *>(dst + e * P + b * CSPLIT_XB) =
                                        make_float2(acc[u][b][2 * e], acc[u][b][2 * e + 1]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            if (ga + e >= L) continue;
#pragma unroll
                            for (int b = 0; b < NBX; ++b) {
                                const int gx = gx_lane + b * CSPLIT_XB;
                                if (gx < w) dst[e * P + b * CSPLIT_XB] = acc[u][b][2 * e];
                                if (gx + 1 < w) dst[e * P + b * CSPLIT_XB + 1] = acc[u][b][2 * e + 1];
                            }
                        }
                    }
                }
            }
            // the other buffer was last read before the barrier that ended the previous item
            if (more)
                store_tile<G, THREADS>(regs, 0, threadIdx.x, planes + (cur ^ 1) * G::BUF, h, w, ty2 * th - R,
                                       tx2 * TW - R - G::SHX, ph);
            __syncthreads();
            cur ^= 1;
            n = n2; ty = ty2; tx = tx2;
        }
    }
}

// Output rows that share their pixel operands, wavefronts per workgroup and tile rows of maps that take several
// tiles, per patch size.  (Tile rows, measured on 128 x 128 maps in one process: k = 5 writes 5.4-5.9 TB/s in tiles
// of 16 rows against 5.0-5.1 in tiles of 32 and 3.6 in tiles of 4; k = 7 and 9 lose 3 % from 32 to 16 rows at two
// workgroups per compute unit -- k = 9 takes 16 rows for its three, CSPLIT_TH1 above.)
template <int KS> struct SplitShape { static constexpr int RU = 1, WAVES = 4, TH = CSPLIT_TH1<KS>; };
template <> struct SplitShape<7> { static constexpr int RU = 2, WAVES = 4, TH = CSPLIT_TH_MAX; };
template <> struct SplitShape<5> { static constexpr int RU = 1, WAVES = 4, TH = 16; };
template <> struct SplitShape<3> { static constexpr int RU = 2, WAVES = 4, TH = CSPLIT_TH_MAX; };

template <int KS, int NBX, bool VEC4, bool CODES>
static int conv_split_launch_vec(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L,
                                 float *out, unsigned char *codes)
{
    constexpr int RU = SplitShape<KS>::RU, WAVES = SplitShape<KS>::WAVES;
    typedef SplitConv<KS, NBX, RU> G;
    static_assert(2 * G::BUF * 4 * CSPLIT_WG_PER_CU<KS> <= 160 * 1024, "the workgroups of a compute unit must fit in LDS");
    static bool attr_set[MAX_DEVICES] = {};      // per device: the attribute is set on that device's code object
    if (!attr_set[ctx->device]) {
        DDCCA_HIP(ctx, hipFuncSetAttribute((const void *)conv_split_kernel<KS, NBX, RU, WAVES, VEC4, CODES>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 2 * G::BUF * 4));
        attr_set[ctx->device] = true;
    }
    ConvSplitParams p;
    p.in = in; p.W = W; p.out = out; p.codes = codes; p.h = h; p.w = w; p.L = L;
    p.tiles_x = (w + G::TW - 1) / G::TW;
    // a map of at most CSPLIT_TH1 rows is one tile row; a higher one goes in equal tile heights of at most
    // SplitShape::TH rows; a multiple of the rows one pass of the workgroup covers either way
    constexpr int PASS = RU * WAVES;
    const int cap = h <= CSPLIT_TH1<KS> ? CSPLIT_TH1<KS> : SplitShape<KS>::TH;
    const int nty = (h + cap - 1) / cap;
    p.th = std::min(cap, ((h + nty - 1) / nty + PASS - 1) / PASS * PASS);
    p.tiles_y = (h + p.th - 1) / p.th;
    p.n_items = (long long)n * p.tiles_x * p.tiles_y;
    unsigned grid = (unsigned)std::min(p.n_items, (long long)CSPLIT_WG_PER_CU<KS> * ctx->n_cu);
    // Workgroup b takes items b, b + grid, ...: with a grid that shares a factor with the tiles of an image, a
    // workgroup would meet only some of an image's tiles over and over -- and when the last tile row or column is
    // smaller than the others, always the small ones or never (112 rows in tiles of 32: a quarter of the
    // workgroups idle half of the time).  A grid coprime to the tile count deals every kind of tile to every
    // workgroup.
    const int tiles = p.tiles_x * p.tiles_y;
    if ((h % p.th != 0 || w % G::TW != 0) && p.n_items > grid) {
        auto gcd = [](unsigned a, unsigned b) { while (b) { const unsigned t = a % b; a = b; b = t; } return a; };
        while (grid > 1 && gcd(grid, (unsigned)tiles) != 1) --grid;
    }
    hipLaunchKernelGGL((conv_split_kernel<KS, NBX, RU, WAVES, VEC4, CODES>), dim3(grid), dim3(WAVES * 64), 2 * G::BUF * 4,
                       ctx->stream, p);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

template <int KS, int NBX, bool CODES>
static int conv_split_launch_nbx(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L,
                                 float *out, unsigned char *codes)
{
    // 16-byte loads when every image row starts on a 16-byte boundary
    if ((w & 3) == 0 && (((uintptr_t)in) & 15) == 0)
        return conv_split_launch_vec<KS, NBX, true, CODES>(ctx, in, n, h, w, W, L, out, codes);
    return conv_split_launch_vec<KS, NBX, false, CODES>(ctx, in, n, h, w, W, L, out, codes);
}

template <int KS, bool CODES>
static int conv_split_launch(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int L,
                             float *out, unsigned char *codes)
{
    // equal-width tiles of at most CSPLIT_MAX_NBX column blocks
    const int xblocks = (w + CSPLIT_XB - 1) / CSPLIT_XB;
    const int tiles_x = (xblocks + CSPLIT_MAX_NBX - 1) / CSPLIT_MAX_NBX;
    const int nbx = (xblocks + tiles_x - 1) / tiles_x;
    switch (nbx) {
        case 1: return conv_split_launch_nbx<KS, 1, CODES>(ctx, in, n, h, w, W, L, out, codes);
        case 2: return conv_split_launch_nbx<KS, 2, CODES>(ctx, in, n, h, w, W, L, out, codes);
        case 3: return conv_split_launch_nbx<KS, 3, CODES>(ctx, in, n, h, w, W, L, out, codes);
        default: return conv_split_launch_nbx<KS, 4, CODES>(ctx, in, n, h, w, W, L, out, codes);
    }
}

int launch_conv_split(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L,
                      float *out)
{
    ProfScope prof(ctx, DDCCA_K_CONV);
    switch (k) {
        case 3: return conv_split_launch<3, false>(ctx, in, n, h, w, W, L, out, nullptr);
        case 5: return conv_split_launch<5, false>(ctx, in, n, h, w, W, L, out, nullptr);
        case 7: return conv_split_launch<7, false>(ctx, in, n, h, w, W, L, out, nullptr);
        case 9: return conv_split_launch<9, false>(ctx, in, n, h, w, W, L, out, nullptr);
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
}

// The hash codes (Eq. 7-9) of the L maps this convolution would write: codes[n][ceil(L/8)][h][w], byte i of a pixel
// = bits 8i .. 8i+7 of its code.
int launch_conv_split_codes(ddcca_ctx *ctx, const float *in, int64_t n, int h, int w, const float *W, int k, int L,
                            unsigned char *codes)
{
    ProfScope prof(ctx, DDCCA_K_CONV_HASH_HIST);
    switch (k) {
        case 3: return conv_split_launch<3, true>(ctx, in, n, h, w, W, L, nullptr, codes);
        case 5: return conv_split_launch<5, true>(ctx, in, n, h, w, W, L, nullptr, codes);
        case 7: return conv_split_launch<7, true>(ctx, in, n, h, w, W, L, nullptr, codes);
        case 9: return conv_split_launch<9, true>(ctx, in, n, h, w, W, L, nullptr, codes);
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
}

}  // namespace ddcca
