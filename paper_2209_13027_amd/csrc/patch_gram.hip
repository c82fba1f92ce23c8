// Patch Gram accumulation (Section II-A matrices, Section III Eq. 15 batching):
//   for every pixel of every map pair, z = [x1; x2] (the two k*k patches, 2D entries) and
//   G += z z^T.
// The patch matrix of Eq. 1 is never formed: an image tile with its halo is staged in LDS and
// the MFMA operands are read straight from the tile with a per-lane window offset.  The
// contraction runs on v_mfma_f32_16x16x4_f32 (K = 4 consecutive patches of a tile row per
// instruction).  For a Gram the A operand of row block bi and the B operand of column block
// bj have the same register layout (lane l: stacked row 16*b + l%16, patch l/16), so one LDS
// read per block feeds every tile of that block row and block column.
//
// Mean removal: the mean-removed patch is H x with H = I - 11^T/D, and H annihilates
// constant vectors, so H x = H (x - c 1) for ANY per-patch constant c.  The kernel uses
// c = the patch's own centre pixel: y = x - x_centre has a zero at the centre position, so
// only D-1 entries per view are contracted (2(D-1) = 16, 48, 96, 160 stacked rows for
// k = 3, 5, 7, 9: whole 16-row blocks, no padding), and the export step rebuilds
// sum (H x)(H x)^T = H (sum y y^T) H in fp64.  Differences to the centre pixel also carry no
// DC level, which keeps the fp32 accumulators well scaled; on top of that each tile is
// shifted by an estimate of its mean pixel value (harmless, and it keeps the staged values
// themselves small).
//
// Optional arithmetic (DDCCA_GRAM_BF16X3): the contraction on the bf16 matrix pipeline with every operand
// y split exactly into three bf16 pieces and the six significant piece products summed in fp32 (see
// conv_split.h).  K = 32 consecutive patches per instruction; the pieces of a block's operand (8 patches
// per lane) are made in registers right after the centre subtraction, so tiles, slots, flushes and the
// export are those of the fp32 kernel.  The bf16 matrix instructions run beside the vector ALU, which the
// fp32 ones do not, so the splitting work hides behind the matrix work of the other resident wavefront.
//
// Maps recomputed in the tile staging (Section II-B on Section II-A, DDCCA_MAPS_RECOMPUTED): when the maps
// are the previous stage's convolution of given inputs, a workgroup can hold the INPUT tile (halo of both
// stages) in LDS and produce the tile of each of the L_prev maps from it right into the pixel buffer the
// contraction reads, so the maps never exist in HBM.  Items are then (input map, tile, filter) with the
// filter innermost: the input tile is loaded once per L_prev items.  The convolution runs on the vector
// ALU (8 outputs of a row per thread and pass, the filter taps as scalar operands).
#include <type_traits>

#include "conv_split.h"

namespace ddcca {

constexpr int GRAM_THREADS = 256;          // 4 wavefronts
constexpr int GRAM_TH = 16;                // patch rows per tile
constexpr int GRAM_TW_MAX = 128;           // patch columns per tile (multiple of 4)
constexpr size_t LDS_BYTES_PER_CU = 160 * 1024;
constexpr int GRAM_KU = 2;                 // k-steps whose operand reads and centre subtractions are grouped

struct GramParams {
    const float *v1, *v2;                  // [n_maps][h][w]
    int64_t n_items;                       // n_maps * tiles_y * tiles_x
    int h, w, tiles_x, tiles_y, tw;        // tw: tile width in patches
    int pitch;                             // LDS row pitch of the pixel tile (floats)
    int view_stride;                       // LDS floats per view's pixel tile
    int buf_stride;                        // LDS floats per tile buffer (two views); two buffers
    int dc_off;                            // LDS float offset of the 2x2 DC-estimate cells
    int flush_items;                       // items between fp64 flushes
    double *slots;                         // [n_slots][NT*256]
    int slots_valid;                       // slots below this hold earlier partial sums
    // maps recomputed in the staging (FUSE kernels): v1, v2 are the INPUTS [n_inputs][h][w] and
    // n_items = n_inputs * tiles * Lp
    const float *Wp1, *Wp2;                // [Lp][KS][KS] filters of the previous stage per view
    int Lp;
    int raw_off, raw_pitch, raw_view_stride;   // LDS floats: input tiles after the DC cells
};

// Compile-time geometry.  TSPLIT wavefronts share one group of patch rows and split the
// tile list between them (tile t belongs to role t % TSPLIT), which keeps the
// accumulators of one wavefront within the register budget for large k.
// CROSS restricts the tile list to the view-1 x view-2 block (all the class-conditioned
// matrices need).
template <int KS, int TSPLIT_, bool CROSS_>
struct GramGeom {
    static constexpr int D = KS * KS;
    static constexpr int R = (KS - 1) / 2;
    static constexpr int DR = D - 1;                     // contracted entries per view (centre dropped)
    static constexpr int CEN = (D - 1) / 2;              // patch index of the centre pixel
    static constexpr int NB = (2 * DR) / 16;
    // centre-pixel operands per k-step: one per view when no 16-row block mixes the views,
    // else one per block
    static constexpr bool STRADDLE = (DR % 16) != 0;
    static constexpr int NCEN = STRADDLE ? NB : 2;
    static constexpr int cen_index(int b) { return STRADDLE ? b : (b >= NB / 2 ? 1 : 0); }
    static_assert((2 * DR) % 16 == 0, "2(k^2-1) is a multiple of 16 for odd k");
    static constexpr int NT = NB * (NB + 1) / 2;         // slot layout always covers the full triangle
    static constexpr int TSPLIT = TSPLIT_;
    static constexpr bool CROSS = CROSS_;
    static constexpr int NPG = 4 / TSPLIT_;              // patch-row groups per workgroup
    static constexpr int B1_END = (DR + 15) / 16;        // blocks [0, B1_END) contain view-1 rows
    static constexpr int B2_BEGIN = DR / 16;             // blocks [B2_BEGIN, NB) contain view-2 rows
    static constexpr bool tile_used(int bi, int bj) { return !CROSS_ || (bi < B1_END && bj >= B2_BEGIN); }
    static constexpr int used_tiles()
    {
        int n = 0;
        for (int bi = 0; bi < NB; ++bi)
            for (int bj = bi; bj < NB; ++bj) n += tile_used(bi, bj) ? 1 : 0;
        return n;
    }
    static constexpr int NACC = (used_tiles() + TSPLIT_ - 1) / TSPLIT_;   // accumulator tiles per wavefront
    // groups of k-steps per run of the fp32 contraction's loop (one set of operand addresses per run)
    static constexpr int GU = 8;
};

template <typename G, int ROLE>
__device__ __forceinline__ void gram_mfma_step(const float (&z)[G::NB], floatx4 (&acc)[G::NACC])
{
    int u = 0;       // index among used tiles
#pragma unroll
    for (int bi = 0; bi < G::NB; ++bi)
#pragma unroll
        for (int bj = bi; bj < G::NB; ++bj) {
            if (G::tile_used(bi, bj)) {
                if (u % G::TSPLIT == ROLE)
                    acc[u / G::TSPLIT] = __builtin_amdgcn_mfma_f32_16x16x4f32(z[bi], z[bj], acc[u / G::TSPLIT], 0, 0, 0);
                ++u;
            }
        }
}

// All k-steps of this wavefront's patch rows of the staged tile.
template <typename G, int ROLE>
__device__ __forceinline__ void gram_rows(const float *pix, int pitch, int rows, int cols, int pg, int q,
                                          const int (&pix_off)[G::NB], const int (&cen_off)[G::NCEN],
                                          floatx4 (&acc)[G::NACC])
{
    constexpr int NB = G::NB;
    const int full = cols >> 2, tail = cols & 3;
    for (int py = pg; py < rows; py += G::NPG) {
        const float *prow = pix + py * pitch;
        // KU k-steps per iteration, in phases: the LDS reads of the next KU steps (the two steps of a block
        // pair up in one two-address read), the MFMAs of the KU current ones, then the centre subtractions
        // of the next KU.  The fp32 matrix instructions do not overlap with the vector ALU on a SIMD, and
        // every LDS read instruction costs the matrix pipeline about as much as two vector instructions
        // (measured: 8 and 4 cycles per MFMA-free slot), so fewer, wider reads are what pays; more than two
        // steps per group gain nothing further.
        constexpr int KU = GRAM_KU;
        float z[KU][NB];
        const int groups = full / KU;
        if (groups > 0) {
#pragma unroll
            for (int u = 0; u < KU; ++u)
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    z[u][b] = prow[pix_off[b] + 4 * u] - prow[cen_off[G::cen_index(b)] + 4 * u];
        }
        // One group: the LDS reads of the group at column nx of pk (with GU > 1 the group after the last one reads
        // 4 * KU columns past the row's last patch: inside the row pitch or the 16 floats that follow every view's
        // tile, and never used), the MFMAs of the current one, the centre subtractions of the next.
        auto group = [&](const float *pk, int nx) {
            float pa[KU][NB], pc[KU][G::NCEN];
#pragma unroll
            for (int u = 0; u < KU; ++u) {
#pragma unroll
                for (int b = 0; b < NB; ++b) pa[u][b] = pk[pix_off[b] + nx + 4 * u];
#pragma unroll
                for (int v = 0; v < G::NCEN; ++v) pc[u][v] = pk[cen_off[v] + nx + 4 * u];
            }
            // three fenced phases: left to itself the scheduler moves the subtractions up to right behind the reads
            // they use, where they wait for the LDS with one MFMA between
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < KU; ++u) gram_mfma_step<G, ROLE>(z[u], acc);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < KU; ++u)
#pragma unroll
                for (int b = 0; b < NB; ++b) z[u][b] = pa[u][b] - pc[u][G::cen_index(b)];
            __builtin_amdgcn_sched_barrier(0);
        };
        // GU groups per iteration share one set of operand addresses (the later ones add an immediate offset)
        constexpr int GU = G::GU;
        if constexpr (GU == 1) {
            // (the last group reads its own columns again)
            for (int kg = 0; kg < groups; ++kg) group(prow, 4 * KU * (kg + 1 < groups ? kg + 1 : kg));
        } else {
            // runs of GU, GU/2, .. 1 groups, each run with one address update for all its groups
            int kg = 0;
            auto run = [&](auto n) {
                constexpr int N = decltype(n)::value;
                const float *pk = prow + 4 * KU * kg;
#pragma unroll
                for (int j = 0; j < N; ++j) group(pk, 4 * KU * (j + 1));
                kg += N;
            };
            while (kg + GU <= groups) run(std::integral_constant<int, GU>{});
            if constexpr (GU >= 8) if (kg + 4 <= groups) run(std::integral_constant<int, 4>{});
            if constexpr (GU >= 4) if (kg + 2 <= groups) run(std::integral_constant<int, 2>{});
            if (kg < groups) run(std::integral_constant<int, 1>{});
        }
        for (int kx = groups * KU; kx < full; ++kx) {
            float z0[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) z0[b] = prow[pix_off[b] + 4 * kx] - prow[cen_off[G::cen_index(b)] + 4 * kx];
            gram_mfma_step<G, ROLE>(z0, acc);
        }
        float z0[NB];
        if (tail) {                                   // ragged end of the row: patches past the image add 0
            const bool ok = q < tail;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float v = prow[pix_off[b] + 4 * full] - prow[cen_off[G::cen_index(b)] + 4 * full];
                z0[b] = ok ? v : 0.f;
            }
            gram_mfma_step<G, ROLE>(z0, acc);
        }
    }
}

// ---- three-piece bf16 operands --------------------------------------------------------------------------
// One K = 32 step: six piece products per tile, product by product across the tiles (consecutive
// instructions write different accumulators), small terms first.
template <typename G, int ROLE>
__device__ __forceinline__ void gram_mfma_step_split(const SplitOperand (&zh)[G::NB], const SplitOperand (&zm)[G::NB],
                                                     const SplitOperand (&zl)[G::NB], floatx4 (&acc)[G::NACC])
{
#pragma unroll
    for (int pr = 0; pr < 6; ++pr) {
        int u = 0;
#pragma unroll
        for (int bi = 0; bi < G::NB; ++bi)
#pragma unroll
            for (int bj = bi; bj < G::NB; ++bj) {
                if (G::tile_used(bi, bj)) {
                    if (u % G::TSPLIT == ROLE) {
                        const bf16x8 a = pr == 1 ? zl[bi].v : (pr == 2 || pr == 4) ? zm[bi].v : zh[bi].v;
                        const bf16x8 b = pr == 0 ? zl[bj].v : (pr == 2 || pr == 3) ? zm[bj].v : zh[bj].v;
                        acc[u / G::TSPLIT] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[u / G::TSPLIT], 0, 0, 0);
                    }
                    ++u;
                }
            }
    }
}

// All K = 32 steps of this wavefront's patch rows of the staged tile.  pix_off / cen_off point at the first
// of the lane's 8 consecutive patches (8 * (lane / 16)).
template <typename G, int ROLE>
__device__ __forceinline__ void gram_rows_split(const float *pix, int pitch, int rows, int cols, int pg, int q,
                                                const int (&pix_off)[G::NB], const int (&cen_off)[G::NCEN],
                                                floatx4 (&acc)[G::NACC])
{
    constexpr int NB = G::NB;
    const int steps = (cols + 31) >> 5;
    for (int py = pg; py < rows; py += G::NPG) {
        const float *prow = pix + py * pitch;
        for (int ks = 0; ks < steps; ++ks) {
            const int x0 = 32 * ks;
            const bool partial = x0 + 32 > cols;          // ragged end of the row: patches past the tile add 0
            const int valid = cols - x0 - 8 * q;          // this lane's patches j < valid exist
            float cen[G::NCEN][8];
#pragma unroll
            for (int v = 0; v < G::NCEN; ++v)
#pragma unroll
                for (int j = 0; j < 8; ++j) cen[v][j] = prow[cen_off[v] + x0 + j];
            SplitOperand zh[NB], zm[NB], zl[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float y[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) y[j] = prow[pix_off[b] + x0 + j] - cen[G::cen_index(b)][j];
                if (partial) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) y[j] = j < valid ? y[j] : 0.f;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) split3_pair(y[2 * i], y[2 * i + 1], zh[b].w[i], zm[b].w[i], zl[b].w[i]);
            }
            gram_mfma_step_split<G, ROLE>(zh, zm, zl, acc);
        }
    }
}

// Tile number (position in the full upper block triangle) of the u-th used tile.
template <typename G>
struct GramTileTable {
    int t[G::NT];
    constexpr GramTileTable() : t()
    {
        int u = 0, idx = 0;
        for (int bi = 0; bi < G::NB; ++bi)
            for (int bj = bi; bj < G::NB; ++bj, ++idx)
                if (G::tile_used(bi, bj)) t[u++] = idx;
        for (; u < G::NT; ++u) t[u] = 0;
    }
};

// Add this wavefront's accumulators into the workgroup's fp32 staging buffer (first writer
// stores, later ones add) and clear them.
template <typename G>
__device__ __forceinline__ void gram_stage_acc(floatx4 (&acc)[G::NACC], float *stage, int lane, bool first)
{
#pragma unroll
    for (int a = 0; a < G::NACC; ++a) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float *dst = stage + (a * 4 + v) * 64 + lane;
            *dst = first ? acc[a][v] : *dst + acc[a][v];
        }
        acc[a] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
}

// Workgroup-wide flush: the patch-row groups' fp32 accumulators are summed in LDS (one role
// at a time) and folded into the workgroup's fp64 slot.  Must be called by all threads.
template <typename G>
__device__ __forceinline__ void gram_flush(floatx4 (&acc)[G::NACC], float *stage, double *slot, int pg, int role,
                                           bool rmw)
{
    static constexpr GramTileTable<G> table{};
    const int lane = threadIdx.x & 63;
    for (int r = 0; r < G::TSPLIT; ++r) {
        for (int g = 0; g < G::NPG; ++g) {
            if (pg == g && role == r) gram_stage_acc<G>(acc, stage, lane, g == 0);
            __syncthreads();
        }
        for (int e = threadIdx.x; e < G::NACC * 256; e += GRAM_THREADS) {
            const int u = (e >> 8) * G::TSPLIT + r;
            if (u < G::used_tiles()) {
                double *dst = slot + (size_t)table.t[u] * 256 + (e & 255);
                const double add = (double)stage[e];
                *dst = rmw ? *dst + add : add;
            }
        }
        __syncthreads();
    }
}

// Tile staging.  Thread (wave w, lane l) owns tile elements (row w + 4*jy, column l + 64*jx).
template <int KS>
struct GramStage {
    static constexpr int R = (KS - 1) / 2;
    static constexpr int PH = GRAM_TH + 2 * R;
    static constexpr int NJY = (PH + 3) / 4;
    static constexpr int NJX = (GRAM_TW_MAX + 2 * R + 63) / 64;
};

// Issue the global loads of one tile (both views) into registers; elements outside the image
// (zero padding) or outside the tile read as 0.
template <int KS>
__device__ __forceinline__ void gram_tile_fetch(const GramParams &p, int64_t m, int ty, int tx, int pw,
                                                float (&ra)[GramStage<KS>::NJY][GramStage<KS>::NJX],
                                                float (&rb)[GramStage<KS>::NJY][GramStage<KS>::NJX])
{
    using S = GramStage<KS>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int gy0 = ty * GRAM_TH - S::R + wave, gx0 = tx * p.tw - S::R + lane;
    const int64_t P = (int64_t)p.h * p.w;
    const float *s1 = p.v1 + m * P, *s2 = p.v2 + m * P;
#pragma unroll
    for (int jy = 0; jy < S::NJY; ++jy) {
        const int gy = gy0 + 4 * jy;
        const bool yok = gy >= 0 && gy < p.h && wave + 4 * jy < S::PH;
#pragma unroll
        for (int jx = 0; jx < S::NJX; ++jx) {
            const int gx = gx0 + 64 * jx;
            float a = 0.f, b = 0.f;
            if (yok && gx >= 0 && gx < p.w && lane + 64 * jx < pw) {
                const int64_t o = (int64_t)gy * p.w + gx;
                a = s1[o];
                b = s2[o];
            }
            ra[jy][jx] = a;
            rb[jy][jx] = b;
        }
    }
}

// Write a fetched tile into an LDS buffer, shifted by the DC estimates (c1, c2); wavefront 0
// leaves the mean of its own share of the tile as the DC estimate for the next tile.
template <int KS>
__device__ __forceinline__ void gram_tile_store(const GramParams &p, float *buf, int pw, float c1, float c2,
                                                const float (&ra)[GramStage<KS>::NJY][GramStage<KS>::NJX],
                                                const float (&rb)[GramStage<KS>::NJY][GramStage<KS>::NJX],
                                                float *dc_next)
{
    using S = GramStage<KS>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int jy = 0; jy < S::NJY; ++jy) {
        const int yy = wave + 4 * jy;
#pragma unroll
        for (int jx = 0; jx < S::NJX; ++jx) {
            const int xx = lane + 64 * jx;
            if (yy < S::PH && xx < pw) {
                buf[yy * p.pitch + xx] = ra[jy][jx] - c1;
                buf[p.view_stride + yy * p.pitch + xx] = rb[jy][jx] - c2;
                s1 += ra[jy][jx];
                s2 += rb[jy][jx];
            }
        }
    }
    if (wave == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            s1 += __shfl_xor(s1, o);
            s2 += __shfl_xor(s2, o);
        }
        if (lane == 0) {
            const float inv = 1.0f / (float)(((S::PH + 3) / 4) * pw);
            dc_next[0] = s1 * inv;
            dc_next[1] = s2 * inv;
        }
    }
}

// Tile staging by aligned chunks of four pixels, for images whose rows start on 16-byte boundaries (w a multiple
// of 4, aligned views): a fifth of the load and LDS-write instructions of the element-wise staging above, which
// matters because the vector instructions of the staging run while the matrix pipeline of their SIMD waits.  Same
// LDS layout.  Chunk e of a tile is row e / NCX, tile columns X0 + 4*(e % NCX) .. + 3; X0 <= 0 is such that the
// chunk's image column is a multiple of 4 (tile widths are multiples of 4), so a chunk lies wholly inside the
// image or outside.  Thread t carries chunks t, t + 256, ...
template <int KS>
struct GramStageV {
    static constexpr int R = (KS - 1) / 2;
    static constexpr int PH = GRAM_TH + 2 * R;
    static constexpr int X0 = -((4 - R % 4) % 4);
    static constexpr int NCX = (GRAM_TW_MAX + 2 * R - X0 + 3) / 4;
    static constexpr int NV = (PH * NCX + GRAM_THREADS - 1) / GRAM_THREADS;
    __device__ static void chunk(int j, int &yy, int &xx)
    {
        const int e = threadIdx.x + GRAM_THREADS * j;
        yy = e / NCX;
        xx = X0 + 4 * (e - yy * NCX);
    }
};

template <int KS>
__device__ __forceinline__ void gram_tile_fetch_v(const GramParams &p, int64_t m, int ty, int tx, int pw,
                                                  float4 (&va)[GramStageV<KS>::NV], float4 (&vb)[GramStageV<KS>::NV])
{
    using S = GramStageV<KS>;
    const int gy0 = ty * GRAM_TH - S::R, gx0 = tx * p.tw - S::R;
    const int64_t P = (int64_t)p.h * p.w;
    const float *s1 = p.v1 + m * P, *s2 = p.v2 + m * P;
#pragma unroll
    for (int j = 0; j < S::NV; ++j) {
        int yy, xx;
        S::chunk(j, yy, xx);
        const int gy = gy0 + yy, gx = gx0 + xx;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
        // (one condition, not a chain: one masked region per chunk instead of nested branches)
        const bool ok = (yy < S::PH) & (xx < pw) & (gy >= 0) & (gy < p.h) & (gx >= 0) & (gx < p.w);
        if (ok) {
            const int64_t o = (int64_t)gy * p.w + gx;
            a = *reinterpret_cast<const float4 *>(s1 + o);
            b = *reinterpret_cast<const float4 *>(s2 + o);
        }
        va[j] = a;
        vb[j] = b;
    }
}

// The DC estimate of a fetched tile: the mean over the second chunk of every lane of the last wavefront (256 pixels
// of rows in the middle of the tile; the last wavefront carries the fewest chunks).  Called by that wavefront.
template <int KS>
__device__ __forceinline__ void gram_tile_mean_v(int pw, const float4 (&va)[GramStageV<KS>::NV],
                                                 const float4 (&vb)[GramStageV<KS>::NV], float *dc_out)
{
    using S = GramStageV<KS>;
    static_assert(S::NV >= 2 && 2 * GRAM_THREADS <= S::PH * S::NCX, "every lane has a second chunk inside the tile");
    int yy, xx;
    S::chunk(1, yy, xx);
    const float a[4] = {va[1].x, va[1].y, va[1].z, va[1].w}, b[4] = {vb[1].x, vb[1].y, vb[1].z, vb[1].w};
    float s1 = 0.f, s2 = 0.f, cnt = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (xx + i >= 0 && xx + i < pw) {
            s1 += a[i];
            s2 += b[i];
            cnt += 1.f;
        }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        s1 += __shfl_xor(s1, o);
        s2 += __shfl_xor(s2, o);
        cnt += __shfl_xor(cnt, o);
    }
    if ((threadIdx.x & 63) == 0) {
        dc_out[0] = s1 / cnt;
        dc_out[1] = s2 / cnt;
    }
}

// The LDS rows of a tile staged by chunks begin XS = -X0 columns before tile column 0, so that every chunk is stored
// whole at a multiple of four columns (the readers start XS columns in; the row pitch covers the last chunk).  The
// pitch is a multiple of 4 floats for k = 5 and 9 and even for k = 3 and 7.
template <int KS>
__device__ __forceinline__ void gram_chunk_store(float *dst, float4 v)
{
    if constexpr (KS == 5 || KS == 9) {
        *reinterpret_cast<float4 *>(dst) = v;
    } else {
        *reinterpret_cast<float2 *>(dst) = make_float2(v.x, v.y);
        *reinterpret_cast<float2 *>(dst + 2) = make_float2(v.z, v.w);
    }
}

template <int KS>
__device__ __forceinline__ void gram_tile_store_v(const GramParams &p, float *buf, int pw, float c1, float c2,
                                                  const float4 (&va)[GramStageV<KS>::NV],
                                                  const float4 (&vb)[GramStageV<KS>::NV], float *dc_next)
{
    using S = GramStageV<KS>;
#pragma unroll
    for (int j = 0; j < S::NV; ++j) {
        int yy, xx;
        S::chunk(j, yy, xx);
        if ((yy < S::PH) & (xx < pw)) {
            float *dst = buf + yy * p.pitch + (xx - S::X0);
            gram_chunk_store<KS>(dst, make_float4(va[j].x - c1, va[j].y - c1, va[j].z - c1, va[j].w - c1));
            gram_chunk_store<KS>(dst + p.view_stride,
                                 make_float4(vb[j].x - c2, vb[j].y - c2, vb[j].z - c2, vb[j].w - c2));
        }
    }
    if (threadIdx.x >= GRAM_THREADS - 64) gram_tile_mean_v<KS>(pw, va, vb, dc_next);
}

// ---- maps recomputed from an input tile ------------------------------------------------------------------
template <int KS>
struct GramRaw {
    static constexpr int R = (KS - 1) / 2;
    static constexpr int PH = GRAM_TH + 2 * R;             // map rows of a tile with its halo
    static constexpr int RH = PH + 2 * R;                  // input rows under them
    static constexpr int RUN = 8;                          // outputs of a row per thread and pass
    static constexpr int SEG = (RUN + 2 * R + 3) & ~3;     // input columns under a run, whole float4s
    static constexpr int runs_x(int pw) { return (pw + RUN - 1) / RUN; }
    static constexpr int pitch(int pw) { return RUN * (runs_x(pw) - 1) + SEG; }
    static constexpr int NE = (RH * pitch(GRAM_TW_MAX + 2 * R) + GRAM_THREADS - 1) / GRAM_THREADS;
};

// The input tile under (input map n, tile t) of both views into LDS; outside the image: 0 (Eq. 6 pads with
// zeros).  Element (y, x) is image pixel (ty*TH - 2R + y, tx*tw - 2R + x).
template <int KS>
__device__ __forceinline__ void gram_raw_load(const GramParams &p, int64_t nt, int tiles, float *raw)
{
    using S = GramRaw<KS>;
    const int64_t n = nt / tiles;
    const int t = (int)(nt - n * tiles);
    const int ty = t / p.tiles_x, tx = t - ty * p.tiles_x;
    const int gy0 = ty * GRAM_TH - 2 * S::R, gx0 = tx * p.tw - 2 * S::R;
    const int64_t P = (int64_t)p.h * p.w;
    const float *s1 = p.v1 + n * P, *s2 = p.v2 + n * P;
    const int total = S::RH * p.raw_pitch;
    float a[S::NE], b[S::NE];
#pragma unroll
    for (int i = 0; i < S::NE; ++i) {
        const int e = threadIdx.x + GRAM_THREADS * i;
        const int y = e / p.raw_pitch, x = e - y * p.raw_pitch;
        const int gy = gy0 + y, gx = gx0 + x;
        a[i] = 0.f;
        b[i] = 0.f;
        if (e < total && gy >= 0 && gy < p.h && gx >= 0 && gx < p.w) {
            const int64_t o = (int64_t)gy * p.w + gx;
            a[i] = s1[o];
            b[i] = s2[o];
        }
    }
#pragma unroll
    for (int i = 0; i < S::NE; ++i) {
        const int e = threadIdx.x + GRAM_THREADS * i;
        if (e < total) {
            raw[e] = a[i];
            raw[p.raw_view_stride + e] = b[i];
        }
    }
}

// Map l of the input tile into a pixel buffer: element (y, x) of the map tile is map pixel
// (ty*TH - R + y, tx*tw - R + x) = sum_{dy,dx} W[l][dy][dx] * input(y + dy, x + dx) in tile coordinates
// (Eq. 6), and 0 outside the image (the next stage pads the MAP with zeros).  Wavefronts 0, 1 take view 1,
// wavefronts 2, 3 view 2, so that the taps are scalar operands.  Stored shifted by the DC estimates (c1, c2);
// wavefronts 0 and 2 leave the mean of their own share as the estimate for the next tile.
template <int KS>
__device__ __forceinline__ void gram_tile_conv(const GramParams &p, const float *raw, float *buf, int l, int ty,
                                               int tx, int pw, float c1, float c2, float *dc_next)
{
    using S = GramRaw<KS>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int view = __builtin_amdgcn_readfirstlane(wave >> 1);
    const float *__restrict__ W = (view ? p.Wp2 : p.Wp1) + (size_t)l * KS * KS;
    const float *rv = raw + view * p.raw_view_stride;
    float *bv = buf + view * p.view_stride;
    const float c = view ? c2 : c1;
    const int nrx = S::runs_x(pw), nruns = S::PH * nrx;
    const int gy0 = ty * GRAM_TH - S::R, gx0 = tx * p.tw - S::R;
    float sum = 0.f, cnt = 0.f;
    for (int run = threadIdx.x & 127; run < nruns; run += 128) {
        const int y = run / nrx, x0 = (run - y * nrx) * S::RUN;
        float acc[S::RUN];
#pragma unroll
        for (int j = 0; j < S::RUN; ++j) acc[j] = 0.f;
        // (one filter row at a time: unrolled, all rows' input segments and taps would be in registers at once,
        // next to the Gram accumulators that live across this phase)
#pragma unroll 1
        for (int dy = 0; dy < KS; ++dy) {
            const float4 *rr = reinterpret_cast<const float4 *>(rv + (y + dy) * p.raw_pitch + x0);
            float seg[S::SEG];
#pragma unroll
            for (int v = 0; v < S::SEG / 4; ++v) {
                const float4 f = rr[v];
                seg[4 * v] = f.x;
                seg[4 * v + 1] = f.y;
                seg[4 * v + 2] = f.z;
                seg[4 * v + 3] = f.w;
            }
#pragma unroll
            for (int dx = 0; dx < KS; ++dx) {
                const float wv = W[dy * KS + dx];
#pragma unroll
                for (int j = 0; j < S::RUN; ++j) acc[j] = fmaf(wv, seg[j + dx], acc[j]);
            }
        }
        const int gy = gy0 + y;
        const bool yok = gy >= 0 && gy < p.h;
#pragma unroll
        for (int j = 0; j < S::RUN; ++j) {
            const int x = x0 + j, gx = gx0 + x;
            const float v = (yok && gx >= 0 && gx < p.w) ? acc[j] : 0.f;
            if (x < pw) {
                bv[y * p.pitch + x] = v - c;
                sum += v;
                cnt += 1.f;
            }
        }
    }
    if ((wave & 1) == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            sum += __shfl_xor(sum, o);
            cnt += __shfl_xor(cnt, o);
        }
        if (lane == 0) dc_next[view] = sum / cnt;          // (lane 0 holds at least one run: cnt > 0)
    }
}

template <int KS, int TSPLIT, bool CROSS, int WAVES_PER_EU, bool SPLIT, bool FUSE, bool VEC>
__global__ __launch_bounds__(GRAM_THREADS, WAVES_PER_EU) void patch_gram_kernel(GramParams p)
{
    static_assert(!(FUSE && CROSS), "maps are recomputed for the full Gram only");
    static_assert(!(FUSE && VEC), "the staging by chunks is for maps read from memory");
    using G = GramGeom<KS, TSPLIT, CROSS>;
    using S = GramStage<KS>;
    constexpr int R = G::R, NB = G::NB, NT = G::NT;
    extern __shared__ float lds[];
    float *dc = lds + p.dc_off;                            // [2][2] DC estimates, double-buffered
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, i = lane & 15;
    const int pg = wave / TSPLIT, role = wave % TSPLIT;

    // per-lane operand offsets for each 16-row block of the stacked vector: stacked row
    // 16*b + i is entry a' of view v (v = row / DR); entries at and after the centre shift by one
    int pix_off[NB], cen_off[G::NCEN];
    const int lane_patch = SPLIT ? 8 * q : q;             // first patch of the lane within a k-step
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int row = 16 * b + i;
        const int view = row >= G::DR ? 1 : 0;
        const int ar = row - view * G::DR;
        const int a = ar >= G::CEN ? ar + 1 : ar;
        const int dy = a / KS, dx = a - dy * KS;
        pix_off[b] = view * p.view_stride + dy * p.pitch + dx + lane_patch;
        if (G::STRADDLE) cen_off[b] = view * p.view_stride + R * p.pitch + R + lane_patch;
    }
    if (!G::STRADDLE) {
        cen_off[0] = R * p.pitch + R + lane_patch;
        cen_off[1] = p.view_stride + R * p.pitch + R + lane_patch;
    }

    floatx4 acc[G::NACC];
#pragma unroll
    for (int t = 0; t < G::NACC; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};

    // contiguous range of work items for this workgroup
    const int64_t per = p.n_items / gridDim.x, extra = p.n_items % gridDim.x;
    const int64_t first = blockIdx.x * per + min((int64_t)blockIdx.x, extra);
    const int64_t count = per + (blockIdx.x < extra ? 1 : 0);
    const int tiles = p.tiles_x * p.tiles_y;
    double *my_slot = p.slots + (size_t)blockIdx.x * NT * 256;
    bool rmw = (int)blockIdx.x < p.slots_valid;
    int since_flush = 0;
    const int pw = p.tw + 2 * R;

    float *raw = lds + p.raw_off;                          // FUSE: the input tiles of both views
    // FUSE: an item is (input map n, tile t, filter l) = ((n * tiles + t) * Lp + l)
    auto tile_of = [&](int64_t item, int &ty, int &tx) {
        const int64_t nt = FUSE ? item / p.Lp : item;
        const int t = (int)(nt % tiles);
        ty = t / p.tiles_x;
        tx = t - ty * p.tiles_x;
    };
    // maps from memory: the workgroup's items are consecutive tiles, so the position (map, tile row, tile column)
    // of the current tile and of the one in flight is stepped, not divided out of the item number per tile
    int64_t m_cur = 0, m_nxt = 0;
    int ty_cur = 0, tx_cur = 0, ty_nxt = 0, tx_nxt = 0;
    if constexpr (!FUSE) {
        m_cur = first / tiles;
        const int t = (int)(first - m_cur * tiles);
        ty_cur = t / p.tiles_x;
        tx_cur = t - ty_cur * p.tiles_x;
    }
    // the tile in flight: by elements, or by aligned chunks of four (VEC)
    using SV = GramStageV<KS>;
    float ra[VEC ? 1 : S::NJY][VEC ? 1 : S::NJX], rb[VEC ? 1 : S::NJY][VEC ? 1 : S::NJX];
    float4 va[VEC ? SV::NV : 1], vb[VEC ? SV::NV : 1];
    if (FUSE && count > 0) {
        // first tile: once unshifted for its DC estimate, then again shifted by it
        int ty, tx;
        tile_of(first, ty, tx);
        const int l = (int)(first % p.Lp);
        gram_raw_load<KS>(p, first / p.Lp, tiles, raw);
        __syncthreads();
        gram_tile_conv<KS>(p, raw, lds, l, ty, tx, pw, 0.f, 0.f, dc + 2);
        __syncthreads();
        gram_tile_conv<KS>(p, raw, lds, l, ty, tx, pw, dc[2], dc[3], dc);
        __syncthreads();
    }
    if constexpr (VEC) {
        if (count > 0) {
            // first tile: its own DC estimate, then into buffer 0
            gram_tile_fetch_v<KS>(p, m_cur, ty_cur, tx_cur, pw, va, vb);
            if (wave == GRAM_THREADS / 64 - 1) gram_tile_mean_v<KS>(pw, va, vb, dc + 2);
            __syncthreads();
            gram_tile_store_v<KS>(p, lds, pw, dc[2], dc[3], va, vb, dc);
            __syncthreads();
        }
    }
    if constexpr (!FUSE && !VEC) if (count > 0) {
        // first tile: its own DC estimate, then into buffer 0
        gram_tile_fetch<KS>(p, m_cur, ty_cur, tx_cur, pw, ra, rb);
        float s1 = 0.f, s2 = 0.f;
        if (wave == 0) {
#pragma unroll
            for (int jy = 0; jy < S::NJY; ++jy)
#pragma unroll
                for (int jx = 0; jx < S::NJX; ++jx)
                    if (4 * jy < S::PH && lane + 64 * jx < pw) {
                        s1 += ra[jy][jx];
                        s2 += rb[jy][jx];
                    }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                s1 += __shfl_xor(s1, o);
                s2 += __shfl_xor(s2, o);
            }
            if (lane == 0) {
                const float inv = 1.0f / (float)(((S::PH + 3) / 4) * pw);
                dc[2] = s1 * inv;
                dc[3] = s2 * inv;
            }
        }
        __syncthreads();
        gram_tile_store<KS>(p, lds, pw, dc[2], dc[3], ra, rb, dc);
        __syncthreads();
    }

    for (int64_t it = 0; it < count; ++it) {
        const int64_t item = first + it;
        const int cur = (int)(it & 1);
        const float *pix = lds + cur * p.buf_stride + (VEC ? -SV::X0 : 0);
        const bool more = it + 1 < count;
        // the next tile travels from HBM to registers while this one is contracted
        if constexpr (!FUSE) {
            m_nxt = m_cur; ty_nxt = ty_cur; tx_nxt = tx_cur + 1;
            if (tx_nxt == p.tiles_x) {
                tx_nxt = 0;
                if (++ty_nxt == p.tiles_y) { ty_nxt = 0; ++m_nxt; }
            }
        }
        if constexpr (VEC) {
            if (more) gram_tile_fetch_v<KS>(p, m_nxt, ty_nxt, tx_nxt, pw, va, vb);
        } else if (!FUSE && more) {
            gram_tile_fetch<KS>(p, m_nxt, ty_nxt, tx_nxt, pw, ra, rb);
        }

        int ty = ty_cur, tx = tx_cur;
        if constexpr (FUSE) tile_of(item, ty, tx);
        const int rows = min(GRAM_TH, p.h - ty * GRAM_TH);
        const int cols = min(p.tw, p.w - tx * p.tw);
        if constexpr (SPLIT) {
            if (TSPLIT == 1 || role == 0) gram_rows_split<G, 0>(pix, p.pitch, rows, cols, pg, q, pix_off, cen_off, acc);
            else gram_rows_split<G, TSPLIT - 1>(pix, p.pitch, rows, cols, pg, q, pix_off, cen_off, acc);
        } else {
            if (TSPLIT == 1 || role == 0) gram_rows<G, 0>(pix, p.pitch, rows, cols, pg, q, pix_off, cen_off, acc);
            else gram_rows<G, TSPLIT - 1>(pix, p.pitch, rows, cols, pg, q, pix_off, cen_off, acc);
        }

        if (++since_flush >= p.flush_items || !more) {
            __syncthreads();                              // every wavefront is done with the tile
            gram_flush<G>(acc, lds, my_slot, pg, role, rmw);
            rmw = true;
            since_flush = 0;
        }
        if (FUSE && more) {
            // (the input tile is read between barriers only, by gram_tile_conv: no wavefront is still in it)
            const int64_t nx = item + 1;
            const int l = (int)(nx % p.Lp);
            if (l == 0) {
                gram_raw_load<KS>(p, nx / p.Lp, tiles, raw);
                __syncthreads();
            }
            int ny, nxx;
            tile_of(nx, ny, nxx);
            gram_tile_conv<KS>(p, raw, lds + (cur ^ 1) * p.buf_stride, l, ny, nxx, pw, dc[2 * cur], dc[2 * cur + 1],
                               dc + 2 * (cur ^ 1));
            __syncthreads();
        }
        if (!FUSE && more) {
            // DC shift of tile it+1 = estimate left by tile it (cells cur), new estimate into the other cells
            if constexpr (VEC)
                gram_tile_store_v<KS>(p, lds + (cur ^ 1) * p.buf_stride, pw, dc[2 * cur], dc[2 * cur + 1], va, vb,
                                      dc + 2 * (cur ^ 1));
            else
                gram_tile_store<KS>(p, lds + (cur ^ 1) * p.buf_stride, pw, dc[2 * cur], dc[2 * cur + 1], ra, rb,
                                    dc + 2 * (cur ^ 1));
            __syncthreads();
        }
        m_cur = m_nxt; ty_cur = ty_nxt; tx_cur = tx_nxt;
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

// Entry (r,c) of the stacked 2(D-1) x 2(D-1) Gram from its tile storage (upper block triangle).
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

// Entry (a,b) of the D x D block (view va, view vb) of sum y y^T, y = x - x_centre: the centre
// row and column are zero, the others come from the reduced stacked Gram.
__device__ inline double patch_block_entry(const double *st, int NB, int D, int va, int a, int vb, int b)
{
    const int cen = (D - 1) / 2;
    if (a == cen || b == cen) return 0.0;
    const int ra = va * (D - 1) + (a > cen ? a - 1 : a);
    const int rb = vb * (D - 1) + (b > cen ? b - 1 : b);
    return stacked_entry(st, NB, ra, rb);
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
                v = 0.5 * (patch_block_entry(st_main, NB, D, 0, a, 0, b) + patch_block_entry(st_main, NB, D, 0, b, 0, a)); break;
            case 1:
                v = 0.5 * (patch_block_entry(st_main, NB, D, 1, a, 1, b) + patch_block_entry(st_main, NB, D, 1, b, 1, a)); break;
            case 2: v = patch_block_entry(st_main, NB, D, 0, a, 1, b); break;
            case 3: v = patch_block_entry(st_cls, NB, D, 0, a, 1, b); break;
            default: v = patch_block_entry(st_tot, NB, D, 0, a, 1, b); break;
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

// Launch shape per patch size: wavefronts sharing a patch-row group, wavefronts per SIMD the
// register budget is set for, workgroups per compute unit.
struct GramShape { int tsplit, waves_per_eu; };
static GramShape gram_shape(int k)
{
    switch (k) {
        case 3: return {1, 4};
        case 5: return {1, 3};
        case 7: return {1, 2};
        default: return {2, 2};
    }
}

// one slot per resident workgroup
int max_gram_slots(ddcca_ctx *ctx, int k) { return ctx->n_cu * gram_shape(k).waves_per_eu; }

template <int KS, int TSPLIT, bool CROSS, int WPE, bool SPLIT, bool FUSE, bool VEC>
static int gram_launch(ddcca_ctx *ctx, const GramParams &p, int grid, size_t lds)
{
    static bool attr_set[MAX_DEVICES] = {};      // per device: the attribute is set on that device's code object
    if (!attr_set[ctx->device]) {
        DDCCA_HIP(ctx, hipFuncSetAttribute((const void *)patch_gram_kernel<KS, TSPLIT, CROSS, WPE, SPLIT, FUSE, VEC>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
        attr_set[ctx->device] = true;
    }
    hipLaunchKernelGGL((patch_gram_kernel<KS, TSPLIT, CROSS, WPE, SPLIT, FUSE, VEC>), dim3(grid), dim3(GRAM_THREADS), lds,
                       ctx->stream, p);
    DDCCA_HIP(ctx, hipGetLastError());
    return DDCCA_OK;
}

// LDS layout of a launch with column tiles of at most tw_max patches; returns the bytes.
static size_t gram_layout(GramParams &p, int k, int tw_max, bool split, bool fuse, bool vec)
{
    const int w4 = (p.w + 3) & ~3;
    // split wide images into equal column tiles of at most tw_max patches
    const int ntx = (w4 + tw_max - 1) / tw_max;
    p.tw = (((w4 + ntx - 1) / ntx) + 3) & ~3;
    p.tiles_x = (p.w + p.tw - 1) / p.tw;
    p.tiles_y = (p.h + GRAM_TH - 1) / GRAM_TH;
    const int r = (k - 1) / 2;
    // row pitch: >= tile width + halo, and congruent to k+3 mod 32 so that the window
    // rows a lane group touches fall into distinct LDS banks
    // (three-piece operands read whole groups of 32 patches: the pitch covers the rounded-up width)
    int pitch = (split ? (p.tw + 31) / 32 * 32 : p.tw) + 2 * r;
    // (tiles staged by chunks of four: the rows begin (4 - r % 4) % 4 columns early and end with a whole chunk)
    if (vec) pitch = std::max(pitch, (p.tw + 2 * r + (4 - r % 4) % 4 + 3) & ~3);
    while (pitch % 32 != (k + 3) % 32) ++pitch;
    p.pitch = pitch;
    p.view_stride = (GRAM_TH + 2 * r) * pitch + 16;      // +16: shift view 2 by half the banks
    p.buf_stride = 2 * p.view_stride;
    const int tsplit = gram_shape(k).tsplit;
    const size_t tile_floats = (size_t)2 * p.buf_stride;
    const size_t stage_floats = (size_t)((gram_tiles(k) + tsplit - 1) / tsplit) * 256;
    p.dc_off = (int)std::max(tile_floats, stage_floats);
    size_t floats = (size_t)p.dc_off + 4;
    p.raw_off = p.raw_pitch = p.raw_view_stride = 0;
    if (fuse) {
        // input tile under the map tile: 8-column runs, the last one read as whole float4s
        const int pw = p.tw + 2 * r, seg = (8 + 2 * r + 3) & ~3;
        p.raw_off = (int)floats;                                     // (a multiple of 4 floats)
        p.raw_pitch = 8 * ((pw + 7) / 8 - 1) + seg;
        p.raw_view_stride = (GRAM_TH + 4 * r) * p.raw_pitch;
        floats += (size_t)2 * p.raw_view_stride;
    }
    return floats * sizeof(float);
}

static int gram_run(ddcca_ctx *ctx, GramParams &p, int64_t n_maps, int k, bool cross_only, bool fuse, int max_slots,
                    int *slots_valid)
{
    const bool split = ctx->gram_arith == DDCCA_GRAM_BF16X3;
    const GramShape shape = gram_shape(k);
    // image rows on 16-byte boundaries: the tiles travel as aligned chunks of four pixels
    const bool vec = !fuse && (p.w & 3) == 0 && (((uintptr_t)p.v1 | (uintptr_t)p.v2) & 15) == 0;
    size_t lds = gram_layout(p, k, GRAM_TW_MAX, split, fuse, vec);
    // (with the input tiles next to the pixel buffers: narrower tiles until every resident workgroup fits)
    for (int tw_max = GRAM_TW_MAX - 32; fuse && tw_max >= 32 && lds * shape.waves_per_eu > LDS_BYTES_PER_CU;
         tw_max -= 32)
        lds = gram_layout(p, k, tw_max, split, fuse, vec);
    p.n_items = n_maps * p.tiles_x * p.tiles_y;
    const int npg = 4 / shape.tsplit;
    // about 16k patches between fp64 flushes per wavefront
    const int patches_per_group_item = (GRAM_TH / npg) * p.tw;
    p.flush_items = std::max(1, 16384 / patches_per_group_item);
    p.slots_valid = *slots_valid;
    // one workgroup per resident position: what the register budget allows per SIMD, unless the tiles of that
    // many workgroups do not fit a compute unit's LDS (k = 5 at the full tile width: three, not four) -- a grid
    // larger than what is resident would run its surplus as a second, thinly occupied round
    const int resident = std::min<int>(shape.waves_per_eu, (int)std::max<size_t>(1, LDS_BYTES_PER_CU / lds));
    const int max_grid = std::min(max_slots, ctx->n_cu * resident);
    const int grid = (int)std::min<int64_t>(max_grid, std::max<int64_t>(p.n_items, 1));
    int rc;
#define GRAM_VEC(KS, TS, CR, WPE, SP)                                                                  \
    (vec ? gram_launch<KS, TS, CR, WPE, SP, false, true>(ctx, p, grid, lds)                            \
         : gram_launch<KS, TS, CR, WPE, SP, false, false>(ctx, p, grid, lds))
#define GRAM_PICK(KS, TS, WPE, SP)                                                                     \
    (fuse ? gram_launch<KS, TS, false, WPE, SP, true, false>(ctx, p, grid, lds)                        \
          : cross_only ? GRAM_VEC(KS, TS, true, WPE, SP) : GRAM_VEC(KS, TS, false, WPE, SP))
#define GRAM_CASE(KS, TS, WPE)                                                                         \
    case KS: rc = split ? GRAM_PICK(KS, TS, WPE, true) : GRAM_PICK(KS, TS, WPE, false); break;
    switch (k) {
        GRAM_CASE(3, 1, 4)
        GRAM_CASE(5, 1, 3)
        GRAM_CASE(7, 1, 2)
        GRAM_CASE(9, 2, 2)
        default: return fail(ctx, DDCCA_EINVAL, "unsupported k");
    }
#undef GRAM_CASE
#undef GRAM_PICK
#undef GRAM_VEC
    if (rc) return rc;
    // slots below the old mark that this grid did not touch keep their data; new ones were initialised
    *slots_valid = std::max(*slots_valid, grid);
    return DDCCA_OK;
}

int launch_patch_gram(ddcca_ctx *ctx, const float *v1, const float *v2, int64_t n_maps, int h, int w, int k,
                      bool cross_only, double *slots, int max_slots, int *slots_valid)
{
    ProfScope prof(ctx, cross_only ? DDCCA_K_GRAM_CROSS : DDCCA_K_GRAM);
    GramParams p;
    p.v1 = v1; p.v2 = v2; p.h = h; p.w = w;
    p.Wp1 = p.Wp2 = nullptr; p.Lp = 0;
    p.slots = slots;
    return gram_run(ctx, p, n_maps, k, cross_only, false, max_slots, slots_valid);
}

int launch_patch_gram_recomputed(ddcca_ctx *ctx, const float *in1, const float *in2, int64_t n_inputs, int h, int w,
                                 int k, const float *Wp1, const float *Wp2, int L_prev, double *slots, int max_slots,
                                 int *slots_valid)
{
    ProfScope prof(ctx, DDCCA_K_GRAM);
    GramParams p;
    p.v1 = in1; p.v2 = in2; p.h = h; p.w = w;
    p.Wp1 = Wp1; p.Wp2 = Wp2; p.Lp = L_prev;
    p.slots = slots;
    return gram_run(ctx, p, n_inputs * L_prev, k, false, true, max_slots, slots_valid);
}

int launch_gram_reduce(ddcca_ctx *ctx, const double *slots, int n_slots, int k, double *stacked)
{
    return launch_reduce_slots(ctx, slots, n_slots, gram_tiles(k) * 256, stacked);
}

int launch_reduce_slots(ddcca_ctx *ctx, const double *slots, int n_slots, int E, double *stacked)
{
    ProfScope prof(ctx, DDCCA_K_REDUCE);
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
