// Stage convolution (Eq. 6) with every fp32 operand split into three bf16 pieces.
//
// x = h + m + l with h = bf16(x), m = bf16(x - h), l = bf16(x - h - m) (round to nearest even; both
// differences are exact in fp32), so the three pieces carry 24 significant bits.  A product of two such
// numbers is taken as the six piece products that matter,
//     x*y ~ h*h' + (h*m' + m*h') + m*m' + (h*l' + l*h'),
// the dropped ones (m*l', l*m', l*l') being below 2^-24 relative.  Each piece product is exact in fp32 and
// the products are summed in fp32 by v_mfma_f32_16x16x32_bf16, so the result has the accuracy of an fp32
// dot product while running on the bf16 matrix pipeline: 6 instructions of 16 cycles for 32 taps instead of
// 8 instructions of 32 cycles, and, unlike the fp32 matrix instructions, concurrently with the vector ALU.
//
// Implicit GEMM, as in the fp32 kernel: rows = (filter g, x-shift s), columns = 16 pixel positions
// x0 + 2c of one image row.  K runs over the taps (dy, dx'), dx' in 0..k (both shifts: k+1 columns, an even
// number), in row-major order, cut into groups of 8 = four pairs (dx', dx'+1), dx' even.  A pair is one
// 32-bit word of a tile stored as packed bf16 pairs, so a lane feeds the instruction from four words (a
// group may run over the end of a tap row into the next).  One instruction covers four groups (lane / 16):
// 1 / 1 / 2 / 3 instructions per piece product for k = 3 / 5 / 7 / 9.
#pragma once

#include "ddcca_internal.h"

namespace ddcca {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

union SplitOperand {
    bf16x8 v;
    unsigned int w[4];
};

template <int KS, int NBX, int TH>
struct SplitGeom {
    static constexpr int R = (KS - 1) / 2;
    static constexpr int KW = KS + 1;              // tap columns incl. the shift (even)
    static constexpr int PAIRS = KS * KW / 2;      // tap pairs
    static constexpr int KG = (PAIRS + 3) / 4;     // groups of four pairs
    static constexpr int STEPS = (KG + 3) / 4;     // matrix instructions per piece product
    static constexpr int TW = NBX * 32;
    static constexpr int PH = TH + 2 * R;
    static constexpr int COLS = (TW + KW + 6) / 4 * 4;   // staged pixels per tile row (row start a multiple of 4, <= 3 slack)
    static constexpr int V4 = COLS / 4;
    static constexpr int PWORDS = COLS / 2;        // packed pairs per tile row and plane
    static constexpr int PLANE = PH * PWORDS;      // words per plane
};

__device__ __forceinline__ unsigned bf16_bits(__bf16 b) { return (unsigned)__builtin_bit_cast(unsigned short, b); }

// The three bf16 pieces of x, as 16-bit patterns.
__device__ __forceinline__ void split3(float x, unsigned &h, unsigned &m, unsigned &l)
{
    const __bf16 bh = (__bf16)x;
    const float r1 = x - (float)bh;
    const __bf16 bm = (__bf16)r1;
    const float r2 = r1 - (float)bm;
    const __bf16 bl = (__bf16)r2;
    h = bf16_bits(bh);
    m = bf16_bits(bm);
    l = bf16_bits(bl);
}

// Store the pieces of the pixel pair (a, b) as word `idx` of the three planes.
__device__ __forceinline__ void split_store_pair(unsigned int *planes, int plane_words, int idx, float a, float b)
{
    unsigned ah, am, al, bh, bm, bl;
    split3(a, ah, am, al);
    split3(b, bh, bm, bl);
    planes[idx] = ah | (bh << 16);
    planes[plane_words + idx] = am | (bm << 16);
    planes[2 * plane_words + idx] = al | (bl << 16);
}

// A operand of lane (q, c): row `c` of the instruction is filter g, shift s; per step and piece the four tap
// pairs of group 4*step + q.  ROW_GS: row = 2*g' + s (pairs of x-shifts side by side, the order of the fp32
// convolution); otherwise row = 8*s + g'.
template <class G, int KS, bool ROW_GS>
__device__ __forceinline__ void split_weights(const float *W, int L, int g0, int q, int c, SplitOperand (&wa)[G::STEPS][3])
{
    const int g = g0 + (ROW_GS ? (c >> 1) : (c & 7)), s = ROW_GS ? (c & 1) : (c >> 3);
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int pair = 4 * (4 * t + q) + i;
            const int dy = (2 * pair) / G::KW, dx = 2 * pair - dy * G::KW;       // taps (dy, dx) and (dy, dx + 1)
            float v0 = 0.f, v1 = 0.f;
            if (pair < G::PAIRS && g < L) {
                if (dx - s >= 0 && dx - s < KS) v0 = W[(g * KS + dy) * KS + dx - s];
                if (dx + 1 - s >= 0 && dx + 1 - s < KS) v1 = W[(g * KS + dy) * KS + dx + 1 - s];
            }
            unsigned h0, m0, l0, h1, m1, l1;
            split3(v0, h0, m0, l0);
            split3(v1, h1, m1, l1);
            wa[t][0].w[i] = h0 | (h1 << 16);
            wa[t][1].w[i] = m0 | (m1 << 16);
            wa[t][2].w[i] = l0 | (l1 << 16);
        }
    }
}

// Word offsets (inside a plane, relative to the lane's pixel pair of tile row 0) of the four tap pairs of this
// lane's group, per step.
template <class G>
__device__ __forceinline__ void split_offsets(int q, int (&toff)[G::STEPS][4])
{
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int pair = 4 * (4 * t + q) + i;
            const int dy = (2 * pair) / G::KW, dx = 2 * pair - dy * G::KW;
            toff[t][i] = pair < G::PAIRS ? dy * G::PWORDS + dx / 2 : 0;
        }
}

// RU tile rows (rstride words apart), NBX column blocks, planes `plane` words apart: acc[u][b] = the 16 x 16 outputs of the instruction
// layout.  prow: word of the lane's first pixel pair (tile row of the first output row, plane of the h pieces).
template <class G, int NBX, int RU>
__device__ __forceinline__ void split_rows(const unsigned int *prow, int rstride, int plane, const int (&toff)[G::STEPS][4],
                                           const SplitOperand (&wa)[G::STEPS][3], floatx4 (&acc)[RU][NBX])
{
    constexpr bool CONTIG = G::KW % 8 == 0;       // a group never runs over the end of a tap row: 4 consecutive words
#pragma unroll
    for (int u = 0; u < RU; ++u)
#pragma unroll
        for (int b = 0; b < NBX; ++b) acc[u][b] = floatx4{0.f, 0.f, 0.f, 0.f};
    constexpr int CB = NBX >= 2 ? 2 : 1;          // column blocks whose pieces are held at a time
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
#pragma unroll
        for (int u = 0; u < RU; ++u) {
#pragma unroll
            for (int b0 = 0; b0 < NBX; b0 += CB) {
                // the pieces of CB column blocks first, then piece product by piece product across the blocks:
                // consecutive instructions belong to different accumulators
                SplitOperand ph[CB], pm[CB], pl[CB];
#pragma unroll
                for (int b = 0; b < CB; ++b) {
                    if (b0 + b >= NBX) continue;
                    const unsigned int *src = prow + u * rstride + (b0 + b) * 16;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int o = CONTIG ? toff[t][0] + i : toff[t][i];
                        ph[b].w[i] = src[o];
                        pm[b].w[i] = src[plane + o];
                        pl[b].w[i] = src[2 * plane + o];
                    }
                }
                // small terms first: (h,l') (l,h') (m,m') (h,m') (m,h') (h,h')
                constexpr int WP[6] = {0, 2, 1, 0, 1, 0};
#pragma unroll
                for (int pr = 0; pr < 6; ++pr)
#pragma unroll
                    for (int b = 0; b < CB; ++b) {
                        if (b0 + b >= NBX) continue;
                        const bf16x8 pix = pr == 0 ? pl[b].v : (pr == 2 || pr == 3) ? pm[b].v : ph[b].v;
                        acc[u][b0 + b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[t][WP[pr]].v, pix, acc[u][b0 + b], 0, 0, 0);
                    }
            }
        }
    }
}

}  // namespace ddcca
