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
// x0 + 2c of one image row.  K runs over groups of 8 consecutive tap columns of one tap row:
//   group kg = dy * CH + j  ->  taps (dy, dx' = 8j .. 8j+7),  dx' in 0..k (both shifts),  CH = ceil((k+1)/8)
// so that the 8 K-values a lane feeds to the instruction are 8 consecutive pixels of one tile row, i.e. four
// 32-bit words of a tile stored as packed bf16 pairs.  One instruction covers four groups (lane / 16).
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
    static constexpr int KW = KS + 1;              // tap columns incl. the shift
    static constexpr int CH = (KW + 7) / 8;        // groups of 8 tap columns per tap row
    static constexpr int KG = KS * CH;             // groups
    static constexpr int STEPS = (KG + 3) / 4;     // matrix instructions per piece product
    static constexpr int TW = NBX * 32;
    static constexpr int PH = TH + 2 * R;
    static constexpr int COLS = TW + 8 * CH + 4;   // staged pixels per tile row (row start a multiple of 4, <= 3 slack)
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

// A operand of lane (q, c): row `c` of the instruction is filter g, shift s; per step and piece the 8 taps
// of group 4*step + q.  ROW_GS: row = 2*g' + s (pairs of x-shifts side by side, the order of the fp32
// convolution); otherwise row = 8*s + g'.
template <class G, int KS, bool ROW_GS>
__device__ __forceinline__ void split_weights(const float *W, int L, int g0, int q, int c, SplitOperand (&wa)[G::STEPS][3])
{
    const int g = g0 + (ROW_GS ? (c >> 1) : (c & 7)), s = ROW_GS ? (c & 1) : (c >> 3);
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
        const int kg = 4 * t + q;
        const int dy = kg / G::CH, j = kg - dy * G::CH;
        unsigned hh[8], mm[8], ll[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int dxw = 8 * j + i - s;
            float v = 0.f;
            if (kg < G::KG && dxw >= 0 && dxw < KS && g < L) v = W[(g * KS + dy) * KS + dxw];
            split3(v, hh[i], mm[i], ll[i]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            wa[t][0].w[i] = hh[2 * i] | (hh[2 * i + 1] << 16);
            wa[t][1].w[i] = mm[2 * i] | (mm[2 * i + 1] << 16);
            wa[t][2].w[i] = ll[2 * i] | (ll[2 * i + 1] << 16);
        }
    }
}

// Word offsets (inside a plane, relative to the lane's pixel pair of tile row 0) of this lane's group per step.
template <class G>
__device__ __forceinline__ void split_offsets(int q, int (&toff)[G::STEPS])
{
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
        const int kg = 4 * t + q;
        const int dy = kg / G::CH, j = kg - dy * G::CH;
        toff[t] = kg < G::KG ? dy * G::PWORDS + 4 * j : 0;
    }
}

// RU tile rows (RSTRIDE words apart), NBX column blocks: acc[u][b] = the 16 x 16 outputs of the instruction
// layout.  prow: word of the lane's first pixel pair (tile row of the first output row, plane of the h pieces).
template <class G, int NBX, int RU, int RSTRIDE>
__device__ __forceinline__ void split_rows(const unsigned int *prow, const int (&toff)[G::STEPS],
                                           const SplitOperand (&wa)[G::STEPS][3], floatx4 (&acc)[RU][NBX])
{
#pragma unroll
    for (int u = 0; u < RU; ++u)
#pragma unroll
        for (int b = 0; b < NBX; ++b) acc[u][b] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int t = 0; t < G::STEPS; ++t) {
        const unsigned int *pk = prow + toff[t];
#pragma unroll
        for (int u = 0; u < RU; ++u) {
            // the pieces of all column blocks first, then piece product by piece product across the blocks:
            // consecutive instructions belong to different accumulators
            SplitOperand ph[NBX], pm[NBX], pl[NBX];
#pragma unroll
            for (int b = 0; b < NBX; ++b) {
                const unsigned int *src = pk + u * RSTRIDE + b * 16;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ph[b].w[i] = src[i];
                    pm[b].w[i] = src[G::PLANE + i];
                    pl[b].w[i] = src[2 * G::PLANE + i];
                }
            }
            // small terms first
#pragma unroll
            for (int b = 0; b < NBX; ++b)
                acc[u][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[t][0].v, pl[b].v, acc[u][b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NBX; ++b)
                acc[u][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[t][2].v, ph[b].v, acc[u][b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NBX; ++b)
                acc[u][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[t][1].v, pm[b].v, acc[u][b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NBX; ++b)
                acc[u][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[t][0].v, pm[b].v, acc[u][b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NBX; ++b)
                acc[u][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[t][1].v, ph[b].v, acc[u][b], 0, 0, 0);
#pragma unroll
            for (int b = 0; b < NBX; ++b)
                acc[u][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[t][0].v, ph[b].v, acc[u][b], 0, 0, 0);
        }
    }
}

}  // namespace ddcca
