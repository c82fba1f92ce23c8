// Device helpers shared by the output-layer kernels (hashing + block histograms, Eq. 7-12).
#pragma once

#include "ddcca_internal.h"

#include <hip/hip_fp16.h>

namespace ddcca {

constexpr int IQ_LUT_MAX = 2048;   // information-quality table entries (counts 0..2047); larger counts are computed directly

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

template <int OUT> struct HistOut;
template <> struct HistOut<DDCCA_FEAT_COUNT_U16> { typedef uint16_t type; };
template <> struct HistOut<DDCCA_FEAT_IQ_F32> { typedef float type; };
template <> struct HistOut<DDCCA_FEAT_IQ_F16> { typedef __half type; };

__device__ __forceinline__ float iq_value(unsigned c, const float *lut, int lut_n, double log_total)
{
    return (int)c < lut_n ? lut[c] : (float)(log_total - log((double)(c + 1u)));
}

template <int OUT> __device__ __forceinline__ typename HistOut<OUT>::type hist_convert(unsigned c, const float *lut,
                                                                                      int lut_n, double log_total);
template <> __device__ __forceinline__ uint16_t hist_convert<DDCCA_FEAT_COUNT_U16>(unsigned c, const float *, int,
                                                                                   double)
{
    return (uint16_t)c;
}
template <> __device__ __forceinline__ float hist_convert<DDCCA_FEAT_IQ_F32>(unsigned c, const float *lut, int lut_n,
                                                                             double log_total)
{
    return iq_value(c, lut, lut_n, log_total);
}
template <> __device__ __forceinline__ __half hist_convert<DDCCA_FEAT_IQ_F16>(unsigned c, const float *lut, int lut_n,
                                                                              double log_total)
{
    return __float2half_rn(iq_value(c, lut, lut_n, log_total));
}

}  // namespace ddcca
