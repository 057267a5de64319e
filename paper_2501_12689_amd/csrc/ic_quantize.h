// Row preparation: unit-normalise fp32 rows and write them in a store format.
// Used for cache rows on append (IC-Cache workflow step 4 / update_cache) and
// for the query block of every search (the embedding handed to
// GetSimilarExamples, Algorithm 1).
#pragma once
#include "ic_common.h"

namespace ic {

// bfloat16 bits of f, round to nearest, ties to even (finite inputs).
__device__ __forceinline__ uint32_t bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// OCP FP8 E4M3 code of t: nearest representable value, ties to even mantissa,
// magnitudes above 448 clamp to 448.  Works on the value: scale the magnitude so
// that one unit is the spacing of the target binade and round to an integer.
__device__ __forceinline__ uint32_t e4m3_bits(float t) {
    const uint32_t sign = (__float_as_uint(t) >> 24) & 0x80u;
    const float a = fabsf(t);
    if (!(a < 448.0f)) return sign | 0x7Eu;
    if (a < 0.015625f)                       // below 2^-6: fixed spacing 2^-9
        return sign | (uint32_t)rintf(a * 512.0f);
    int e;
    (void)frexpf(a, &e);                     // a = m * 2^e, m in [0.5, 1)
    int E = e - 1;                           // a in [2^E, 2^(E+1)), -6 <= E <= 8
    float r = rintf(ldexpf(a, 3 - E));       // in [8, 16]
    if (r == 16.0f) { r = 8.0f; E += 1; }
    return sign | ((uint32_t)(E + 7) << 3) | ((uint32_t)r - 8u);
}

// One wavefront per row.  X is [n_src, d] fp32; rows [n_src, n_total) of the
// destination are written as zeros (padding of the query block).  Row i goes to
// dst + i * row_bytes; columns [d, row_bytes / elem) are zero.  fp8 also writes
// scale_dst[i].  util_src may be NULL (utility 0); util_dst may be NULL.  If panel is not NULL
// every row is also written into the step-major copy the tiled scan reads, as its row
// panel_first + i (layout: panel_word_offset in ic_common.h).
//
// Arithmetic: the norm is accumulated in fp64, x / norm is formed in fp64 and
// rounded once to fp32, and that fp32 value is what gets quantised.  fp8:
// scale = fp32(max|unit| / 448) (1 for a zero row), code = e4m3(fp32(unit / scale))
// with the quotient in fp64.
template <int ET>  // 0 = bf16, 1 = fp8 e4m3
__global__ __launch_bounds__(256) void quantize_rows(const float *__restrict__ X, int64_t n_src,
                                                     int64_t n_total, int d, int row_bytes,
                                                     uint8_t *__restrict__ dst,
                                                     float *__restrict__ scale_dst,
                                                     const float *__restrict__ util_src,
                                                     float *__restrict__ util_dst,
                                                     uint8_t *__restrict__ panel, int64_t panel_first) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    constexpr int G = (ET == 0) ? 2 : 4;      // elements per 32-bit store
    const int groups = row_bytes / 4;         // 32-bit words per destination row

    for (int64_t i = wave; i < n_total; i += nwaves) {
        uint32_t *out = reinterpret_cast<uint32_t *>(dst + i * (int64_t)row_bytes);
        if (i >= n_src) {
            for (int w = lane; w < groups; w += 64) {
                out[w] = 0u;
                if (panel) *reinterpret_cast<uint32_t *>(panel + panel_word_offset(panel_first + i, w, row_bytes)) = 0u;
            }
            if (ET == 1 && lane == 0) scale_dst[i] = 1.0f;
            continue;
        }
        const float *x = X + i * (int64_t)d;
        double ss = 0.0;
        for (int j = lane; j < d; j += 64) {
            double v = (double)x[j];
            ss += v * v;
        }
        const double nrm = sqrt(wave_sum(ss));
        const bool live = nrm > 0.0;

        float sc = 1.0f;
        if (ET == 1) {
            float amax = 0.0f;
            if (live)
                for (int j = lane; j < d; j += 64) amax = fmaxf(amax, fabsf((float)((double)x[j] / nrm)));
            amax = wave_max(amax);
            if (amax > 0.0f) sc = (float)((double)amax / 448.0);
            if (lane == 0) scale_dst[i] = sc;
        }
        for (int w = lane; w < groups; w += 64) {
            uint32_t word = 0u;
#pragma unroll
            for (int g = 0; g < G; ++g) {
                const int j = w * G + g;
                float unit = 0.0f;
                if (j < d && live) unit = (float)((double)x[j] / nrm);
                if (ET == 0) {
                    word |= bf16_bits(unit) << (16 * g);
                } else {
                    const float t = (float)((double)unit / (double)sc);
                    word |= e4m3_bits(t) << (8 * g);
                }
            }
            out[w] = word;
            if (panel) *reinterpret_cast<uint32_t *>(panel + panel_word_offset(panel_first + i, w, row_bytes)) = word;
        }
        if (util_dst && lane == 0) util_dst[i] = util_src ? util_src[i] : 0.0f;
    }
}

}  // namespace ic
