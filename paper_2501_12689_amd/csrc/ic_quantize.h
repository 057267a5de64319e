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

// fp32(x / div), the fp64 quotient rounded once more to fp32, without dividing wherever that provably
// changes nothing.  inv = 1 / div (correctly rounded), so q = x * inv lies within 2^-52 (relative) of
// the true quotient and the correctly rounded fp64 quotient within 2^-53 of it: both lie between
// q (1 - 2^-50) and q (1 + 2^-50).  Rounding to fp32 is monotonic, so when the two ends round to the same
// fp32 value that value is fp32(fp64(x / div)).  Otherwise (a quotient within 2^-49 of a rounding
// boundary of fp32: about 3 elements in 10^8) `doubt` is set and the caller divides.
__device__ __forceinline__ float quotient_f32(double x, double inv, bool &doubt) {
    const double q = x * inv;
    const float lo = (float)(q * (1.0 - 0x1p-50)), hi = (float)(q * (1.0 + 0x1p-50));
    doubt |= lo != hi;
    return lo;
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
//
// A lane owns columns 256 t + 4 lane + {0, 1, 2, 3}, t < NT (NT = steps of 256 columns that a
// destination row has, at most 8), and keeps them in registers: the row is read once, 16 bytes per lane
// and a contiguous kilobyte per wavefront and instruction, all loads issued before the first is used.
// The squares are added in that order per lane (columns past d count as zeros), then across lanes by
// wave_sum, whatever the alignment of X, so a row's norm does not depend on how it was handed over.
// The quotients are formed by quotient_f32; a row in which any lane is in doubt about any column (rare)
// is done again with the divisions themselves, from the row as reloaded.
constexpr int kQuantSteps = 8;   // 256 columns each: d <= 2048

template <int ET, int NT>  // ET: 0 = bf16, 1 = fp8 e4m3
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
    const int groups = row_bytes / 4;         // 32-bit words per destination row
    const int row_elems = (ET == 0) ? row_bytes / 2 : row_bytes;   // columns of a destination row (a multiple of 64)
    // 16-byte loads need d % 4 == 0 and an aligned X (then every row starts aligned)
    const bool vec = (d % 4 == 0) && ((reinterpret_cast<uintptr_t>(X) & 15u) == 0);

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
        auto load_row = [&](f32x4 (&v)[NT]) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                v[t] = f32x4{0.f, 0.f, 0.f, 0.f};
                const int j = 256 * t + 4 * lane;
                if (j < d) {
                    if (vec) {
                        v[t] = *reinterpret_cast<const f32x4 *>(x + j);
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (j + c < d) v[t][c] = x[j + c];
                    }
                }
            }
        };
        f32x4 v[NT];
        load_row(v);
        double ss = 0.0;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const double e = (double)v[t][c];
                ss += e * e;
            }
        const double nrm = sqrt(wave_sum(ss));
        const bool live = nrm > 0.0;
        const double inv_nrm = live ? 1.0 / nrm : 0.0;

        // unit values (columns past d, and every column of a zero row, are zeros)
        bool doubt = false;
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int c = 0; c < 4; ++c) v[t][c] = quotient_f32((double)v[t][c], inv_nrm, doubt);
        if (__builtin_amdgcn_ballot_w64(doubt) != 0ull) {
            load_row(v);
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int c = 0; c < 4; ++c) v[t][c] = live ? (float)((double)v[t][c] / nrm) : 0.0f;
        }
        float sc = 1.0f;
        if (ET == 1) {
            float amax = 0.0f;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int c = 0; c < 4; ++c) amax = fmaxf(amax, fabsf(v[t][c]));
            amax = wave_max(amax);
            if (amax > 0.0f) sc = (float)((double)amax / 448.0);
            if (lane == 0) scale_dst[i] = sc;
        }
        if (ET == 0) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (256 * t + 4 * lane < row_elems) {
                    // two 32-bit words of two bf16 each: words 128 t + 2 lane and the next, in one granule
                    const int w = 128 * t + 2 * lane;
                    uint2 word;
                    word.x = bf16_bits(v[t][0]) | (bf16_bits(v[t][1]) << 16);
                    word.y = bf16_bits(v[t][2]) | (bf16_bits(v[t][3]) << 16);
                    *reinterpret_cast<uint2 *>(out + w) = word;
                    if (panel) *reinterpret_cast<uint2 *>(panel + panel_word_offset(panel_first + i, w, row_bytes)) = word;
                }
            }
        } else {
            const double scd = (double)sc, inv_sc = 1.0 / scd;
            f32x4 tq[NT];
            bool doubt2 = false;
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int c = 0; c < 4; ++c) tq[t][c] = quotient_f32((double)v[t][c], inv_sc, doubt2);
            if (__builtin_amdgcn_ballot_w64(doubt2) != 0ull) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int c = 0; c < 4; ++c) tq[t][c] = (float)((double)v[t][c] / scd);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (256 * t + 4 * lane < row_elems) {
                    const int w = 64 * t + lane;
                    uint32_t word = 0u;
#pragma unroll
                    for (int c = 0; c < 4; ++c) word |= e4m3_bits(tq[t][c]) << (8 * c);
                    out[w] = word;
                    if (panel) *reinterpret_cast<uint32_t *>(panel + panel_word_offset(panel_first + i, w, row_bytes)) = word;
                }
            }
        }
        if (util_dst && lane == 0) util_dst[i] = util_src ? util_src[i] : 0.0f;
    }
}

// Host side: the instance for a destination row of row_bytes bytes (NT = steps of 256 columns).
template <int ET, int NT>
inline void launch_quantize_rows_nt(unsigned grid, hipStream_t st, const float *X, int64_t n_src, int64_t n_total, int d,
                                    int row_bytes, uint8_t *dst, float *scale_dst, const float *util_src, float *util_dst,
                                    uint8_t *panel, int64_t panel_first) {
    hipLaunchKernelGGL((quantize_rows<ET, NT>), dim3(grid), dim3(256), 0, st, X, n_src, n_total, d, row_bytes, dst, scale_dst,
                       util_src, util_dst, panel, panel_first);
}

inline void launch_quantize_rows(int et, unsigned grid, hipStream_t st, const float *X, int64_t n_src, int64_t n_total, int d,
                                 int row_bytes, uint8_t *dst, float *scale_dst, const float *util_src, float *util_dst,
                                 uint8_t *panel, int64_t panel_first) {
    const int row_elems = et == 0 ? row_bytes / 2 : row_bytes;
    const int nt = (row_elems + 255) / 256;   // 1 .. 4 for bf16 (d <= 1024), 1 .. 8 for fp8 (d <= 2048)
#define IC_QUANT_CASE(ET, NT)                                                                                          \
    case NT:                                                                                                           \
        launch_quantize_rows_nt<ET, NT>(grid, st, X, n_src, n_total, d, row_bytes, dst, scale_dst, util_src, util_dst, \
                                        panel, panel_first);                                                           \
        break;
    if (et == 0) {
        switch (nt) {
            IC_QUANT_CASE(0, 1) IC_QUANT_CASE(0, 2) IC_QUANT_CASE(0, 3) IC_QUANT_CASE(0, 4)
            default: break;   // longer rows are refused when the index is created
        }
    } else {
        switch (nt) {
            IC_QUANT_CASE(1, 1) IC_QUANT_CASE(1, 2) IC_QUANT_CASE(1, 3) IC_QUANT_CASE(1, 4)
            IC_QUANT_CASE(1, 5) IC_QUANT_CASE(1, 6) IC_QUANT_CASE(1, 7) IC_QUANT_CASE(1, 8)
            default: break;
        }
    }
#undef IC_QUANT_CASE
}

}  // namespace ic
