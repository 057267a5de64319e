// Shared device helpers: vector types, the totally ordered 64-bit (score, id)
// key, and wave reductions.  gfx950 only (64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ic {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(2))) long i64x2;

constexpr int kWave = 64;

// ---------------------------------------------------------------------------
// Selection key.  The result order is (score descending, id ascending); both
// are folded into one unsigned 64-bit key so that "better" is "greater":
//   high 32 bits: the fp32 score mapped monotonically onto unsigned integers
//                 (-0 is first turned into +0 so that equal scores share bits)
//   low  32 bits: 0xFFFFFFFF - id
// Keys are unique per example.  kKeyFloor is the largest key a score of -inf
// can produce; invalid rows get score -inf and therefore never beat it, and
// any key <= kKeyFloor means "no example".
// ---------------------------------------------------------------------------
constexpr uint64_t kKeyFloor = 0x007FFFFFFFFFFFFFull;

__device__ __forceinline__ uint32_t ord_of_score(float s) {
    uint32_t b = (s == 0.0f) ? 0u : __float_as_uint(s);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float score_of_ord(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}
__device__ __forceinline__ uint64_t make_key(float s, uint32_t id) {
    return ((uint64_t)ord_of_score(s) << 32) | (uint64_t)(0xFFFFFFFFu - id);
}
__device__ __forceinline__ float key_score(uint64_t key) { return score_of_ord((uint32_t)(key >> 32)); }
// Starting threshold of a query whose pilot found fewer than k rows with a score: a score below every
// real one (cosines lie in [-1, 1] and lambda * utility is taken to stay above -1e30) and above -inf, the
// score of masked, evicted and invisible rows.  Every row with a score passes it, no row without one does,
// so a mask that leaves a handful of rows leaves the scans' candidate lists nearly empty instead of full.
constexpr float kNoThresholdScore = -1e30f;
__device__ __forceinline__ uint32_t key_id(uint64_t key) { return 0xFFFFFFFFu - (uint32_t)key; }

// ---------------------------------------------------------------------------
// Step-major copy ("panel") of an array of rows, the layout the tiled scan reads: tile t = 256 rows
// is stored as row_bytes / 64 steps of 16 KB, step s holding bytes [64 s, 64 s + 64) of the tile's
// rows, 64 B per row, with granule g (16 bytes) of row r at position g ^ ((r / 4) % 4), which is the
// image the scan keeps of the step in LDS.  Byte offset of 32-bit word `word` of row `row`:
// ---------------------------------------------------------------------------
constexpr int kPanelRows = 256;
constexpr int kPanelStepBytes = 64;
__host__ __device__ __forceinline__ int64_t panel_word_offset(int64_t row, int word, int row_bytes) {
    const int r = (int)(row & (kPanelRows - 1));
    const int s = word >> 4, g = (word >> 2) & 3;
    return (row >> 8) * ((int64_t)kPanelRows * row_bytes) + ((int64_t)s * kPanelRows + r) * kPanelStepBytes +
           ((g ^ ((r >> 2) & 3)) << 4) + ((word & 3) << 2);
}

// Butterfly reductions: after the loop every lane holds the same bits, because
// each step combines the two partners' values with a commutative operation.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, kWave));
    return v;
}

}  // namespace ic
