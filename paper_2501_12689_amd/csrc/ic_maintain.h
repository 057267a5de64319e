// Store maintenance for the Example Manager (Sec. 4.3, "Capping Example Cache Size over Time"):
// utilities are refreshed and decayed (the paper applies a factor of 0.9 every hour), evicted
// examples are marked invalid, and a compaction squeezes the invalid rows out so that they stop
// costing bandwidth in every scan.
#pragma once
#include "ic_common.h"

namespace ic {

constexpr int kScanBlock = 1024;  // rows per block of the validity prefix sum

// util[ids[j]] = u[j]; ids outside [0, size) are ignored.
__global__ void set_utility(const int64_t *__restrict__ ids, const float *__restrict__ u, int64_t n,
                            float *__restrict__ util, int64_t size) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n) return;
    const int64_t id = ids[j];
    if (id >= 0 && id < size) util[id] = u[j];
}

// domain[ids[j]] = dom[j]; ids outside [0, size) are skipped; of duplicate ids any one wins
__global__ void set_domains(const int64_t *__restrict__ ids, const int32_t *__restrict__ dom, int64_t n,
                            int32_t *__restrict__ domain, int64_t size) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n) return;
    const int64_t id = ids[j];
    if (id >= 0 && id < size) domain[id] = dom[j];
}

// util[i] *= factor (one fp32 multiplication per row)
__global__ void scale_utility(float *__restrict__ util, int64_t size, float factor) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < size) util[i] = util[i] * factor;
}

__global__ void fill_bytes(uint8_t *__restrict__ p, int64_t n, uint8_t v) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// valid[ids[j]] = 0; ids outside [0, size) are ignored.
__global__ void invalidate_rows(const int64_t *__restrict__ ids, int64_t n, uint8_t *__restrict__ valid,
                                int64_t size) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= n) return;
    const int64_t id = ids[j];
    if (id >= 0 && id < size) valid[id] = 0;
}

// ---- compaction, step 1: new position of every surviving row (exclusive prefix sum of valid)

// block_sums[b] = valid rows in block b
__global__ __launch_bounds__(256) void count_valid(const uint8_t *__restrict__ valid, int64_t size,
                                                   int64_t *__restrict__ block_sums) {
    __shared__ int part[4];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock;
    int c = 0;
    for (int t = threadIdx.x; t < kScanBlock; t += 256) {
        const int64_t i = base + t;
        c += (i < size && valid[i] != 0) ? 1 : 0;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) c += __shfl_xor(c, m, kWave);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) block_sums[blockIdx.x] = (int64_t)part[0] + part[1] + part[2] + part[3];
}

// in place: block_sums[b] -> number of valid rows before block b; block_sums[nblocks] = total.
// One workgroup; the block count is at most a few million, handled in strides of 256.
__global__ __launch_bounds__(256) void scan_block_sums(int64_t *__restrict__ block_sums, int64_t nblocks) {
    __shared__ int64_t tile[256];
    __shared__ int64_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t lo = 0; lo < nblocks; lo += 256) {
        const int64_t i = lo + threadIdx.x;
        const int64_t v = i < nblocks ? block_sums[i] : 0;
        tile[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {  // inclusive scan of the tile
            const int64_t add = (int)threadIdx.x >= off ? tile[threadIdx.x - off] : 0;
            __syncthreads();
            tile[threadIdx.x] += add;
            __syncthreads();
        }
        if (i < nblocks) block_sums[i] = carry + tile[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 0) carry += tile[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) block_sums[nblocks] = carry;
}

// id_map[i] = new id of row i, or -1 if the row is dropped
__global__ __launch_bounds__(256) void write_id_map(const uint8_t *__restrict__ valid, int64_t size,
                                                    const int64_t *__restrict__ block_offsets,
                                                    int64_t *__restrict__ id_map) {
    __shared__ int wave_tot[4];
    const int64_t base = (int64_t)blockIdx.x * kScanBlock;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    int64_t running = block_offsets[blockIdx.x];
    for (int t0 = 0; t0 < kScanBlock; t0 += 256) {  // four passes of 256 consecutive rows
        const int64_t i = base + t0 + threadIdx.x;
        const int v = (i < size && valid[i] != 0) ? 1 : 0;
        const uint64_t bal = __ballot(v);
        const int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_tot[w] = __popcll(bal);
        __syncthreads();
        int wbase = 0;
        for (int x = 0; x < w; ++x) wbase += wave_tot[x];
        const int pass_total = wave_tot[0] + wave_tot[1] + wave_tot[2] + wave_tot[3];
        if (i < size) id_map[i] = v ? running + wbase + before : (int64_t)-1;
        running += pass_total;
        __syncthreads();
    }
}

// every stride-th block offset, for the host's plan of the moves (one small copy)
__global__ void pick_offsets(const int64_t *__restrict__ block_offsets, int64_t stride, int count,
                             int64_t *__restrict__ out) {
    const int i = threadIdx.x;
    if (i < count) out[i] = block_offsets[(int64_t)i * stride];
}

// ---- compaction, step 2: move the surviving rows of one chunk [lo, hi) of the store (lo a
// multiple of kScanBlock; hi too, or hi = size).  Chunks are processed in order, one pair of
// launches each.  Once at least a chunk's worth of rows has been dropped before the chunk, its
// destination lies entirely before lo, where every row has already been moved: gather_rows
// writes the rows straight to their final place and store_rows does nothing.  Until then the
// destination overlaps the chunk's own unread rows, so gather_rows packs them into a bounce
// buffer and store_rows copies the packed rows to their place afterwards.
__device__ __forceinline__ bool chunk_moves_directly(int64_t lo, int64_t hi, int64_t first_new) {
    return lo - first_new >= hi - lo;
}
// If the index keeps a step-major copy (panel != NULL) a moved row is written to its new place there as
// well (by gather_rows when the chunk moves directly, by store_rows otherwise): the copy is a different
// buffer, so it has no overlap to mind, and nothing has to be read twice to rebuild it.
__global__ __launch_bounds__(256) void gather_rows(const uint8_t *rows, int row_bytes,
                                                   const int64_t *__restrict__ id_map,
                                                   const int64_t *__restrict__ block_offsets, int64_t lo,
                                                   int64_t hi, uint8_t *bounce, uint8_t *panel) {
    const int64_t first_new = block_offsets[lo / kScanBlock];
    const bool direct = chunk_moves_directly(lo, hi, first_new);
    uint8_t *out = direct ? const_cast<uint8_t *>(rows) + first_new * (int64_t)row_bytes : bounce;
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t r = lo + wave; r < hi; r += nwaves) {
        const int64_t to = id_map[r];
        if (to < 0) continue;
        const i32x4 *src = reinterpret_cast<const i32x4 *>(rows + r * (int64_t)row_bytes);
        i32x4 *dst = reinterpret_cast<i32x4 *>(out + (to - first_new) * (int64_t)row_bytes);
        for (int c = lane; c < row_bytes / 16; c += 64) {
            const i32x4 g = src[c];
            dst[c] = g;
            if (direct && panel) *reinterpret_cast<i32x4 *>(panel + panel_word_offset(to, c * 4, row_bytes)) = g;
        }
    }
}

__global__ __launch_bounds__(256) void store_rows(uint8_t *__restrict__ rows, int row_bytes,
                                                  const int64_t *__restrict__ block_offsets, int64_t lo,
                                                  int64_t hi, int64_t hi_block,
                                                  const uint8_t *__restrict__ bounce, uint8_t *__restrict__ panel) {
    const int64_t first_new = block_offsets[lo / kScanBlock];
    if (chunk_moves_directly(lo, hi, first_new)) return;
    const int64_t count = block_offsets[hi_block] - first_new;
    const int per_row = row_bytes / 16;
    const int64_t vecs = count * (int64_t)per_row;
    const i32x4 *src = reinterpret_cast<const i32x4 *>(bounce);
    i32x4 *dst = reinterpret_cast<i32x4 *>(rows + first_new * (int64_t)row_bytes);
    for (int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x; v < vecs; v += (int64_t)gridDim.x * 256) {
        const i32x4 g = src[v];
        dst[v] = g;
        if (panel) {
            const int64_t row = first_new + v / per_row;
            *reinterpret_cast<i32x4 *>(panel + panel_word_offset(row, (int)(v % per_row) * 4, row_bytes)) = g;
        }
    }
}

// per-row fp32 side arrays (utility, fp8 scale): scatter into a scratch array, then copy back
__global__ void scatter_f32(const float *__restrict__ src, const int64_t *__restrict__ id_map, int64_t size,
                            float *__restrict__ tmp) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < size && id_map[i] >= 0) tmp[id_map[i]] = src[i];
}
__global__ void copy_f32_counted(const float *__restrict__ tmp, const int64_t *__restrict__ total,
                                 float *__restrict__ dst) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < *total) dst[i] = tmp[i];
}

}  // namespace ic
