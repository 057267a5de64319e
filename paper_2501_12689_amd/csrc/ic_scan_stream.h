// Streaming scan: similarity of a block of up to 64 queries with every cached
// row, fused with the per-slice partial top-k.  This is the O(N) step of
// IC-Cache's stage-1 relevance selection (Sec. 4.1; GetSimilarExamples in
// Algorithm 1) for small query batches, where the work is bound by reading the
// store from HBM once.
//
// Shape of the computation
//   * A workgroup (4 wavefronts) owns slice s of the cache: the 16-row tiles
//     s, s+S, s+2S, ...  and one block of QG*16 queries.
//   * The embedding dimension is split over the 4 wavefronts: wavefront w owns
//     CPW consecutive 64-byte chunks of every row.  Its share of the query block
//     stays in registers for the whole kernel (QG*CPW 16-byte fragments), and
//     its share of each row tile goes from global memory straight into the MFMA
//     operand registers: lane (r = lane%16, c = lane/16) reads 16 bytes of row
//     r at chunk offset 16*c, which is exactly the A-operand layout of
//     v_mfma_f32_16x16x32 (row r, 8 consecutive k).  Queries use the same byte
//     mapping for the B operand, so every product pairs equal coordinates.
//   * The 4 partial 16x16 score tiles are exchanged through LDS and summed in a
//     fixed order by wavefront g < QG, which owns query group g from then on:
//     score = dot * scales + lambda * utility, -inf for invalid rows.
//   * Selection: each query has a candidate region of `cap` keys in global
//     memory (private to this workgroup) and a threshold key in LDS.  A score
//     that beats the threshold is appended; when the region is full the owning
//     wavefront ranks its keys, keeps the best k (sorted) and raises the
//     threshold to the k-th.  Only candidates that beat the k-th best so far are
//     ever written, so the score matrix never leaves registers.
//   * At the end the region sizes are written out; a merge kernel combines the
//     S regions of every query.
#pragma once
#include "ic_common.h"

namespace ic {

struct ScanArgs {
    const uint8_t *store;    // [n] rows, row_bytes apart
    int64_t n;               // rows in the index
    int row_bytes;           // multiple of 128
    const float *row_scale;  // [n] (fp8) or NULL
    const float *util;       // [>= round_up(n,4)] or NULL when lambda == 0
    const uint8_t *mask;     // [n] or NULL
    float lambda;
    const uint8_t *qbuf;     // prepared queries, [gridDim.y * QG*16] rows, row_bytes apart
    const float *q_scale;    // per prepared query (fp8) or NULL
    int Q;                   // real queries in qbuf
    int k;
    int cap;                 // region capacity: multiple of 64, k < cap <= 256
    int S;                   // slices == gridDim.x
    uint64_t *regions;       // [Q][S][cap] keys
    int32_t *counts;         // [Q][S] keys in use
};

constexpr int kScanWaves = 4;
constexpr int kMaxCap = 256;

// Keep the best k of a full region (sorted, best first) and publish the new
// threshold.  Runs on one whole wavefront; `scr` is that wavefront's LDS
// scratch of kMaxCap keys.  Keys are unique, so rank = number of greater keys
// is a permutation.
__device__ __forceinline__ void compact_region(uint64_t *region, int c, int k, uint64_t *scr,
                                               uint64_t *thr_slot, uint32_t *cnt_slot, int lane) {
    uint64_t mine[kMaxCap / 64];
#pragma unroll
    for (int t = 0; t < kMaxCap / 64; ++t) {
        const int idx = lane + 64 * t;
        mine[t] = 0;
        if (idx < c) {
            mine[t] = __hip_atomic_load(region + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            scr[idx] = mine[t];
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    int rank[kMaxCap / 64];
#pragma unroll
    for (int t = 0; t < kMaxCap / 64; ++t) rank[t] = 0;
    for (int i = 0; i < c; ++i) {
        const uint64_t other = scr[i];
#pragma unroll
        for (int t = 0; t < kMaxCap / 64; ++t) rank[t] += (other > mine[t]) ? 1 : 0;
    }
#pragma unroll
    for (int t = 0; t < kMaxCap / 64; ++t) {
        const int idx = lane + 64 * t;
        if (idx < c && rank[t] < k) {
            region[rank[t]] = mine[t];
            if (rank[t] == k - 1) *thr_slot = mine[t];
        }
    }
    if (lane == 0) *cnt_slot = (uint32_t)(c < k ? c : k);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <int ET, int QG, int CPW>
__global__ __launch_bounds__(256) void scan_stream(const ScanArgs a) {
    constexpr int QB = QG * 16;
    __shared__ f32x4 part[2][kScanWaves][QG][64];
    __shared__ uint64_t thr_key[QB];
    __shared__ uint32_t cnt[QB];
    __shared__ uint64_t scratch[kScanWaves][kMaxCap];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int r16 = lane & 15;  // row within tile (A operand) / query within group (B, D)
    const int c4 = lane >> 4;   // 16-byte column within a 64-byte chunk; D rows 4*c4 .. 4*c4+3
    const int s = blockIdx.x;
    const int qb = blockIdx.y;
    const int nchunks = a.row_bytes >> 6;
    const int chunk0 = w * CPW;

    if (tid < QB) {
        thr_key[tid] = kKeyFloor;
        cnt[tid] = 0u;
    }

    // query fragments owned by this wavefront, resident for the whole kernel
    i32x4 qf[QG][CPW];
#pragma unroll
    for (int g = 0; g < QG; ++g) {
        const uint8_t *qrow = a.qbuf + (int64_t)(qb * QB + g * 16 + r16) * a.row_bytes + c4 * 16;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            qf[g][c] = i32x4{0, 0, 0, 0};
            if (chunk0 + c < nchunks) qf[g][c] = *reinterpret_cast<const i32x4 *>(qrow + (chunk0 + c) * 64);
        }
    }

    // selection state of the query this lane serves in the epilogue (wave g == w)
    const int jl = w * 16 + r16;            // query within block (meaningful when w < QG)
    const int jq = qb * QB + jl;            // query within this launch
    const bool q_live = (w < QG) && (jq < a.Q);
    float q_scale = 1.0f;
    if (ET == 1 && q_live) q_scale = a.q_scale[jq];
    uint64_t *region = a.regions + ((int64_t)(q_live ? jq : 0) * a.S + s) * a.cap;
    float thr_s = -INFINITY;
    uint64_t thr_k = kKeyFloor;

    __syncthreads();

    const int64_t ntiles = (a.n + 15) >> 4;
    const int64_t last_row = a.n - 1;
    const uint8_t *lane_base = a.store + chunk0 * 64 + c4 * 16;

    i32x4 rows[3][CPW];
    auto load_tile = [&](int64_t t, i32x4 *dst) {
        int64_t r = t * 16 + r16;
        if (r > last_row) r = last_row;  // ragged tail: re-read a valid row, masked out later
        const uint8_t *p = lane_base + r * (int64_t)a.row_bytes;
#pragma unroll
        for (int c = 0; c < CPW; ++c)
            if (chunk0 + c < nchunks) dst[c] = *reinterpret_cast<const i32x4 *>(p + c * 64);
    };

    int64_t t = s;
    if (t < ntiles) load_tile(t, rows[0]);
    if (t + a.S < ntiles) load_tile(t + a.S, rows[1]);
    int pb = 0;

    while (t < ntiles) {
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            if (t < ntiles) {
                if (t + 2 * (int64_t)a.S < ntiles) load_tile(t + 2 * (int64_t)a.S, rows[(b + 2) % 3]);

                // epilogue inputs for this tile, requested early
                const int64_t i0 = t * 16 + c4 * 4;
                f32x4 bias = {0.f, 0.f, 0.f, 0.f};
                f32x4 rsc = {1.f, 1.f, 1.f, 1.f};
                uint32_t valid = 0;
                if (w < QG) {
                    if (a.util) {
                        const f32x4 u = *reinterpret_cast<const f32x4 *>(a.util + i0);
                        bias = u * a.lambda;
                    }
                    if (ET == 1) rsc = *reinterpret_cast<const f32x4 *>(a.row_scale + i0);
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int64_t i = i0 + v;
                        bool ok = i < a.n;
                        if (ok && a.mask) ok = a.mask[i] != 0;
                        valid |= (ok ? 1u : 0u) << v;
                    }
                }

                f32x4 acc[QG];
#pragma unroll
                for (int g = 0; g < QG; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int c = 0; c < CPW; ++c) {
                    if (chunk0 + c < nchunks) {
#pragma unroll
                        for (int g = 0; g < QG; ++g) {
                            if (ET == 0) {
                                acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                    __builtin_bit_cast(bf16x8, rows[b][c]),
                                    __builtin_bit_cast(bf16x8, qf[g][c]), acc[g], 0, 0, 0);
                            } else {
                                const i64x2 ra = __builtin_bit_cast(i64x2, rows[b][c]);
                                const i64x2 qa = __builtin_bit_cast(i64x2, qf[g][c]);
                                acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(ra.x, qa.x, acc[g], 0, 0, 0);
                                acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(ra.y, qa.y, acc[g], 0, 0, 0);
                            }
                        }
                    }
                }
#pragma unroll
                for (int g = 0; g < QG; ++g) part[pb][w][g][lane] = acc[g];
                __syncthreads();

                if (w < QG) {
                    f32x4 sum = part[pb][0][w][lane];
                    sum += part[pb][1][w][lane];
                    sum += part[pb][2][w][lane];
                    sum += part[pb][3][w][lane];

                    uint64_t key[4];
                    uint32_t pend = 0;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float sc = (ET == 1) ? sum[v] * (rsc[v] * q_scale) + bias[v] : sum[v] + bias[v];
                        if (!((valid >> v) & 1u)) sc = -INFINITY;
                        key[v] = 0;
                        if (q_live && sc >= thr_s) {
                            key[v] = make_key(sc, (uint32_t)(i0 + v));
                            if (key[v] > thr_k) pend |= 1u << v;
                        }
                    }
                    // rare path: at least one lane of this wavefront has a candidate
                    while (__ballot(pend != 0) != 0ull) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            if ((pend >> v) & 1u) {
                                const uint32_t pos = atomicAdd(&cnt[jl], 1u);
                                if (pos < (uint32_t)a.cap) {
                                    region[pos] = key[v];
                                    pend &= ~(1u << v);
                                }
                            }
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                        const bool full = q_live && cnt[jl] >= (uint32_t)a.cap;
                        const uint32_t fullmask = (uint32_t)(__ballot(full) & 0xFFFFull);
                        if (fullmask) {
                            __threadfence();  // appended keys reach L2 before they are read back
                            for (int j = 0; j < 16; ++j) {
                                if ((fullmask >> j) & 1u) {
                                    const int qq = qb * QB + w * 16 + j;
                                    uint64_t *reg = a.regions + ((int64_t)qq * a.S + s) * a.cap;
                                    compact_region(reg, a.cap, a.k, scratch[w], &thr_key[w * 16 + j],
                                                   &cnt[w * 16 + j], lane);
                                }
                            }
                            __threadfence();
                            thr_k = thr_key[jl];
                            thr_s = key_score(thr_k);
#pragma unroll
                            for (int v = 0; v < 4; ++v)
                                if (((pend >> v) & 1u) && !(key[v] > thr_k)) pend &= ~(1u << v);
                        }
                    }
                }
                pb ^= 1;
                t += a.S;
            }
        }
    }

    if (q_live && c4 == 0) {
        const uint32_t c = cnt[jl];
        a.counts[(int64_t)jq * a.S + s] = (int32_t)(c < (uint32_t)a.cap ? c : (uint32_t)a.cap);
    }
}

}  // namespace ic
