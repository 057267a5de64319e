// Cross-slice merge: combine the candidate lists that the scan kernels leave
// per (query, slice) into the final top-k of each query (the "keep the most
// similar examples" step of IC-Cache stage 1, Sec. 4.1).
//
// One workgroup takes up to kMergeKeys keys of one query (a group of segments),
// sorts them in LDS with a bitonic network under the (score desc, id asc) key
// order and writes the best k.  The host chains launches until one group per
// query is left; the last launch decodes keys into (fp32 score, int64 id).
#pragma once
#include "ic_common.h"

namespace ic {

constexpr int kMergeKeys = 2048;

struct MergeArgs {
    const uint64_t *src;       // keys of query q start at src + q * q_stride
    int64_t q_stride;
    int seg_stride;            // keys between consecutive segments
    int seg_cap;               // most keys in a segment (slots reserved per segment in LDS)
    const int32_t *seg_counts; // [Q][nseg] keys in use, or NULL: every segment holds seg_cap keys
    int nseg;                  // segments per query
    int segs_per_wg;           // segs_per_wg * seg_cap <= kMergeKeys
    int k;
    uint64_t *dst;             // non-final: lists [Q][gridDim.y][k]
    float *out_scores;         // final: [Q][k], or NULL
    int64_t *out_ids;          // final: [Q][k], or NULL
    uint64_t *kth_out;         // final: [Q] key of the k-th best (0 if there are fewer), or NULL
};

__global__ __launch_bounds__(256) void merge_lists(const MergeArgs a) {
    __shared__ uint64_t buf[kMergeKeys];
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    const int g = blockIdx.y;
    const int seg0 = g * a.segs_per_wg;
    const int used = a.segs_per_wg * a.seg_cap;
    int P = 2;
    while (P < used) P <<= 1;
    if (P < a.k) {
        while (P < a.k) P <<= 1;
    }

    const uint64_t *src = a.src + (int64_t)q * a.q_stride;
    for (int e = tid; e < P; e += 256) {
        uint64_t key = 0;
        if (e < used) {
            const int si = e / a.seg_cap;
            const int idx = e - si * a.seg_cap;
            const int seg = seg0 + si;
            if (seg < a.nseg) {
                int c = a.seg_cap;
                if (a.seg_counts) {
                    c = a.seg_counts[(int64_t)q * a.nseg + seg];
                    c = c < a.seg_cap ? c : a.seg_cap;
                }
                if (idx < c) key = src[(int64_t)seg * a.seg_stride + idx];
            }
        }
        buf[e] = key;
    }

    for (int size = 2; size <= P; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            __syncthreads();
            for (int e = tid; e < (P >> 1); e += 256) {
                const int i = 2 * e - (e & (stride - 1));
                const int j = i + stride;
                const bool descending = (i & size) == 0;
                const uint64_t x = buf[i], y = buf[j];
                if ((x < y) == descending) {
                    buf[i] = y;
                    buf[j] = x;
                }
            }
        }
    }
    __syncthreads();

    for (int r = tid; r < a.k; r += 256) {
        const uint64_t key = buf[r];
        if (a.dst) {
            a.dst[((int64_t)q * gridDim.y + g) * a.k + r] = key;
        } else if (a.out_scores) {
            const bool none = key <= kKeyFloor;
            a.out_scores[(int64_t)q * a.k + r] = none ? -INFINITY : key_score(key);
            a.out_ids[(int64_t)q * a.k + r] = none ? (int64_t)-1 : (int64_t)key_id(key);
        }
    }
    if (!a.dst && a.kth_out && tid == 0) a.kth_out[q] = buf[a.k - 1];
}

}  // namespace ic
