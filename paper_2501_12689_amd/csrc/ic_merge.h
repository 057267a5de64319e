// Cross-slice merge: combine the candidate lists that the scan kernels leave per query into the
// final top-k of each query (the "keep the most similar examples" step of IC-Cache stage 1,
// Sec. 4.1).
//
// One workgroup takes a group of segments of one query, packs their keys into LDS, sorts them
// with a bitonic network under the (score desc, id asc) key order and writes the best k.  Only
// the keys present are loaded (nearly empty segments are the usual case once the scan starts from
// the pilot's threshold) and the network is sized to them (256 to 2048 keys; mostly in registers
// and by lane shuffles).  A group that holds more than kMergeKeys keys is taken in rounds that
// keep the best k so far.
// The host chains launches until one group per query is left; the last launch decodes keys into
// (fp32 score, int64 id).
#pragma once
#include "ic_common.h"

namespace ic {

constexpr int kMergeKeys = 2048;
constexpr int kMergeMaxSegs = 64;  // segments one workgroup takes when they may be full
constexpr int kMergeWideSegs = 1024;  // most segments one workgroup can take (sparse segments: one level for all slices)

struct MergeArgs {
    const uint64_t *src;        // keys of query q start at src + q * q_stride
    int64_t q_stride;
    int seg_stride;             // keys between consecutive segments
    int seg_cap;                // most keys in a segment
    // keys in use per segment, one of: seg_counts[q][nseg]; or total_counts[q] keys laid out
    // contiguously over the segments (segment s holds keys [s*seg_cap, (s+1)*seg_cap) of them,
    // anything beyond nseg*seg_cap is ignored); or, when both are NULL, seg_cap in every segment
    const int32_t *seg_counts;
    const int32_t *total_counts;
    int nseg;                   // segments per query
    int segs_per_wg;            // <= kMergeWideSegs
    int k;
    uint64_t *dst;              // non-final: lists [Q][gridDim.y][k]
    float *out_scores;          // final: [Q][k], or NULL
    int64_t *out_ids;           // final: [Q][k], or NULL
    uint64_t *kth_out;          // final: [Q] key of the k-th best (a key of kNoThresholdScore if there are fewer), or NULL
    const int32_t *only_flagged;  // if not NULL, queries whose block of 64 has flag 0 are left alone
    float min_score;            // final: entries whose score is below it are dropped (-inf: none)
    int32_t *out_counts;        // final: [Q] entries kept, or NULL
    int64_t self_first;         // final: >= 0: query q is stored row self_first + q and is left out of its
                                // own result (k_out = k - 1 entries are written); -1: off
    int k_out;                  // final: entries per row of the result
    const int32_t *id_map;      // if not NULL: the keys' ids are positions in a reordered copy of the store;
                                // they are replaced by id_map[position] as the keys are loaded, so that ties
                                // are broken by the examples' own ids
};

// Sort the first 256 * R keys of buf in descending order (256 threads; buf complete and visible
// on entry, sorted and visible on return).  Bitonic network over element index e = R * tid + r:
// thread tid keeps elements R*tid .. R*tid + R - 1 in registers, so the compare-exchange stages
// with a distance below R stay inside a thread, those with a distance up to 32 * R exchange with
// another lane of the wavefront (shuffles), and only the few with a larger distance go through
// LDS (3 of the 66 stages for R = 8).
template <int R>
__device__ __forceinline__ void sort_buffer(uint64_t *buf, int tid) {
    constexpr int kLevels = (R == 1) ? 8 : (R == 2) ? 9 : (R == 4) ? 10 : 11;
    static_assert(R == 1 || R == 2 || R == 4 || R == 8, "keys per thread");
    static_assert(256 * 8 == kMergeKeys, "the largest network covers the buffer");
    uint64_t x[R];
#pragma unroll
    for (int r = 0; r < R; ++r) x[r] = buf[R * tid + r];
    const int base = R * tid;
#pragma unroll
    for (int lvl = 1; lvl <= kLevels; ++lvl) {
        const int size = 1 << lvl;  // sorted runs of this length alternate in direction (the last level: all descending)
#pragma unroll
        for (int sb = lvl - 1; sb >= 0; --sb) {
            const int stride = 1 << sb;
            if (stride < R) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    if ((r & stride) == 0) {
                        const bool descending = ((base + r) & size) == 0;
                        const int r2 = (r + stride) < R ? r + stride : r;  // always r + stride here
                        const uint64_t lo = x[r] < x[r2] ? x[r] : x[r2];
                        const uint64_t hi = x[r] < x[r2] ? x[r2] : x[r];
                        x[r] = descending ? hi : lo;
                        x[r2] = descending ? lo : hi;
                    }
                }
            } else {
                const bool descending = (base & size) == 0;
                const bool keep_max = descending == ((base & stride) == 0);
                uint64_t y[R];
                if (stride < 64 * R) {
#pragma unroll
                    for (int r = 0; r < R; ++r) y[r] = __shfl_xor(x[r], stride / R, kWave);
                } else {
                    __syncthreads();  // the previous readers of buf are done
#pragma unroll
                    for (int r = 0; r < R; ++r) buf[base + r] = x[r];
                    __syncthreads();
#pragma unroll
                    for (int r = 0; r < R; ++r) y[r] = buf[(base ^ stride) + r];
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const bool take_other = keep_max ? (y[r] > x[r]) : (y[r] < x[r]);
                    x[r] = take_other ? y[r] : x[r];
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < R; ++r) buf[base + r] = x[r];
    __syncthreads();
}

__global__ __launch_bounds__(256) void merge_lists(const MergeArgs a) {
    __shared__ uint64_t buf[kMergeKeys];
    __shared__ int seg_cnt[kMergeWideSegs];
    __shared__ int seg_off[kMergeWideSegs + 1];
    __shared__ int wave_tot[4];
    __shared__ int kept;
    __shared__ int self_pos;
    const int tid = threadIdx.x;
    const int q = blockIdx.x;
    const int g = blockIdx.y;
    if (a.only_flagged && a.only_flagged[q >> 6] == 0) return;
    const int seg0 = g * a.segs_per_wg;

    // keys in use per segment and their exclusive prefix sums: thread t owns the kPer consecutive
    // segments from kPer * t on; wavefronts combine by shuffles, the four wavefronts through LDS
    constexpr int kPer = kMergeWideSegs / 256;
    int mine[kPer], run = 0;
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        const int sl = kPer * tid + e, seg = seg0 + sl;
        int c = 0;
        if (sl < a.segs_per_wg && seg < a.nseg) {
            if (a.seg_counts) c = a.seg_counts[(int64_t)q * a.nseg + seg];
            else if (a.total_counts) c = a.total_counts[q] - seg * a.seg_cap;
            else c = a.seg_cap;
            c = c < 0 ? 0 : (c > a.seg_cap ? a.seg_cap : c);
        }
        mine[e] = c;
        run += c;
    }
    int incl = run;   // inclusive sum over the lanes of this wavefront
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) {
        const int o = __shfl_up(incl, m, kWave);
        if ((tid & 63) >= m) incl += o;
    }
    if ((tid & 63) == 63) wave_tot[tid >> 6] = incl;
    __syncthreads();
    int before = incl - run;
    for (int w = 0; w < (tid >> 6); ++w) before += wave_tot[w];
#pragma unroll
    for (int e = 0; e < kPer; ++e) {
        const int sl = kPer * tid + e;
        if (sl < a.segs_per_wg) {
            seg_cnt[sl] = mine[e];
            seg_off[sl] = before;
        }
        before += mine[e];
    }
    if (tid == 255) seg_off[a.segs_per_wg] = before;   // the last thread's running sum is the total
    __syncthreads();
    const int total = seg_off[a.segs_per_wg];
    const uint64_t *src = a.src + (int64_t)q * a.q_stride;
    auto fetch = [&](const uint64_t *sp, int idx) -> uint64_t {
        uint64_t key = sp[idx];
        if (a.id_map && key > kKeyFloor)
            key = (key & 0xFFFFFFFF00000000ull) | (uint64_t)(0xFFFFFFFFu - (uint32_t)a.id_map[key_id(key)]);
        return key;
    };

    // The group's keys, segment after segment, form one sequence of `total` keys.  Usually it fits
    // the buffer and is sorted in one go.  If not (full regions, many segments), it is taken in
    // rounds: the best k so far stay at the front of the buffer, the rest of the buffer is
    // refilled with the next keys of the sequence, and the buffer is sorted again.
    int have = 0, consumed = 0;
    do {
        const int room = kMergeKeys - have;
        const int take = total - consumed < room ? total - consumed : room;
        if (take == total && a.segs_per_wg <= 256) {  // everything at once: all segments in parallel, a few threads each
            const int tps = 256 / a.segs_per_wg;  // threads per segment
            const int s = tid / tps;
            if (s < a.segs_per_wg) {
                const int c = seg_cnt[s];
                const uint64_t *sp = src + (int64_t)(seg0 + s) * a.seg_stride;
                uint64_t *dp = buf + seg_off[s];
                for (int idx = tid % tps; idx < c; idx += tps) dp[idx] = fetch(sp, idx);
            }
        } else if (take == total) {  // more segments than threads (sparse ones): a thread takes several
            for (int s = tid; s < a.segs_per_wg; s += 256) {
                const int c = seg_cnt[s];
                const uint64_t *sp = src + (int64_t)(seg0 + s) * a.seg_stride;
                uint64_t *dp = buf + seg_off[s];
                for (int idx = 0; idx < c; ++idx) dp[idx] = fetch(sp, idx);
            }
        } else {  // keys [consumed, consumed + take) of the sequence: find each key's segment
            for (int e = tid; e < take; e += 256) {
                const int pos = consumed + e;
                int lo = 0, hi = a.segs_per_wg;  // seg_off[lo] <= pos < seg_off[hi]
                while (hi - lo > 1) {
                    const int mid = (lo + hi) >> 1;
                    if (seg_off[mid] <= pos) lo = mid;
                    else hi = mid;
                }
                buf[have + e] = fetch(src + (int64_t)(seg0 + lo) * a.seg_stride, pos - seg_off[lo]);
            }
        }
        const int n = have + take;
        int P = 256;  // the network is sized to the keys present
        while (P < n || P < a.k) P <<= 1;
        for (int e = n + tid; e < P; e += 256) buf[e] = 0;  // padding sorts to the end
        __syncthreads();
        if (P == 256) sort_buffer<1>(buf, tid);
        else if (P == 512) sort_buffer<2>(buf, tid);
        else if (P == 1024) sort_buffer<4>(buf, tid);
        else sort_buffer<8>(buf, tid);
        consumed += take;
        have = n < a.k ? n : a.k;
    } while (consumed < total);

    if (tid == 0) {
        kept = 0;
        self_pos = a.k;  // position of the query's own row among the best k keys (a.k: not there)
    }
    __syncthreads();
    if (!a.dst && a.out_scores && a.self_first >= 0) {
        for (int r = tid; r < a.k; r += 256)
            if (buf[r] > kKeyFloor && (int64_t)key_id(buf[r]) == a.self_first + q) self_pos = r;
        __syncthreads();
    }
    for (int r = tid; r < a.k; r += 256) {
        if (a.dst) {
            a.dst[((int64_t)q * gridDim.y + g) * a.k + r] = buf[r];
        } else if (a.out_scores && r < a.k_out) {
            const uint64_t key = buf[r + (r >= self_pos ? 1 : 0)];  // skip the query's own row
            const bool none = key <= kKeyFloor || key_score(key) < a.min_score;
            a.out_scores[(int64_t)q * a.k_out + r] = none ? -INFINITY : key_score(key);
            a.out_ids[(int64_t)q * a.k_out + r] = none ? (int64_t)-1 : (int64_t)key_id(key);
            if (!none) atomicAdd(&kept, 1);
        }
    }
    if (!a.dst && a.kth_out && tid == 0) {
        const uint64_t kth = buf[a.k - 1];
        a.kth_out[q] = kth > kKeyFloor ? kth : make_key(kNoThresholdScore, 0u);
    }
    if (!a.dst && a.out_scores && a.out_counts) {
        __syncthreads();
        if (tid == 0) a.out_counts[q] = kept;
    }
}

}  // namespace ic
