// Cluster pruning in front of the scan (Sec. 4.1, "Two-Stage Scalable Example Selection"): the
// cached examples are clustered offline into K groups with K-Means; online a request is compared
// with the K centroids first and then only with the examples of the nearest clusters, K + N/K
// comparisons instead of N, smallest at K = sqrt(N).
//
// Kernels of the offline part: lists from an assignment (histogram, offsets, scatter), the copy of
// the store sorted by cluster that the online scan reads as contiguous ranges, and the K-Means
// update step (mean direction of every cluster).
#pragma once
#include "ic_common.h"
#include "ic_merge.h"

namespace ic {

// ---- online part: the (query, list) pairs of a batch, grouped by list --------------------------------
//
// A list that several queries of a batch probe is read once for up to 16 of them: the pairs are sorted by
// list, and every run of equal lists is cut into tasks of at most 16 pairs.  One workgroup; at most
// kTaskPairs pairs.  probe[p] is the list of pair p (pair = query * nprobe + rank; a value outside
// [0, K) means no list).  task_list[t] = the list of task t, task_pair[16 t + j] = the pair in slot j of
// task t, -1 where there is none; both hold `pairs` tasks, the most there can be.  The order of the tasks
// and of the pairs inside a task is fixed by the sort (descending list id, descending pair), so a search
// does the same thing every time it is run.  The kernel also zeroes region_counts[0, n_counts), the
// per-(pair, slice) counts that the scan tasks then fill in for the pairs they serve.
constexpr int kTaskPairs = kMergeKeys;   // pairs of one pass: what one workgroup sorts at once
constexpr int kTaskSlots = 16;           // query slots of a task (= the queries of a scan workgroup)

// R = sorted keys per thread: 256 R >= pairs.
template <int R>
__global__ __launch_bounds__(256) void ivf_group_tasks(const int64_t *__restrict__ probe, int pairs, int32_t K,
                                                       int64_t *__restrict__ task_list, int32_t *__restrict__ task_pair,
                                                       int32_t *__restrict__ region_counts, int n_counts) {
    __shared__ uint64_t key[kMergeKeys];
    __shared__ int32_t part[2][256];
    const int tid = threadIdx.x;
    // (the barriers of the sort below order these stores before the ones that fill the tasks in)
    for (int i = tid; i < pairs; i += 256) task_list[i] = -1;
    for (int i = tid; i < pairs * kTaskSlots; i += 256) task_pair[i] = -1;
    for (int i = tid; i < n_counts; i += 256) region_counts[i] = 0;
    // key = (list + 1, pair); 0 for a pair without a list and for the padding: those sort to the end
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int p = R * tid + r;
        uint64_t k64 = 0ull;
        if (p < pairs) {
            const int64_t c = probe[p];
            if (c >= 0 && c < K) k64 = ((uint64_t)(c + 1) << 32) | (uint64_t)(uint32_t)p;
        }
        key[p] = k64;
    }
    __syncthreads();
    sort_buffer<R>(key, tid);
    // element e = R tid + r of the sorted keys.  head: first pair of its list.  Every thread finds, for its
    // elements, the start of the run they are in (a prefix maximum over the heads' positions) ...
    uint64_t mine[R];
    int head_at[R];   // position of the last head at or before the element, -1 if none in this thread yet
#pragma unroll
    for (int r = 0; r < R; ++r) mine[r] = key[R * tid + r];
    const uint64_t before = tid > 0 ? key[R * tid - 1] : 0ull;
    int last_head = -1;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const uint64_t prev = r > 0 ? mine[r - 1] : before;
        const bool head = mine[r] != 0ull && (R * tid + r == 0 || (prev >> 32) != (mine[r] >> 32));
        if (head) last_head = R * tid + r;
        head_at[r] = last_head;
    }
    // exclusive prefix maximum of last_head over the threads
    int src = 0;
    part[0][tid] = last_head;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int v = part[src][tid];
        const int o = tid >= off ? part[src][tid - off] : -1;
        part[src ^ 1][tid] = v > o ? v : o;
        src ^= 1;
        __syncthreads();
    }
    const int head_before = tid > 0 ? part[src][tid - 1] : -1;
    __syncthreads();
    // ... then which of them open a task (every 16th pair of a run), and how many tasks were opened before
    int opens = 0;
    bool open[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int start = head_at[r] >= 0 ? head_at[r] : head_before;
        open[r] = mine[r] != 0ull && ((R * tid + r - start) % kTaskSlots) == 0;
        head_at[r] = start;
        opens += open[r] ? 1 : 0;
    }
    src = 0;
    part[0][tid] = opens;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        const int v = part[src][tid];
        const int o = tid >= off ? part[src][tid - off] : 0;
        part[src ^ 1][tid] = v + o;
        src ^= 1;
        __syncthreads();
    }
    int task = (tid > 0 ? part[src][tid - 1] : 0) - 1;   // index of the task open before this thread's first element
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (mine[r] == 0ull) continue;
        if (open[r]) {
            ++task;
            task_list[task] = (int64_t)(mine[r] >> 32) - 1;
        }
        task_pair[task * kTaskSlots + (R * tid + r - head_at[r]) % kTaskSlots] = (int32_t)(uint32_t)mine[r];
    }
}

// assign[i] = cluster of row i from its key (score of the best centroid, its id); 0 = no key: -1
__global__ void ivf_take_assignment(const uint64_t *__restrict__ keys, int64_t n, int32_t *__restrict__ assign) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) assign[i] = keys[i] > kKeyFloor ? (int32_t)key_id(keys[i]) : -1;
}

__global__ void ivf_zero_i64(int64_t *__restrict__ p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// counts[c] = live rows assigned to cluster c (rows with assign outside [0, K) or live == 0 are in no list)
__global__ void ivf_histogram(const int32_t *__restrict__ assign, const uint8_t *__restrict__ live, int64_t n,
                              int32_t K, int64_t *__restrict__ counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t c = assign[i];
    if (c >= 0 && c < K && live[i] != 0) atomicAdd(reinterpret_cast<unsigned long long *>(counts + c), 1ull);
}

// offsets[c] = rows in clusters before c, offsets[K] = rows in lists; cursor[c] = offsets[c].
// counts and offsets may not alias.  One workgroup.
__global__ __launch_bounds__(256) void ivf_offsets(const int64_t *__restrict__ counts, int32_t K,
                                                   int64_t *__restrict__ offsets, int64_t *__restrict__ cursor) {
    __shared__ int64_t tile[256];
    __shared__ int64_t carry;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int32_t lo = 0; lo < K; lo += 256) {
        const int32_t c = lo + threadIdx.x;
        const int64_t v = c < K ? counts[c] : 0;
        tile[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {
            const int64_t add = (int)threadIdx.x >= off ? tile[threadIdx.x - off] : 0;
            __syncthreads();
            tile[threadIdx.x] += add;
            __syncthreads();
        }
        if (c < K) {
            offsets[c] = carry + tile[threadIdx.x] - v;
            cursor[c] = carry + tile[threadIdx.x] - v;
        }
        __syncthreads();
        if (threadIdx.x == 0) carry += tile[255];
        __syncthreads();
    }
    if (threadIdx.x == 0) offsets[K] = carry;
}

// perm[position] = row, positions of a cluster handed out by an atomic cursor (the order inside a
// list is not fixed; nothing depends on it: ids are mapped back before ties are broken)
__global__ void ivf_scatter(const int32_t *__restrict__ assign, const uint8_t *__restrict__ live, int64_t n,
                            int32_t K, int64_t *__restrict__ cursor, int32_t *__restrict__ perm) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int32_t c = assign[i];
    if (c < 0 || c >= K || live[i] == 0) return;
    const int64_t pos = (int64_t)atomicAdd(reinterpret_cast<unsigned long long *>(cursor + c), 1ull);
    perm[pos] = (int32_t)i;
}

// sorted copy: row j of dst = row perm[j] of src, with its utility and scale
__global__ __launch_bounds__(256) void ivf_gather(const uint8_t *__restrict__ src_rows, const float *__restrict__ src_util,
                                                  const float *__restrict__ src_scale, int row_bytes,
                                                  const int32_t *__restrict__ perm, const int64_t *__restrict__ total,
                                                  uint8_t *__restrict__ dst_rows, float *__restrict__ dst_util,
                                                  float *__restrict__ dst_scale, uint8_t *__restrict__ dst_live) {
    const int lane = threadIdx.x & 63;
    const int64_t wave = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    const int64_t n = *total;
    for (int64_t j = wave; j < n; j += nwaves) {
        const int64_t r = perm[j];
        const i32x4 *s = reinterpret_cast<const i32x4 *>(src_rows + r * (int64_t)row_bytes);
        i32x4 *d = reinterpret_cast<i32x4 *>(dst_rows + j * (int64_t)row_bytes);
        for (int c = lane; c < row_bytes / 16; c += 64) d[c] = s[c];
        if (lane == 0) {
            dst_util[j] = src_util[r];
            if (src_scale) dst_scale[j] = src_scale[r];
            dst_live[j] = 1;
        }
    }
}

// value of an OCP E4M3 code (no infinities; the two NaN codes do not occur in a store)
__device__ __forceinline__ float e4m3_value(uint32_t c) {
    const uint32_t e = (c >> 3) & 15u, m = c & 7u;
    const float mag = e == 0 ? (float)m * 0x1p-9f : __uint_as_float(((e + 120u) << 23) | (m << 20));
    return (c & 0x80u) ? -mag : mag;
}

// element e of a stored row as fp32 (without the fp8 row scale)
template <int ET>
__device__ __forceinline__ float stored_element(const uint8_t *row, int e) {
    if (ET == 0) return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(row)[e] << 16);
    return e4m3_value(row[e]);
}

// element i of 16 stored bytes held in registers, as fp32 (without the fp8 row scale)
template <int ET>
__device__ __forceinline__ float piece_element(const i32x4 v, int i) {
    if (ET == 0) {
        const uint32_t word = (uint32_t)v[i >> 1];
        return __uint_as_float((i & 1) ? (word & 0xFFFF0000u) : (word << 16));
    }
    return e4m3_value((uint8_t)(((uint32_t)v[i >> 2] >> (8 * (i & 3))) & 0xFFu));
}

// K-Means update, first step: acc[c][e] += sum over a share of cluster c's rows of element e, as
// 64-bit fixed point with 30 fractional bits.  rows are the sorted copy, so the cluster is the range
// [offsets[c], offsets[c + 1]); workgroup (c, y) takes the y-th of gridDim.y equal shares of it, adds
// its rows in fp64 in a fixed order (lane l owns the 16-byte pieces l and l + 64 of every row, the
// four wavefronts take rows round robin, their partial sums are added in wavefront order), rounds
// each sum once to fixed point and adds it to acc with an integer atomic.  Integer addition is
// associative, so the result does not depend on the order in which the workgroups finish.  Elements
// of unit rows are at most 1 in magnitude: a share's sum stays below 2^31, its fixed-point value
// below 2^61, and the rounding error of a cluster's sum is at most gridDim.y * 2^-31.
constexpr double kIvfFixedOne = 1073741824.0;  // 2^30
template <int ET>
__global__ __launch_bounds__(256) void ivf_cluster_sums(const uint8_t *__restrict__ rows, const float *__restrict__ scale,
                                                        int row_bytes, int d, const int64_t *__restrict__ offsets,
                                                        long long *__restrict__ acc) {
    constexpr int E16 = (ET == 0) ? 8 : 16;  // elements in 16 bytes
    constexpr int kRowsAhead = 4;            // rows a wavefront requests before it adds them
    __shared__ double part[4][64];
    const int c = blockIdx.x;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t lo = offsets[c], hi = offsets[c + 1];
    const int64_t share = (hi - lo + gridDim.y - 1) / gridDim.y;
    const int64_t first = lo + (int64_t)blockIdx.y * share;
    const int64_t last = first + share < hi ? first + share : hi;
    if (first >= last) return;  // whole workgroup: an empty cluster or an empty share
    const int npieces = row_bytes / 16;  // at most 128
    const bool own0 = lane < npieces, own1 = lane + 64 < npieces;
    double sum[2][E16];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int i = 0; i < E16; ++i) sum[p][i] = 0.0;
    for (int64_t r0 = first + w * kRowsAhead; r0 < last; r0 += 4 * kRowsAhead) {
        i32x4 piece[kRowsAhead][2];
        float sc[kRowsAhead];
#pragma unroll
        for (int u = 0; u < kRowsAhead; ++u) {
            const int64_t r = r0 + u < last ? r0 + u : last - 1;  // past the share: re-read, not added
            const uint8_t *row = rows + r * (int64_t)row_bytes;
            piece[u][0] = own0 ? *reinterpret_cast<const i32x4 *>(row + lane * 16) : i32x4{0, 0, 0, 0};
            piece[u][1] = own1 ? *reinterpret_cast<const i32x4 *>(row + (lane + 64) * 16) : i32x4{0, 0, 0, 0};
            sc[u] = (ET == 1) ? scale[r] : 1.0f;
        }
#pragma unroll
        for (int u = 0; u < kRowsAhead; ++u) {
            if (r0 + u >= last) break;
            const double s64 = (double)sc[u];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int i = 0; i < E16; ++i) sum[p][i] += (double)piece_element<ET>(piece[u][p], i) * s64;
        }
    }
#pragma unroll
    for (int p = 0; p < 2; ++p) {
#pragma unroll
        for (int i = 0; i < E16; ++i) {
            part[w][lane] = sum[p][i];
            __syncthreads();
            if (w == 0) {
                const int e = (lane + 64 * p) * E16 + i;
                if (e < d) {
                    const double total = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
                    atomicAdd(reinterpret_cast<unsigned long long *>(acc + (int64_t)c * d + e),
                              (unsigned long long)__double2ll_rn(total * kIvfFixedOne));
                }
            }
            __syncthreads();
        }
    }
}

// K-Means update, second step: sums[c] = acc[c] as fp32 [K, d]; a cluster without rows keeps its
// centroid (its stored row is decoded instead).
template <int ET>
__global__ void ivf_finish_sums(const long long *__restrict__ acc, const int64_t *__restrict__ offsets, int d,
                                const uint8_t *__restrict__ cent_rows, int row_bytes,
                                const float *__restrict__ cent_scale, float *__restrict__ sums) {
    const int c = blockIdx.x;
    const bool empty = offsets[c] == offsets[c + 1];
    const uint8_t *row = cent_rows + (int64_t)c * row_bytes;
    const float sc = (ET == 1) ? cent_scale[c] : 1.0f;
    for (int e = threadIdx.x; e < d; e += blockDim.x)
        sums[(int64_t)c * d + e] = empty ? stored_element<ET>(row, e) * sc
                                         : (float)((double)acc[(int64_t)c * d + e] * (1.0 / kIvfFixedOne));
}

// K-Means start: sums[c] = the stored row at position floor(c * n / K), decoded to fp32 [K, d]
template <int ET>
__global__ void ivf_rows_as_centroids(const uint8_t *__restrict__ rows, const float *__restrict__ scale,
                                      int row_bytes, int d, int64_t n, int32_t K, float *__restrict__ sums) {
    const int c = blockIdx.x;
    const int64_t r = (int64_t)c * n / K;
    const uint8_t *row = rows + r * (int64_t)row_bytes;
    const float sc = (ET == 1) ? scale[r] : 1.0f;
    for (int e = threadIdx.x; e < d; e += blockDim.x) sums[(int64_t)c * d + e] = stored_element<ET>(row, e) * sc;
}

}  // namespace ic
