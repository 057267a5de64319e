// Host side of the C ABI declared in include/iccache.h: argument checks, the
// layout of the caller's arena, and kernel launches.  No device memory is
// allocated here and nothing synchronises the host except the timing query.
#include "../../include/iccache.h"

#include <hip/hip_runtime.h>

#include <mutex>
#include <new>
#include <vector>

#include "ic_common.h"
#include "ic_merge.h"
#include "ic_quantize.h"
#include "ic_ivf.h"
#include "ic_maintain.h"
#include "ic_scan_gemm.h"
#include "ic_scan_stream.h"

namespace {

constexpr int64_t kAlign = IC_ARENA_ALIGN;
constexpr int kMaxRowBytes = 2048;     // widest row the streaming scan holds in registers
constexpr int kQueryChunkMax = 8192;   // queries per pass over the store
constexpr int kSliceBudgetMax = 1024;  // most workgroups a scan launch may use
constexpr int kPilotSlices = 512;           // slices of the threshold pilot (>= IC_MAX_K)
constexpr int kPilotMinQueries = 9;         // smaller batches select cheaply without a pilot, unless k is large
constexpr int64_t kPilotMinWork = 128;      // ... that is, unless queries x k reaches this (with at least 8 queries)
constexpr int64_t kPilotMinTiles = (int64_t)kPilotSlices * 4;       // streaming pilot: at least every 4th tile is skipped
constexpr int64_t kGemmMinTiles = (int64_t)kPilotSlices * 8 * 4;    // the tiled scan is used from 262,144 rows on,
constexpr int64_t kGemmSmallTiles = (int64_t)kPilotSlices * 8;      // and from 65,536 rows on for more than 128 queries,
constexpr int64_t kGemmTinyTiles = (int64_t)kPilotSlices * 2;       // from 16,384 rows on if also k <= 16 (a larger k needs
                                                                    // a pilot as dense as the scan itself on so few rows)
constexpr int kComputeUnitsDefault = 256;   // MI355X
constexpr size_t kLdsPerCu = 160 * 1024;
constexpr size_t kMaxTimedEvents = 1 << 16;  // event pairs kept while timing is on
constexpr int64_t kRegionSlots = 64 * (int64_t)kSliceBudgetMax;  // bound on queries x slices
constexpr int kRedoSlices = 64;             // slices of the streaming pass that redoes query blocks of the tiled scan
constexpr int kGemmMinQueries = 65;         // batches from here on use the MFMA-tiled scan (one tile is 256 queries wide, but from
                                            // 65 queries on it already beats two passes of the streaming scan: 4.1 vs 4.7 ms at d=768)
constexpr int kGemmListSeg = ic::kMergeKeys;  // candidate lists are merged in segments of this many keys
constexpr uint32_t kGemmOverCap = 65536;      // tiles of one tiled scan that may be left to its second launch
constexpr int kGemmListMax = 8 * kGemmListSeg;
constexpr size_t kL2Share = 2u << 20;       // query-block bytes of a group of XCDs: half of an XCD's 4 MB L2, the other half
                                            // holds the row tiles its 32 workgroups are on (with the whole L2 given to queries
                                            // the fp8 scan of 4096 queries re-read the store 9 times and ran 6 % slower)

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Candidates a scan workgroup keeps per query between compactions.
// Sized so that, with 64 queries per workgroup, two workgroups fit the LDS of a compute unit
// for k <= 64 (64 * 112 * 8 B = 56 KB of regions each).
inline int region_cap(int k) { return k <= 32 ? 64 : (k <= 64 ? 112 : ic::kMaxCap); }
// With 64 queries per workgroup and 64 < k <= 100 the regions are kept at 112 keys as well, so that
// two workgroups still fit a compute unit; the slack above k is small, which is fine because such
// batches start from the pilot's threshold and a slice rarely sees more than a few dozen candidates
// (a region that does fill up is compacted more often, nothing else changes).
inline int region_cap_for(int k, int qg_idx) { return (qg_idx == 2 && k > 64 && k <= 100) ? 112 : region_cap(k); }

// Keys of the per-query candidate list of the MFMA-tiled scan.  Starting from the pilot's
// threshold about 64*k rows pass (the pilot sees every 64th tile); over 4096 queries with
// k = 16 the largest list seen was 2.1 times that mean, so the list holds 128*k and never
// fewer than 4096.  An overflow is still handled exactly (the block is redone).
inline int gemm_list_cap(int k) {
    int64_t c = round_up(std::min<int64_t>(std::max<int64_t>(128 * (int64_t)k, 2 * kGemmListSeg), kGemmListMax), kGemmListSeg);
    return (int)c;
}

struct Layout {
    int esize = 0, row_bytes = 0, q_chunk = 0;
    int64_t cap_pad = 0;
    size_t off_rows = 0, off_scale = 0, off_util = 0, off_qbuf = 0, off_qscale = 0, off_regions = 0,
           off_counts = 0, off_list_a = 0, off_list_b = 0, off_consts = 0, off_bias = 0, off_pilot = 0, off_thr = 0, off_glist = 0, off_gcount = 0,
           off_redo = 0, off_over = 0, off_valid = 0, off_blocks = 0, off_domain = 0, off_panel = 0, off_qpanel = 0,
           total = 0;
    bool panel = false;  // the store has a step-major copy for the tiled scan
    int64_t list_slots = 0;
    int64_t region_slots = 0;  // queries x slices that the candidate regions hold
    int q_rows = 0;  // rows of the prepared query block
};

// with_panel = false: an index that is only ever scanned by the streaming kernels (the sorted copy behind
// cluster pruning) goes without the step-major copy of its rows
bool make_layout(int32_t d, ic_dtype store, int64_t capacity, int64_t max_q, int32_t max_k, Layout &L,
                 bool with_panel = true) {
    if (store != IC_STORE_BF16 && store != IC_STORE_FP8_E4M3) return false;
    if (d < 1 || capacity < 1 || max_q < 1 || max_k < 1 || max_k > IC_MAX_K) return false;
    if (capacity > (int64_t)1 << 31) return false;
    L.esize = (store == IC_STORE_BF16) ? 2 : 1;
    const int64_t rb = round_up((int64_t)d * L.esize, 128);
    if (rb > kMaxRowBytes) return false;
    L.row_bytes = (int)rb;
    L.cap_pad = round_up(capacity, ic::kGemmTile);
    L.q_chunk = (int)std::min<int64_t>(round_up(max_q, 64), kQueryChunkMax);
    L.q_rows = (int)round_up(L.q_chunk, ic::kGemmTile);
    const bool gemm = L.q_chunk >= kGemmMinQueries;
    // A block of 64 queries that the tiled scan hands back is redone by one streaming pass over the store;
    // that pass gets kRedoSlices workgroups for the block whatever the size of the batch, so the regions of
    // an index that serves large batches hold that many slices for every query of a pass.
    L.region_slots = gemm ? std::max<int64_t>(kRegionSlots, (int64_t)L.q_chunk * kRedoSlices) : kRegionSlots;
    L.list_slots = std::max<int64_t>(kRegionSlots / 8 + L.q_chunk, gemm ? (int64_t)L.q_chunk * (kGemmListMax / kGemmListSeg) : 0);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = (size_t)round_up((int64_t)(off + bytes), kAlign);
        return at;
    };
    L.off_rows = take((size_t)L.cap_pad * (size_t)L.row_bytes);
    L.off_scale = take(store == IC_STORE_FP8_E4M3 ? (size_t)L.cap_pad * 4 : 0);
    L.off_util = take((size_t)L.cap_pad * 4);
    L.off_qbuf = take((size_t)L.q_rows * (size_t)L.row_bytes);
    L.off_qscale = take((size_t)L.q_rows * 4);
    L.off_regions = take((size_t)L.region_slots * (size_t)region_cap(max_k) * 8);
    L.off_counts = take((size_t)L.region_slots * 4);
    L.off_list_a = take((size_t)L.list_slots * (size_t)max_k * 8);
    L.off_list_b = take((size_t)L.list_slots * (size_t)max_k * 8);
    L.off_consts = take(64);
    L.off_bias = take((size_t)L.cap_pad * 4);
    L.off_pilot = take((size_t)L.q_chunk * kPilotSlices * 8);
    L.off_thr = take((size_t)L.q_chunk * 8);
    L.off_glist = take(gemm ? (size_t)L.q_chunk * (size_t)gemm_list_cap(max_k) * 8 : 0);
    L.off_gcount = take(gemm ? (size_t)L.q_chunk * 4 : 0);
    L.off_redo = take(gemm ? (size_t)(L.q_chunk / 64 + 1) * 4 : 0);
    L.off_over = take(gemm ? 8 + (size_t)kGemmOverCap * 8 : 0);
    L.off_valid = take((size_t)L.cap_pad);                                          // persistent validity, 1 B/row
    L.off_blocks = take((size_t)(L.cap_pad / ic::kScanBlock + 2) * 8);              // compaction: block offsets
    L.off_domain = take((size_t)L.cap_pad * 4);                                      // sharing domain, 4 B/row
    // the tiled scan reads both operands from step-major copies (see ic_scan_gemm.h): the store's, as large as
    // the store itself, and the query block's
    L.panel = gemm && with_panel;
    L.off_panel = take(L.panel ? (size_t)L.cap_pad * (size_t)L.row_bytes : 0);
    L.off_qpanel = take(L.panel ? (size_t)L.q_rows * (size_t)L.row_bytes : 0);
    L.total = off;
    return true;
}

// 64-byte chunks of a row per wavefront of the streaming scan.  An even number lets a wavefront fetch whole
// 128-byte lines, so rows of 18 or 20 chunks (1152, 1280 bytes) are dealt 6 to a wavefront instead of 5 (the last
// wavefront gets 0 or 2 and multiplies its surplus by zeros).  Measured on stores of 1 M rows and of 6 GB: 4-10 %
// faster for every batch size (on 100 k rows, which the caches hold: the same up to 32 queries, 7 % slower for 64).
// Rows of 10, 12, 26 and 28 chunks keep the odd deal: the even one gains 7-10 % for up to 32 queries on large
// stores at 12, 26 and 28 chunks but costs 64 queries 5-13 % there, and on 100 k rows of 12 chunks it costs every
// batch size 2-3 us.  The deal depends on the row length only, because it fixes the order in which a row's
// products are added: a query's scores must not depend on the batch it came in, nor on whether the search was
// pruned by clusters.
inline int chunks_per_wavefront(int nchunks) {
    int cpw = (nchunks + ic::kScanWaves - 1) / ic::kScanWaves;
    if (nchunks == 18 || nchunks == 20) cpw += 1;
    return cpw;
}

// 64 zero bytes: the score bias of a search that has neither utility weight nor mask.
__global__ void init_consts(uint32_t *c) {
    if (threadIdx.x < 16) c[threadIdx.x] = 0u;
}

using ScanFn = void (*)(dim3, hipStream_t, const ic::ScanArgs &);

template <int ET, int QG, int CPW, bool PILOT, bool DOM = false>
void launch_scan(dim3 grid, hipStream_t st, const ic::ScanArgs &a) {
    // more than 64 KB of dynamic LDS has to be allowed once per kernel
    static const hipError_t allowed = hipFuncSetAttribute(
        reinterpret_cast<const void *>(&ic::scan_stream<ET, QG, CPW, PILOT, false, DOM>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)ic::scan_lds_bytes(QG, ic::kMaxCap));
    (void)allowed;
    hipLaunchKernelGGL((ic::scan_stream<ET, QG, CPW, PILOT, false, DOM>), grid, dim3(256),
                       ic::scan_lds_bytes(QG, PILOT ? 0 : a.cap), st, a);
}

#define IC_SCAN_ROW(ET, QG, P)                                                                  \
    {                                                                                           \
        launch_scan<ET, QG, 1, P>, launch_scan<ET, QG, 2, P>, launch_scan<ET, QG, 3, P>,         \
            launch_scan<ET, QG, 4, P>, launch_scan<ET, QG, 5, P>, launch_scan<ET, QG, 6, P>,     \
            launch_scan<ET, QG, 7, P>, launch_scan<ET, QG, 8, P>                                 \
    }
// [pilot][element type][query groups: 1, 2, 4][chunks per wavefront - 1]
const ScanFn kScanTable[2][2][3][8] = {
    {{IC_SCAN_ROW(0, 1, false), IC_SCAN_ROW(0, 2, false), IC_SCAN_ROW(0, 4, false)},
     {IC_SCAN_ROW(1, 1, false), IC_SCAN_ROW(1, 2, false), IC_SCAN_ROW(1, 4, false)}},
    {{IC_SCAN_ROW(0, 1, true), IC_SCAN_ROW(0, 2, true), IC_SCAN_ROW(0, 4, true)},
     {IC_SCAN_ROW(1, 1, true), IC_SCAN_ROW(1, 2, true), IC_SCAN_ROW(1, 4, true)}},
};
#undef IC_SCAN_ROW
#define IC_SCAN_ROW(ET, QG, P)                                                                              \
    {                                                                                                       \
        launch_scan<ET, QG, 1, P, true>, launch_scan<ET, QG, 2, P, true>, launch_scan<ET, QG, 3, P, true>,   \
            launch_scan<ET, QG, 4, P, true>, launch_scan<ET, QG, 5, P, true>, launch_scan<ET, QG, 6, P, true>, \
            launch_scan<ET, QG, 7, P, true>, launch_scan<ET, QG, 8, P, true>                                 \
    }
// the same kernels with the per-query sharing-domain test compiled in
const ScanFn kScanTableDom[2][2][3][8] = {
    {{IC_SCAN_ROW(0, 1, false), IC_SCAN_ROW(0, 2, false), IC_SCAN_ROW(0, 4, false)},
     {IC_SCAN_ROW(1, 1, false), IC_SCAN_ROW(1, 2, false), IC_SCAN_ROW(1, 4, false)}},
    {{IC_SCAN_ROW(0, 1, true), IC_SCAN_ROW(0, 2, true), IC_SCAN_ROW(0, 4, true)},
     {IC_SCAN_ROW(1, 1, true), IC_SCAN_ROW(1, 2, true), IC_SCAN_ROW(1, 4, true)}},
};
#undef IC_SCAN_ROW

template <int ET, int CPW>
void launch_scan_task(dim3 grid, hipStream_t st, const ic::ScanArgs &a) {
    static const hipError_t allowed = hipFuncSetAttribute(
        reinterpret_cast<const void *>(&ic::scan_stream<ET, 1, CPW, false, true>),
        hipFuncAttributeMaxDynamicSharedMemorySize, (int)ic::scan_lds_bytes(1, ic::kMaxCap));
    (void)allowed;
    hipLaunchKernelGGL((ic::scan_stream<ET, 1, CPW, false, true>), grid, dim3(256), ic::scan_lds_bytes(1, a.cap), st, a);
}
// cluster-range scans: [element type][chunks per wavefront - 1]
const ScanFn kTaskTable[2][8] = {
    {launch_scan_task<0, 1>, launch_scan_task<0, 2>, launch_scan_task<0, 3>, launch_scan_task<0, 4>,
     launch_scan_task<0, 5>, launch_scan_task<0, 6>, launch_scan_task<0, 7>, launch_scan_task<0, 8>},
    {launch_scan_task<1, 1>, launch_scan_task<1, 2>, launch_scan_task<1, 3>, launch_scan_task<1, 4>,
     launch_scan_task<1, 5>, launch_scan_task<1, 6>, launch_scan_task<1, 7>, launch_scan_task<1, 8>},
};

template <int ET, bool PILOT, bool DOM, bool AGAIN = false>
void launch_gemm_one(int grid, hipStream_t st, const ic::GemmArgs &a) {
    static const hipError_t allowed =
        hipFuncSetAttribute(reinterpret_cast<const void *>(&ic::scan_gemm<ET, PILOT, DOM, false, AGAIN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)ic::gemm_lds_bytes());
    (void)allowed;
    hipLaunchKernelGGL((ic::scan_gemm<ET, PILOT, DOM, false, AGAIN>), dim3(grid), dim3(ic::kGemmThreads),
                       ic::gemm_lds_bytes(), st, a);
}
template <int ET>
void launch_gemm_rowmax(int grid, hipStream_t st, const ic::GemmArgs &a) {
    static const hipError_t allowed =
        hipFuncSetAttribute(reinterpret_cast<const void *>(&ic::scan_gemm<ET, false, false, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)ic::gemm_lds_bytes());
    (void)allowed;
    hipLaunchKernelGGL((ic::scan_gemm<ET, false, false, true>), dim3(grid), dim3(ic::kGemmThreads), ic::gemm_lds_bytes(),
                       st, a);
}
template <int ET, bool PILOT>
void launch_gemm(int grid, hipStream_t st, const ic::GemmArgs &a) {
    if (a.q_dom) launch_gemm_one<ET, PILOT, true>(grid, st, a);
    else launch_gemm_one<ET, PILOT, false>(grid, st, a);
}
// the tiles the selection launch left undone (it listed them), each computed again and tested score by score
template <int ET>
void launch_gemm_again(int grid, hipStream_t st, const ic::GemmArgs &a) {
    if (a.q_dom) launch_gemm_one<ET, false, true, true>(grid, st, a);
    else launch_gemm_one<ET, false, false, true>(grid, st, a);
}

}  // namespace

// Per-search scratch: everything the kernels of one search write besides the result.  An index
// keeps one inside the caller's arena; the entry point that allocates nothing builds one over
// the library's static device array instead.
struct Workspace {
    uint8_t *qbuf = nullptr;        // prepared query block, [q_rows] rows in the store's format
    uint8_t *qpanel = nullptr;      // its step-major copy for the tiled scan, or NULL
    float *qscale = nullptr;        // [q_rows]
    uint64_t *regions = nullptr;    // candidate keys per (query, slice)
    int32_t *counts = nullptr;
    uint64_t *list_a = nullptr, *list_b = nullptr;  // ping-pong between merge levels
    uint8_t *consts = nullptr;      // 64 zero bytes (the bias of a search that has none)
    float *bias = nullptr;          // [cap_pad] per-row additive term of the current search
    uint64_t *pilot_keys = nullptr; // [q_chunk][kPilotSlices]
    uint64_t *thr_init = nullptr;   // [q_chunk]
    uint64_t *glist = nullptr;      // [q_chunk][gemm_list_cap(max_k)], NULL when the tiled scan is not available
    int32_t *gcount = nullptr;      // [q_chunk]
    int32_t *redo = nullptr;        // [q_chunk/64 + 1]
    uint32_t *over = nullptr;       // [0]: tiles left to the second launch of the tiled scan; from [2] on: the (tile, block) pairs
    int q_chunk = 0;                // queries per pass over the store
    int64_t region_slots = 0;       // bound on queries x slices of one streaming launch
    bool *consts_ready = nullptr;   // host flag: consts has been written on this device
    bool timed = true;              // scan launches may be bracketed with events (creates events on first use)
};

struct ic_index {
    int32_t d;
    ic_dtype store;
    int64_t capacity;
    int64_t max_q;
    int32_t max_k;
    Layout L;
    int64_t n;
    hipStream_t stream;
    int slice_budget;  // 0 = derive from occupancy; otherwise forced (benchmark sweeps)
    int compute_units;
    int device;        // the GPU that was current at creation
    uint8_t *rows;
    uint8_t *panel;        // step-major copy of rows for the tiled scan ([cap_pad / 256] tiles), or NULL
    float *scale;
    float *util;
    uint8_t *valid;        // [cap_pad] 1 = row is live, 0 = invalidated (evicted) and waiting for compaction
    int64_t *block_offsets;  // compaction scratch
    bool any_invalid;      // some row has been invalidated since the last compaction
    int32_t *domain;       // [cap_pad] sharing domain of every row; 0 = shared with every domain
    Workspace ws;          // the search scratch inside the arena
    int last_nblk64 = 0;   // blocks of 64 queries of the last batch that took the tiled scan
    int gemm_list_cap_override;  // tests: shrink the candidate lists to force the overflow path
    bool consts_ready;  // written by the first search (creation launches nothing)
    bool timing;
    std::vector<hipEvent_t> events;  // pairs (start, stop)
    size_t events_used;
};

extern "C" {

const char *ic_status_string(ic_status s) {
    switch (s) {
        case IC_OK: return "ok";
        case IC_ERR_INVALID_ARG: return "invalid argument";
        case IC_ERR_OOM: return "out of host memory";
        case IC_ERR_CAPACITY: return "capacity exceeded";
        case IC_ERR_DEVICE: return "HIP call failed";
        case IC_ERR_UNSUPPORTED: return "unsupported configuration";
    }
    return "unknown status";
}

size_t ic_workspace_bytes(int32_t d, ic_dtype store, int64_t capacity_rows, int64_t max_queries,
                          int32_t max_k) {
    Layout L;
    if (!make_layout(d, store, capacity_rows, max_queries, max_k, L)) return 0;
    return L.total;
}

static ic_status create_index(ic_index **out, int32_t d, ic_dtype store, int64_t capacity_rows,
                              int64_t max_queries, int32_t max_k, void *arena_dev, size_t arena_bytes,
                              void *stream, bool with_panel) {
    if (!out || !arena_dev) return IC_ERR_INVALID_ARG;
    if (((uintptr_t)arena_dev % kAlign) != 0) return IC_ERR_INVALID_ARG;
    Layout L;
    if (!make_layout(d, store, capacity_rows, max_queries, max_k, L, with_panel)) return IC_ERR_INVALID_ARG;
    if (arena_bytes < L.total) return IC_ERR_CAPACITY;
    ic_index *ix = new (std::nothrow) ic_index();
    if (!ix) return IC_ERR_OOM;
    ix->d = d;
    ix->store = store;
    ix->capacity = capacity_rows;
    ix->max_q = max_queries;
    ix->max_k = max_k;
    ix->L = L;
    ix->n = 0;
    ix->stream = (hipStream_t)stream;
    ix->slice_budget = 0;
    ix->compute_units = kComputeUnitsDefault;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
        ix->compute_units = cus;
    ix->device = dev;
    (void)hipGetLastError();
    uint8_t *base = (uint8_t *)arena_dev;
    ix->rows = base + L.off_rows;
    ix->panel = L.panel ? base + L.off_panel : nullptr;
    ix->scale = (store == IC_STORE_FP8_E4M3) ? (float *)(base + L.off_scale) : nullptr;
    ix->util = (float *)(base + L.off_util);
    ix->valid = base + L.off_valid;
    ix->block_offsets = (int64_t *)(base + L.off_blocks);
    ix->any_invalid = false;
    ix->domain = (int32_t *)(base + L.off_domain);
    Workspace &W = ix->ws;
    W.qbuf = base + L.off_qbuf;
    W.qpanel = L.panel ? base + L.off_qpanel : nullptr;
    W.qscale = (float *)(base + L.off_qscale);
    W.regions = (uint64_t *)(base + L.off_regions);
    W.counts = (int32_t *)(base + L.off_counts);
    W.list_a = (uint64_t *)(base + L.off_list_a);
    W.list_b = (uint64_t *)(base + L.off_list_b);
    W.consts = base + L.off_consts;
    W.bias = (float *)(base + L.off_bias);
    W.pilot_keys = (uint64_t *)(base + L.off_pilot);
    W.thr_init = (uint64_t *)(base + L.off_thr);
    const bool gemm = L.q_chunk >= kGemmMinQueries;
    W.glist = gemm ? (uint64_t *)(base + L.off_glist) : nullptr;
    W.gcount = gemm ? (int32_t *)(base + L.off_gcount) : nullptr;
    W.redo = gemm ? (int32_t *)(base + L.off_redo) : nullptr;
    W.over = gemm ? (uint32_t *)(base + L.off_over) : nullptr;
    W.q_chunk = L.q_chunk;
    W.region_slots = L.region_slots;
    W.consts_ready = &ix->consts_ready;
    ix->gemm_list_cap_override = 0;
    ix->timing = false;
    ix->events_used = 0;
    ix->consts_ready = false;
    *out = ix;
    return IC_OK;
}

ic_status ic_index_create(ic_index **out, int32_t d, ic_dtype store, int64_t capacity_rows,
                          int64_t max_queries, int32_t max_k, void *arena_dev, size_t arena_bytes,
                          void *stream) {
    return create_index(out, d, store, capacity_rows, max_queries, max_k, arena_dev, arena_bytes, stream, true);
}

ic_status ic_index_destroy(ic_index *index) {
    if (!index) return IC_ERR_INVALID_ARG;
    for (hipEvent_t e : index->events) (void)hipEventDestroy(e);
    delete index;
    return IC_OK;
}

int64_t ic_index_size(const ic_index *index) { return index ? index->n : -1; }

ic_status ic_index_set_stream(ic_index *index, void *stream) {
    if (!index) return IC_ERR_INVALID_ARG;
    index->stream = (hipStream_t)stream;
    return IC_OK;
}

ic_status ic_index_set_tuning(ic_index *index, int32_t slices, int32_t list_keys) {
    if (!index || slices < 0 || slices > kSliceBudgetMax || list_keys < 0 || list_keys > gemm_list_cap(index->max_k))
        return IC_ERR_INVALID_ARG;
    index->slice_budget = slices;
    index->gemm_list_cap_override = list_keys;
    return IC_OK;
}

ic_status ic_index_store_view(const ic_index *index, const void **rows_dev, int64_t *row_stride_bytes,
                              const float **scale_dev, const float **util_dev) {
    if (!index) return IC_ERR_INVALID_ARG;
    if (rows_dev) *rows_dev = index->rows;
    if (row_stride_bytes) *row_stride_bytes = index->L.row_bytes;
    if (scale_dev) *scale_dev = index->scale;
    if (util_dev) *util_dev = index->util;
    return IC_OK;
}

ic_status ic_index_set_timing(ic_index *index, int enable) {
    if (!index) return IC_ERR_INVALID_ARG;
    index->timing = enable != 0;
    index->events_used = 0;
    return IC_OK;
}

ic_status ic_index_scan_time_ms(ic_index *index, float *ms, int64_t *launches) {
    if (!index || !ms) return IC_ERR_INVALID_ARG;
    float total = 0.f;
    for (size_t i = 0; i + 1 < index->events_used; i += 2) {
        if (hipEventSynchronize(index->events[i + 1]) != hipSuccess) return IC_ERR_DEVICE;
        float t = 0.f;
        if (hipEventElapsedTime(&t, index->events[i], index->events[i + 1]) != hipSuccess)
            return IC_ERR_DEVICE;
        total += t;
    }
    *ms = total;
    if (launches) *launches = (int64_t)(index->events_used / 2);
    return IC_OK;
}

ic_status ic_index_tiled_scan_counts(ic_index *index, int64_t *tiles_again, int64_t *blocks_redone) {
    if (!index) return IC_ERR_INVALID_ARG;
    if (tiles_again) *tiles_again = 0;
    if (blocks_redone) *blocks_redone = 0;
    if (!index->ws.over || index->last_nblk64 == 0) return IC_OK;
    if (hipStreamSynchronize(index->stream) != hipSuccess) return IC_ERR_DEVICE;
    uint32_t listed = 0;
    std::vector<int32_t> flags((size_t)index->last_nblk64);
    if (hipMemcpy(&listed, index->ws.over, sizeof(listed), hipMemcpyDeviceToHost) != hipSuccess) return IC_ERR_DEVICE;
    if (hipMemcpy(flags.data(), index->ws.redo, flags.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess)
        return IC_ERR_DEVICE;
    if (tiles_again) *tiles_again = (int64_t)listed;
    if (blocks_redone)
        for (int32_t f : flags) *blocks_redone += f != 0;
    return IC_OK;
}

// Bring the step-major copy of the store up to date for rows [first, last): they are copied, and the
// rest of the last tile they touch is zeroed (rows past the end of the store must not hold stale
// bytes: the tiled scan multiplies whole tiles).
static void panel_rows(ic_index *index, int64_t first, int64_t last) {
    const int64_t fill_to = round_up(last, ic::kGemmTile);
    const int64_t granules = (fill_to - first) * (index->L.row_bytes / 16);
    if (granules <= 0) return;
    const int grid = (int)std::min<int64_t>((granules + 255) / 256, 65536);
    hipLaunchKernelGGL(ic::to_panel, dim3(grid), dim3(256), 0, index->stream, (const uint8_t *)index->rows,
                       index->L.row_bytes, first, last, fill_to, index->panel);
}

ic_status ic_index_append(ic_index *index, const float *emb_dev, const float *util_dev, int64_t n,
                          int64_t *first_id) {
    if (!index || n < 0 || (n > 0 && !emb_dev)) return IC_ERR_INVALID_ARG;
    if (index->n + n > index->capacity) return IC_ERR_CAPACITY;
    if (first_id) *first_id = index->n;
    if (n == 0) return IC_OK;
    const int64_t at = index->n;
    const int grid = (int)std::min<int64_t>((n + 3) / 4, 65536);
    uint8_t *dst = index->rows + at * (int64_t)index->L.row_bytes;
    float *util_dst = index->util + at;
    ic::launch_quantize_rows(index->store == IC_STORE_BF16 ? 0 : 1, (unsigned)grid, index->stream, emb_dev, n, n, index->d,
                             index->L.row_bytes, dst, index->store == IC_STORE_BF16 ? nullptr : index->scale + at, util_dev,
                             util_dst, index->panel, at);
    hipLaunchKernelGGL(ic::fill_bytes, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, index->stream,
                       index->valid + at, n, (uint8_t)1);
    hipLaunchKernelGGL(ic::fill_bytes, dim3((unsigned)((n * 4 + 255) / 256)), dim3(256), 0, index->stream,
                       (uint8_t *)(index->domain + at), n * 4, (uint8_t)0);  // new rows are shared with everyone
    // quantize_rows wrote the new rows into the step-major copy as well; the rest of their last tile is zeroed
    if (index->panel && (at + n) % ic::kGemmTile != 0) panel_rows(index, at + n, at + n);
    if (hipGetLastError() != hipSuccess) return IC_ERR_DEVICE;
    index->n += n;
    return IC_OK;
}

// ---- Example Manager maintenance (Sec. 4.3) --------------------------------------------------

ic_status ic_index_set_utility(ic_index *index, const int64_t *ids_dev, const float *util_dev, int64_t n) {
    if (!index || n < 0 || (n > 0 && (!ids_dev || !util_dev))) return IC_ERR_INVALID_ARG;
    if (n == 0) return IC_OK;
    hipLaunchKernelGGL(ic::set_utility, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, index->stream, ids_dev,
                       util_dev, n, index->util, index->n);
    return hipGetLastError() == hipSuccess ? IC_OK : IC_ERR_DEVICE;
}

ic_status ic_index_scale_utility(ic_index *index, float factor) {
    if (!index) return IC_ERR_INVALID_ARG;
    if (index->n == 0) return IC_OK;
    hipLaunchKernelGGL(ic::scale_utility, dim3((unsigned)((index->n + 255) / 256)), dim3(256), 0, index->stream,
                       index->util, index->n, factor);
    return hipGetLastError() == hipSuccess ? IC_OK : IC_ERR_DEVICE;
}

ic_status ic_index_invalidate(ic_index *index, const int64_t *ids_dev, int64_t n) {
    if (!index || n < 0 || (n > 0 && !ids_dev)) return IC_ERR_INVALID_ARG;
    if (n == 0) return IC_OK;
    hipLaunchKernelGGL(ic::invalidate_rows, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, index->stream, ids_dev,
                       n, index->valid, index->n);
    index->any_invalid = true;
    return hipGetLastError() == hipSuccess ? IC_OK : IC_ERR_DEVICE;
}

ic_status ic_index_set_domains(ic_index *index, const int64_t *ids_dev, const int32_t *domains_dev, int64_t n) {
    if (!index || n < 0 || (n > 0 && (!ids_dev || !domains_dev))) return IC_ERR_INVALID_ARG;
    if (n == 0) return IC_OK;
    hipLaunchKernelGGL(ic::set_domains, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, index->stream, ids_dev,
                       domains_dev, n, index->domain, index->n);
    return hipGetLastError() == hipSuccess ? IC_OK : IC_ERR_DEVICE;
}

ic_status ic_index_compact(ic_index *index, int64_t *id_map_dev, int64_t *new_size) {
    if (!index || !id_map_dev) return IC_ERR_INVALID_ARG;
    const int64_t n = index->n;
    if (new_size) *new_size = n;
    if (n == 0) return IC_OK;
    hipStream_t st = index->stream;
    const Layout &L = index->L;
    const int64_t nblocks = (n + ic::kScanBlock - 1) / ic::kScanBlock;
    int64_t *offs = index->block_offsets;
    hipLaunchKernelGGL(ic::count_valid, dim3((unsigned)nblocks), dim3(256), 0, st, index->valid, n, offs);
    hipLaunchKernelGGL(ic::scan_block_sums, dim3(1), dim3(256), 0, st, offs, nblocks);
    hipLaunchKernelGGL(ic::write_id_map, dim3((unsigned)nblocks), dim3(256), 0, st, index->valid, n, offs, id_map_dev);
    // rows, chunk by chunk through the candidate-region scratch (free between searches)
    uint8_t *bounce = (uint8_t *)index->ws.regions;
    const size_t bounce_bytes = (size_t)kRegionSlots * (size_t)region_cap(index->max_k) * 8;
    const int64_t chunk = std::max<int64_t>(ic::kScanBlock,
                                            (int64_t)(bounce_bytes / (size_t)L.row_bytes) / ic::kScanBlock * ic::kScanBlock);
    const int grid = std::max(8, index->compute_units) * 4;
    // A few block offsets come to the host (this call synchronises anyway): every `stride`-th, at most 64 of
    // them, which is a copy small enough to take the driver's quick path.  With the number of rows dropped
    // before a chunk known, a chunk that moves directly can be as long as that number, so the chunks grow as
    // the gap widens and a few dozen launches do what fixed chunks need hundreds for.  Between two sampled
    // offsets the chunks have the fixed size and the kernels decide for themselves, as they always can.
    int64_t stride = chunk / ic::kScanBlock;                 // in blocks; sampled positions are chunk boundaries
    while ((nblocks + stride - 1) / stride > 64) stride *= 2;
    const int picked = (int)((nblocks + stride - 1) / stride);
    int64_t *picked_dev = reinterpret_cast<int64_t *>(index->ws.bias);   // scratch of the searches, not in use here yet
    int64_t picked_h[64];
    hipLaunchKernelGGL(ic::pick_offsets, dim3(1), dim3(64), 0, st, offs, stride, picked, picked_dev);
    if (hipMemcpyAsync(picked_h, picked_dev, (size_t)picked * sizeof(int64_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return IC_ERR_DEVICE;
    const int64_t span = stride * ic::kScanBlock;            // rows between two sampled offsets
    for (int64_t lo = 0; lo < n;) {
        int64_t hi = std::min(n, lo + chunk);
        bool direct = false;
        if (lo % span == 0) {
            const int64_t dropped = lo - picked_h[lo / span];
            if (dropped >= span) {   // gather_rows sees lo - first_new >= hi - lo and writes the rows in place
                hi = std::min(n, lo + dropped / span * span);
                direct = true;
            }
        }
        hipLaunchKernelGGL(ic::gather_rows, dim3(grid), dim3(256), 0, st, index->rows, L.row_bytes, id_map_dev, offs, lo, hi,
                           bounce, index->panel);
        if (!direct)
            hipLaunchKernelGGL(ic::store_rows, dim3(grid), dim3(256), 0, st, index->rows, L.row_bytes, offs, lo, hi,
                               (hi + ic::kScanBlock - 1) / ic::kScanBlock, bounce, index->panel);
        lo = hi;
    }
    // side arrays through the per-search bias scratch
    const unsigned g1 = (unsigned)((n + 255) / 256);
    hipLaunchKernelGGL(ic::scatter_f32, dim3(g1), dim3(256), 0, st, index->util, id_map_dev, n, index->ws.bias);
    hipLaunchKernelGGL(ic::copy_f32_counted, dim3(g1), dim3(256), 0, st, index->ws.bias, offs + nblocks, index->util);
    if (index->scale) {
        hipLaunchKernelGGL(ic::scatter_f32, dim3(g1), dim3(256), 0, st, index->scale, id_map_dev, n, index->ws.bias);
        hipLaunchKernelGGL(ic::copy_f32_counted, dim3(g1), dim3(256), 0, st, index->ws.bias, offs + nblocks, index->scale);
    }
    // the domains are moved as 32-bit words (the copies do no arithmetic)
    hipLaunchKernelGGL(ic::scatter_f32, dim3(g1), dim3(256), 0, st, (const float *)index->domain, id_map_dev, n, index->ws.bias);
    hipLaunchKernelGGL(ic::copy_f32_counted, dim3(g1), dim3(256), 0, st, index->ws.bias, offs + nblocks, (float *)index->domain);
    hipLaunchKernelGGL(ic::fill_bytes, dim3(g1), dim3(256), 0, st, index->valid, n, (uint8_t)1);
    int64_t total = 0;
    if (hipMemcpyAsync(&total, offs + nblocks, sizeof(int64_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return IC_ERR_DEVICE;
    index->n = total;
    index->any_invalid = false;
    if (new_size) *new_size = total;
    if (index->panel) panel_rows(index, total, total);   // the moved rows wrote their copies; the rest of the last tile is zeroed
    return hipGetLastError() == hipSuccess ? IC_OK : IC_ERR_DEVICE;
}

namespace {

// Chain merge_lists launches from the given first level down to one group per query, then
// write the final rows.  `m` describes the first level; out pointers are for this query block.
struct FinalOpts {          // how the last merge level writes a query's row of the result
    float min_score;        // entries below it are dropped (threshold mode); -inf: keep all
    int32_t *counts;        // [qc] entries kept per query, or NULL
    int64_t self_first;     // self-search: query j of the block is stored row self_first + j, which is
                            // left out of its own result (the lists then hold k + 1 keys); -1: off
};

void run_merge(ic_index *index, const Workspace &W, ic::MergeArgs m, int qc, int k, float *out_scores, int64_t *out_ids,
               const int32_t *only_flagged, const FinalOpts &fo) {
    hipStream_t st = index->stream;
    uint64_t *ping = W.list_a, *pong = W.list_b;
    m.k = k;
    m.kth_out = nullptr;
    m.out_scores = out_scores;
    m.out_ids = out_ids;
    m.only_flagged = only_flagged;
    m.min_score = fo.min_score;
    m.out_counts = fo.counts;
    m.self_first = fo.self_first;
    m.k_out = fo.self_first >= 0 ? k - 1 : k;
    for (;;) {
        const int G = std::max(1, (m.nseg + m.segs_per_wg - 1) / m.segs_per_wg);
        m.dst = (G == 1) ? nullptr : ping;
        hipLaunchKernelGGL(ic::merge_lists, dim3(qc, G), dim3(256), 0, st, m);
        if (G == 1) break;
        m.src = ping;
        m.q_stride = (int64_t)G * k;
        m.seg_stride = k;
        m.seg_cap = k;
        m.seg_counts = nullptr;
        m.total_counts = nullptr;
        m.id_map = nullptr;  // applied by the first level
        m.nseg = G;
        m.segs_per_wg = std::min(ic::kMergeMaxSegs, ic::kMergeKeys / k);
        std::swap(ping, pong);
    }
}

struct Timer {  // brackets the dominant kernel of a search with events when timing is on
    ic_index *index;
    bool on;
    bool allowed;
    Timer(ic_index *ix, bool may) : index(ix), on(false), allowed(may) {}
    bool start() {
        on = allowed && index->timing && index->events_used + 2 <= kMaxTimedEvents;
        if (!on) return true;
        while (index->events.size() < index->events_used + 2) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return false;
            index->events.push_back(e);
        }
        (void)hipEventRecord(index->events[index->events_used], index->stream);
        return true;
    }
    void stop() {
        if (!on) return;
        (void)hipEventRecord(index->events[index->events_used + 1], index->stream);
        index->events_used += 2;
    }
};

}  // namespace

namespace {
struct SearchReq {                      // where the queries come from and how the result rows are written
    const float *q_dev = nullptr;       // [Q, d] fp32 queries to normalise and quantise, or
    const uint8_t *q_rows = nullptr;    // [Q] rows already in the store's format, row_bytes apart,
    const float *q_row_scale = nullptr; //     with their scales (fp8)
    int64_t self_first = -1;            // q_rows are this index's own rows from here on: each is left out
    float min_score = -INFINITY;        // threshold mode
    int32_t *counts = nullptr;
    const int32_t *q_domain = nullptr;  // [Q] sharing domain of every query: rows of other domains are not returned
};
ic_status search_impl(ic_index *index, const Workspace &W, int64_t Q, int32_t k, float lambda,
                      const uint8_t *mask_dev, float *out_scores_dev, int64_t *out_ids_dev, const SearchReq &req);
}

ic_status ic_search(const ic_index *cindex, const float *q_dev, int64_t Q, int32_t k, float lambda,
                    const uint8_t *mask_dev, float *out_scores_dev, int64_t *out_ids_dev) {
    SearchReq r;
    r.q_dev = q_dev;
    if (Q > 0 && !q_dev) return IC_ERR_INVALID_ARG;
    return search_impl(const_cast<ic_index *>(cindex), cindex->ws, Q, k, lambda, mask_dev, out_scores_dev, out_ids_dev, r);
}

ic_status ic_self_search(const ic_index *cindex, int64_t first_row, int64_t count, int32_t k, float lambda,
                         const uint8_t *mask_dev, float *out_scores_dev, int64_t *out_ids_dev) {
    if (!cindex || first_row < 0 || count < 0 || first_row + count > cindex->n) return IC_ERR_INVALID_ARG;
    if (k < 1 || k + 1 > cindex->max_k) return IC_ERR_INVALID_ARG;  // the lists hold the row itself as well
    SearchReq r;
    r.q_rows = cindex->rows + first_row * (int64_t)cindex->L.row_bytes;
    r.q_row_scale = cindex->scale ? cindex->scale + first_row : nullptr;
    r.self_first = first_row;
    return search_impl(const_cast<ic_index *>(cindex), cindex->ws, count, k, lambda, mask_dev, out_scores_dev, out_ids_dev, r);
}

ic_status ic_search_domains(const ic_index *cindex, const float *q_dev, int64_t Q, int32_t k, float lambda,
                            const uint8_t *mask_dev, const int32_t *query_domain_dev, float *out_scores_dev,
                            int64_t *out_ids_dev) {
    if (Q > 0 && (!q_dev || !query_domain_dev)) return IC_ERR_INVALID_ARG;
    SearchReq r;
    r.q_dev = q_dev;
    r.q_domain = query_domain_dev;
    return search_impl(const_cast<ic_index *>(cindex), cindex->ws, Q, k, lambda, mask_dev, out_scores_dev, out_ids_dev, r);
}

ic_status ic_search_threshold(const ic_index *cindex, const float *q_dev, int64_t Q, int32_t k, float lambda,
                              const uint8_t *mask_dev, float min_score, float *out_scores_dev,
                              int64_t *out_ids_dev, int32_t *out_counts_dev) {
    if (min_score != min_score) return IC_ERR_INVALID_ARG;  // NaN
    SearchReq r;
    r.q_dev = q_dev;
    r.min_score = min_score;
    r.counts = out_counts_dev;
    if (Q > 0 && !q_dev) return IC_ERR_INVALID_ARG;
    return search_impl(const_cast<ic_index *>(cindex), cindex->ws, Q, k, lambda, mask_dev, out_scores_dev, out_ids_dev, r);
}

namespace {
ic_status search_impl(ic_index *index, const Workspace &W, int64_t Q, int32_t k_out, float lambda,
                      const uint8_t *mask_dev, float *out_scores_dev, int64_t *out_ids_dev, const SearchReq &req) {
    const float *q_dev = req.q_dev;
    const float min_score = req.min_score;
    int32_t *out_counts_dev = req.counts;
    const int64_t self_first = req.self_first;
    const bool self = self_first >= 0;
    const int32_t k = self ? k_out + 1 : k_out;  // what the scans and merges select
    if (!index || Q < 0 || k_out < 1 || k > index->max_k) return IC_ERR_INVALID_ARG;
    if (Q == 0) return IC_OK;
    if ((!q_dev && !req.q_rows) || !out_scores_dev || !out_ids_dev) return IC_ERR_INVALID_ARG;

    const Layout &L = index->L;
    const int et = (index->store == IC_STORE_BF16) ? 0 : 1;
    const int nchunks = L.row_bytes / 64;
    const int cpw = chunks_per_wavefront(nchunks);
    const int64_t n = index->n;
    const int64_t ntiles = (n + 15) / 16;
    hipStream_t st = index->stream;
    const bool pilot_ok = ntiles >= kPilotMinTiles;
    // batches large enough for the matrix cores to be the bound take the MFMA-tiled scan; it
    // needs the pilot's thresholds and the per-query candidate lists
    // (measured on 100k-250k rows: 1.5 to 2 times faster than the streaming scan from 256 queries on,
    // about even at 128)
    auto gemm_for = [&](int64_t queries) {
        return W.glist != nullptr && index->panel != nullptr && W.qpanel != nullptr && queries >= kGemmMinQueries &&
               (ntiles >= kGemmMinTiles || (ntiles >= kGemmSmallTiles && queries > 128) ||
                (ntiles >= kGemmTinyTiles && queries > 128 && k <= 16));
    };

    if (!*W.consts_ready) {
        hipLaunchKernelGGL(init_consts, dim3(1), dim3(64), 0, st, (uint32_t *)W.consts);
        *W.consts_ready = true;
    }

    // a4 (first half): per-row additive term, once per search.  The tiled scan always reads it
    // (it marks the padding rows of the last tile); the streaming scan only if it is not all zero.
    const bool any_gemm = gemm_for(std::min<int64_t>(Q, W.q_chunk));
    const bool use_bias = (lambda != 0.0f) || mask_dev != nullptr || any_gemm || index->any_invalid;
    if (use_bias && n > 0) {
        const int64_t n_pad = round_up(n, ic::kGemmTile);
        const int grid = (int)std::min<int64_t>((n_pad + 255) / 256, 4096);
        hipLaunchKernelGGL(ic::make_bias, dim3(grid), dim3(256), 0, st,
                           (lambda != 0.0f) ? (const float *)index->util : (const float *)nullptr, mask_dev,
                           index->any_invalid ? (const uint8_t *)index->valid : (const uint8_t *)nullptr, n, n_pad,
                           lambda, W.bias);
    }

    for (int64_t q0 = 0; q0 < Q; q0 += W.q_chunk) {
        const int qc = (int)std::min<int64_t>(W.q_chunk, Q - q0);
        const bool gemm = gemm_for(qc);
        const int qg_idx = gemm ? 2 : (qc <= 16 ? 0 : (qc <= 32 ? 1 : 2));
        const int qb_rows = 16 << qg_idx;
        const int cap = region_cap_for(k, qg_idx);
        const int nqb = (qc + qb_rows - 1) / qb_rows;                      // blocks of the streaming scan
        const int nqb_gemm = (qc + ic::kGemmTile - 1) / ic::kGemmTile;     // blocks of the tiled scan
        const int q_pad = gemm ? nqb_gemm * ic::kGemmTile : nqb * qb_rows;
        float *out_s = out_scores_dev + q0 * (int64_t)k_out;
        int64_t *out_i = out_ids_dev + q0 * (int64_t)k_out;
        const FinalOpts fo{min_score, out_counts_dev ? out_counts_dev + q0 : nullptr, self ? self_first + q0 : -1};

        // a2: unit-normalise the queries and write them in the store's format; a self-search
        // takes the rows as they are stored (same format, already normalised)
        if (req.q_rows) {
            if (hipMemcpyAsync(W.qbuf, req.q_rows + q0 * (int64_t)L.row_bytes, (size_t)qc * L.row_bytes,
                               hipMemcpyDeviceToDevice, st) != hipSuccess)
                return IC_ERR_DEVICE;
            if (et == 1 && hipMemcpyAsync(W.qscale, req.q_row_scale + q0, (size_t)qc * 4,
                                          hipMemcpyDeviceToDevice, st) != hipSuccess)
                return IC_ERR_DEVICE;
            if (q_pad > qc)   // the padding queries of the last block: zero rows, like the ones quantize_rows writes
                hipLaunchKernelGGL(ic::fill_bytes, dim3((unsigned)(((int64_t)(q_pad - qc) * L.row_bytes + 255) / 256)),
                                   dim3(256), 0, st, W.qbuf + (int64_t)qc * L.row_bytes,
                                   (int64_t)(q_pad - qc) * L.row_bytes, (uint8_t)0);
        } else {
            const int grid = (q_pad + 3) / 4;
            const float *src = q_dev + q0 * (int64_t)index->d;
            ic::launch_quantize_rows(et, (unsigned)grid, st, src, (int64_t)qc, (int64_t)q_pad, index->d, L.row_bytes, W.qbuf,
                                     et == 0 ? nullptr : W.qscale, nullptr, nullptr, gemm ? W.qpanel : nullptr, 0);
        }

        if (gemm && req.q_rows) {   // stored rows as queries: their step-major copy (quantize_rows writes both at once)
            const int64_t granules = (int64_t)q_pad * (L.row_bytes / 16);
            hipLaunchKernelGGL(ic::to_panel, dim3((unsigned)std::min<int64_t>((granules + 255) / 256, 65536)), dim3(256), 0, st,
                               (const uint8_t *)W.qbuf, L.row_bytes, (int64_t)0, (int64_t)q_pad, (int64_t)q_pad, W.qpanel);
        }

        if (n == 0) {  // nothing to scan: the merge of zero segments writes the padding rows
            ic::MergeArgs m{};
            m.src = W.regions;
            m.q_stride = 0;
            m.seg_stride = cap;
            m.seg_cap = cap;
            m.seg_counts = W.counts;
            m.nseg = 0;
            m.segs_per_wg = 1;
            run_merge(index, W, m, qc, k, out_s, out_i, nullptr, fo);
            continue;
        }

        // a3-a5: similarity, score epilogue and selection
        ic::ScanArgs a{};
        a.store = index->rows;
        a.n = n;
        a.row_bytes = L.row_bytes;
        a.row_scale = index->scale;
        a.bias = use_bias ? W.bias : (const float *)W.consts;
        a.bias_stride = use_bias ? 1 : 0;
        a.qbuf = W.qbuf;
        a.q_scale = W.qscale;
        a.Q = qc;
        a.k = k;
        a.cap = cap;
        a.regions = W.regions;
        a.counts = W.counts;
        a.pilot_out = W.pilot_keys;
        a.thr_init = nullptr;
        a.redo = nullptr;
        a.thr_slack = 0.0f;
        a.tile_mul = 1;
        a.row_dom = index->domain;
        a.q_dom = req.q_domain ? req.q_domain + q0 : nullptr;
        const auto &scan_table = req.q_domain ? kScanTableDom : kScanTable;

        // slices of the streaming scan: one workgroup per slice and query block; by default as
        // many as are resident at once (two per compute unit by registers, fewer when the
        // candidate regions fill the LDS)
        int budget = index->slice_budget;
        if (budget == 0) {
            const size_t lds = ic::scan_lds_bytes(1 << qg_idx, cap);
            const int per_cu = (int)std::min<size_t>(2, std::max<size_t>(1, kLdsPerCu / lds));
            budget = std::min(kSliceBudgetMax, index->compute_units * per_cu);
        }
        budget = (int)std::min<int64_t>(budget, W.region_slots / qb_rows);   // what the candidate regions hold
        int S = (int)std::min<int64_t>(std::max<int64_t>(1, budget / nqb), ntiles);
        // after the tiled scan the streaming kernel only redoes flagged blocks (nearly always none, and the
        // other workgroups return at once): a block gets kRedoSlices workgroups, not its share of one resident grid
        if (gemm && index->slice_budget == 0)
            S = (int)std::min<int64_t>(std::max<int64_t>(S, std::min<int64_t>(kRedoSlices, W.region_slots / ((int64_t)nqb * qb_rows))), ntiles);
        // Threshold pilot: a pass over a strided sample of the rows that keeps the best score
        // per (query, slice); the k-th largest of a query's slice maxima is reached by at least
        // k rows, so the full scan may start from it.
        const int gemm_grid = std::max(8, index->compute_units / 8 * 8);
        bool sparse_regions = false;   // the streaming pilot leaves so few candidates that one merge level will do
        ic::GemmArgs g{};
        int64_t gemm_stride = 1;       // row stride of the tiled scan's pilot
        if (gemm) {
            g.store = index->rows;
            g.panel = index->panel;
            g.qpanel = W.qpanel;
            g.n = n;
            g.row_bytes = L.row_bytes;
            g.row_scale = index->scale;
            g.bias = W.bias;
            g.qbuf = W.qbuf;
            g.q_scale = W.qscale;
            g.Q = qc;
            g.nqb = nqb_gemm;
            g.ntiles = (n + ic::kGemmTile - 1) / ic::kGemmTile;
            g.row_stride = 1;
            g.n_sampled = n;
            g.self_first = fo.self_first;
            g.row_dom = index->domain;
            g.q_dom = a.q_dom;
            g.gq = 1;  // query-block groups: enough that a group's blocks stay in an XCD's L2
            while (g.gq < 8 && (size_t)((nqb_gemm + g.gq - 1) / g.gq) * ic::kGemmTile * L.row_bytes > kL2Share) g.gq *= 2;
        }
        if (gemm) {
            // The pilot of the tiled scan is the tiled scan itself over every 32nd (small k: 64th)
            // row of the store; a tile takes 256 sampled rows spread evenly over the whole store and
            // a slice is the set of tiles with the same index modulo kPilotSlices, so every slice is
            // a uniform sample even when the rows arrived sorted by topic.  Starting from its
            // threshold about stride * k rows per query pass.
            ic::GemmArgs p = g;
            const int64_t want = (k <= 16) ? 64 : 32;
            // at least max(k, 64) sampled tiles, so that the k-th largest slice maximum exists
            // and dense enough that a tile of 256 x 256 scores has about 24 or fewer above the thresholds
            // (256 queries x stride * k rows per query x 256 / n rows): the per-tile hit list holds 96
            const int64_t by_hits = g.ntiles * 3 / (32 * (int64_t)k);
            const int64_t most = std::min<int64_t>(want, g.ntiles / std::max(k, 64));
            p.row_stride = std::max<int64_t>(1, std::min<int64_t>(by_hits, most));
            // a pilot of a few rounds of the grid: a slightly sparser sample (up to half again as many hits per
            // tile) that saves a whole round is the cheaper one
            auto rounds = [&](int64_t stride) {
                const int64_t tiles = ((n + stride - 1) / stride + ic::kGemmTile - 1) / ic::kGemmTile * nqb_gemm;
                return (tiles + gemm_grid - 1) / gemm_grid;
            };
            if (rounds(p.row_stride) <= 3) {
                for (int64_t s2 = p.row_stride + 1; s2 <= std::min<int64_t>(most, p.row_stride * 3 / 2); ++s2) {
                    if (rounds(s2) < rounds(p.row_stride)) {
                        p.row_stride = s2;
                        break;
                    }
                }
            }
            gemm_stride = p.row_stride;
            p.n_sampled = (n + p.row_stride - 1) / p.row_stride;
            p.ntiles = (p.n_sampled + ic::kGemmTile - 1) / ic::kGemmTile;
            p.pilot_out = W.pilot_keys;
            p.pilot_stride = kPilotSlices;
            const int64_t nkeys = (int64_t)qc * kPilotSlices;
            hipLaunchKernelGGL(ic::gemm_reset, dim3((unsigned)((nkeys + 255) / 256)), dim3(256), 0, st, W.pilot_keys, nkeys,
                               W.gcount, qc, W.redo, (qc + 63) / 64, W.over);
            if (et == 0) launch_gemm<0, true>(gemm_grid, st, p);
            else launch_gemm<1, true>(gemm_grid, st, p);
            ic::MergeArgs m{};
            m.src = W.pilot_keys;
            m.q_stride = kPilotSlices;
            m.seg_stride = kPilotSlices;
            m.seg_cap = (int)std::min<int64_t>(kPilotSlices, p.ntiles);
            m.nseg = 1;
            m.segs_per_wg = 1;
            m.k = k;
            m.kth_out = W.thr_init;
            hipLaunchKernelGGL(ic::merge_lists, dim3(qc, 1), dim3(256), 0, st, m);
            a.thr_init = W.thr_init;
        } else if (pilot_ok && ((qc >= 8 && (int64_t)qc * k >= kPilotMinWork) || (qc >= 4 && (int64_t)qc * k >= 6 * kPilotMinWork) ||
                                (qc >= kPilotMinQueries && ntiles >= kGemmMinTiles))) {
            // It pays when the selection is a visible part of the scan: several queries and a k that
            // is not tiny (measured break-even: about 8 queries x k = 16), always from 9 queries on
            // a large store; a single query never needs it.
            // Stride of the sample: every slice of the pilot keeps at least one tile, and starting
            // from its threshold about stride * k rows per query pass, which should leave a region
            // of the full scan (S of them per query) with 8 candidates or fewer (more of them cost
            // more in the merges than the sparser pilot saves).
            ic::ScanArgs p = a;
            p.S = kPilotSlices;
            const int64_t by_regions = std::max<int64_t>(4, 8 * (int64_t)S / k);
            p.tile_mul = (int)std::min<int64_t>(std::min<int64_t>(128, ntiles / kPilotSlices), by_regions);
            sparse_regions = (int64_t)p.tile_mul * k <= ic::kMergeKeys / 2;   // about tile_mul * k rows pass per query
            scan_table[1][et][qg_idx][cpw - 1](dim3(kPilotSlices, nqb), st, p);
            ic::MergeArgs m{};
            m.src = W.pilot_keys;
            m.q_stride = kPilotSlices;
            m.seg_stride = kPilotSlices;
            m.seg_cap = kPilotSlices;
            m.nseg = 1;
            m.segs_per_wg = 1;
            m.k = k;
            m.kth_out = W.thr_init;
            hipLaunchKernelGGL(ic::merge_lists, dim3(qc, 1), dim3(256), 0, st, m);
            a.thr_init = W.thr_init;
        }

        a.S = S;
        Timer timer(index, W.timed);

        if (gemm) {
            const int gcap = index->gemm_list_cap_override ? index->gemm_list_cap_override : gemm_list_cap(k);
            const int nblk64 = (qc + 63) / 64;
            index->last_nblk64 = nblk64;
            g.thr_init = W.thr_init;
            g.glist = W.glist;
            g.gcap = gcap;
            g.gcount = W.gcount;
            g.redo = W.redo;
            g.over_n = W.over;
            g.over_list = reinterpret_cast<uint2 *>(W.over + 2);
            g.over_cap = kGemmOverCap;
            if (!timer.start()) return IC_ERR_DEVICE;
            if (et == 0) launch_gemm<0, false>(gemm_grid, st, g);
            else launch_gemm<1, false>(gemm_grid, st, g);
            timer.stop();
            // tiles with more hits than the per-tile list holds were listed instead: a second launch
            // does them again (its workgroups find the list empty, nearly always, and return)
            if (et == 0) launch_gemm_again<0>(gemm_grid, st, g);
            else launch_gemm_again<1>(gemm_grid, st, g);

            // blocks whose candidate lists overflowed are redone by the streaming scan; the
            // thresholds come from the other kernel, hence the slack (1e-4 bounds the difference
            // between two fp32 summation orders of a dot product of unit vectors)
            a.redo = W.redo;
            a.thr_slack = 1e-4f;
            scan_table[0][et][qg_idx][cpw - 1](dim3(S, nqb), st, a);

            ic::MergeArgs m{};
            m.src = W.glist;
            m.q_stride = gcap;
            m.seg_cap = std::min(gcap, kGemmListSeg);
            m.seg_stride = m.seg_cap;
            m.total_counts = W.gcount;
            m.nseg = (gcap + m.seg_cap - 1) / m.seg_cap;
            // about stride * k keys per query passed the pilot's threshold: when that is well inside one
            // sort, one workgroup per query takes the whole list (one launch; a longer list is merged in
            // rounds), otherwise the segments are sorted side by side and merged by a second level
            m.segs_per_wg = (gemm_stride * k <= kGemmListSeg / 2) ? m.nseg : 1;
            run_merge(index, W, m, qc, k, out_s, out_i, nullptr, fo);
        } else {
            if (!timer.start()) return IC_ERR_DEVICE;
            scan_table[0][et][qg_idx][cpw - 1](dim3(S, nqb), st, a);
            timer.stop();
        }

        // a6: merge the S candidate regions of every query (after the tiled scan: only the
        // blocks that were redone)
        ic::MergeArgs m{};
        m.src = W.regions;
        m.q_stride = (int64_t)S * cap;
        m.seg_stride = cap;
        m.seg_cap = cap;
        m.seg_counts = W.counts;
        m.nseg = S;
        // after a pilot the regions hold a handful of keys each, so a workgroup takes as many as
        // it may (fewer, smaller lists for the next level; a rare full group is merged in rounds);
        // without one they may be full, and more workgroups with one round each are faster
        m.segs_per_wg = a.thr_init ? ic::kMergeMaxSegs : std::min(ic::kMergeMaxSegs, ic::kMergeKeys / cap);
        // few candidates in all (a pilot that sampled densely, on a small store): one workgroup per query
        // takes every slice, one launch instead of two (more than it can sort at once is merged in rounds)
        if (sparse_regions && S <= ic::kMergeWideSegs) m.segs_per_wg = S;
        // after the tiled scan only flagged blocks have regions at all (nearly always none): one launch
        if (gemm && S <= ic::kMergeWideSegs) m.segs_per_wg = S;
        run_merge(index, W, m, qc, k, out_s, out_i, gemm ? W.redo : nullptr, fo);
    }
    if (hipGetLastError() != hipSuccess) return IC_ERR_DEVICE;
    return IC_OK;
}
}  // namespace

// ---- a search whose scratch is a static device array (for callers that cannot allocate) -------

namespace {
constexpr int kStaticQueries = IC_STATIC_MAX_QUERIES;
constexpr int64_t kStaticRows = IC_STATIC_MAX_ROWS;
constexpr int64_t kStaticRegionSlots = (int64_t)kStaticQueries * 512;   // 64 queries x 512 slices
constexpr int kStaticDevices = 64;

struct StaticLayout {
    size_t off_qbuf, off_qscale, off_consts, off_pilot, off_thr, off_counts, off_list_a, off_list_b, off_bias,
        off_regions, total;
};
constexpr size_t static_up(size_t x) { return (x + (size_t)kAlign - 1) / (size_t)kAlign * (size_t)kAlign; }
constexpr StaticLayout make_static_layout() {
    StaticLayout S{};
    size_t off = 0;
    S.off_qbuf = off;     off = static_up(off + (size_t)kStaticQueries * kMaxRowBytes);
    S.off_qscale = off;   off = static_up(off + (size_t)kStaticQueries * 4);
    S.off_consts = off;   off = static_up(off + 64);
    S.off_pilot = off;    off = static_up(off + (size_t)kStaticQueries * kPilotSlices * 8);
    S.off_thr = off;      off = static_up(off + (size_t)kStaticQueries * 8);
    S.off_counts = off;   off = static_up(off + (size_t)kStaticRegionSlots * 4);
    S.off_list_a = off;   off = static_up(off + (size_t)(kStaticRegionSlots / 8 + kStaticQueries) * IC_MAX_K * 8);
    S.off_list_b = off;   off = static_up(off + (size_t)(kStaticRegionSlots / 8 + kStaticQueries) * IC_MAX_K * 8);
    S.off_bias = off;     off = static_up(off + (size_t)kStaticRows * 4);
    S.off_regions = off;  off = static_up(off + (size_t)kStaticRegionSlots * ic::kMaxCap * 8);
    S.total = off;
    return S;
}
constexpr StaticLayout kStaticLayout = make_static_layout();
static_assert(kStaticLayout.total <= (size_t)IC_STATIC_SCRATCH_BYTES, "the static scratch holds the workspace");
}  // namespace

// The scratch itself: one copy per GPU the library runs on, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress; the device address it yields is what
// the kernels get.
static __device__ __align__(256) unsigned char scratch[IC_STATIC_SCRATCH_BYTES];

namespace {
struct StaticState {
    unsigned char *ptr = nullptr;   // device address of `scratch` on this GPU
    bool consts_ready = false;
};
StaticState g_static[kStaticDevices];
std::mutex g_static_mutex;
}  // namespace

extern "C" ic_status ic_search_static(const ic_index *cindex, const float *q_dev, int64_t Q, int32_t k, float lambda,
                                      const uint8_t *mask_dev, float *out_scores_dev, int64_t *out_ids_dev) {
    if (!cindex || Q < 0 || (Q > 0 && !q_dev)) return IC_ERR_INVALID_ARG;
    if (Q > kStaticQueries || round_up(cindex->n, ic::kGemmTile) > kStaticRows) return IC_ERR_UNSUPPORTED;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return IC_ERR_DEVICE;
    if (dev < 0 || dev >= kStaticDevices) return IC_ERR_UNSUPPORTED;
    if (dev != cindex->device) return IC_ERR_INVALID_ARG;   // the index lives on another GPU than the current one
    std::lock_guard<std::mutex> lock(g_static_mutex);
    StaticState &st = g_static[dev];
    if (!st.ptr) {   // once per device, with that device current: every GPU has its own copy at its own address
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return IC_ERR_DEVICE;
        }
        st.ptr = static_cast<unsigned char *>(p);
    }
    constexpr StaticLayout S = kStaticLayout;
    Workspace W;
    W.qbuf = st.ptr + S.off_qbuf;
    W.qscale = (float *)(st.ptr + S.off_qscale);
    W.consts = st.ptr + S.off_consts;
    W.pilot_keys = (uint64_t *)(st.ptr + S.off_pilot);
    W.thr_init = (uint64_t *)(st.ptr + S.off_thr);
    W.counts = (int32_t *)(st.ptr + S.off_counts);
    W.list_a = (uint64_t *)(st.ptr + S.off_list_a);
    W.list_b = (uint64_t *)(st.ptr + S.off_list_b);
    W.bias = (float *)(st.ptr + S.off_bias);
    W.regions = (uint64_t *)(st.ptr + S.off_regions);
    W.q_chunk = kStaticQueries;
    W.region_slots = kStaticRegionSlots;
    W.consts_ready = &st.consts_ready;
    W.timed = false;   // timing creates events; this call creates nothing
    SearchReq r;
    r.q_dev = q_dev;
    return search_impl(const_cast<ic_index *>(cindex), W, Q, k, lambda, mask_dev, out_scores_dev, out_ids_dev, r);
}

// ---- cluster pruning (Sec. 4.1: K-Means clusters offline, nearest clusters first online) ------

struct ic_ivf {
    ic_index *base;      // the index being accelerated (not owned)
    ic_index *cent;      // K centroids, same format as the store
    ic_index *sorted;    // copy of the live rows of base, sorted by cluster
    int32_t K, max_probe;
    int32_t *assign;     // [base size] cluster of every row
    int32_t *perm;       // [rows in lists] sorted position -> id in base
    int64_t *counts, *offsets, *cursor;  // [K], [K + 1], [K]
    float *sums;         // [K, d] K-Means update scratch
    long long *acc64;    // [K, d] fixed-point sums of the update in progress
    int64_t *tmp_ids;    // [base capacity] assignment search result
    float *tmp_scores;
    int64_t *probe_ids;  // [query chunk, max_probe]
    float *probe_scores;
    int64_t *task_list;  // [kTaskPairs] list of every scan task of a pass
    int32_t *task_pair;  // [kTaskPairs, kTaskSlots] (query, list) pairs a task serves
    bool lists_ready;
};

namespace {
constexpr int64_t kIvfCentQueries = 4096;  // query chunk of the centroid index (assignment passes)
constexpr int kIvfShares = 16;             // workgroups that share the rows of one cluster in the K-Means update

struct IvfLayout {
    size_t off_cent = 0, off_sorted = 0, off_assign = 0, off_perm = 0, off_counts = 0, off_offsets = 0,
           off_cursor = 0, off_sums = 0, off_acc64 = 0, off_tmp_ids = 0, off_tmp_scores = 0, off_probe_ids = 0,
           off_probe_scores = 0, off_task_list = 0, off_task_pair = 0, total = 0;
    size_t cent_bytes = 0, sorted_bytes = 0;
};

bool make_ivf_layout(const ic_index *base, int32_t K, int32_t max_probe, IvfLayout &V) {
    if (!base || K < 1 || K > (1 << 20) || max_probe < 1 || max_probe > IC_MAX_K) return false;
    V.cent_bytes = ic_workspace_bytes(base->d, base->store, K, kIvfCentQueries, max_probe);
    Layout LS;   // the sorted copy is only scanned list by list (streaming kernel): no step-major copy of its rows
    V.sorted_bytes = make_layout(base->d, base->store, base->capacity, base->max_q, base->max_k, LS, false) ? LS.total : 0;
    if (!V.cent_bytes || !V.sorted_bytes) return false;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = (size_t)round_up((int64_t)(off + bytes), kAlign);
        return at;
    };
    const size_t cap = (size_t)base->L.cap_pad;
    V.off_cent = take(V.cent_bytes);
    V.off_sorted = take(V.sorted_bytes);
    V.off_assign = take(cap * 4);
    V.off_perm = take(cap * 4);
    V.off_counts = take((size_t)K * 8);
    V.off_offsets = take((size_t)(K + 1) * 8);
    V.off_cursor = take((size_t)K * 8);
    V.off_sums = take((size_t)K * (size_t)base->d * 4);
    V.off_acc64 = take((size_t)K * (size_t)base->d * 8);
    V.off_tmp_ids = take(cap * 8);
    V.off_tmp_scores = take(cap * 4);
    V.off_probe_ids = take((size_t)base->L.q_chunk * (size_t)max_probe * 8);
    V.off_probe_scores = take((size_t)base->L.q_chunk * (size_t)max_probe * 4);
    V.off_task_list = take((size_t)ic::kTaskPairs * 8);
    V.off_task_pair = take((size_t)ic::kTaskPairs * ic::kTaskSlots * 4);
    V.total = off;
    return true;
}

// lists and sorted copy from ivf->assign
ic_status ivf_build_lists(ic_ivf *v) {
    ic_index *b = v->base, *s = v->sorted;
    hipStream_t st = b->stream;
    const int64_t n = b->n;
    const unsigned gk = (unsigned)((v->K + 255) / 256), gn = (unsigned)((std::max<int64_t>(n, 1) + 255) / 256);
    hipLaunchKernelGGL(ic::ivf_zero_i64, dim3(gk), dim3(256), 0, st, v->counts, (int64_t)v->K);
    if (n > 0)
        hipLaunchKernelGGL(ic::ivf_histogram, dim3(gn), dim3(256), 0, st, v->assign, b->valid, n, v->K, v->counts);
    hipLaunchKernelGGL(ic::ivf_offsets, dim3(1), dim3(256), 0, st, v->counts, v->K, v->offsets, v->cursor);
    if (n > 0) {
        hipLaunchKernelGGL(ic::ivf_scatter, dim3(gn), dim3(256), 0, st, v->assign, b->valid, n, v->K, v->cursor, v->perm);
        const int grid = std::max(8, b->compute_units) * 4;
        hipLaunchKernelGGL(ic::ivf_gather, dim3(grid), dim3(256), 0, st, b->rows, b->util, b->scale, b->L.row_bytes,
                           v->perm, v->offsets + v->K, s->rows, s->util, s->scale, s->valid);
    }
    int64_t total = 0;
    if (hipMemcpyAsync(&total, v->offsets + v->K, sizeof(int64_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return IC_ERR_DEVICE;
    s->n = total;
    s->any_invalid = false;
    s->stream = st;
    v->lists_ready = true;
    return hipGetLastError() == hipSuccess ? IC_OK : IC_ERR_DEVICE;
}

ic_status ivf_load_centroids(ic_ivf *v, const float *centroids_dev) {  // normalise, quantise, store
    v->cent->n = 0;
    v->cent->stream = v->base->stream;
    return ic_index_append(v->cent, centroids_dev, nullptr, v->K, nullptr);
}
}  // namespace

size_t ic_ivf_workspace_bytes(const ic_index *base, int32_t K, int32_t max_probe) {
    IvfLayout V;
    return make_ivf_layout(base, K, max_probe, V) ? V.total : 0;
}

ic_status ic_ivf_create(ic_ivf **out, ic_index *base, int32_t K, int32_t max_probe, void *arena_dev,
                        size_t arena_bytes) {
    if (!out || !base || !arena_dev || ((uintptr_t)arena_dev % kAlign) != 0) return IC_ERR_INVALID_ARG;
    IvfLayout V;
    if (!make_ivf_layout(base, K, max_probe, V)) return IC_ERR_INVALID_ARG;
    if (arena_bytes < V.total) return IC_ERR_CAPACITY;
    ic_ivf *v = new (std::nothrow) ic_ivf();
    if (!v) return IC_ERR_OOM;
    uint8_t *p = (uint8_t *)arena_dev;
    v->base = base;
    v->K = K;
    v->max_probe = max_probe;
    v->cent = nullptr;
    v->sorted = nullptr;
    ic_status st = ic_index_create(&v->cent, base->d, base->store, K, kIvfCentQueries, max_probe, p + V.off_cent,
                                   V.cent_bytes, base->stream);
    if (st == IC_OK)
        st = create_index(&v->sorted, base->d, base->store, base->capacity, base->max_q, base->max_k,
                          p + V.off_sorted, V.sorted_bytes, base->stream, false);
    if (st != IC_OK) {
        if (v->cent) ic_index_destroy(v->cent);
        delete v;
        return st;
    }
    v->assign = (int32_t *)(p + V.off_assign);
    v->perm = (int32_t *)(p + V.off_perm);
    v->counts = (int64_t *)(p + V.off_counts);
    v->offsets = (int64_t *)(p + V.off_offsets);
    v->cursor = (int64_t *)(p + V.off_cursor);
    v->sums = (float *)(p + V.off_sums);
    v->acc64 = (long long *)(p + V.off_acc64);
    v->tmp_ids = (int64_t *)(p + V.off_tmp_ids);
    v->tmp_scores = (float *)(p + V.off_tmp_scores);
    v->probe_ids = (int64_t *)(p + V.off_probe_ids);
    v->probe_scores = (float *)(p + V.off_probe_scores);
    v->task_list = (int64_t *)(p + V.off_task_list);
    v->task_pair = (int32_t *)(p + V.off_task_pair);
    v->lists_ready = false;
    *out = v;
    return IC_OK;
}

ic_status ic_ivf_destroy(ic_ivf *ivf) {
    if (!ivf) return IC_ERR_INVALID_ARG;
    ic_index_destroy(ivf->cent);
    ic_index_destroy(ivf->sorted);
    delete ivf;
    return IC_OK;
}

ic_status ic_ivf_set_centroids(ic_ivf *ivf, const float *centroids_dev) {
    if (!ivf || !centroids_dev) return IC_ERR_INVALID_ARG;
    ivf->lists_ready = false;
    return ivf_load_centroids(ivf, centroids_dev);
}

ic_status ic_ivf_assign(ic_ivf *ivf) {
    if (!ivf || ivf->cent->n != ivf->K) return IC_ERR_INVALID_ARG;
    ic_index *b = ivf->base;
    ivf->cent->stream = b->stream;
    if (b->n > 0) {
        // The tiled scan with the roles turned around: the rows are the rows, the K centroids are the
        // block of "queries", and instead of the best rows per query it keeps the best query per
        // row (ties to the lowest centroid id) as one key per row.
        hipStream_t st = b->stream;
        const Layout &L = b->L;
        ic::GemmArgs g{};
        g.store = b->rows;
        g.n = b->n;
        g.row_bytes = L.row_bytes;
        g.row_scale = b->scale;
        g.qbuf = ivf->cent->rows;       // padded to whole tiles of 256 rows; what lies past K is never selected
        g.q_scale = ivf->cent->scale;
        g.Q = ivf->K;
        g.nqb = (ivf->K + ic::kGemmTile - 1) / ic::kGemmTile;
        g.ntiles = (b->n + ic::kGemmTile - 1) / ic::kGemmTile;
        g.row_stride = 1;
        g.n_sampled = g.n;
        g.self_first = -1;
        g.row_best = (uint64_t *)ivf->tmp_ids;
        g.gq = 1;
        while (g.gq < 8 && (size_t)((g.nqb + g.gq - 1) / g.gq) * ic::kGemmTile * L.row_bytes > kL2Share) g.gq *= 2;
        hipLaunchKernelGGL(ic::ivf_zero_i64, dim3((unsigned)((b->n + 255) / 256)), dim3(256), 0, st, ivf->tmp_ids, b->n);
        const int grid = std::max(8, b->compute_units / 8 * 8);
        if (b->store == IC_STORE_BF16) launch_gemm_rowmax<0>(grid, st, g);
        else launch_gemm_rowmax<1>(grid, st, g);
        hipLaunchKernelGGL(ic::ivf_take_assignment, dim3((unsigned)((b->n + 255) / 256)), dim3(256), 0, st,
                           (const uint64_t *)ivf->tmp_ids, b->n, ivf->assign);
        if (hipGetLastError() != hipSuccess) return IC_ERR_DEVICE;
    }
    return ivf_build_lists(ivf);
}

ic_status ic_ivf_set_assignment(ic_ivf *ivf, const int32_t *assign_dev) {
    if (!ivf || (ivf->base->n > 0 && !assign_dev)) return IC_ERR_INVALID_ARG;
    if (ivf->base->n > 0 &&
        hipMemcpyAsync(ivf->assign, assign_dev, (size_t)ivf->base->n * 4, hipMemcpyDeviceToDevice,
                       ivf->base->stream) != hipSuccess)
        return IC_ERR_DEVICE;
    return ivf_build_lists(ivf);
}

ic_status ic_ivf_update_centroids(ic_ivf *ivf) {
    if (!ivf || !ivf->lists_ready || ivf->cent->n != ivf->K) return IC_ERR_INVALID_ARG;
    ic_index *s = ivf->sorted, *c = ivf->cent;
    hipStream_t st = ivf->base->stream;
    // every cluster's rows are shared out over kIvfShares workgroups (the lists are uneven: one
    // workgroup per cluster left the chip waiting for the longest list)
    const int64_t cells = (int64_t)ivf->K * s->d;
    hipLaunchKernelGGL(ic::ivf_zero_i64, dim3((unsigned)((cells + 255) / 256)), dim3(256), 0, st,
                       (int64_t *)ivf->acc64, cells);
    if (s->store == IC_STORE_BF16) {
        hipLaunchKernelGGL((ic::ivf_cluster_sums<0>), dim3(ivf->K, kIvfShares), dim3(256), 0, st, s->rows, s->scale,
                           s->L.row_bytes, s->d, ivf->offsets, ivf->acc64);
        hipLaunchKernelGGL((ic::ivf_finish_sums<0>), dim3(ivf->K), dim3(256), 0, st, ivf->acc64, ivf->offsets, s->d,
                           c->rows, c->L.row_bytes, c->scale, ivf->sums);
    } else {
        hipLaunchKernelGGL((ic::ivf_cluster_sums<1>), dim3(ivf->K, kIvfShares), dim3(256), 0, st, s->rows, s->scale,
                           s->L.row_bytes, s->d, ivf->offsets, ivf->acc64);
        hipLaunchKernelGGL((ic::ivf_finish_sums<1>), dim3(ivf->K), dim3(256), 0, st, ivf->acc64, ivf->offsets, s->d,
                           c->rows, c->L.row_bytes, c->scale, ivf->sums);
    }
    if (hipGetLastError() != hipSuccess) return IC_ERR_DEVICE;
    return ivf_load_centroids(ivf, ivf->sums);
}

ic_status ic_ivf_train(ic_ivf *ivf, int32_t iters) {
    if (!ivf || iters < 0 || ivf->base->n < 1) return IC_ERR_INVALID_ARG;
    ic_index *b = ivf->base;
    if (b->store == IC_STORE_BF16)
        hipLaunchKernelGGL((ic::ivf_rows_as_centroids<0>), dim3(ivf->K), dim3(256), 0, b->stream, b->rows, b->scale,
                           b->L.row_bytes, b->d, b->n, ivf->K, ivf->sums);
    else
        hipLaunchKernelGGL((ic::ivf_rows_as_centroids<1>), dim3(ivf->K), dim3(256), 0, b->stream, b->rows, b->scale,
                           b->L.row_bytes, b->d, b->n, ivf->K, ivf->sums);
    ic_status st = ivf_load_centroids(ivf, ivf->sums);
    for (int32_t it = 0; st == IC_OK && it < iters; ++it) {
        st = ic_ivf_assign(ivf);
        if (st == IC_OK) st = ic_ivf_update_centroids(ivf);
    }
    if (st == IC_OK) st = ic_ivf_assign(ivf);
    return st;
}

ic_status ic_ivf_view(const ic_ivf *ivf, const int32_t **assign_dev, const int64_t **offsets_dev,
                      const int32_t **perm_dev, const ic_index **centroids, const ic_index **sorted) {
    if (!ivf) return IC_ERR_INVALID_ARG;
    if (assign_dev) *assign_dev = ivf->assign;
    if (offsets_dev) *offsets_dev = ivf->offsets;
    if (perm_dev) *perm_dev = ivf->perm;
    if (centroids) *centroids = ivf->cent;
    if (sorted) *sorted = ivf->sorted;
    return IC_OK;
}

ic_status ic_ivf_search(ic_ivf *ivf, const float *q_dev, int64_t Q, int32_t k, int32_t nprobe, float lambda,
                        float *out_scores_dev, int64_t *out_ids_dev) {
    if (!ivf || Q < 0 || k < 1 || nprobe < 1 || nprobe > ivf->max_probe) return IC_ERR_INVALID_ARG;
    ic_index *s = ivf->sorted, *c = ivf->cent;
    if (k > s->max_k || !ivf->lists_ready || c->n != ivf->K) return IC_ERR_INVALID_ARG;
    if (Q == 0) return IC_OK;
    if (!q_dev || !out_scores_dev || !out_ids_dev) return IC_ERR_INVALID_ARG;
    hipStream_t st = ivf->base->stream;
    c->stream = st;
    s->stream = st;
    const Layout &L = s->L;
    const int et = (s->store == IC_STORE_BF16) ? 0 : 1;
    const int cpw = chunks_per_wavefront(L.row_bytes / 64);
    const int cap = region_cap_for(k, 0);
    const int64_t n = s->n;
    if (!s->consts_ready) {
        hipLaunchKernelGGL(init_consts, dim3(1), dim3(64), 0, st, (uint32_t *)s->ws.consts);
        s->consts_ready = true;
    }
    const bool use_bias = lambda != 0.0f && n > 0;
    if (use_bias) {
        const int64_t n_pad = round_up(n, ic::kGemmTile);
        hipLaunchKernelGGL(ic::make_bias, dim3((int)std::min<int64_t>((n_pad + 255) / 256, 4096)), dim3(256), 0, st,
                           (const float *)s->util, (const uint8_t *)nullptr, (const uint8_t *)nullptr, n, n_pad, lambda,
                           s->ws.bias);
    }
    // slices per list: about 12 tiles of 16 rows each, at most 16 slices; with few (query, list) tasks more,
    // up to 64 and down to 2 tiles of an average list, so that about 4096 workgroups are launched: lists are
    // uneven (a head cluster's can be 20 times the average), and the longest one sets the time of the launch
    const int64_t avg_tiles = std::max<int64_t>(1, n / std::max<int64_t>(1, ivf->K) / 16);
    const int64_t tasks = std::min<int64_t>(Q, std::min<int64_t>(L.q_chunk, ivf->base->L.q_chunk)) * nprobe;
    const int64_t by_tasks = std::min<int64_t>(std::min<int64_t>(64, 4096 / std::max<int64_t>(1, tasks)), avg_tiles / 2);
    const int S = (int)std::max<int64_t>(std::min<int64_t>(16, std::max<int64_t>(1, avg_tiles / 12)), by_tasks);
    // a pass takes as many queries as the candidate regions hold (one per pair and slice) and as one
    // workgroup can group by list (kTaskPairs pairs)
    const int64_t qmax = std::min<int64_t>(std::min<int64_t>(std::min<int64_t>(L.q_chunk, ivf->base->L.q_chunk),
                                                             std::max<int64_t>(1, kRegionSlots / ((int64_t)nprobe * S))),
                                           std::max<int64_t>(1, ic::kTaskPairs / nprobe));
    for (int64_t q0 = 0; q0 < Q; q0 += qmax) {
        const int qc = (int)std::min<int64_t>(qmax, Q - q0);
        // the nprobe nearest centroids of every query
        SearchReq r;
        r.q_dev = q_dev + q0 * (int64_t)s->d;
        ic_status rc = search_impl(c, c->ws, qc, nprobe, 0.0f, nullptr, ivf->probe_scores, ivf->probe_ids, r);
        if (rc != IC_OK) return rc;
        // the queries in the store's format, then scan tasks: one per list and up to 16 queries that probe it
        const int grid = (qc + 3) / 4;
        ic::launch_quantize_rows(et, (unsigned)grid, st, r.q_dev, (int64_t)qc, (int64_t)qc, s->d, L.row_bytes, s->ws.qbuf,
                                 et == 0 ? nullptr : s->ws.qscale, nullptr, nullptr, nullptr, 0);
        float *out_s = out_scores_dev + q0 * (int64_t)k;
        int64_t *out_i = out_ids_dev + q0 * (int64_t)k;
        const FinalOpts fo{-INFINITY, nullptr, -1};
        ic::MergeArgs m{};
        m.src = s->ws.regions;
        m.seg_stride = cap;
        m.seg_cap = cap;
        m.seg_counts = s->ws.counts;
        m.segs_per_wg = std::min(ic::kMergeMaxSegs, ic::kMergeKeys / cap);
        if (n == 0) {
            m.q_stride = 0;
            m.nseg = 0;
            m.segs_per_wg = 1;
            run_merge(s, s->ws, m, qc, k, out_s, out_i, nullptr, fo);
            continue;
        }
        ic::ScanArgs a{};
        a.store = s->rows;
        a.n = n;
        a.row_bytes = L.row_bytes;
        a.row_scale = s->scale;
        a.bias = use_bias ? s->ws.bias : (const float *)s->ws.consts;
        a.bias_stride = use_bias ? 1 : 0;
        a.qbuf = s->ws.qbuf;
        a.q_scale = s->ws.qscale;
        a.Q = qc;
        a.k = k;
        a.cap = cap;
        a.S = S;
        a.regions = s->ws.regions;
        a.counts = s->ws.counts;
        a.tile_mul = 1;
        // the pairs grouped by list: a list that several queries probe is read once for up to 16 of them
        const int pairs = qc * nprobe;
        auto group = pairs <= 256 ? ic::ivf_group_tasks<1> : pairs <= 512 ? ic::ivf_group_tasks<2>
                   : pairs <= 1024 ? ic::ivf_group_tasks<4> : ic::ivf_group_tasks<8>;   // the sort is sized to the pairs
        hipLaunchKernelGGL(group, dim3(1), dim3(256), 0, st, (const int64_t *)ivf->probe_ids, pairs, ivf->K, ivf->task_list,
                           ivf->task_pair, s->ws.counts, pairs * S);
        a.task_cluster = ivf->task_list;
        a.task_offsets = ivf->offsets;
        a.task_pair = ivf->task_pair;
        a.task_nprobe = nprobe;
        kTaskTable[et][cpw - 1](dim3(S, pairs), st, a);
        m.q_stride = (int64_t)nprobe * S * cap;
        m.nseg = nprobe * S;
        m.id_map = ivf->perm;
        run_merge(s, s->ws, m, qc, k, out_s, out_i, nullptr, fo);
    }
    return hipGetLastError() == hipSuccess ? IC_OK : IC_ERR_DEVICE;
}

}  // extern "C"
