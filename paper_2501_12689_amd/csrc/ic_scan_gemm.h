// Large-batch scan: similarity of blocks of 256 queries with tiles of 256 cached rows as a
// register-tiled MFMA contraction, fused with threshold selection.  This is the same O(N) step of
// IC-Cache's stage-1 relevance selection (Sec. 4.1; GetSimilarExamples in Algorithm 1) as the
// streaming scan, for batches large enough that the matrix cores, not HBM, bound the work.
//
// Shape of the computation
//   * One output tile = 256 rows x 256 queries over the whole embedding dimension.  A workgroup has
//     8 wavefronts (4 x 2, each 64 rows x 128 queries = 2 x 4 MFMA tiles of 32x32, 128 accumulator
//     registers), two per SIMD: while one issues loads or LDS reads the other keeps the matrix pipe
//     fed (with one wavefront per SIMD every direct load cost about 27 cycles of idle pipe).
//   * A pipeline step is 64 bytes of every row of the tile (512 rows x 64 B = 32 KB).  An LDS ring
//     of 4 slots holds the step being multiplied and up to three in flight.  Operands are copied
//     from global memory straight into LDS (global_load_lds_dwordx4: no staging registers, no LDS
//     store instructions).  The wait before a step's barrier is counted (vmcnt): only the next
//     step's loads must have landed, so a load has three steps to arrive.
//   * LDS layout: row-major, 64 B per row; granule g (16 bytes) of row r sits at position
//     g ^ ((r / 4) % 4).  A 128-bit LDS read is served 16 lanes at a time, and 16 consecutive rows
//     then cover all sixteen 16-byte slots of the 256-byte bank span exactly once.  A direct load
//     writes lane l of a wavefront to (wave's LDS base + 16*l), i.e. 16 rows x 4 granules per
//     instruction, so the swizzle is applied on the global side: the lane fetches the granule that
//     belongs at its position (the step-major copies described below hold the granules in that
//     order already).
//   * Operand mapping: lane (r = lane%32, h = lane/32) reads granule 2*p + h of row r for MFMA
//     step p (0, 1); rows and queries use the same mapping, so each MFMA pairs equal coordinates
//     (the order of the coordinates inside a dot product is free).  bf16: one
//     v_mfma_f32_32x32x16_bf16 per granule pair; fp8: one v_mfma_f32_32x32x64_f8f6f4 per step, whose
//     32-byte operand is both of the lane's granules.
//   * Where the operands come from.  Selection launches (and their second launch) read both operands
//     from step-major copies ("panels"): tile t of 256 rows is stored as its pipeline steps one
//     after the other, a step being 16 KB = 64 B of each of the 256 rows with the granules already in
//     their swizzled positions, i.e. exactly the image the step has in LDS.  A direct load then moves
//     1 KB of contiguous memory (eight full 128-byte lines) instead of half a line of each of 16
//     rows, which halves the requests the L2 has to answer (it served 64-byte requests at 140 G/s
//     when the rows were read from the row-major store, and a copy-only pipeline measured 950 against
//     630 cycles per step).  The panel of the store is written by to_panel() when rows are appended
//     or moved, the panel of the query block once per search.  Pilot and row-maximum launches
//     read the row-major store (a pilot's rows are a strided sample).
//   * Workgroups are persistent and XCD-aware: workgroup id modulo 8 is the XCD it runs on; an XCD
//     owns a group of query blocks small enough to stay in its L2 and a class of row tiles, and
//     walks query blocks fastest so that a row tile is used by consecutive tiles.  The load
//     pipeline runs across tile boundaries: a cursor walks the same tile sequence 4 steps ahead.
//   * Scores: bf16 accumulators start at their row's bias (lambda * utility, -inf for rows that may
//     not be selected), passed as the addend of the tile's first MFMAs, so the finished accumulator
//     is the score; fp8 multiplies by the row's and the query's scale and adds the bias afterwards.
//   * Selection: thresholds come from the pilot (per query a key, score then row, that at least k rows
//     reach; rows with exactly its score pass only up to its row, so copies of one row cannot flood a list).
//     A tile's 65,536 scores are compared 16 at a time (max, then one compare); a lane whose 16
//     scores reach the threshold copies them to an LDS list, the workgroup then tests those few
//     blocks exactly, one score per thread, and parks what passes (about 17 candidates per tile)
//     in a second LDS list.  That list is flushed to the queries' candidate lists in global
//     memory (slot = atomic counter per query) while the next tile is being computed: the atomics
//     are issued in that tile's last step and their results used after it, so nobody waits for an
//     L2 round trip.  A tile with more such blocks than the LDS list holds keeps nothing and is
//     noted in a list; a second, small launch (AGAIN = true) computes the listed tiles again and
//     tests every score.  If a query's candidate list in global memory overflows, its block of 64
//     queries is flagged and redone by the streaming scan, so the result stays exact whatever the data.
//   * Pilot launches (PILOT = true) run the same pipeline over a strided sample of the rows (every
//     row_stride-th row; a tile takes 256 of them spread evenly over the whole store) and keep, per
//     query and slice, only the best key: the best score and the row it belongs to.
//   * Row-maximum launches (ROWMAX = true) turn the selection around: for every cached row the
//     best of the "queries" (with ties to the lowest query id), as one 64-bit key per row.  This
//     is the assignment step of K-Means (Sec. 4.1): the queries are the centroids.
#pragma once
#include <type_traits>

#include "ic_common.h"

namespace ic {

typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kGemmTile = 256;        // rows and queries per output tile (= kPanelRows: a tile of the step-major copies)
constexpr int kGemmStageBytes = 128;  // rows are padded to a multiple of this
constexpr int kGemmHalfBytes = 64;    // bytes of every row per pipeline step (= kPanelStepBytes)
static_assert(kGemmTile == kPanelRows && kGemmHalfBytes == kPanelStepBytes, "the step-major copies are laid out for this kernel");
constexpr int kGemmSlots = 4;         // LDS ring: pipeline steps resident or in flight
constexpr int kGemmThreads = 512;     // 8 wavefronts, two per SIMD: one issues MFMAs while the other issues loads

struct GemmArgs {
    const uint8_t *panel;    // selection launches: step-major copy of the store, [ceil(n/256)] tiles of 256 * row_bytes bytes
    const uint8_t *qpanel;   // selection launches: step-major copy of the prepared queries, [nqb] tiles
    const uint8_t *store;    // [n] rows, row_bytes apart
    int64_t n;
    int row_bytes;           // multiple of 128
    const float *row_scale;  // fp8: [round_up(n,256)]
    const float *bias;       // [round_up(n,256)]: lambda*utility, -inf for invalid and padding rows
    const uint8_t *qbuf;     // prepared queries, [nqb*256] rows
    const float *q_scale;    // fp8: per prepared query
    int Q;                   // real queries
    const uint64_t *thr_init;  // [Q] a key that >= k rows reach, as this kernel computes their scores (or the key of
                               // kNoThresholdScore: every row with a score passes)
    uint64_t *glist;         // [Q][gcap] candidate keys
    int gcap;
    int32_t *gcount;         // [Q] candidates appended (may exceed gcap: the list overflowed)
    int32_t *redo;           // [ceil(Q/64)] set to 1 when a list of the block overflowed
    uint32_t *over_n;        // tiles that listed more blocks than the per-tile list holds ...
    uint2 *over_list;        // ... as (row tile, query block), [over_cap]; AGAIN launches walk this list
    uint32_t over_cap;
    int nqb;                 // query blocks of 256
    int64_t ntiles;          // row tiles of 256
    uint64_t *pilot_out;     // pilot launches: [Q][pilot_stride] keys (best score over the slice so far, and the row it belongs to)
    int pilot_stride;
    int64_t row_stride;      // PILOT: the launch scores rows 0, row_stride, 2 * row_stride, ... only.  Row r of its
                             // t-th tile is row r * ntiles + t of that sample, so every tile, and with it every
                             // slice, is a uniform sample of the store whatever the order the rows arrived in
    int64_t n_sampled;       // PILOT: rows of the sample, ceil(n / row_stride); ntiles = ceil(n_sampled / 256)
    const int32_t *row_dom;  // DOM: sharing domain of every row (0 = public), [round_up(n,256)]
    const int32_t *q_dom;    // DOM: domain of every query, [Q]; row i is visible to q if row_dom[i] is 0 or q_dom[q]
    int64_t self_first;      // self-search: query q is stored row self_first + q and must not select
                             // itself (a tile on the diagonal would otherwise list 256 hits); -1: off
    uint64_t *row_best;      // ROWMAX: [n] keys (score of the best query, its id), zeroed before the launch
    int gq;                  // XCD mapping: query-block groups (1, 2, 4 or 8); 8/gq row classes
};

constexpr int kGemmPark = 512;        // candidates a workgroup can park per tile (one flusher thread each)
constexpr int kGemmHits = 96;         // blocks of 16 scores a workgroup can list per tile

struct HitEntry {   // 16 scores of one lane's block that reached its query's threshold
    f32x4 sc[4];
    uint64_t thr;   // the query's pilot key
    uint32_t q;
    uint32_t row;   // row of score 0
};

constexpr size_t gemm_lds_bytes() {
    return (size_t)kGemmSlots * 2 * kGemmTile * kGemmHalfBytes + 2 * kGemmTile * 4 + (size_t)kGemmPark * 12 + 16 +
           (size_t)kGemmHits * sizeof(HitEntry) + kGemmTile * 4;
}

template <int ET, bool PILOT, bool DOM = false, bool ROWMAX = false, bool AGAIN = false>
__global__ __launch_bounds__(kGemmThreads) void scan_gemm(const GemmArgs a) {
    static_assert(!ROWMAX || (!PILOT && !DOM), "row maxima take neither thresholds nor domains");
    static_assert(!AGAIN || (!PILOT && !ROWMAX), "only the selection launch leaves tiles to be done again");
    // bf16 launches that score (selection and its pilot, which must round alike: the pilot's threshold
    // is a score the selection has to reach again) start every accumulator at its row's bias instead
    // of at zero, so the score is what the MFMAs leave behind and the epilogue adds nothing (128
    // additions per lane and tile less, at a time when the matrix pipe is idle).  The bias of a tile is
    // fetched during the tile before it.  fp8 scores need the two scales first and keep the addition.
    constexpr bool kBiasInit = ET == 0 && !ROWMAX;
    // selection launches read both operands from the step-major copies (a tile covers the same byte
    // range in either layout, so a tile's base address is computed the same way)
    constexpr bool kPanel = !PILOT && !ROWMAX;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_dyn[];
    uint8_t *lds = static_cast<uint8_t *>(__builtin_assume_aligned(lds_dyn, 16));
    constexpr int kSlot = 2 * kGemmTile * kGemmHalfBytes;  // 32 KB: 256 rows then 256 queries, 64 B each
    float *bias_t = reinterpret_cast<float *>(lds + kGemmSlots * kSlot);
    float *scale_t = bias_t + kGemmTile;
    uint64_t *park_key = reinterpret_cast<uint64_t *>(scale_t + kGemmTile);  // [kGemmPark]
    uint32_t *park_q = reinterpret_cast<uint32_t *>(park_key + kGemmPark);    // [kGemmPark]
    uint32_t *park_n = park_q + kGemmPark;   // [0] parked candidates, [1] listed blocks
    uint32_t *hit_n = park_n + 1;
    HitEntry *hits = reinterpret_cast<HitEntry *>(park_n + 4);  // [kGemmHits]
    int32_t *dom_t = reinterpret_cast<int32_t *>(hits + kGemmHits);  // [kGemmTile] sharing domains of the tile's rows (DOM)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // 4 x 2 wavefronts of 64 rows x 128 queries.  A batch of one block with at most 128 real queries
    // gives its first 128 queries to wavefronts 0-3 (one per SIMD), so that all four SIMDs work;
    // otherwise the two wavefronts of a SIMD (w, w + 4) share their queries (measured slightly faster).
    const bool half_block = a.nqb == 1 && a.Q <= 128;
    const int wm = half_block ? (w & 3) : (w >> 1), wn = half_block ? (w >> 2) : (w & 1);
    const int r32 = lane & 31, h = lane >> 5;
    const int nhs = a.row_bytes / kGemmHalfBytes;  // pipeline steps per tile (even, >= 2)

    // ---- which tiles this workgroup walks
    const int xcd = blockIdx.x & 7;
    const int gr = 8 / a.gq;                          // row classes
    const int qgroup = xcd % a.gq, rclass = xcd / a.gq;
    const int nq_x = (a.nqb - qgroup + a.gq - 1) / a.gq;              // query blocks of this XCD
    const int64_t nr_x = (a.ntiles - rclass + gr - 1) / gr;           // row tiles of this XCD
    // AGAIN: the jobs are the entries of over_list, dealt to the workgroups in turn
    const uint32_t listed = AGAIN ? *a.over_n : 0u;
    const int64_t work = AGAIN ? (int64_t)(listed < a.over_cap ? listed : a.over_cap) : (int64_t)nq_x * nr_x;
    const int64_t step = AGAIN ? gridDim.x : gridDim.x >> 3;
    const int64_t first_job = AGAIN ? blockIdx.x : blockIdx.x >> 3;
    if (first_job >= work) return;  // nothing to do: no load is ever issued

    // Everything a tile needs to address its operands.
    struct Tile {
        int qb;
        int last;  // last valid row of the tile, relative to its first row (0 .. 255)
        int64_t row0;
        const uint8_t *rows_base;
        const uint8_t *q_base;
    };
    auto locate = [&](int ql, int64_t rl, Tile &t) {  // ql-th query block, rl-th row tile of this XCD
        t.qb = qgroup + a.gq * ql;
        if (AGAIN) {
            const uint2 e = a.over_list[rl];   // ql is 0
            t.qb = (int)e.y;
            t.row0 = (int64_t)e.x * kGemmTile;
        }
        t.q_base = (kPanel ? a.qpanel : a.qbuf) + (size_t)t.qb * kGemmTile * a.row_bytes;
        if (PILOT) {
            t.row0 = rclass + gr * rl;   // the tile's index: its row r is row r * ntiles + row0 of the sample
            t.rows_base = a.store + t.row0 * a.row_stride * a.row_bytes;
            t.last = (int)((a.n_sampled - 1 - t.row0) / a.ntiles);   // 0 .. 255 since ntiles = ceil(n_sampled / 256)
        } else {
            if (!AGAIN) t.row0 = (rclass + gr * rl) * kGemmTile;
            t.rows_base = (kPanel ? a.panel : a.store) + t.row0 * a.row_bytes;
            const int64_t last = a.n - 1 - t.row0;
            t.last = (int)(last < kGemmTile - 1 ? last : kGemmTile - 1);
        }
    };
    // job = rl * nq_x + ql walks query blocks fastest; the pair is advanced without divisions
    struct Walk {
        int ql;
        int64_t rl;
        int64_t job;
    };
    const int nq_w = AGAIN ? 1 : nq_x;   // query blocks of the walk (a list is walked entry by entry)
    const int step_q = (int)(step % nq_w);
    const int64_t step_r = step / nq_w;
    auto walk_next = [&](Walk &x) {
        x.job += step;
        x.ql += step_q;
        x.rl += step_r;
        if (x.ql >= nq_w) {
            x.ql -= nq_w;
            x.rl += 1;
        }
    };
    Walk tw;  // the tile being computed
    tw.job = first_job;
    tw.ql = (int)(tw.job % nq_w);
    tw.rl = tw.job / nq_w;

    // ---- copy plan.  One direct load moves 16 rows x 64 B per wavefront: lane l lands at the
    // wavefront's LDS base + 16*l, i.e. row l/4, position l%4, and therefore fetches granule
    // (l%4) ^ ((row/4)%4).  Per pipeline step a wavefront issues 4 loads: row groups w and w+8 (of 16
    // rows each) of the cached rows and the same groups of the queries.  From a panel the same
    // load reads 1 KB of contiguous memory: lane l fetches byte 16*l of the group's kilobyte (rows
    // past the end of the store are zeros there, so nothing is clamped).
    typedef const void __attribute__((address_space(1))) *gptr_t;
    typedef void __attribute__((address_space(3))) *lptr_t;
    const int crow = lane >> 2;
    const int cg = (lane & 3) ^ ((lane >> 4) & 3);
    // byte offsets from a tile's first query / first row (rows clamped per tile; 64 bits only for a
    // pilot, whose rows lie ntiles * row_stride rows apart)
    uint32_t off_q[2];
    typename std::conditional<PILOT, uint64_t, uint32_t>::type off_r[2];
    const uint64_t row_pitch = PILOT ? (uint64_t)a.ntiles * (uint64_t)a.row_stride * (uint64_t)a.row_bytes : (uint64_t)a.row_bytes;
#pragma unroll
    for (int u = 0; u < 2; ++u) off_q[u] = (uint32_t)(((w + 8 * u) * 16 + crow) * a.row_bytes + cg * 16);
    Walk cw = tw;   // the load cursor runs kGemmSlots pipeline steps ahead of the computation
    const uint8_t *c_rows, *c_q;
    int c_hs;
    auto cursor_tile = [&]() {
        Tile t;
        locate(cw.ql, cw.rl, t);
        c_rows = t.rows_base;
        c_q = t.q_base;
        c_hs = 0;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            int r = (w + 8 * u) * 16 + crow;
            r = r < t.last ? r : t.last;  // ragged last tile: rows past the end re-read the last valid row (bias -inf)
            if (PILOT) off_r[u] = (uint64_t)r * row_pitch + (uint64_t)(cg * 16);
            else off_r[u] = (uint32_t)(r * a.row_bytes + cg * 16);
        }
    };
    const uint32_t lane16 = (uint32_t)lane * 16u;
    auto issue = [&](int slot, auto half_c) {  // request the cursor's step into an LDS slot
        uint8_t *dst = lds + slot * kSlot + w * (16 * kGemmHalfBytes);  // wave-uniform
        constexpr int kQueryLoads = decltype(half_c)::value ? 1 : 2;   // kHalf: the second half of the block is never read
        if (kPanel) {
            // step c_hs of a tile is the 16 KB from c_hs * 16 KB on; row group g is its g-th kilobyte
            const uint8_t *ra = c_rows + (size_t)c_hs * (kGemmTile * kGemmHalfBytes) + w * (16 * kGemmHalfBytes);
            const uint8_t *qa = c_q + (size_t)c_hs * (kGemmTile * kGemmHalfBytes) + w * (16 * kGemmHalfBytes);
#pragma unroll
            for (int u = 0; u < 2; ++u)
                __builtin_amdgcn_global_load_lds((gptr_t)(ra + u * 128 * kGemmHalfBytes + lane16),
                                                 (lptr_t)(dst + u * 128 * kGemmHalfBytes), 16, 0, 0);
#pragma unroll
            for (int u = 0; u < kQueryLoads; ++u)
                __builtin_amdgcn_global_load_lds((gptr_t)(qa + u * 128 * kGemmHalfBytes + lane16),
                                                 (lptr_t)(dst + (kGemmTile + u * 128) * kGemmHalfBytes), 16, 0, 0);
            return;
        }
        const uint8_t *ra = c_rows + c_hs * kGemmHalfBytes;
        const uint8_t *qa = c_q + c_hs * kGemmHalfBytes;
#pragma unroll
        for (int u = 0; u < 2; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(ra + off_r[u]), (lptr_t)(dst + u * 128 * kGemmHalfBytes), 16, 0, 0);
#pragma unroll
        for (int u = 0; u < kQueryLoads; ++u)
            __builtin_amdgcn_global_load_lds((gptr_t)(qa + off_q[u]),
                                             (lptr_t)(dst + (kGemmTile + u * 128) * kGemmHalfBytes), 16, 0, 0);
    };
    auto advance = [&]() {  // move the cursor one step on (uniform control flow)
        if (++c_hs == nhs) {
            // past the last tile the same tile is requested again; those loads are never used
            if (cw.job + step < work) walk_next(cw);
            cursor_tile();
        }
    };

    // ---- operand read plan: byte offset inside a slot of this lane's granule for step p (0, 1):
    // granule 2*p + h of row r sits at position (2*p + h) ^ ((r / 4) % 4)
    uint32_t frag_off[2];
#pragma unroll
    for (int p = 0; p < 2; ++p)
        frag_off[p] = (uint32_t)(r32 * kGemmHalfBytes + (((2 * p + h) ^ ((r32 >> 2) & 3)) * 16));
    const uint32_t a_base = (uint32_t)(wm * 64 * kGemmHalfBytes);
    const uint32_t b_base = (uint32_t)((kGemmTile + wn * 128) * kGemmHalfBytes);

    // Barrier for data exchanged through LDS only: unlike __syncthreads() it does not wait for this
    // wavefront's outstanding global loads and stores (the direct loads in flight, the list flushes).
    auto lds_barrier = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // append one candidate to its query's list (slot from the query's atomic counter)
    auto append_global = [&](uint32_t q, uint64_t key, int pos) {
        if (pos < a.gcap) a.glist[(size_t)q * a.gcap + pos] = key;
        else a.redo[q >> 6] = 1;
    };
    if (tid == 0) {
        *park_n = 0u;
        *hit_n = 0u;
    }

    // The two wavefronts of a SIMD (w and w + 4) issue their direct loads half a step apart, so
    // that one of them always has nothing but MFMAs and LDS reads to issue: the first four refill
    // a slot right after the barrier that frees it, the other four during the first half of the
    // following step.
    const bool late = w >= 4;
    // fill the ring: the first kGemmSlots steps of this workgroup's work (the late wavefronts
    // request their share of the last one during the first step)
    // bias of rows 4 * tid .. 4 * tid + 3 of the tile that starts at (pilot: has the index) r0
    auto bias_of = [&](int64_t r0) {
        f32x4 b;
        if (PILOT) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int64_t sampled = (int64_t)(tid * 4 + e) * a.ntiles + r0;
                b[e] = sampled < a.n_sampled ? a.bias[sampled * a.row_stride] : -INFINITY;
            }
        } else {
            b = *reinterpret_cast<const f32x4 *>(a.bias + r0 + tid * 4);
        }
        return b;
    };
    if (kBiasInit && tid < 64) {   // bias of this workgroup's first tile; the barrier below publishes it
        Tile first;
        locate(tw.ql, tw.rl, first);
        *reinterpret_cast<f32x4 *>(bias_t + tid * 4) = bias_of(first.row0);
    }
    cursor_tile();
#pragma unroll
    for (int sl = 0; sl < kGemmSlots; ++sl) {
        if (sl + 1 < kGemmSlots || !late) {
            issue(sl, std::false_type{});
            advance();
        }
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    int hslot = 0;  // ring slot of the step being computed
    // At a step's barrier this wavefront's loads for the next step must have landed; those of the two
    // steps after it (4 loads each; 3 when the second half of the query block is not copied) may be
    // in flight.
    auto wait_next_step = [&](auto half_c) {
        if (decltype(half_c)::value) asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
    };
    // kDead: the batch is a single query block with at most 128 real queries and this wavefront's
    // 128 queries are all padding.  It keeps its part in the copies and the barriers and skips the
    // operand reads and the MFMAs, so such a batch costs half the matrix work and the scan is bound
    // by reading the store.  (In a batch of several blocks only the last block can have such
    // wavefronts; they are not worth a second copy of the loop there.)
    auto run_tiles = [&](auto late_c, auto dead_c, auto half_c) {
    constexpr bool kLate = decltype(late_c)::value;
    constexpr bool kDead = decltype(dead_c)::value;
    for (; tw.job < work; walk_next(tw)) {
        Tile cur;
        locate(tw.ql, tw.rl, cur);
        const int qb = cur.qb;
        const int64_t row0 = cur.row0;

        // bf16 selection launches: the first MFMA of every accumulator tile takes the bias of the
        // tile's rows as its addend (accumulator v of tile (i, j) belongs to row
        // wm*64 + i*32 + 8*(v/4) + 4*h + v%4, whatever j); everything else starts from zero
        f32x16 acc[2][4];
        f32x16 bvec[2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                f32x4 b = {0.f, 0.f, 0.f, 0.f};
                if (kBiasInit) b = *reinterpret_cast<const f32x4 *>(bias_t + wm * 64 + i * 32 + 8 * u + 4 * h);
#pragma unroll
                for (int e = 0; e < 4; ++e) bvec[i][4 * u + e] = b[e];
            }
        if (ET == 1 || kDead) {   // the fp8 loop has no first step of its own; idle wavefronts issue no MFMA at all
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = bvec[i];
        }
        // the tile after this one (kBiasInit: its bias is fetched in this tile's last step)
        int64_t row0_next = row0;
        if (kBiasInit && tw.job + step < work) {
            Walk nx = tw;
            walk_next(nx);
            Tile nt;
            locate(nx.ql, nx.rl, nt);
            row0_next = nt.row0;
        }

        // What the previous tile parked is flushed during this tile: slots are claimed (one atomic
        // per candidate) in the tile's last step and the keys are written after it.
        int fl_pos = -1;
        uint64_t thr_raw[4];
        float qs[4];
        f32x4 bias_r = {0.f, 0.f, 0.f, 0.f}, scale_r = {1.f, 1.f, 1.f, 1.f};
        i32x4 dom_r = {0, 0, 0, 0};   // DOM: the tile's row domains and this lane's query domains
        int qd[4] = {0, 0, 0, 0};

        // bias, scale and domain of rows 4 * tid .. 4 * tid + 3 of the tile (threads 0-63)
        auto row_terms = [&]() {
            bias_r = bias_of(kBiasInit ? row0_next : row0);
            if (PILOT) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t sampled = (int64_t)(tid * 4 + e) * a.ntiles + row0;
                    const bool in = sampled < a.n_sampled;
                    const int64_t at = in ? sampled * a.row_stride : 0;   // the sampled row's place in the store
                    if (ET == 1) scale_r[e] = in ? a.row_scale[at] : 1.0f;
                    if (DOM) dom_r[e] = in ? a.row_dom[at] : 0;
                }
            } else {
                if (ET == 1) scale_r = *reinterpret_cast<const f32x4 *>(a.row_scale + row0 + tid * 4);
                if (DOM) dom_r = *reinterpret_cast<const i32x4 *>(a.row_dom + row0 + tid * 4);
            }
        };

        i32x4 fa[2][2], fb[2][4];
        auto read_frags = [&](int slot, int p, i32x4 *xa, i32x4 *xb) {
            const uint8_t *sa = lds + slot * kSlot + a_base + frag_off[p];
            const uint8_t *sb = lds + slot * kSlot + b_base + frag_off[p];
#pragma unroll
            for (int i = 0; i < 2; ++i) xa[i] = *reinterpret_cast<const i32x4 *>(sa + i * 32 * kGemmHalfBytes);
#pragma unroll
            for (int j = 0; j < 4; ++j) xb[j] = *reinterpret_cast<const i32x4 *>(sb + j * 32 * kGemmHalfBytes);
        };
        auto mfma8 = [&](const i32x4 *xa, const i32x4 *xb, auto first_c) {
            constexpr bool kFirst = decltype(first_c)::value;   // the tile's first MFMAs: addend = bias (or zero)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, xa[i]), __builtin_bit_cast(bf16x8, xb[j]),
                        kFirst ? bvec[i] : acc[i][j], 0, 0, 0);
                }
        };
        constexpr int kPer = 1;  // MFMA instructions per accumulator tile and 32-byte half step (bf16)

        // One pipeline step = 64 B of every row = two MFMA steps of 8 accumulator tiles.
        //   first half:  MFMAs on the operands read earlier; the second half's operands are read
        //   barrier:     this wavefront's loads for the next step have landed (at most the two
        //                younger steps are still in flight) and it has read all it needs from the
        //                current slot; after the barrier that holds for every wavefront
        //   second half: the current slot is refilled with the step kGemmSlots ahead, the next
        //                step's first operands are read, MFMAs on the second operands
        // Nothing waits for a load younger than three steps, and LDS reads are always one MFMA
        // step ahead of their use.
        auto half = [&](auto last_c, auto first_c) {
            constexpr bool kLast = decltype(last_c)::value;
            if (kLate) issue((hslot + kGemmSlots - 1) & (kGemmSlots - 1), half_c);  // the slot freed by the previous barrier
            if (!kDead) {
                read_frags(hslot, 1, fa[1], fb[1]);
                mfma8(fa[0], fb[0], first_c);
#pragma unroll
                for (int g = 0; g < 6; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, kPer, 0);  // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);     // LDS read
                    if (kLate && g < 4) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // direct load
                }
                __builtin_amdgcn_sched_group_barrier(0x008, 2 * kPer, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (kLate) advance();
            wait_next_step(half_c);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            if (kLast) {
                // what the epilogue needs from global memory, and the slots of the parked candidates
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int q = qb * kGemmTile + wn * 128 + j * 32 + r32;
                    if (q >= a.Q) q = a.Q - 1;  // padding query: read something valid, masked below
                    thr_raw[j] = (PILOT || ROWMAX) ? 0ull : a.thr_init[q];
                    qs[j] = (ET == 1) ? a.q_scale[q] : 1.0f;
                    if (DOM) qd[j] = a.q_dom[q];
                }
                if (tid < 64 && !ROWMAX) row_terms();
                if (!PILOT && !ROWMAX) {
                    const uint32_t parked = min(*park_n, (uint32_t)kGemmPark);  // final: barriers since it was written
                    if ((uint32_t)tid < parked) fl_pos = atomicAdd(a.gcount + park_q[tid], 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (!kLate) issue(hslot, half_c);
            const int nslot = (hslot + 1) & (kGemmSlots - 1);
            if (!kDead) {
                if (!kLast) read_frags(nslot, 0, fa[0], fb[0]);
                mfma8(fa[1], fb[1], std::false_type{});
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, kPer, 0);
                    if (!kLate) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // direct load
                    if (!kLast) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
                if (!kLast) {
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x008, kPer, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (!kLate) advance();
            hslot = nslot;
        };
        // fp8: one v_mfma_f32_32x32x64_f8f6f4 per accumulator tile and step (twice the flops per
        // cycle of the 32x32x16 forms).  Its operand is 32 bytes per lane: both granules (p = 0, 1)
        // of the lane's row, so all 12 operand reads of a step are done one step ahead, into the
        // other half of a double buffer, and the step's 8 MFMAs sit 4 before and 4 after the barrier.
        i32x8 ga[2][2], gb[2][4];
        auto read_frags8 = [&](int slot, i32x8 *xa, i32x8 *xb) {
            const uint8_t *sa = lds + slot * kSlot + a_base;
            const uint8_t *sb = lds + slot * kSlot + b_base;
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                xa[i].lo = *reinterpret_cast<const i32x4 *>(sa + frag_off[0] + i * 32 * kGemmHalfBytes);
                xa[i].hi = *reinterpret_cast<const i32x4 *>(sa + frag_off[1] + i * 32 * kGemmHalfBytes);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                xb[j].lo = *reinterpret_cast<const i32x4 *>(sb + frag_off[0] + j * 32 * kGemmHalfBytes);
                xb[j].hi = *reinterpret_cast<const i32x4 *>(sb + frag_off[1] + j * 32 * kGemmHalfBytes);
            }
        };
        auto half8 = [&](auto last_c, auto par_c) {
            constexpr bool kLast = decltype(last_c)::value;
            constexpr int kPar = decltype(par_c)::value;
            if (kLate) issue((hslot + kGemmSlots - 1) & (kGemmSlots - 1), half_c);  // the slot freed by the previous barrier
            if (!kDead) {
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ga[kPar][i], gb[kPar][j], acc[i][j], 0,
                                                                                     0, 0, 0, 0, 0);
                if (kLate) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
                        __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);  // direct load
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (kLate) advance();
            wait_next_step(half_c);
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_sched_barrier(0);
            if (kLast) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int q = qb * kGemmTile + wn * 128 + j * 32 + r32;
                    if (q >= a.Q) q = a.Q - 1;  // padding query: read something valid, masked below
                    thr_raw[j] = (PILOT || ROWMAX) ? 0ull : a.thr_init[q];
                    qs[j] = a.q_scale[q];
                    if (DOM) qd[j] = a.q_dom[q];
                }
                if (tid < 64 && !ROWMAX) row_terms();
                if (!PILOT && !ROWMAX) {
                    const uint32_t parked = min(*park_n, (uint32_t)kGemmPark);  // final: barriers since it was written
                    if ((uint32_t)tid < parked) fl_pos = atomicAdd(a.gcount + park_q[tid], 1);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (!kLate) issue(hslot, half_c);
            const int nslot = (hslot + 1) & (kGemmSlots - 1);
            if (!kDead) {
                if (!kLast) read_frags8(nslot, ga[kPar ^ 1], gb[kPar ^ 1]);
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 2; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ga[kPar][i], gb[kPar][j], acc[i][j], 0,
                                                                                     0, 0, 0, 0, 0);
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    if (!kLast) __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);      // LDS reads
                    if (!kLate) __builtin_amdgcn_sched_group_barrier(0x010, 1, 0);      // direct load
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (!kLate) advance();
            hslot = nslot;
        };
        if constexpr (ET == 0) {
            if (!kDead) read_frags(hslot, 0, fa[0], fb[0]);  // the step landed before the barrier of the step before it
            half(std::false_type{}, std::true_type{});   // the number of steps is at least 2
            for (int hs = 1; hs + 1 < nhs; ++hs) half(std::false_type{}, std::false_type{});
            half(std::true_type{}, std::false_type{});
        } else {
            if (!kDead) read_frags8(hslot, ga[0], gb[0]);
            for (int hs = 0; hs + 2 < nhs; hs += 2) {  // the number of steps is even
                half8(std::false_type{}, std::integral_constant<int, 0>{});
                half8(std::false_type{}, std::integral_constant<int, 1>{});
            }
            half8(std::false_type{}, std::integral_constant<int, 0>{});
            half8(std::true_type{}, std::integral_constant<int, 1>{});
        }

        if (ROWMAX) {
            // Row maxima: for each of the tile's rows the best of this block's queries.  A row's
            // positive scale does not change which query is best, so only the queries' scales enter.
            // A lane holds 4 queries of 32 rows.  It first picks, per row, the best of its 4 queries on
            // the fp32 scores (equal scores: the lower query) and only then forms the row's 64-bit key.
            // The 32 lanes that share those rows combine their keys with a butterfly that halves the
            // values a lane carries at every step (a lane keeps the rows whose index has its own lane
            // bit and hands the others to its partner: 16 + 8 + 4 + 2 + 1 exchanges instead of 5 x 32),
            // which leaves lane r32 of the group with the finished key of the group's r32-th row; it
            // adds that key to the row's key in global memory (64-bit atomic maximum; the other query
            // blocks and the other half of this block do the same).
            int qn[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) qn[j] = qb * kGemmTile + wn * 128 + j * 32 + r32;
            uint64_t val[32];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float bs = -INFINITY;
                    int bq = -1;
#pragma unroll
                    for (int j = 3; j >= 0; --j) {   // downwards: on equal scores the lower query stays
                        const float x = (ET == 1) ? acc[i][j][v] * qs[j] : acc[i][j][v];
                        if (qn[j] < a.Q && (bq < 0 || x >= bs)) {
                            bs = x;
                            bq = qn[j];
                        }
                    }
                    val[i * 16 + v] = bq >= 0 ? make_key(bs, (uint32_t)bq) : 0ull;
                }
#pragma unroll
            for (int bit = 4; bit >= 0; --bit) {
                const int half = 1 << bit;                     // values a lane still carries after this step
                const bool upper = ((r32 >> bit) & 1) != 0;    // this lane keeps the upper half of what it carries
#pragma unroll
                for (int t = 0; t < half; ++t) {
                    const uint64_t keep = upper ? val[half + t] : val[t];
                    const uint64_t send = upper ? val[t] : val[half + t];
                    const uint64_t got = __shfl_xor(send, half, kWave);   // the partner keeps the other half
                    val[t] = keep > got ? keep : got;
                }
            }
            const uint64_t mine = val[0];   // row index r32 = i * 16 + v of this group's rows
            {
                const int i = r32 >> 4, v = r32 & 15;
                const int r = wm * 64 + i * 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                if (r <= cur.last && mine > 0ull)
                    atomicMax(reinterpret_cast<unsigned long long *>(a.row_best) + row0 + r, (unsigned long long)mine);
            }
            continue;
        }
        if (PILOT) {
            // Pilot launch: the best key (score, then row) of every query over this tile's 256 sampled rows,
            // combined into the query's slice (tile of the sample modulo pilot_stride) with a 64-bit atomic
            // maximum.  The key names the row the score belongs to, so that the k-th largest key of a query's
            // slices is a key that k rows of the store reach, row ids included: among rows with exactly the
            // threshold's score (copies of one row) only those up to that id pass the selection.
            uint64_t *pmax = reinterpret_cast<uint64_t *>(hits);  // [kGemmTile] best key per query
            if (tid < 64) {
                *reinterpret_cast<f32x4 *>(bias_t + tid * 4) = bias_r;
                if (ET == 1) *reinterpret_cast<f32x4 *>(scale_t + tid * 4) = scale_r;
                if (DOM) *reinterpret_cast<i32x4 *>(dom_t + tid * 4) = dom_r;
            }
            if (tid < kGemmTile) pmax[tid] = 0ull;
            lds_barrier();
            float best[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            int brow[4] = {0, 0, 0, 0};   // row of the best score within the lane's rows: i * 32 + 8 * (v / 4) + v % 4
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                f32x4 bs[4], rs[4];
                i32x4 ds[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int rr = wm * 64 + i * 32 + 8 * u + 4 * h;
                    if (!kBiasInit) bs[u] = *reinterpret_cast<const f32x4 *>(bias_t + rr);
                    if (ET == 1) rs[u] = *reinterpret_cast<const f32x4 *>(scale_t + rr);
                    if (DOM) ds[u] = *reinterpret_cast<const i32x4 *>(dom_t + rr);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        float x = (ET == 1) ? acc[i][j][v] * (rs[v >> 2][v & 3] * qs[j]) + bs[v >> 2][v & 3]
                                            : acc[i][j][v];   // bf16: the bias is in it from the start
                        if (DOM && ds[v >> 2][v & 3] != 0 && ds[v >> 2][v & 3] != qd[j]) x = -INFINITY;
                        if (x > best[j]) {
                            best[j] = x;
                            brow[j] = i * 32 + 8 * (v >> 2) + (v & 3);
                        }
                    }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // row r of the tile is row r * ntiles + row0 of the sample, which is every row_stride-th row
                const int64_t sampled = (int64_t)(wm * 64 + 4 * h + brow[j]) * a.ntiles + row0;
                atomicMax(reinterpret_cast<unsigned long long *>(pmax) + wn * 128 + j * 32 + r32,
                          (unsigned long long)make_key(best[j], (uint32_t)(sampled * a.row_stride)));
            }
            lds_barrier();
            if (tid < kGemmTile) {
                const int q = qb * kGemmTile + tid;
                const uint32_t slice = (uint32_t)(row0 % a.pilot_stride);
                if (q < a.Q)
                    atomicMax(reinterpret_cast<unsigned long long *>(a.pilot_out) + (size_t)q * a.pilot_stride + slice,
                              (unsigned long long)pmax[tid]);
            }
            continue;  // the K-loop barriers of the next tile separate these reads from the next reset
        }
        if (fl_pos >= 0) append_global(park_q[tid], park_key[tid], fl_pos);
        if (tid < 64) {  // every wavefront is past the previous tile's epilogue (it has met this tile's barriers)
            *reinterpret_cast<f32x4 *>(bias_t + tid * 4) = bias_r;   // kBiasInit: the next tile's, read at its start
            if (ET == 1) *reinterpret_cast<f32x4 *>(scale_t + tid * 4) = scale_r;
            if (DOM) *reinterpret_cast<i32x4 *>(dom_t + tid * 4) = dom_r;
        }
        lds_barrier();   // the parked entries have been read by their flushers
        if (tid == 0) {
            *park_n = 0u;
            *hit_n = 0u;
        }
        lds_barrier();

        // ---- epilogue: score = dot * scales + bias (bf16: the accumulator as it is), compare with the query's threshold
        // accumulator v of tile (i, j) is row wm*64 + i*32 + 8*(v/4) + 4*h + v%4, query column wn*128 + j*32 + r32
        float thr_s[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = qb * kGemmTile + wn * 128 + j * 32 + r32;
            thr_s[j] = thr_raw[j] > kKeyFloor ? key_score(thr_raw[j]) : -INFINITY;
            if (q >= a.Q) thr_s[j] = __builtin_nanf("");  // padding query: no comparison with it holds, so nothing passes
        }
        // self-search: in the (at most two) row tiles that hold this query block's own rows, the
        // dot product of a query with itself is replaced by -inf before the scores are examined
        // (scales are positive, so the score stays -inf)
        const int64_t self0 = a.self_first + (int64_t)qb * kGemmTile;  // stored row of the block's first query
        if (a.self_first >= 0 && row0 < self0 + kGemmTile && row0 + kGemmTile > self0) {
            const int d0 = (int)(row0 - self0) + wm * 64 + 4 * h - wn * 128 - r32;  // row - query at i = j = v = 0
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (d0 + i * 32 + 8 * (v >> 2) + (v & 3) - j * 32 == 0) acc[i][j][v] = -INFINITY;
        }
        // sharing domains: the dot product of a query with a row it may not see becomes -inf, so that
        // such rows neither count against the threshold nor fill the lists
        if (DOM) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                i32x4 ds[4];
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    ds[u] = *reinterpret_cast<const i32x4 *>(dom_t + wm * 64 + i * 32 + 8 * u + 4 * h);
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        if (ds[v >> 2][v & 3] != 0 && ds[v >> 2][v & 3] != qd[j]) acc[i][j][v] = -INFINITY;
            }
        }
        if (AGAIN) {
            // A tile that listed more blocks than the list holds: every score is tested exactly by
            // the lane that holds it, and what passes is appended to its query's list at once.
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                f32x4 bs[4], rs[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int rr = wm * 64 + i * 32 + 8 * u + 4 * h;
                    if (!kBiasInit) bs[u] = *reinterpret_cast<const f32x4 *>(bias_t + rr);
                    if (ET == 1) rs[u] = *reinterpret_cast<const f32x4 *>(scale_t + rr);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int q = qb * kGemmTile + wn * 128 + j * 32 + r32;
                    if (q >= a.Q) continue;
                    const uint64_t t0 = thr_raw[j];
                    const uint64_t thr_k = t0 > kKeyFloor ? t0 - 1ull : kKeyFloor;   // the pilot's key itself passes
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float x = (ET == 1) ? acc[i][j][v] * (rs[v >> 2][v & 3] * qs[j]) + bs[v >> 2][v & 3]
                                                  : acc[i][j][v];   // bf16: the bias is in it from the start
                        const uint32_t row = (uint32_t)(row0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * h + (v & 3));
                        const uint64_t key = make_key(x, row);
                        if (key > thr_k && x > -INFINITY) append_global((uint32_t)q, key, atomicAdd(a.gcount + q, 1));
                    }
                }
            }
            continue;
        }
        // pass 1: 8 blocks of 16 scores per lane.  A lane whose block reaches the query's
        // threshold (about 17 lanes per tile) copies the block's scores to a small LDS list.
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            f32x4 bs[4], rs[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int rr = wm * 64 + i * 32 + 8 * u + 4 * h;
                if (!kBiasInit) bs[u] = *reinterpret_cast<const f32x4 *>(bias_t + rr);
                if (ET == 1) rs[u] = *reinterpret_cast<const f32x4 *>(scale_t + rr);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                f32x4 sc[4];
                float best = -INFINITY;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float x = (ET == 1) ? acc[i][j][v] * (rs[v >> 2][v & 3] * qs[j]) + bs[v >> 2][v & 3]
                                              : acc[i][j][v];   // bf16: the bias is in it from the start
                    sc[v >> 2][v & 3] = x;
                    best = fmaxf(best, x);
                }
                if (best >= thr_s[j]) {
                    const uint32_t slot = atomicAdd(hit_n, 1u);
                    const int q = qb * kGemmTile + wn * 128 + j * 32 + r32;
                    if (slot < (uint32_t)kGemmHits) {
                        HitEntry &e = hits[slot];
#pragma unroll
                        for (int u = 0; u < 4; ++u) e.sc[u] = sc[u];
                        e.q = (uint32_t)q;
                        e.row = (uint32_t)(row0 + wm * 64 + i * 32 + 4 * h);  // row of score 0; score v: + 8*(v/4) + v%4
                        e.thr = thr_raw[j];
                    }   // list full: the whole tile is left to a second launch, see below
                }
            }
        }
        lds_barrier();
        // pass 2: the listed blocks, one score per thread; what passes the exact key test is parked
        {
            // A tile that listed more blocks than the list holds (rows that suit many of the block's
            // queries at once, e.g. a high utility) keeps nothing: it goes on the list of tiles that a
            // second launch does again, testing every score; if that list is full too, the block's
            // queries are redone by the streaming scan.
            uint32_t nh = *hit_n;
            if (nh > (uint32_t)kGemmHits) {
                if (tid == 0) {
                    const uint32_t slot = atomicAdd(a.over_n, 1u);
                    if (slot < a.over_cap) {
                        a.over_list[slot] = make_uint2((uint32_t)(row0 / kGemmTile), (uint32_t)qb);
                    } else {
                        for (int b = qb * 4; b < qb * 4 + 4 && b * 64 < a.Q; ++b) a.redo[b] = 1;
                    }
                }
                nh = 0u;
            }
            const int v = tid & 15;
            for (uint32_t e = tid >> 4; e < nh; e += kGemmThreads / 16) {
                const HitEntry &he = hits[e];
                const float x = he.sc[v >> 2][v & 3];
                const uint64_t t0 = he.thr;
                const uint64_t thr_k = t0 > kKeyFloor ? t0 - 1ull : kKeyFloor;   // the pilot's key itself passes
                const uint32_t row = he.row + 8 * (v >> 2) + (v & 3);
                const uint64_t key = make_key(x, row);
                if (key > thr_k && x > -INFINITY) {
                    const uint32_t slot = atomicAdd(park_n, 1u);
                    if (slot < (uint32_t)kGemmPark) {
                        park_key[slot] = key;
                        park_q[slot] = he.q;
                    } else {   // more than kGemmPark candidates in one tile: appended at once
                        append_global(he.q, key, atomicAdd(a.gcount + he.q, 1));
                    }
                }
            }
        }
    }
    };
    const bool dead = half_block && wn == 1;  // wave-uniform; these are wavefronts 4-7, the late ones
    if (dead) run_tiles(std::true_type{}, std::true_type{}, std::true_type{});
    else if (half_block) run_tiles(std::false_type{}, std::false_type{}, std::true_type{});
    else if (late) run_tiles(std::true_type{}, std::false_type{}, std::false_type{});
    else run_tiles(std::false_type{}, std::false_type{}, std::false_type{});

    // the last tile's parked candidates; the direct loads of the unused extra stage must have landed
    // before the workgroup gives up its LDS
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const uint32_t parked = min(*park_n, (uint32_t)kGemmPark);
    for (uint32_t e = tid; e < parked; e += kGemmThreads) {
        const uint32_t q = park_q[e];
        append_global(q, park_key[e], atomicAdd(a.gcount + q, 1));
    }
}

// Step-major copy (layout: panel_word_offset in ic_common.h) of rows [first, last) of a row-major
// array, row_bytes apart.  Rows [last, fill_to) are written as zeros (the rest of the last tile:
// fill_to = last rounded up to a multiple of 256).  One thread per 16-byte granule.
__global__ __launch_bounds__(256) void to_panel(const uint8_t *__restrict__ rows, int row_bytes, int64_t first,
                                                int64_t last, int64_t fill_to, uint8_t *__restrict__ panel) {
    const int gpr = row_bytes >> 4;   // granules per row
    const int64_t total = (fill_to - first) * gpr;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = first + idx / gpr;
        const int gi = (int)(idx % gpr);
        i32x4 v = {0, 0, 0, 0};
        if (i < last) v = *reinterpret_cast<const i32x4 *>(rows + i * row_bytes + gi * 16);
        *reinterpret_cast<i32x4 *>(panel + panel_word_offset(i, gi * 4, row_bytes)) = v;
    }
}

// One launch before a tiled search: zero the slice maxima of the pilot, and the per-query counters,
// the redo flags and the list of overflowed tiles of the selection launch (count >= nq >= nblk).
__global__ void gemm_reset(uint64_t *keys, int64_t count, int32_t *gcount, int nq, int32_t *redo, int nblk,
                           uint32_t *over_n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) keys[i] = 0ull;
    if (i < nq) gcount[i] = 0;
    if (i < nblk) redo[i] = 0;
    if (i == 0) *over_n = 0u;
}

}  // namespace ic
