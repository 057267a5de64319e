// Streaming scan: similarity of a block of up to 64 queries with every cached
// row, fused with the per-slice partial top-k.  This is the O(N) step of
// IC-Cache's stage-1 relevance selection (Sec. 4.1; GetSimilarExamples in
// Algorithm 1) for small query batches, where the work is bound by reading the
// store from HBM once.
//
// Shape of the computation
//   * A workgroup (4 wavefronts) owns slice s of the cache, a contiguous range of
//     16-row tiles (a pilot: the tiles s, s+S, s+2S, ... of its sample), and one
//     block of QG*16 queries.
//   * The embedding dimension is split over the 4 wavefronts: wavefront w owns
//     CPW consecutive 64-byte chunks of every row.  Its share of the query block
//     stays in registers for the whole kernel (QG*CPW 16-byte fragments).  The
//     MFMA operand layout is: lane (r = lane%16, c = lane/16) holds 16 bytes of
//     row r at chunk offset 16*c, the A-operand layout of v_mfma_f32_16x16x32
//     (row r, 8 consecutive k).  Queries use the same byte mapping for the B
//     operand, so every product pairs equal coordinates.
//   * Row tiles are loaded several tiles ahead into register stages.  With an
//     even CPW a wavefront's share of a row is whole 128-byte lines, and a load
//     instruction fetches one full line of each of 8 rows, non-temporal (the
//     memory system serves that pattern about 12 % faster than half a line of
//     each of 16 rows); when a stage is consumed its fragments pass through a
//     small LDS buffer private to the wavefront into the operand layout.  With
//     an odd CPW the loads are made directly in the operand layout.
//   * The 4 partial 16x16 score tiles are exchanged through LDS (one buffer,
//     two barriers per tile) and summed in a fixed order by wavefront g < QG, which owns query group g from then on:
//     score = dot * scales + bias, where bias = lambda * utility, or -inf for an
//     invalid row (make_bias prepares it once per search).
//   * Selection: each query has a candidate region of `cap` keys and a
//     threshold key in LDS.  A score that beats the threshold is appended; when
//     the region is full the owning wavefront ranks its keys, keeps the best k
//     (sorted) and raises the threshold to the k-th.  Only candidates that beat
//     the k-th best so far are ever kept, so the score matrix never leaves
//     registers, and the rare path touches LDS only: it never waits on the row
//     loads that are in flight.
//   * At the end the regions and their sizes are written out; a merge kernel
//     combines the S regions of every query.
//   * Pilot variant (PILOT = true).  The same kernel run over every tile_mul-th row (a uniform
//     sample of the rows, 16 sampled rows to a tile) keeps, per query, only the best score of its slice.  With S >= k slices the k-th
//     largest of those S maxima is a score that at least k rows reach, i.e. a
//     valid starting threshold for the full scan, which then appends only the few
//     rows that beat it instead of warming its thresholds up slice by slice.
#pragma once
#include "ic_common.h"

namespace ic {

struct ScanArgs {
    const uint8_t *store;    // [n] rows, row_bytes apart
    int64_t n;               // rows in the index (>= 1)
    int row_bytes;           // multiple of 128
    const float *row_scale;  // fp8: [round_up(n,16)] fp32.  bf16: unused
    // Additive term of the score, read as bias[i * bias_stride]: lambda * utility for valid
    // rows and -inf for invalid ones ([round_up(n,16)] fp32, stride 1, written by make_bias),
    // or four zeros with stride 0 when the search has neither utility weight nor mask, so
    // that the load in the main loop is unconditional.
    const float *bias;
    int bias_stride;
    const uint8_t *qbuf;     // prepared queries, [gridDim.y * QG*16] rows, row_bytes apart
    const float *q_scale;    // per prepared query (fp8) or NULL
    int Q;                   // real queries in qbuf
    int k;
    int cap;                 // region capacity: multiple of 16, k < cap <= kMaxCap
    int S;                   // slices == gridDim.x
    uint64_t *regions;       // [Q][S][cap] keys
    int32_t *counts;         // [Q][S] keys in use
    int tile_mul;            // PILOT kernels score rows 0, tile_mul, 2*tile_mul, ... only
    uint64_t *pilot_out;     // PILOT kernels: [Q][S] keys (best score of the slice, id = slice)
    const uint64_t *thr_init;  // full scan: per query, key of a score that >= k rows reach, or NULL
    const int32_t *redo;     // if not NULL (QG == 4 only): query blocks whose flag is 0 are skipped
    // Set when thr_init was computed by a different kernel (the tiled scan's pilot): that kernel adds
    // the products in another order, so the score it saw for the k-th row may be a few ulps above
    // what this kernel computes for the same row, which would then miss its own threshold.  The
    // starting score s is lowered by this much (absolute) plus 2^-17 (|s| + 2).  The tiled bf16 scan
    // starts its sums at the bias b, so each of its d/16 <= 64 partial sums is rounded at the magnitude
    // |b| + 1, and the two kernels differ by at most about 65 * 2^-24 (|b| + 1) on a row; a row whose
    // score lies that close to s has |b| <= |s| + 1, and rows further above s pass anyway.  A lower
    // start only admits more candidates, the selection stays exact.
    float thr_slack;
    // Task launches (TASK = true, one query group): workgroup column y is one list of a cluster-pruned
    // search together with up to 16 (query, list) pairs that probe it, so that the list is read once
    // for all of them.  The list is the contiguous range [offsets[c], offsets[c + 1]) of a store sorted
    // by cluster, c = task_cluster[y] (-1: no task).  Query slot j of the workgroup serves pair
    // task_pair[16 y + j] (-1: empty slot), i.e. query pair / task_nprobe; regions / counts are indexed
    // by the pair instead of the query, and the counts of pairs no task serves are left as the caller
    // set them (zero).
    const int64_t *task_cluster;
    const int64_t *task_offsets;
    const int32_t *task_pair;
    int task_nprobe;
    // Sharing domains (DOM = true): row i is visible to query q if row_dom[i] == 0 (public) or
    // row_dom[i] == q_dom[q].  row_dom is [round_up(n,16)] int32, q_dom [Q] int32.
    const int32_t *row_dom;
    const int32_t *q_dom;
};

constexpr int kScanWaves = 4;
constexpr int kMaxCap = 192;
// Line-mode loads (even CPW): a wavefront's private LDS buffer in which a pair of 64-byte chunks of
// 16 rows is turned from the layout it was loaded in (8 rows x 128 B per instruction) into the MFMA
// operand layout.  144 B per row: the 16 lanes that read the same column of 16 rows hit 16 different banks.
constexpr int kTransRow = 144;
constexpr int kTransBytes = 16 * kTransRow;

// Dynamic LDS of scan_stream for a block of QG*16 queries with region capacity cap.
__host__ __device__ constexpr size_t scan_lds_bytes(int qg, int cap) {
    return (size_t)kScanWaves * qg * 64 * 16 * (qg < 4 ? 2 : 1)   // partial score tiles (two sets when they are small)
           + (size_t)qg * 16 * cap * 8         // candidate regions
           + (size_t)qg * 16 * (8 + 4)         // threshold keys, region sizes
           + (qg < 4 ? (size_t)kScanWaves * kTransBytes : 0);  // transposition buffers (QG = 4: inside the partial tiles)
}

// Score bias of every row for one search: lambda * utility where the row is valid, -inf
// where the mask excludes it, where the row has been invalidated (live[i] == 0) and for the
// padding rows [n, n_pad).  util, mask and live may be NULL.
__global__ __launch_bounds__(256) void make_bias(const float *__restrict__ util,
                                                 const uint8_t *__restrict__ mask,
                                                 const uint8_t *__restrict__ live, int64_t n,
                                                 int64_t n_pad, float lambda, float *__restrict__ bias) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t step = (int64_t)gridDim.x * 256;
    for (; i < n_pad; i += step) {
        float b = -INFINITY;
        if (i < n && (!mask || mask[i] != 0) && (!live || live[i] != 0)) b = util ? lambda * util[i] : 0.0f;
        bias[i] = b;
    }
}

// Keep the best k keys of a full region of c keys (c a multiple of 4, at most 64*NT; the
// survivors end up sorted, best first) and publish the k-th as the new threshold.  Runs on
// one whole wavefront, in LDS only.  Keys are unique, so rank = number of greater keys is a
// permutation of 0..c-1.
template <int NT>
__device__ __forceinline__ void compact_region(uint64_t *reg, int c, int k, uint64_t *thr_slot,
                                               uint32_t *cnt_slot, int lane) {
    typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
    uint64_t mine[NT];
    int rank[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int idx = lane + 64 * t;
        mine[t] = (idx < c) ? reg[idx] : 0ull;
        rank[t] = 0;
    }
#pragma unroll 2
    for (int i = 0; i < c; i += 4) {
        const u64x2 o01 = *reinterpret_cast<const u64x2 *>(reg + i);
        const u64x2 o23 = *reinterpret_cast<const u64x2 *>(reg + i + 2);
#pragma unroll
        for (int t = 0; t < NT; ++t)
            rank[t] += (int)(o01.x > mine[t]) + (int)(o01.y > mine[t]) + (int)(o23.x > mine[t]) +
                       (int)(o23.y > mine[t]);
    }
    __builtin_amdgcn_wave_barrier();  // every lane has read the region before any lane rewrites it
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int idx = lane + 64 * t;
        if (idx < c && rank[t] < k) {
            reg[rank[t]] = mine[t];
            if (rank[t] == k - 1) *thr_slot = mine[t];
        }
    }
    if (lane == 0) *cnt_slot = (uint32_t)(c < k ? c : k);
    __builtin_amdgcn_wave_barrier();
}

template <int ET, int QG, int CPW, bool PILOT, bool TASK = false, bool DOM = false>
__global__ __launch_bounds__(256) void scan_stream(const ScanArgs a) {
    static_assert(!TASK || (QG == 1 && !PILOT), "task launches use one query group and no pilot");
    constexpr int QB = QG * 16;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_dyn[];
    uint8_t *lds_raw = static_cast<uint8_t *>(__builtin_assume_aligned(lds_dyn, 16));
    typedef f32x4 PartTile[kScanWaves][QG][64];
    // With one or two query groups the partial tiles are small and there are two sets of them, used
    // by alternate tiles: a wavefront then cannot overwrite a set before every wavefront has passed
    // the next tile's barrier, i.e. has read it, and one barrier per tile is enough.
    constexpr bool kTwoSets = QG < 4;
    PartTile *parts = reinterpret_cast<PartTile *>(lds_raw);
    uint64_t *regs = reinterpret_cast<uint64_t *>(lds_raw + sizeof(PartTile) * (kTwoSets ? 2 : 1));  // [QB][cap]
    uint64_t *thr_key = regs + QB * (PILOT ? 0 : a.cap);                          // [QB]; a pilot has no regions
    uint32_t *cnt = reinterpret_cast<uint32_t *>(thr_key + QB);                   // [QB]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront index, kept scalar
    // Line mode: with an even number of chunks per wavefront its share of a row is whole 128-byte
    // lines, and a load instruction fetches one line of each of 8 rows (non-temporal) instead of
    // half a line of each of 16; the fragments then pass through this wavefront's LDS buffer.
    // With QG = 4 the buffer is the wavefront's own 4 KB of the partial tiles: it is used before
    // the wavefront writes its partial sums, and nobody reads those until the barrier after.
    constexpr bool LINES = (CPW % 2 == 0);
    uint8_t *trans = (QG == 4) ? reinterpret_cast<uint8_t *>(&parts[0][w][0][0])
                               : reinterpret_cast<uint8_t *>(cnt + QB) + w * kTransBytes;
    static_assert(QG < 4 || sizeof(f32x4) * QG * 64 >= (size_t)kTransBytes, "partial tiles hold the buffer");
    const int r16 = lane & 15;  // row within tile (A operand) / query within group (B, D)
    const int c4 = lane >> 4;   // 16-byte column within a 64-byte chunk; D rows 4*c4 .. 4*c4+3
    const int s = blockIdx.x;
    const int qb = blockIdx.y;
    // rows this workgroup may select from: the whole store, or one cluster's range
    int64_t row_lo = 0, row_hi = a.n;
    if (TASK) {
        const int64_t c = a.task_cluster[qb];
        row_lo = c >= 0 ? a.task_offsets[c] : 0;
        row_hi = c >= 0 ? a.task_offsets[c + 1] : 0;
        if (row_lo >= row_hi) return;  // no task, or an empty list: the pairs' counts stay zero
    }
    const int nchunks = a.row_bytes >> 6;
    const int chunk0 = w * CPW;
    if (a.redo && a.redo[qb] == 0) return;  // whole workgroup: this block needs no second pass

    // Starting threshold of a query: nothing, or "any row whose score reaches the pilot's
    // score" (the key just below the smallest key with that score).
    auto start_threshold = [&](int q) -> uint64_t {
        if (!a.thr_init || q >= a.Q) return kKeyFloor;
        const uint64_t t0 = a.thr_init[q];
        if (t0 <= kKeyFloor) return kKeyFloor;
        if (a.thr_slack > 0.0f) {
            const float s0 = key_score(t0);
            const float s1 = s0 - (a.thr_slack + (fabsf(s0) + 2.0f) * 0x1p-17f);
            return ((uint64_t)ord_of_score(s1) << 32) - 1ull;
        }
        return ((t0 >> 32) << 32) - 1ull;
    };
    if (tid < QB && !PILOT) {
        thr_key[tid] = TASK ? kKeyFloor : start_threshold(qb * QB + tid);
        cnt[tid] = 0u;
    }

    // Byte offset of each chunk this wavefront owns.  When the row has fewer chunks than
    // 4*CPW the surplus slots re-read the last chunk against a zero query fragment, which
    // keeps the main loop free of branches.
    int coff[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) coff[c] = (chunk0 + c < nchunks ? chunk0 + c : nchunks - 1) * 64;
    // line mode: byte offset of each line this wavefront owns (a surplus line re-reads the row's last)
    int loff[(CPW + 1) / 2];
#pragma unroll
    for (int j = 0; j < (CPW + 1) / 2; ++j) loff[j] = (chunk0 + 2 * j < nchunks ? chunk0 + 2 * j : nchunks - 2) * 64;
    const int l8 = lane >> 3;   // line mode: row within a half tile, and the lane's 16 bytes of the line
    const int p8 = lane & 7;

    // task launches: the pair and the query of this lane's slot
    const int task_p = TASK ? a.task_pair[(int64_t)qb * 16 + r16] : -1;
    const int task_q = task_p >= 0 ? task_p / a.task_nprobe : 0;
    // query fragments owned by this wavefront, resident for the whole kernel
    i32x4 qf[QG][CPW];
#pragma unroll
    for (int g = 0; g < QG; ++g) {
        // task launches: slot r16 holds the query of the pair it serves (an empty slot: query 0, never live)
        const uint8_t *qrow = a.qbuf + (int64_t)(TASK ? task_q : qb * QB + g * 16 + r16) * a.row_bytes + c4 * 16;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            qf[g][c] = *reinterpret_cast<const i32x4 *>(qrow + coff[c]);
            if (chunk0 + c >= nchunks) qf[g][c] = i32x4{0, 0, 0, 0};
        }
    }

    // selection state of the query this lane serves in the epilogue (wave g == w)
    const int jl = (w < QG ? w : 0) * 16 + r16;  // query within block
    const int jq = TASK ? task_q : qb * QB + jl;  // query within this launch
    const bool q_live = (w < QG) && (jq < a.Q) && (!TASK || task_p >= 0);
    float q_scale = 1.0f;
    if (ET == 1 && q_live) q_scale = a.q_scale[jq];
    int q_dom = 0;
    if (DOM && q_live) q_dom = a.q_dom[jq];
    uint64_t *region = regs + jl * a.cap;
    uint64_t thr_k = (q_live && !TASK) ? start_threshold(jq) : kKeyFloor;
    float thr_s = thr_k > kKeyFloor ? key_score(thr_k + 1ull) : -INFINITY;
    float best = -INFINITY;  // pilot mode: best score of this lane's rows

    __syncthreads();

    // A pilot scores rows 0, tile_mul, 2 * tile_mul, ... only, and row r of its t-th tile is row
    // r * ntiles + t of that sample: every tile, and with it every slice, is a uniform sample of the
    // store whatever the order the rows arrived in.  Below, last_row of a pilot counts sampled rows.
    const int64_t tile_mul = PILOT ? a.tile_mul : 1;
    const int64_t tile0 = row_lo >> 4;  // first tile of the range (0 unless TASK)
    const int64_t last_row = PILOT ? (row_hi - 1) / tile_mul : row_hi - 1;
    const int64_t ntiles = ((last_row + 16) >> 4) - tile0;  // tiles this launch visits
    const int64_t S = a.S;

    // Everything a tile needs from global memory, requested kStages - 1 tiles ahead: two tiles for
    // long rows, four when a wavefront's share of a row is at most 4 chunks (the stages are small
    // then, and short rows need more tiles in flight to cover the memory latency).  The loads are
    // unconditional (indices are clamped), so the only waits in the loop are counted waits for the
    // oldest stage.
    constexpr int kStages = (CPW <= 4) ? 5 : 3;
    struct Stage {
        i32x4 rows[CPW];
        f32x4 bias;
        i32x4 dom;   // DOM only
        f32x4 rsc;
    };
    Stage st[kStages];
    auto load_stage = [&](int64_t t, Stage &x) {
        const int64_t tt = tile0 + (t < ntiles ? t : ntiles - 1);
        if (LINES) {
            int64_t r0 = PILOT ? l8 * ntiles + tt : tt * 16 + l8, r1 = r0 + (PILOT ? 8 * ntiles : 8);
            if (r0 > last_row) r0 = last_row;  // ragged tail: re-read a valid row, masked out later
            if (r1 > last_row) r1 = last_row;
            const uint8_t *p0 = a.store + r0 * tile_mul * (int64_t)a.row_bytes + p8 * 16;
            const uint8_t *p1 = a.store + r1 * tile_mul * (int64_t)a.row_bytes + p8 * 16;
#pragma unroll
            for (int c = 0; c < CPW; ++c)
                x.rows[c] = __builtin_nontemporal_load(
                    reinterpret_cast<const i32x4 *>(((c & 1) ? p1 : p0) + loff[c >> 1]));
        } else {
            int64_t r = PILOT ? r16 * ntiles + tt : tt * 16 + r16;
            if (r > last_row) r = last_row;
            const uint8_t *p = a.store + r * tile_mul * (int64_t)a.row_bytes + c4 * 16;
#pragma unroll
            for (int c = 0; c < CPW; ++c) x.rows[c] = *reinterpret_cast<const i32x4 *>(p + coff[c]);
        }
        const int64_t i0 = tt * 16 + c4 * 4;
        if (PILOT) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int64_t sampled = (c4 * 4 + v) * ntiles + tt;
                const int64_t at = (sampled <= last_row ? sampled : last_row) * tile_mul;
                x.bias[v] = a.bias[at * a.bias_stride];
                if (DOM) x.dom[v] = a.row_dom[at];
                if (ET == 1) x.rsc[v] = a.row_scale[at];
            }
        } else {
            x.bias = *reinterpret_cast<const f32x4 *>(a.bias + i0 * a.bias_stride);
            if (DOM) x.dom = *reinterpret_cast<const i32x4 *>(a.row_dom + i0);
            if (ET == 1) x.rsc = *reinterpret_cast<const f32x4 *>(a.row_scale + i0);
        }
    };

    // The loop body is unrolled by kStages so that the stage buffers are addressed statically.
    // Tiles past the end of the slice (when its tile count is not a multiple of kStages) are
    // processed like any other: their loads are clamped and all their rows fall past
    // last_row, so they contribute no candidate.
    // Which tiles a slice takes.  A full scan gives slice s the contiguous range of tiles
    // [s * per, (s + 1) * per): every workgroup then reads one sequential stream, and the streams are
    // spread over the whole store.  (Tiles s, s + S, s + 2S, ... make all workgroups walk the store side
    // by side, inside the same 16 * S rows at any time; the memory system serves that 2 % slower for
    // 1.5 KB rows and 9 % slower for 1 KB rows.)  The selection does not depend on how the tiles are
    // dealt.  A pilot keeps the interleaved order: its tiles are samples spread over the store anyway.
    constexpr bool kBlocked = !PILOT;
    const int64_t per = (ntiles + S - 1) / S;
    const int64_t mine0 = (int64_t)s * per;   // kBlocked: the slice's first tile
    const int64_t my_tiles = kBlocked ? (mine0 < ntiles ? (ntiles - mine0 < per ? ntiles - mine0 : per) : 0)
                                      : ((s < ntiles) ? (ntiles - s + S - 1) / S : 0);
    auto tile_at = [&](int64_t j) -> int64_t {   // the j-th tile this slice visits; past its end: a tile no row is in
        if (j >= my_tiles) return ntiles + s;
        return kBlocked ? mine0 + j : s + j * S;
    };
    int64_t j = 0;
    int64_t t = tile_at(0);
#pragma unroll
    for (int b = 0; b + 1 < kStages; ++b) load_stage(tile_at(b), st[b]);

    int set = 0;   // which set of partial tiles this tile uses
    for (int64_t it = 0; it < my_tiles; it += kStages) {
#pragma unroll
        for (int b = 0; b < kStages; ++b) {
            {
                PartTile &part = parts[kTwoSets ? set : 0];
                set ^= 1;
                load_stage(tile_at(j + kStages - 1), st[(b + kStages - 1) % kStages]);
                const Stage &cur = st[b];

                // operand fragments: lane (r16, c4) holds bytes [16*c4, 16*c4 + 16) of chunk c of row r16
                i32x4 op[CPW];
                if (LINES) {
                    // The LDS unit executes a wavefront's instructions in order, so the reads below
                    // see the writes above them without a wait, and the next pair's writes cannot
                    // overtake these reads; the wave barriers only pin the compiler's order.
#pragma unroll
                    for (int j = 0; j < CPW / 2; ++j) {
                        *reinterpret_cast<i32x4 *>(trans + l8 * kTransRow + p8 * 16) = cur.rows[2 * j];
                        *reinterpret_cast<i32x4 *>(trans + (8 + l8) * kTransRow + p8 * 16) = cur.rows[2 * j + 1];
                        asm volatile("" ::: "memory");
                        __builtin_amdgcn_wave_barrier();
                        op[2 * j] = *reinterpret_cast<const i32x4 *>(trans + r16 * kTransRow + c4 * 16);
                        op[2 * j + 1] = *reinterpret_cast<const i32x4 *>(trans + r16 * kTransRow + 64 + c4 * 16);
                        asm volatile("" ::: "memory");
                        __builtin_amdgcn_wave_barrier();
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < CPW; ++c) op[c] = cur.rows[c];
                }

                f32x4 acc[QG];
#pragma unroll
                for (int g = 0; g < QG; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};
                // fp8: pairs of chunks go through one v_mfma_f32_16x16x128_f8f6f4 (32 bytes per lane and
                // operand, scale operands 0 = unscaled; twice the rate of four 16x16x32 instructions); rows
                // and queries pair the same bytes, and the order inside a dot product is free
                // (only for an even number of chunks: the two forms are not mixed on one accumulator; and
                // only with four query groups, where it is 3-6 % faster on 1 KB rows: with two groups it
                // measured 2-5 % slower, with one the same)
                constexpr int kWide = (ET == 1 && CPW % 2 == 0 && QG == 4) ? CPW : 0;   // chunks that go in pairs
#pragma unroll
                for (int c = 0; c < kWide; c += 2) {
#pragma unroll
                    for (int g = 0; g < QG; ++g) {
                        i32x8 ra, qa;
                        ra.lo = op[c];
                        ra.hi = op[c + 1];
                        qa.lo = qf[g][c];
                        qa.hi = qf[g][c + 1];
                        acc[g] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(ra, qa, acc[g], 0, 0, 0, 0, 0, 0);
                    }
                }
#pragma unroll
                for (int c = kWide; c < CPW; ++c) {
#pragma unroll
                    for (int g = 0; g < QG; ++g) {
                        if (ET == 0) {
                            acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                                __builtin_bit_cast(bf16x8, op[c]), __builtin_bit_cast(bf16x8, qf[g][c]),
                                acc[g], 0, 0, 0);
                        } else {
                            const i64x2 ra = __builtin_bit_cast(i64x2, op[c]);
                            const i64x2 qa = __builtin_bit_cast(i64x2, qf[g][c]);
                            acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(ra.x, qa.x, acc[g], 0, 0, 0);
                            acc[g] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(ra.y, qa.y, acc[g], 0, 0, 0);
                        }
                    }
                }
#pragma unroll
                for (int g = 0; g < QG; ++g) part[w][g][lane] = acc[g];
                __syncthreads();
                f32x4 sum = {0.f, 0.f, 0.f, 0.f};
                if (w < QG) {
                    sum = part[0][w][lane];
                    sum += part[1][w][lane];
                    sum += part[2][w][lane];
                    sum += part[3][w][lane];
                }
                if (!kTwoSets) __syncthreads();  // the partial tiles may be overwritten from here on

                if (w < QG) {
                    // first of this lane's 4 rows; a pilot's are sampled rows i0, i0 + ntiles, ...
                    const int64_t i0 = PILOT ? c4 * 4 * ntiles + t : (tile0 + t) * 16 + c4 * 4;
                    const int64_t i_step = PILOT ? ntiles : 1;
                    uint64_t key[4];
                    uint32_t pend = 0;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        float sc = (ET == 1) ? sum[v] * (cur.rsc[v] * q_scale) + cur.bias[v]
                                             : sum[v] + cur.bias[v];
                        if (i0 + v * i_step > last_row || (PILOT && t >= ntiles)) sc = -INFINITY;
                        if (DOM && cur.dom[v] != 0 && cur.dom[v] != q_dom) sc = -INFINITY;  // another domain's row
                        if (TASK && i0 + v < row_lo) sc = -INFINITY;  // the first tile may start in the previous list
                        if (PILOT) {
                            best = fmaxf(best, sc);
                            continue;
                        }
                        key[v] = 0;
                        if (q_live && sc >= thr_s) {
                            key[v] = make_key(sc, (uint32_t)(i0 + v));
                            if (key[v] > thr_k) pend |= 1u << v;
                        }
                    }
                    // Rare path: at least one lane of this wavefront has a candidate.  A lane
                    // claims as many slots of its query's region as it has candidates with one
                    // LDS atomic and fills the ones that exist; what does not fit stays pending
                    // until the region has been compacted.
                    while (__ballot(pend != 0) != 0ull) {
                        if (pend) {
                            uint32_t slot = atomicAdd(&cnt[jl], (uint32_t)__popc(pend));
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                if (((pend >> v) & 1u) && slot < (uint32_t)a.cap) {
                                    region[slot++] = key[v];
                                    pend &= ~(1u << v);
                                }
                            }
                        }
                        uint64_t over = __ballot(pend != 0);
                        if (over == 0ull) break;
                        // queries whose region overflowed: full by construction, compact them
                        const uint32_t fullmask = (uint32_t)((over | (over >> 16) | (over >> 32) | (over >> 48)) & 0xFFFFull);
                        __builtin_amdgcn_wave_barrier();
                        for (int j = 0; j < 16; ++j) {
                            if ((fullmask >> j) & 1u) {
                                const int ql = w * 16 + j;
                                uint64_t *reg = regs + ql * a.cap;
                                if (a.cap <= 64) compact_region<1>(reg, a.cap, a.k, &thr_key[ql], &cnt[ql], lane);
                                else if (a.cap <= 128) compact_region<2>(reg, a.cap, a.k, &thr_key[ql], &cnt[ql], lane);
                                else compact_region<3>(reg, a.cap, a.k, &thr_key[ql], &cnt[ql], lane);
                            }
                        }
                        thr_k = __hip_atomic_load(&thr_key[jl], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                        thr_s = key_score(thr_k);
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (((pend >> v) & 1u) && !(key[v] > thr_k)) pend &= ~(1u << v);
                    }
                }
                t = tile_at(++j);
            }
        }
    }

    if (PILOT) {
        // best score of the slice per query: combine the four lanes that share a query
        best = fmaxf(best, __shfl_xor(best, 16, kWave));
        best = fmaxf(best, __shfl_xor(best, 32, kWave));
        if (q_live && c4 == 0) a.pilot_out[(int64_t)jq * a.S + s] = make_key(best, (uint32_t)s);
        return;
    }
    // hand the regions to the merge kernel
    if (w < QG) {
        for (int j = 0; j < 16; ++j) {
            const int ql = w * 16 + j;
            const int qq = TASK ? a.task_pair[(int64_t)qb * 16 + j] : qb * QB + ql;     // row of regions / counts
            if (TASK && qq < 0) continue;   // empty slot
            if (!TASK && qq >= a.Q) break;
            uint32_t c = __hip_atomic_load(&cnt[ql], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
            if (c > (uint32_t)a.cap) c = (uint32_t)a.cap;
            uint64_t *out = a.regions + ((int64_t)qq * a.S + s) * a.cap;
            for (int idx = lane; idx < (int)c; idx += 64) out[idx] = regs[ql * a.cap + idx];
            if (lane == 0) a.counts[(int64_t)qq * a.S + s] = (int32_t)c;
        }
    }
}

}  // namespace ic
