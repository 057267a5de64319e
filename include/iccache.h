/*
 * iccache.h -- C ABI of the MI355X example-selection library.
 *
 * The library implements stage 1 of IC-Cache's Example Selector (Sec. 4.1,
 * "Two-Stage Scalable Example Selection"; GetSimilarExamples in Algorithm 1):
 * a batch of request embeddings is compared with every cached example embedding
 * by cosine similarity and the most similar examples are returned.  Two
 * per-example inputs model what the Example Manager (Sec. 4.3) maintains: a
 * utility value that is blended into the score, and a validity flag (evicted
 * rows, rows outside the caller's sharing domain).
 *
 *   score(q, i) = cos(query_q, example_i) + lambda * utility_i
 *   result_q    = the k valid examples with the highest score, ordered by
 *                 (score descending, id ascending)
 *
 * Conventions
 *   - Every pointer named *_dev is DEVICE memory on the GPU that was current
 *     when the index was created; everything else is host memory.
 *   - The caller owns every buffer it passes (arena, inputs, outputs) and keeps
 *     it alive until the stream has drained.  The library owns only the small
 *     host-side handle.  It never allocates or frees device memory.
 *   - All work is enqueued on the index's stream and is asynchronous; calls on
 *     one index are ordered.  No call synchronises the host except
 *     ic_index_scan_time_ms, ic_index_tiled_scan_counts, ic_index_compact and the
 *     ic_ivf_* calls that say so.
 *   - Calls on one index are NOT re-entrant: every search, the const ones included,
 *     uses the index's query block and top-k workspace in the arena and a few host
 *     fields of the handle (timing events, diagnostics).  The caller serialises the
 *     calls on one index (one thread, or a lock); different indices are independent.
 *   - Example ids are append order: 0-based, dense, stable (until ic_index_compact
 *     renumbers the surviving rows).
 *   - Errors are returned as ic_status; nothing throws or aborts.  On error the
 *     outputs are untouched.  Inputs must be finite.
 */
#ifndef ICCACHE_H
#define ICCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ic_index ic_index; /* opaque */

typedef enum {
    IC_OK = 0,
    IC_ERR_INVALID_ARG = 1, /* NULL where forbidden, size out of range, misaligned arena */
    IC_ERR_OOM = 2,         /* host allocation of the handle failed                       */
    IC_ERR_CAPACITY = 3,    /* arena too small, or append beyond capacity_rows            */
    IC_ERR_DEVICE = 4,      /* a HIP call failed                                          */
    IC_ERR_UNSUPPORTED = 5  /* valid request outside what the kernels cover               */
} ic_status;

/* Store formats (one per index).  Rows are unit-normalised on append. */
typedef enum {
    IC_STORE_BF16 = 0,     /* bfloat16, round to nearest even                              */
    IC_STORE_FP8_E4M3 = 1  /* OCP FP8 E4M3 (max 448) with one fp32 scale per row           */
} ic_dtype;

#define IC_MAX_K 128        /* largest k accepted by ic_search                             */
#define IC_MAX_DIM 1024     /* largest embedding dimension for bf16 (2048 for fp8)         */
#define IC_ARENA_ALIGN 256  /* required alignment of the arena pointer, bytes              */

/*
 * Bytes of device memory an index needs: the embedding store (rows padded to a
 * multiple of 128 B), per-row scale, utility and validity arrays, the prepared query
 * block, and the top-k workspace for searches of up to max_queries queries per
 * call with k <= max_k.  With max_queries >= 65 the index also keeps a second copy of
 * the store, ordered for the large-batch scan (as large as the store itself, kept up to
 * date by ic_index_append and ic_index_compact): an index that will only ever see
 * batches of up to 64 queries should say so and gets by with half the memory.
 * Returns 0 if an argument is out of range.
 */
size_t ic_workspace_bytes(int32_t d, ic_dtype store, int64_t capacity_rows,
                          int64_t max_queries, int32_t max_k);

/*
 * Create an empty index over caller-owned device memory: the cache of request-response
 * examples that the Example Manager keeps (Sec. 3, system overview; Sec. 4.3), as the
 * embedding store the selector searches.  Nothing is launched and the arena is not touched.
 *   out            receives the handle
 *   d              embedding dimension, 1 .. IC_MAX_DIM (2*IC_MAX_DIM for fp8)
 *   capacity_rows  most rows the store will ever hold (>= 1)
 *   max_queries    largest Q a single ic_search will be given (>= 1); larger
 *                  batches are still accepted and are processed in pieces
 *   max_k          largest k a search will use, 1 .. IC_MAX_K
 *   arena_dev      device memory, IC_ARENA_ALIGN-aligned, arena_bytes >=
 *                  ic_workspace_bytes(d, store, capacity_rows, max_queries, max_k)
 *   stream         hipStream_t (NULL = default stream) used by every later call
 * Errors: INVALID_ARG, CAPACITY (arena too small), OOM, DEVICE.
 */
ic_status ic_index_create(ic_index **out, int32_t d, ic_dtype store, int64_t capacity_rows,
                          int64_t max_queries, int32_t max_k, void *arena_dev,
                          size_t arena_bytes, void *stream);

/*
 * Append n examples (the update_cache step of the client API, Sec. 3; step 4 of
 * the workflow).  emb_dev is [n, d] fp32 row-major; each row is divided by its
 * Euclidean norm (a zero row stays zero) and stored in the index's format.
 * util_dev is [n] fp32 or NULL (utility 0).  *first_id (host, may be NULL)
 * receives the id of the first appended row.  Cost is O(n); the existing store
 * is not touched.  Appended rows are visible to every later search.
 * Errors: INVALID_ARG, CAPACITY (n would exceed capacity_rows), DEVICE.
 */
ic_status ic_index_append(ic_index *index, const float *emb_dev, const float *util_dev,
                          int64_t n, int64_t *first_id);

/*
 * Top-k selection for Q queries (GetSimilarExamples, Algorithm 1).
 *   q_dev           [Q, d] fp32 row-major; rows need not be unit length
 *   k               1 .. max_k given at creation
 *   lambda          weight of the stored utility (0 = pure cosine); any sign and size as long
 *                   as lambda * utility stays above -1e30 (a score at or below that is
 *                   treated as no score, like a masked row's)
 *   mask_dev        [size] uint8, nonzero = valid, shared by all queries; NULL =
 *                   all rows valid.  size is the index size at the time of call.
 *   out_scores_dev  [Q, k] fp32; out_ids_dev [Q, k] int64.  Rows are sorted by
 *                   (score descending, id ascending).  If fewer than k valid rows
 *                   exist the tail is (score = -inf, id = -1).
 * Q == 0 is a no-op.  Errors: INVALID_ARG, DEVICE.
 */
ic_status ic_search(const ic_index *index, const float *q_dev, int64_t Q, int32_t k,
                    float lambda, const uint8_t *mask_dev, float *out_scores_dev,
                    int64_t *out_ids_dev);

/*
 * ic_search for callers that cannot allocate device memory or hand over a large workspace
 * at the time of the call: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same result (bit for bit) as ic_search,
 * but every buffer the search writes besides its outputs (prepared queries, per-row bias,
 * candidate regions, merge lists, pilot keys) lies in a static device array inside the
 * library (IC_STATIC_SCRATCH_BYTES per GPU the library is used on, held until the process
 * ends) instead of the index's arena; the call allocates nothing and creates no events
 * (kernel timing does not cover it).
 * Limits: Q <= IC_STATIC_MAX_QUERIES, index size <= IC_STATIC_MAX_ROWS (rounded up to 256);
 * beyond them IC_ERR_UNSUPPORTED and nothing is launched.  The index must live on the current
 * GPU (INVALID_ARG otherwise).  Such batches always take the streaming scan.
 * All calls on one GPU share the one array: calls that overlap on a GPU (two streams, two
 * threads, two indices) race; the caller orders them.  Errors otherwise as ic_search.
 */
#define IC_STATIC_MAX_QUERIES 64
#define IC_STATIC_MAX_ROWS 4194304
#define IC_STATIC_SCRATCH_BYTES (80u << 20)
ic_status ic_search_static(const ic_index *index, const float *q_dev, int64_t Q, int32_t k,
                           float lambda, const uint8_t *mask_dev, float *out_scores_dev,
                           int64_t *out_ids_dev);

/*
 * Sharing domains (Sec. 4.3, "How Does IC-Cache Respect Privacy?": cached examples may be shared
 * only within designated user domains).  Every stored row carries a 32-bit domain; 0, the value
 * rows are appended with, means shared with every domain.
 *   ids_dev      [n] int64 row ids (device); ids outside [0, size) are skipped; of duplicate ids
 *                any one wins
 *   domains_dev  [n] int32 (device), read during the call
 * ic_index_compact moves the domains with their rows.  n == 0 is a no-op.
 * Errors: INVALID_ARG, DEVICE.
 */
ic_status ic_index_set_domains(ic_index *index, const int64_t *ids_dev, const int32_t *domains_dev,
                               int64_t n);

/*
 * Top-k selection under access control (same passage).  As ic_search, except that query j only
 * sees the rows whose domain is 0 or query_domain_dev[j]; each query's result is the top k of the
 * rows it may see (mask_dev still applies to all queries).
 *   query_domain_dev  [Q] int32 (device).  A query of domain 0 sees only the rows of domain 0.
 * ic_search and the other searches ignore the rows' domains.  Errors: as ic_search.
 */
ic_status ic_search_domains(const ic_index *index, const float *q_dev, int64_t Q, int32_t k,
                            float lambda, const uint8_t *mask_dev, const int32_t *query_domain_dev,
                            float *out_scores_dev, int64_t *out_ids_dev);

/*
 * Top-k selection with a score threshold (Sec. 4.1, "Selecting Example Combinations": the
 * selector drops examples whose estimated helpfulness falls below a dynamic threshold, so the
 * number of examples varies per query).  Same as ic_search, except that an entry is kept only if
 * its score (the fp32 value that would be returned) is >= min_score; dropped entries are
 * (score = -inf, id = -1) and each row stays sorted, so the kept entries come first.
 *   out_counts_dev  [Q] int32: entries kept for each query (0 .. k); may be NULL
 * min_score = -inf keeps everything.  Errors: as ic_search; INVALID_ARG for a NaN threshold.
 */
ic_status ic_search_threshold(const ic_index *index, const float *q_dev, int64_t Q, int32_t k,
                              float lambda, const uint8_t *mask_dev, float min_score,
                              float *out_scores_dev, int64_t *out_ids_dev, int32_t *out_counts_dev);

/*
 * Self-search: the stored rows first_row .. first_row + count - 1 are the queries, and each is
 * left out of its own result.  This is the measurement behind Sec. 2.3 ("Voluminous requests lead
 * to pervasive similarity": the top-1 similarity of every request to the others) and the lookup a
 * semantic cache performs.  The rows are used as stored (already unit length and quantised), so
 * no query is passed; everything else is as in ic_search.
 *   k               1 .. max_k - 1 (the candidate lists also hold the row itself)
 *   out_scores_dev  [count, k] fp32; out_ids_dev [count, k] int64
 * Errors: INVALID_ARG (range outside the store, k out of range), DEVICE.
 */
ic_status ic_self_search(const ic_index *index, int64_t first_row, int64_t count, int32_t k,
                         float lambda, const uint8_t *mask_dev, float *out_scores_dev,
                         int64_t *out_ids_dev);

/*
 * Maintenance driven by the Example Manager (Sec. 4.3, "Capping Example Cache Size over
 * Time"): the manager keeps a moving average of every example's gain, decays it (factor 0.9
 * per hour in the paper) and evicts low-utility examples.  The four calls below are what the
 * embedding store needs for that.  They are ordered with searches and appends on the stream.
 *
 * ic_index_set_utility   utility[ids_dev[j]] = util_dev[j] for j < n.  ids outside
 *                        [0, size) are ignored; if an id occurs twice either value may win.
 * ic_index_scale_utility utility[i] *= factor for every row (one fp32 multiplication).
 * ic_index_invalidate    marks the rows ids_dev[0..n) as evicted: they are never returned by
 *                        later searches, exactly as if every later mask had a 0 for them.  Ids
 *                        outside [0, size) are ignored.  The rows still occupy the store (and
 *                        cost bandwidth) until ic_index_compact.
 * ic_index_compact       squeezes the invalidated rows out, keeping the order of the others.
 *                        id_map_dev [size before the call] int64 receives the new id of every
 *                        old row, or -1 for a dropped row; *new_size (host, may be NULL) the
 *                        number of rows left.  Ids change: this is the one call after which
 *                        "ids are append order" refers to the surviving rows only, and masks
 *                        given to later searches are indexed by the new ids.  Unlike the other
 *                        calls it waits for the stream (row counts are needed on the host, to
 *                        plan the moves and as the new size).  Cost: every row is read once and
 *                        every surviving row written once (twice in the first few chunks, and
 *                        once more into the second copy of an index that has one), O(size).
 * Errors: INVALID_ARG, DEVICE.
 */
ic_status ic_index_set_utility(ic_index *index, const int64_t *ids_dev, const float *util_dev, int64_t n);
ic_status ic_index_scale_utility(ic_index *index, float factor);
ic_status ic_index_invalidate(ic_index *index, const int64_t *ids_dev, int64_t n);
ic_status ic_index_compact(ic_index *index, int64_t *id_map_dev, int64_t *new_size);

/*
 * Cluster pruning in front of the scan (Sec. 4.1, "Two-Stage Scalable Example Selection": the
 * cached examples are clustered offline into K groups with K-Means; online a request is compared
 * with the K centroids and then only with the examples of the nearest clusters, K + N/K
 * comparisons per request instead of N, smallest at K = sqrt(N)).  The result is approximate: an
 * example outside the probed clusters cannot be returned.
 *
 * An ic_ivf sits on top of an index ("base") and lives in its own caller-owned arena.  It holds K
 * centroids in the store's format, the cluster of every row, and a copy of the base's live rows
 * sorted by cluster, which the online scan reads as contiguous ranges.  It is a snapshot: after
 * appends, evictions or a compaction of the base, call ic_ivf_assign (or train) again.
 *
 * ic_ivf_workspace_bytes  arena bytes for a base index, K clusters (1 .. 2^20) and searches that
 *                         probe up to max_probe (1 .. IC_MAX_K) clusters; 0 if out of range.
 * ic_ivf_create           arena_dev IC_ARENA_ALIGN-aligned.  Uses the base's stream.
 * ic_ivf_set_centroids    centroids_dev [K, d] fp32 from the caller's own clustering; they are
 *                         normalised and stored like examples.  Lists must be rebuilt afterwards.
 * ic_ivf_assign           cluster of a row = its most similar centroid (cosine, ties to the lowest
 *                         centroid id); then builds the lists and the sorted copy.
 * ic_ivf_set_assignment   the same from the caller's assignment, assign_dev [size] int32; rows
 *                         with a cluster outside [0, K) or invalidated rows are in no list.
 * ic_ivf_update_centroids K-Means update: every centroid becomes the mean direction of its list
 *                         (sum of the stored unit rows, normalised); an empty list keeps its centroid.
 * ic_ivf_train            K-Means from the stored rows: the start is the rows at positions
 *                         floor(c * size / K); then iters times (assign, update), then assign.
 * ic_ivf_search           as ic_search without a mask, over the rows of the nprobe (1 .. max_probe)
 *                         nearest clusters of each query only.  Same output conventions.
 * ic_ivf_view             inspection: cluster of every base row [size], list offsets [K + 1] (into the
 *                         sorted copy), base id of every sorted row, and the two internal indices
 *                         (for ic_index_store_view / ic_index_size).  Any out pointer may be NULL.
 * assign, set_assignment and train wait for the stream (the number of listed rows is needed on the
 * host); the other calls are asynchronous.  Errors: INVALID_ARG (also: search or update before the
 * lists exist, assign before centroids exist), CAPACITY, OOM, DEVICE.
 */
typedef struct ic_ivf ic_ivf; /* opaque */
size_t ic_ivf_workspace_bytes(const ic_index *base, int32_t K, int32_t max_probe);
ic_status ic_ivf_create(ic_ivf **out, ic_index *base, int32_t K, int32_t max_probe, void *arena_dev,
                        size_t arena_bytes);
ic_status ic_ivf_destroy(ic_ivf *ivf);
ic_status ic_ivf_set_centroids(ic_ivf *ivf, const float *centroids_dev);
ic_status ic_ivf_assign(ic_ivf *ivf);
ic_status ic_ivf_set_assignment(ic_ivf *ivf, const int32_t *assign_dev);
ic_status ic_ivf_update_centroids(ic_ivf *ivf);
ic_status ic_ivf_train(ic_ivf *ivf, int32_t iters);
ic_status ic_ivf_search(ic_ivf *ivf, const float *q_dev, int64_t Q, int32_t k, int32_t nprobe,
                        float lambda, float *out_scores_dev, int64_t *out_ids_dev);
ic_status ic_ivf_view(const ic_ivf *ivf, const int32_t **assign_dev, const int64_t **offsets_dev,
                      const int32_t **perm_dev, const ic_index **centroids, const ic_index **sorted);

/*
 * Release the handle (the counterpart of the client's stop(), Sec. 3).  Device memory belongs
 * to the caller and is not touched; work already enqueued on the stream still needs the arena,
 * so the caller drains the stream before freeing it.  Errors: INVALID_ARG (NULL).
 */
ic_status ic_index_destroy(ic_index *index);

/* ---- helpers ---------------------------------------------------------- */

/* Number of rows appended so far (-1 for a NULL handle). */
int64_t ic_index_size(const ic_index *index);

/* Replace the stream used by later calls. */
ic_status ic_index_set_stream(ic_index *index, void *stream);

/*
 * Device views of the store for inspection: first row, row stride in bytes,
 * per-row scale (NULL for bf16) and utility arrays.  Any out pointer may be NULL.
 */
ic_status ic_index_store_view(const ic_index *index, const void **rows_dev,
                              int64_t *row_stride_bytes, const float **scale_dev,
                              const float **util_dev);

/*
 * Launch-shape overrides for tests and benchmark sweeps; results never depend on them.
 *   slices     workgroups (slices of the store) per query block of the streaming scan,
 *              1 .. 1024; 0 = as many as are resident at once (the default)
 *   list_keys  keys of a query's candidate list in the tiled scan, at most the default
 *              for max_k; 0 = the default.  Small values force the overflow paths.
 * Applies to later searches.  Errors: INVALID_ARG.
 */
ic_status ic_index_set_tuning(ic_index *index, int32_t slices, int32_t list_keys);

/*
 * Kernel timing for benchmarks.  While enabled, every ic_search brackets each
 * launch of its scan kernel (similarity + fused partial top-k) with events on
 * the index's stream; nothing waits.  ic_index_set_timing (either value) also
 * forgets the launches recorded so far.  ic_index_scan_time_ms waits for the
 * recorded launches to finish and returns their summed duration and, if
 * launches is not NULL, their number (at most 32768 launches are kept).
 */
ic_status ic_index_set_timing(ic_index *index, int enable);
ic_status ic_index_scan_time_ms(ic_index *index, float *ms, int64_t *launches);

/*
 * Diagnostics of the last batch that took the tiled scan (large batches; of its
 * last chunk of max_queries queries if the batch was larger than that): how
 * many (row tile, query block) pairs had more hits than the tile's on-chip list
 * holds and were computed a second time, and how many blocks of 64 queries
 * overflowed their candidate list in device memory and were redone by the
 * streaming scan.  Both are 0 on typical data; they cost time, never
 * exactness.  Waits for the index's stream.  Either out pointer may be NULL.
 * An index too small for the tiled scan reports zeros.
 */
ic_status ic_index_tiled_scan_counts(ic_index *index, int64_t *tiles_again,
                                     int64_t *blocks_redone);

/* Static description of a status code. */
const char *ic_status_string(ic_status s);

#ifdef __cplusplus
}
#endif
#endif /* ICCACHE_H */
