/*
 * proximity.h -- C ABI of the Proximity-FLAT retrieval step on one AMD Instinct GPU.
 *
 * The library implements the per-query retrieval step of an approximate
 * key-value cache placed in front of a vector index (Algorithm 1, Section 3.1):
 * each query embedding is compared with every cached query key (Euclidean
 * distance unless the instance is created with another PROXIMITY_METRIC_*);
 * if the nearest key lies within the tolerance tau the cached list of
 * document indices is returned, otherwise the index is searched exactly for the
 * k nearest documents (the nearest-neighbour search of Section 2.2), the oldest
 * (FIFO) or least recently used (LRU) entry is evicted when the cache already
 * holds c entries (Section 3.3.2), and the query with its result is stored.
 * Options fixed at creation: the re-ranking factor of Section 3.3.4
 * (rerank_factor) and the bucketed cache of Section 3.2 (lsh_bits, lsh_planes).
 *
 * Queries are an ordered stream (Section 3.1 processes one query at a time).
 * A call may hand over many rows; the result is exactly what processing the
 * rows one at a time in row order would give, including hits on keys inserted
 * by earlier rows of the same call and evictions that happen between them.
 *
 * Conventions
 *   - DEVICE pointers are HIP device memory on the handle's device; HOST
 *     pointers are ordinary host memory.  The library never takes ownership of
 *     a caller buffer.
 *   - All matrices are dense row-major.
 *   - Every function returns PROXIMITY_OK (0) or a negative error code.  No
 *     C++ exception or abort crosses this boundary.  Argument errors are found
 *     before any GPU work is enqueued and leave the handle unchanged; the text
 *     of the last error is available from proximity_last_error().
 *   - A handle is an ordered stream consumer and is not thread-safe.  Its workspaces are shared by all
 *     of its calls, so at any time the calls of one handle must be in flight on ONE stream only: before
 *     passing a different stream than the previous call did, wait for that call (hipStreamSynchronize,
 *     or an event the new stream waits on).  Calls that overlap on two streams race.
 *     A flat cache whose max_batch exceeds one probe range (1536 rows; fewer for caches beyond some 40 000
 *     keys, see proximity_probe_row_ranges) owns one stream of its own (default priority): inside a call of
 *     more rows than that the rows are decided there, range by range, beside the distance computation of
 *     the following range on the caller's stream.  The two are tied by events, and the caller's
 *     stream waits for the internal one before the call enqueues what follows, so to the caller the call
 *     is still a piece of work in order on the stream it passed.
 *   - The library allocates all of its device memory in proximity_create().
 *     proximity_search_batch() and proximity_knn_batch() allocate nothing and
 *     never wait for the device: the number of misses is consumed on the
 *     device, and results are valid once the given stream reaches the end of
 *     the call's work.
 */
#ifndef PROXIMITY_H
#define PROXIMITY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PROXIMITY_ABI_VERSION 9u

enum {
  PROXIMITY_OK = 0,
  PROXIMITY_ERR_INVALID_ARG = -1,     /* null pointer, zero size, unsupported value        */
  PROXIMITY_ERR_K_MISMATCH = -2,      /* k differs from the k fixed at creation            */
  PROXIMITY_ERR_BATCH_TOO_LARGE = -3, /* n exceeds max_batch                               */
  PROXIMITY_ERR_BAD_TAU = -4,         /* tau is NaN, infinite or negative                  */
  PROXIMITY_ERR_HIP = -5,             /* a HIP runtime call failed                         */
  PROXIMITY_ERR_OOM = -6              /* device memory for the instance could not be had   */
};

enum { PROXIMITY_DTYPE_F32 = 0, PROXIMITY_DTYPE_BF16 = 1 };
enum { PROXIMITY_POLICY_FIFO = 0, PROXIMITY_POLICY_LRU = 1 };
/* The index's distance function (Section 2.2: Euclidean, inner product or cosine, fixed when
 * the index is built).  Smaller is closer in all three:
 *   L2      sqrt(sum (q_i - x_i)^2)
 *   IP      -(q . x)             (the ranked list is by descending inner product)
 *   COSINE  1 - q.x / (|q| |x|)  (vectors of length zero are not validated)
 * The cache compares a query with its keys by the same function (Section 3.1), except under
 * IP: the negated inner product is no distance between two queries (a query is not nearest
 * to itself), so the cache of an inner-product index compares by Euclidean distance. */
enum { PROXIMITY_METRIC_L2 = 0, PROXIMITY_METRIC_IP = 1, PROXIMITY_METRIC_COSINE = 2 };

/* Limits checked by proximity_create(). */
#define PROXIMITY_MAX_K 240u
#define PROXIMITY_MAX_DIM 4096u
#define PROXIMITY_MAX_BATCH 8192u
#define PROXIMITY_MAX_CAPACITY (1u << 20)
/* Limits of proximity_knn_static(), whose workspace is built into the library. */
#define PROXIMITY_STATIC_MAX_DOCS (1u << 18)
#define PROXIMITY_STATIC_MAX_QUERIES 4u

typedef struct proximity proximity_t;

/*
 * Parameters fixed for the life of an instance (the state Algorithm 1 keeps
 * between queries; Section 3.1: k is chosen once; Section 3.3.1: capacity c;
 * Section 3.3.2: eviction policy).
 */
typedef struct proximity_config {
  uint32_t struct_size;   /* sizeof(proximity_config), for ABI checking                       */
  uint32_t dim;           /* embedding dimension d; multiple of 32, <= PROXIMITY_MAX_DIM     */
  const void* corpus;     /* DEVICE [n_docs][dim], float32 or bfloat16, 16-byte aligned; BORROWED:
                             it must stay allocated and unchanged until proximity_destroy()  */
  uint64_t n_docs;        /* < 2^31.  0 is allowed: misses then return ids -1 / dists +inf
                             (for runs that time the cache probe alone)                      */
  uint32_t corpus_dtype;  /* PROXIMITY_DTYPE_*.  Queries and cache keys are always float32   */
  uint32_t capacity;      /* c; 0 disables the cache: every query misses, nothing is stored  */
  uint32_t k;             /* neighbours per query, 1..PROXIMITY_MAX_K                         */
  uint32_t policy;        /* PROXIMITY_POLICY_*                                               */
  uint32_t max_batch;     /* largest n a call may pass, 1..PROXIMITY_MAX_BATCH                */
  int32_t device;         /* HIP device ordinal                                               */
  uint32_t rerank_factor; /* rho of Section 3.3.4, a whole number >= 1 (0 is read as 1): the
                             index is asked for rho * k neighbours (<= PROXIMITY_MAX_K), all
                             are stored with the key, a miss returns the first k, and a hit
                             returns the k of the stored rho * k documents nearest to the
                             current query, ranked by (distance, index), with those
                             distances.  1: a hit returns the stored list unchanged        */
  uint32_t lsh_bits;      /* L of Section 3.2.  0: one flat cache of `capacity` entries.  1..16: the
                             bucketed cache: 2^L buckets, each a cache of `capacity` entries
                             (b in the paper) with its own FIFO/LRU order; a query is looked
                             up and stored only in the bucket named by its L-bit code.
                             capacity << lsh_bits must not exceed PROXIMITY_MAX_CAPACITY and
                             capacity must be 1..256 then                                    */
  const float* lsh_planes;/* DEVICE [lsh_bits][dim] float32: normals of the L hyperplanes through
                             the origin; bit i of a query's code is 1 exactly when its inner
                             product with row i is >= 0 (evaluated in float64).  Copied at
                             creation; NULL when lsh_bits is 0                               */
  uint32_t metric;        /* PROXIMITY_METRIC_*: ranks the documents, is the unit of tau and of
                             every reported distance.  Keys are the queries as the caller gave
                             them under every metric (proximity_cache_dump returns them so);
                             query-key distances are evaluated in float64, the cosine one as
                             1 - q.k / sqrt((q.q)(k.k)), which is exactly 0 for a key identical
                             to the query, so tau = 0 is an exact-match cache here too          */
  uint32_t flags;         /* PROXIMITY_FLAG_* or 0                                            */
} proximity_config;
/* Never pre-rank on rounded operands (see proximity_coarse_score_error): every batched index search multiplies
 * the corpus as it is stored.  The results are the same either way; this is for comparing the two. */
#define PROXIMITY_FLAG_NO_ROUNDED_SCAN 1u

/* Counters since creation or the last proximity_clear(). */
typedef struct proximity_stats_t {
  uint64_t queries;        /* rows processed                                                 */
  uint64_t hits;           /* rows answered from the cache                                   */
  uint64_t misses;         /* rows that went to the index (= scans = inserts when c > 0)     */
  uint64_t inserts;        /* keys stored                                                    */
  uint64_t evictions;      /* keys removed to make room                                      */
  uint64_t size;           /* keys resident now, <= capacity                                 */
  uint64_t inbatch_hits;   /* hits on a key stored by an earlier row of the same call        */
  uint64_t dense_resolves; /* rows whose nearest key was found by the full-row fallback      */
  uint64_t slack_exhausted;  /* index searches (since creation or the last clear, proximity_knn_batch
                                included) whose float32 candidate list (k + 8 rows; more after a one-plane
                                search, see proximity_coarse_score_error) could not be
                                proven to hold the k nearest under the float32 error bound, and were
                                ranked again from every row within that bound of the k-th          */
  uint64_t slack_unresolved; /* of those, searches that stayed with the float64 ranking of their
                                candidates because the second ranking had no room: more than
                                2048 rows within the bound of the k-th (thousands of identical
                                documents).  0 means every list returned so far is provably exact  */
  uint64_t probe_workspace_bytes; /* device memory the flat cache's probe holds beside keys and values:
                                     float32 scores of two row ranges of a batch against every key, the
                                     candidate lists, the resolver's state between ranges.  Fixed at
                                     creation; at most about 0.5 GiB unless capacity + max_batch
                                     exceeds a million                                              */
  uint64_t coarse_scan_calls; /* since creation: calls whose index search ran on rounded operands (see
                                 proximity_coarse_score_error)                                      */
  uint64_t coarse_scan_fails; /* since creation: lists of such searches that could not be proven to hold
                                 the k nearest (each also counts in slack_exhausted); once they stop
                                 being rare the instance searches on the operands as they are       */
  uint64_t reserved[3];
} proximity_stats_t;

/*
 * One timed launch (see proximity_profile_start), of the corpus-scan distance kernel
 * (kind PROXIMITY_LAUNCH_SCAN) or of the cache probe's (kind PROXIMITY_LAUNCH_PROBE: it
 * probed rows first_query .. first_query+n_queries-1 of its call against the stored keys
 * and the call's earlier rows).  A scan launch handles the misses number first_query .. first_query+n_queries-1 of its
 * call; it streamed the corpus only if the call had more than first_query misses
 * (otherwise it returned at once), which the caller can tell from out_hit.  Where the
 * library launches the kernel in several tile shapes for the same queries (all but one of
 * which return at once: the number of misses is known on the device only), the record is
 * that of the longest of them.
 */
typedef struct proximity_launch_t {
  uint32_t call;         /* ordinal of the search/knn call since proximity_profile_start   */
  uint32_t first_query;  /* index, within the call's miss list, of the launch's first query */
  uint32_t n_queries;    /* queries the launch is compiled to handle at once               */
  float ms;              /* duration from HIP events recorded on the call's stream         */
  uint32_t kind;         /* PROXIMITY_LAUNCH_SCAN or PROXIMITY_LAUNCH_PROBE                 */
} proximity_launch_t;
#define PROXIMITY_LAUNCH_SCAN 0u
#define PROXIMITY_LAUNCH_PROBE 1u

uint32_t proximity_abi_version(void);

/*
 * How far the float32 score by which the index search pre-ranks a row can lie from the row's exact score
 * (host arithmetic, no GPU work).  The search ranks by float32 scores -- |x|^2 - 2 q.x (L2), -2 q.x (IP),
 * -2 q.x / |x| (COSINE) -- keeps the k + 8 best and ranks those by float64 distance (Section 2.2 asks for
 * the exact ranked list).  With E this bound, W the worst kept float32 score and t the k-th smallest exact
 * score among the kept rows, W - E > t proves that no other row belongs to the k nearest; a search for
 * which it fails is ranked again from all rows scoring at most t + E (counted in slack_exhausted).
 *   E = g (X^2 + 2 |q| X)   L2          g = (3 dim + 16) 2^-24 + 2^-17: every product and partial sum of a
 *   E = g 2 |q| X           IP              dim-term inner product rounds once; a bfloat16 corpus is searched with
 *   E = g 4 |q|             COSINE          the query split into bfloat16 terms (up to three products per term),
 *                                           of which the batched scan drops what lies below 2^-18 |q_i|
 * |q| = query_length, X = max_row_length (the longest corpus row).  NaN for a bad argument.
 */
double proximity_score_error_bound(uint32_t metric, uint32_t dim, double query_length, double max_row_length);

/*
 * What a search on rounded operands adds to that bound (host arithmetic, no GPU work).  Calls of more than four
 * rows on a corpus of 768 or 384 float32 columns, or 384 or 256 bfloat16 columns, are pre-ranked on the bfloat16
 * matrix cores with the queries rounded to bfloat16 (the first plane of the split alone) and float32 rows rounded
 * likewise on their way into the matrix instruction: the scan is then bound by HBM alone at up to 128 queries.
 * A rounded value differs from the value by at most 2^-9 of it, hence the score by at most
 *   2^-8 |q| X   (L2, IP)        2^-8 |q|   (COSINE)          bfloat16 corpus: queries rounded
 *   2.002 times that                                          float32 corpus: rows rounded too
 * (times 1.001 for the roundings that follow).  Such a search keeps more candidates than k + 8 -- as many as
 * isotropic rows would put within this error of the k-th, and a margin: 46 for k = 10 in 1 M x 768 float32 rows,
 * 159 for k = 100 in 8 M x 384 bfloat16 rows; it is used when that is at most 248 -- and its exactness check uses
 * E + this term, so the lists it returns are as provably exact as the others; when the check fails more than
 * rarely (coarse_scan_fails) the instance goes back to multiplying the operands as they are.  NaN for a bad
 * argument.
 */
double proximity_coarse_score_error(uint32_t metric, uint32_t corpus_dtype, double query_length,
                                    double max_row_length);

/*
 * How many candidates per query a search on rounded operands hands to the float64 ranking when it is asked for k
 * neighbours (k times the re-ranking factor) of n_docs rows of `dim` columns (host arithmetic, no GPU work):
 *   k + ceil(m + 5 sqrt(m) + 16),   m = k (exp(z delta) - 1),   z = sqrt(2 ln(max(n_docs / k, 2))),
 *   delta = sqrt(dim) / 512  (bfloat16 corpus)  or  2.002 sqrt(dim) / 512  (float32 corpus)
 * -- m is the number of rows that isotropic data puts within the rounding error of the k-th.  Instances for which
 * this exceeds 248 search on the operands as stored.  0 for a bad argument.
 */
uint32_t proximity_rounded_scan_list_length(uint32_t k, uint32_t corpus_dtype, uint32_t dim, uint64_t n_docs);

/*
 * The row ranges in which proximity_search_batch() probes and resolves a call of n rows against a flat cache
 * (host arithmetic, no GPU work; Algorithm 1's distances for the rows of one range are computed while the rows of
 * the range before are decided, in order, beside them).  ends[g] receives the row after the last row of range g;
 * the return value is the number of ranges (1: the whole call at once), 0 for a bad argument or when max_ranges
 * is too small.  Every range but the last ends on a multiple of 64, and none is longer than the number of rows
 * whose float32 probe scores fit the instance's score buffers (which follows from capacity and max_batch).
 *   capacity, max_batch  as in proximity_config
 *   listing              1: Euclidean keys of 768 or 384 columns, probed by the kernel that lists candidates itself
 *                        (range sizes then also balance that kernel's blocks); 0: every other flat cache
 *   n_cu                 compute units of the device (256 on MI355X)
 */
uint32_t proximity_probe_row_ranges(uint32_t n, uint32_t capacity, uint32_t max_batch, uint32_t listing, uint32_t n_cu,
                                    uint32_t* ends, uint32_t max_ranges);

/*
 * Create an instance on cfg->device: computes the squared norm of every corpus
 * row once (one streaming pass over the corpus) and allocates the cache
 * (capacity x dim float32 keys, capacity x rerank_factor*k values) and all
 * workspaces, sized for max_batch.  *out receives the handle.  Blocks until the norms are done.
 * Errors: INVALID_ARG (null, bad struct_size, dim/k/max_batch/capacity/n_docs/
 * rerank_factor*k/lsh_bits outside the limits, unknown dtype/policy/metric, misaligned corpus, lsh_planes
 * null with lsh_bits > 0, corpus null with n_docs > 0), OOM,
 * HIP.  On error *out is set to NULL.
 */
int proximity_create(const proximity_config* cfg, proximity_t** out);

/* Frees everything the instance owns.  NULL is ignored.  Waits for the device. */
void proximity_destroy(proximity_t* h);

/*
 * The lookup procedure of Algorithm 1 for n queries, with the semantics of
 * processing rows 0..n-1 one after the other (and calls in call order).
 *
 *   queries    DEVICE [n][dim] float32, 16-byte aligned (as the corpus must be)
 *   n          1..max_batch (0 is accepted and does nothing)
 *   k          must equal cfg.k
 *   tau        tolerance in the units of the instance's distance function between query
 *              and key (Euclidean, not squared, under L2 and IP; cosine distance under
 *              COSINE); finite, >= 0.
 *              A key at distance exactly tau is a hit.  May differ between calls.
 *   out_ids    DEVICE [n][k] int64: ranked document indices (ascending distance,
 *              equal distances by ascending index; -1 padding when n_docs < k).
 *              On a hit: the list stored with the matched key, unchanged
 *              (rerank_factor 1), or the k of the stored documents nearest to
 *              this query (rerank_factor > 1, Section 3.3.4).
 *   out_dists  DEVICE [n][k] float32 or NULL: the distances (by the instance's distance
 *              function) that go with out_ids (+inf padding).  On a hit with rerank_factor 1 these are
 *              the stored distances to the matched key, not to the query; with
 *              rerank_factor > 1 they are distances to the query.
 *   out_hit    DEVICE [n] uint8: 1 = answered from the cache, 0 = index searched
 *   hip_stream the hipStream_t to enqueue on (NULL = the default stream).
 *
 * Asynchronous; see the conventions above.  Errors: INVALID_ARG, K_MISMATCH,
 * BATCH_TOO_LARGE, BAD_TAU, HIP.
 */
int proximity_search_batch(proximity_t* h, const float* queries, uint32_t n, uint32_t k, float tau,
                           int64_t* out_ids, float* out_dists, uint8_t* out_hit, void* hip_stream);

/*
 * The index search alone (Section 2.2; the retrieveDocumentIndices call of
 * Algorithm 1): exact k nearest corpus rows of each query, cache untouched.
 * Same buffers and rules as proximity_search_batch, without tau and out_hit.
 */
int proximity_knn_batch(proximity_t* h, const float* queries, uint32_t n, uint32_t k,
                        int64_t* out_ids, float* out_dists, void* hip_stream);

/*
 * proximity_knn_batch() for callers that cannot allocate device memory at all -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc -- and so cannot call
 * proximity_create() either.  No instance: the call takes the corpus itself, and the workspace the
 * search needs (row terms, dense scores, per-segment candidate lists: 5.5 MiB) is an array that is part of
 * the loaded library, of which every device holds one copy until the process ends.  The call performs no
 * hipMalloc / hipFree and calls no allocating routine; it is asynchronous like the other search calls.
 *
 *   corpus        DEVICE [n_docs][dim], float32 or bfloat16 (corpus_dtype), 16-byte aligned; read only
 *   n_docs        0..PROXIMITY_STATIC_MAX_DOCS; more is rejected with INVALID_ARG (the workspace has a
 *                 fixed size: use an instance for larger corpora)
 *   dim           multiple of 32, <= PROXIMITY_MAX_DIM
 *   metric        PROXIMITY_METRIC_*
 *   queries       DEVICE [n][dim] float32, 16-byte aligned
 *   n             0..PROXIMITY_STATIC_MAX_QUERIES (more: BATCH_TOO_LARGE).  n = 0 enqueues nothing
 *                 and only performs the set-up described below
 *   k             1..PROXIMITY_MAX_K
 *   out_ids       DEVICE [n][k] int64, out_dists DEVICE [n][k] float32 or NULL: as proximity_knn_batch
 *   device        HIP device ordinal the pointers belong to
 *   hip_stream    the hipStream_t to enqueue on (NULL = the default stream)
 *
 * Results are those of proximity_knn_batch() on an instance over the same corpus, bit for bit (the same
 * kernels run; the squared row norms an instance computes once are recomputed by every call here).
 * The first call on a device looks up the address of that device's copy of the workspace
 * (hipGetSymbolAddress, no allocation); make that call (n = 0 suffices) before starting a graph capture.
 * All calls on one device share that device's workspace, which keeps the last call's contents: every
 * call overwrites what it reads, so nothing needs clearing, but two calls whose work overlaps on one
 * device (different streams, or threads) race -- issue them on one stream, or order them with events.
 * The exactness check behind proximity_stats_t.slack_exhausted runs here as well, but without an instance
 * its counters are not reported.
 * Errors: INVALID_ARG, BATCH_TOO_LARGE, HIP; text from proximity_last_error(NULL).
 */
int proximity_knn_static(const void* corpus, uint64_t n_docs, uint32_t dim, uint32_t corpus_dtype, uint32_t metric,
                         const float* queries, uint32_t n, uint32_t k, int64_t* out_ids, float* out_dists,
                         int32_t device, void* hip_stream);

/* Copies the counters to *out (HOST).  Waits for the handle's last stream. */
int proximity_stats(const proximity_t* h, proximity_stats_t* out);

/*
 * Copies the cache contents to HOST arrays in eviction order (next victim
 * first; the bucketed cache: bucket by bucket in ascending code, each bucket
 * in its own eviction order).  seq[i] is the position, counted from creation or the last clear, of
 * the query that inserted entry i.  keys ([capacity][dim] float32) and ids
 * ([capacity][rerank_factor * k] int64; capacity << lsh_bits rows for the
 * bucketed cache) may be NULL.  *n_live receives the number of entries
 * written.  Waits for the handle's last stream.
 */
int proximity_cache_dump(const proximity_t* h, uint64_t* seq, float* keys, int64_t* ids,
                         uint32_t* n_live);

/* Empties the cache and zeroes counters and the query position.  Waits for the device. */
int proximity_clear(proximity_t* h);

/*
 * Kernel timing for roofline reports.  After proximity_profile_start() every
 * launch of the corpus-scan distance kernel is bracketed with HIP events on the
 * call's stream (at most 8192 launches; later ones are not timed), and so is every
 * launch of the cache probe that lists its candidates itself (Euclidean keys of 768 or
 * 384 columns, calls of 64 rows and more): one record of kind PROXIMITY_LAUNCH_PROBE per
 * row range of the call.
 * proximity_profile_stop() waits for the stream, writes up to cap records to
 * the HOST array `records` (may be NULL with cap 0), sets *n_records to the
 * number written, and stops timing.  Events are created by the start call,
 * not by the search calls.
 */
int proximity_profile_start(proximity_t* h);
int proximity_profile_stop(proximity_t* h, proximity_launch_t* records, uint32_t cap, uint32_t* n_records);

/* Text of the last error on this handle (or of the last failed create when h is NULL). */
const char* proximity_last_error(const proximity_t* h);

#ifdef __cplusplus
}
#endif
#endif /* PROXIMITY_H */
