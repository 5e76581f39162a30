/*
 * ivfadcr.h - C interface of the MI355X (gfx950) IVFADC+R search library.
 *
 * Method: "Searching in one billion vectors: re-rank with source coding".  A database of
 * d-dimensional vectors is indexed by (i) an inverted file over a coarse quantizer with c
 * reproduction values (section 3.3), (ii) an m-byte product-quantizer code q_c of each
 * vector's residual to its coarse centroid (section 2, Eq. (4)), and (iii) an m'-byte
 * refinement code q_r of what q_c leaves (section 3.1, Eq. (7)-(8)).  A query visits the w
 * nearest lists (v in the paper), ranks their entries by the asymmetric distance estimator
 * read from look-up tables (Eq. (5)), keeps the k' best, rebuilds each of those explicitly
 * as  coarse + decode(q_c) + decode(q_r)  (Eq. (9)) and returns the k with the smallest
 * refined squared distance (Eq. (10); query steps 1-3 of section 3.2).
 *
 * Conventions
 *  - Every function returns IVFR_OK (0) or a negative IVFR_ERR_* code; ivfr_last_error()
 *    gives a message for the calling thread's last failure.  Nothing throws across this ABI.
 *  - "host" / "device" in an argument comment says where the memory must live.  Buffers are
 *    owned by the caller; the index and its scratch are owned by the library.
 *  - All matrices are row-major and dense.  Distances are squared L2, fp32.
 *  - 8 bits per sub-quantizer (256 reproduction values), as fixed in sections 2 and 3.1.
 *  - ids are int32 (the 4 bytes per vector of section 3.3); N < 2^31.
 *  - Calls on one index must not overlap in time (one stream of calls per index).
 */
#ifndef IVFADCR_H
#define IVFADCR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IVFR_OK               0
#define IVFR_ERR_INVALID_ARG (-1)  /* null pointer, bad shape, k > k', w > c, ...            */
#define IVFR_ERR_STATE       (-2)  /* call not valid in the index's current state             */
#define IVFR_ERR_OOM         (-3)  /* device or host allocation failed                        */
#define IVFR_ERR_HIP         (-4)  /* a HIP runtime call failed (message names it)            */

typedef struct ivfr_index ivfr_index;   /* opaque */

typedef struct {
    int32_t d;         /* vector dimension; multiple of 8                                   */
    int32_t c;         /* coarse centroids = inverted lists (section 3.3)                   */
    int32_t m;         /* bytes of the first-stage code: 4, 8, 16, 32 or 64; d/m a power of
                          two, at most 32                                                    */
    int32_t m_refine;  /* bytes of the refinement code m'; 0 = plain IVFADC; else a multiple
                          of 4 with d/m' a power of two, at most 32                          */
    int32_t device;    /* HIP device ordinal                                                */
} ivfr_params;

/* Lifetime.  ivfr_create allocates nothing large; ivfr_destroy frees everything. */
int ivfr_create(const ivfr_params* params, ivfr_index** out);
int ivfr_destroy(ivfr_index* index);

/* Offline step 1 of section 3.2: learn the coarse quantizer, q_c and q_r.
 * ivfr_train runs Lloyd k-means on the GPU (initial centroids = distinct training rows drawn
 * from `seed`; an empty cluster keeps its centroid): coarse on the vectors, q_c on the
 * residuals to the coarse centroid, q_r on what q_c leaves.  train: uint8 [n, d], host or
 * device; n >= max(c, 256).
 * ivfr_set_codebooks injects codebooks instead (host fp32): coarse [c, d], pq [m, 256, d/m],
 * rq [m', 256, d/m'] (ignored, may be NULL, when m' = 0).  ivfr_get_codebooks copies them out
 * to host buffers of the same shapes.  Codebooks cannot change once vectors were added. */
int ivfr_train(ivfr_index* index, const uint8_t* train, int64_t n, int32_t iters, uint64_t seed);
int ivfr_set_codebooks(ivfr_index* index, const float* coarse, const float* pq, const float* rq);
int ivfr_get_codebooks(const ivfr_index* index, float* coarse, float* pq, float* rq);

/* Offline steps 2-3 of section 3.2: encode n vectors x (uint8 [n, d], host or device) and
 * stage them for the inverted file.  Vector i gets id id_base + i; successive calls must use
 * increasing, non-overlapping id ranges (lists are kept in ascending id order).
 * ivfr_finalize sorts the staged entries into the inverted lists; afterwards the index is
 * searchable and immutable. */
int ivfr_add(ivfr_index* index, const uint8_t* x, int64_t n, int64_t id_base);
int ivfr_finalize(ivfr_index* index);
int64_t ivfr_ntotal(const ivfr_index* index);   /* vectors added so far (negative: error) */

/* The finished index as flat host arrays: list l holds entries list_offsets[l] ..
 * list_offsets[l+1]-1.  list_offsets int64 [c+1]; ids int32 [N]; codes uint8 [N, m]; rcodes
 * uint8 [N, m'] (may be NULL when m' = 0).  ivfr_import installs such arrays (codebooks must
 * be set first) and leaves the index finalized.  Imported ids must be >= 0 (checked) and
 * distinct (not checked: ties between equal distances are broken by id, and the selections rely
 * on every (distance, id) key being unique). */
int ivfr_export(const ivfr_index* index, int64_t* list_offsets, int32_t* ids, uint8_t* codes, uint8_t* rcodes);
int ivfr_import(ivfr_index* index, int64_t N, const int64_t* list_offsets, const int32_t* ids,
                const uint8_t* codes, const uint8_t* rcodes);

/* Query stage (section 3.2 steps 1-3 on the inverted file of section 3.3).
 * queries: fp32 [nq, d], device.  1 <= w <= c, 1 <= k <= kprime.
 * ids_out int32 [nq, k], dist_out fp32 [nq, k], device: per query ascending by (refined squared
 * distance, id); when fewer than k entries were scanned the tail is id -1, distance +inf.
 * stream: a hipStream_t (NULL = default stream).  The whole query stage is enqueued on it without
 * a host round trip (unit counts, launch shapes and buffer checks are read by the kernels from
 * device memory); the call then waits for the stream once, reads the status words the kernels left
 * (failed buffer checks, queries that are not finite, work counters) and returns, so outputs are
 * valid on return.  Further waits happen only on the rare redo paths: a candidate pool that turned
 * out too small (the pool grows and the batch runs again; it keeps its size for later calls), or
 * queries whose sampled bound failed its check (each is rescanned at most eight times with a
 * tightened bound and at most once without any filter: bound_retries / dense_fallbacks of
 * ivfr_search_stats).
 * Query components must be finite: a query with a NaN or infinite component (or a squared norm
 * beyond fp32) makes the call fail with IVFR_ERR_INVALID_ARG, naming the query.  The workspace of
 * a call grows with nq (about w * m KB of tables per query) and is kept by the index for later calls;
 * IVFR_ERR_OOM is returned before anything is allocated when it cannot fit.
 * Errors: IVFR_ERR_INVALID_ARG for null pointers, parameters outside the ranges above or queries
 * that are not finite, IVFR_ERR_STATE before ivfr_finalize / ivfr_import, IVFR_ERR_OOM /
 * IVFR_ERR_HIP from the runtime; outputs are then undefined. */
int ivfr_search(ivfr_index* index, const float* queries, int64_t nq, int32_t w, int32_t kprime, int32_t k,
                int32_t* ids_out, float* dist_out, void* stream);

/* ivfr_search for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same results (bit for bit) as ivfr_search, but the
 * per-batch arrays and the candidate pool are carved from a fixed array of 128 MiB that the library keeps
 * in device memory (one per GPU it runs on, held until the process ends) instead of from buffers that grow
 * on demand; the call allocates and frees nothing on the device.  Queries are processed in as many internal
 * batches as it takes to fit (look-up tables of w * m KB per query with table mode 0, c * 8 bytes of coarse
 * keys and 24 * kprime bytes of short-list per query, plus the candidate pool).  It fails with IVFR_ERR_OOM,
 * saying what was needed, when one query alone does not fit, when a batch's candidate pool turns out to want
 * more than the array holds, or when a query needs the unfiltered redo pass; with IVFR_ERR_STATE in table
 * mode 1 before a first ivfr_search call has built the per-list table.  Nothing is timed
 * (ivfr_stage_times reports host times only).  All calls on one GPU share that GPU's array, whichever index
 * they search: calls that overlap in time on one GPU race, also on different streams and different indexes. */
int ivfr_search_static(ivfr_index* index, const float* queries, int64_t nq, int32_t w, int32_t kprime, int32_t k,
                       int32_t* ids_out, float* dist_out, void* stream);

/* Same search, additionally exposing intermediate results for verification (any of the extra
 * pointers may be NULL).  All device memory.
 *   probe_out       int32 [nq, w]   visited lists, nearest first (ties: lower list index)
 *   probe_dist_out  fp32  [nq, w]   their squared coarse distances
 *   short_ids_out   int32 [nq, k']  ids of the short-list of step 1 (unordered; tail -1)
 *   short_est_out   fp32  [nq, k']  their ADC estimates (Eq. (5))
 *   short_ref_out   fp32  [nq, k']  their refined distances (Eq. (10))
 *   short_count_out int32 [nq]      short-list length = min(k', entries scanned)          */
int ivfr_search_trace(ivfr_index* index, const float* queries, int64_t nq, int32_t w, int32_t kprime, int32_t k,
                      int32_t* ids_out, float* dist_out,
                      int32_t* probe_out, float* probe_dist_out,
                      int32_t* short_ids_out, float* short_est_out, float* short_ref_out,
                      int32_t* short_count_out, void* stream);

/* Counters of the most recent search call (any pointer may be NULL):
 *   codes_scanned        (query, entry) estimates computed = sum over queries of the visited lists'
 *                        lengths (the "v/c of the database" of section 3.3)
 *   pairs                (query, list) pairs
 *   dense_fallbacks      queries redone without any filter (a buffer for every visited entry): the
 *                        sampled bound kept fewer than k' entries, or ties made tightening it useless
 *   bound_retries        rescans of one query with a tightened bound after its survivors overflowed
 *                        the candidate buffer
 *   codes_streamed       list entries read from memory by the scan (< codes_scanned when lists are
 *                        shared between queries)
 *   codes_scanned_shared / _shared2 / _shared8 / _shared64  parts of codes_scanned computed by the
 *                        shared-list scans of four, two, eight and 64 queries per pass              */
int ivfr_search_stats(const ivfr_index* index, int64_t* codes_scanned, int64_t* pairs, int64_t* dense_fallbacks,
                      int64_t* codes_streamed, int64_t* codes_scanned_shared, int64_t* codes_scanned_shared2,
                      int64_t* codes_scanned_shared8, int64_t* bound_retries, int64_t* codes_scanned_shared64);

/* List sharing.  Queries of one internal batch that visit the same list are scanned together: the
 * list's codes are read once and each code byte fetches all the queries' table entries with one
 * LDS read.  mode -1 (default): mode 2 for batches expected to stream 3e8 codes or more (queries of the
 * batch x entries a query visits, estimated from the list lengths), mode 0 for smaller ones, where the
 * grouping costs more than it saves.  mode 0: every (query, list) pair is scanned on its own.  mode 1
 * (needs m <= 16): units
 * of four and of two queries with fp32 tables (16- and 8-byte LDS reads).  mode 2 (m <= 16):
 * in addition units of eight queries with half-precision tables; an entry whose half-precision
 * estimate could be within the bound is re-evaluated in fp32 before it is kept, so the recorded
 * estimates, and therefore the results, are bit-identical in all modes.  mode 3 (m in {4, 8, 16},
 * sub-vectors of 8, 16 or 32 dimensions, d <= 128; otherwise it acts as mode 2): lists visited by 64 or
 * more queries of the batch are in addition scanned in units of 64 queries on the matrix cores: the
 * estimate ||r||^2 - 2 r.y + ||y||^2 of Eq. (5) against the decoded entry y becomes an fp16 contraction
 * that filters with a rigorous error margin, followed by the same exact fp32 re-evaluation. */
int ivfr_set_list_sharing(ivfr_index* index, int32_t mode);

/* Look-up tables of Eq. (5).  mode 0: one m x 256 table per (query, visited list) pair is computed on
 * the matrix cores and written to the workspace (w * m KB per query), from where the scan kernels
 * load it.  mode 1 (split tables): the entry ||(x - c_l)^j - p_jk||^2 is expanded into
 * ||(x - c_l)^j||^2 + (||p_jk||^2 + 2 c_l^j . p_jk) - 2 x^j . p_jk; the bracket is a c x m x 256 table kept
 * with the index (built by the first search call in this mode, c * m KB), the last term one table per
 * query, the first m scalars per pair, and the scan kernels add the three when a pair's table enters
 * LDS: no per-pair table is written or read back.  Entries then carry the rounding of the larger
 * intermediate terms (about 1e-6 of an estimate instead of 1e-7); all scan kernels evaluate an entry by
 * the same expression, so the list-sharing modes stay bit-identical to one another within a table
 * mode.  With split tables list-sharing mode 3 acts as mode 2. */
int ivfr_set_table_mode(ivfr_index* index, int32_t mode);

/* Internal sizing knobs (defaults in parentheses); 0 keeps the current value.
 *   full_mult   (8)    a query that visits at most full_mult*k' entries keeps every estimate; a
 *                      larger one first scores a sample of its entries (about 16 (k' S)^(1/3) of the S
 *                      visited, at least a fraction 2/k'; the same leading fraction of every visited list,
 *                      or of the nearest ones only when k' is tiny against S) to bound the k'-th smallest
 *                      estimate, and the scan keeps only estimates below the bound
 *   cap_mult    (16)   such a query's candidate buffer holds max(cap_mult*k', min_cap) records, or its
 *   min_cap     (8192) sample, or the survivors expected from the bound plus six deviations, whichever
 *                      is largest; overflowing it triggers a rescan of that query with a tighter bound
 *   batch       (16384) queries processed per internal batch (fewer when w, k' or c are so large that
 *                      a batch's tables would exceed 8 GiB, its short-lists or coarse keys 4 GiB; a call
 *                      that needs several batches is split into equal ones).  Queries of one batch share
 *                      list reads, so larger batches are faster per query.
 *   scan_groups (0 = chosen from the amount of work) workgroups launched by the list-scan kernels          */
int ivfr_set_tuning(ivfr_index* index, int32_t full_mult, int32_t cap_mult, int32_t min_cap, int32_t batch,
                    int32_t scan_groups);

/* Device memory.  ivfr_memory_required is pure host arithmetic (no GPU call): the bytes an index of N
 * vectors with these parameters holds on the device (index_bytes: per vector the m-byte code that the
 * list scan streams plus one record of id, list, code and refinement code - m + m' + 8 bytes rounded
 * up to 32, 64 or 128 - that the re-rank gathers with a single memory access; list table; codebooks)
 * and the workspace a search call with nq queries, w and kprime adds
 * (search_bytes: per-batch arrays plus the candidate pool expected for lists of equal length; a
 * skewed index can want more).  Either output may be NULL.  With available_bytes > 0 it returns
 * IVFR_ERR_OOM when the sum exceeds it.  ivfr_set_memory_limit caps what this index may hold in
 * total (0 = no cap beyond the device's free memory): ivfr_finalize, ivfr_import and ivfr_search
 * check the cap and the free device memory before allocating and fail with IVFR_ERR_OOM, leaving the
 * index as it was. */
int ivfr_memory_required(const ivfr_params* params, int64_t N, int64_t nq, int32_t w, int32_t kprime,
                         int64_t available_bytes, int64_t* index_bytes, int64_t* search_bytes);
int ivfr_set_memory_limit(ivfr_index* index, int64_t bytes);
/* What the index holds on the device now (any pointer may be NULL): the finished inverted file, the
 * search workspace (per-batch arrays, plus the buffer of the unfiltered redo when one was needed), the
 * candidate pool; and how many internal batches of the most recent search call ran twice (the
 * candidate pool had to grow, or a batch of a multi-batch call was brought back for a redo). */
int ivfr_workspace_info(const ivfr_index* index, int64_t* index_bytes, int64_t* workspace_bytes,
                        int64_t* pool_bytes, int64_t* batch_reruns);

/* Per-stage GPU time of the most recent search call, in milliseconds, measured with HIP events
 * on the streams the kernels run on.  ivfr_set_profiling(index, level): 0 = off (default), 1 = only the
 * list-scan launches are timed (the IVFR_STAGE_SCAN* stages; about 0.03 ms of host time per batch), 2 = every
 * stage (about 0.1 ms per batch).  ms: host double
 * [IVFR_N_STAGES], indexed by IVFR_STAGE_*; scan_launches: launches of the list-scan kernels
 * (the IVFR_STAGE_SCAN* stages are exactly those launches), may be NULL. */
#define IVFR_STAGE_COARSE    0   /* query norms + coarse distance GEMM                        */
#define IVFR_STAGE_PROBE     1   /* w nearest lists + plan of (query, list) pairs             */
#define IVFR_STAGE_LUT       2   /* look-up tables of Eq. (5)                                 */
#define IVFR_STAGE_SAMPLE    3   /* sample scoring + bound selection                          */
#define IVFR_STAGE_SCAN      4   /* ADC list scan, one (query, list) pair at a time           */
#define IVFR_STAGE_SHORTLIST 5   /* exact k' smallest of the survivors                        */
#define IVFR_STAGE_RERANK    6   /* Eq. (9)-(10) over the short-list                          */
#define IVFR_STAGE_FINAL     7   /* k smallest refined distances, sorted                      */
#define IVFR_STAGE_SCAN_SHARED 8 /* ADC list scan, four queries per pass over a shared list   */
#define IVFR_STAGE_SCAN_SHARED2 9 /* ADC list scan, two queries per pass over a shared list   */
#define IVFR_STAGE_SCAN_SHARED8 10 /* ADC list scan, eight queries per pass, fp16 tables      */
#define IVFR_STAGE_SCAN_SHARED64 11 /* ADC list scan, 64 queries per pass on the matrix cores */
#define IVFR_STAGE_HOST_ENQUEUE 12 /* host time spent enqueuing the call's work (always measured) */
#define IVFR_STAGE_HOST_WAIT 13  /* host time spent waiting for the stream (always measured)  */
#define IVFR_N_STAGES        14
int ivfr_set_profiling(ivfr_index* index, int32_t enable);
int ivfr_stage_times(const ivfr_index* index, double* ms, int32_t* scan_launches);

const char* ivfr_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IVFADCR_H */
