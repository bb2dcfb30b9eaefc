/*
 * dessert.h -- C ABI of the MI355X (gfx950) library for hashed set-to-set
 * scoring: vector-set search with vector-set queries (DESSERT, arxiv
 * 2210.15748).
 *
 * The paper's problem statement (Sec. 1.1): given N vector sets S_1..S_N and
 * a query set Q, return the sets with the largest F(Q,S) = A(sigma(sim(q,x))).
 * The library implements the paper's estimator of F (Alg. 1 and Alg. 2) with
 * signed-random-projection hashes, sigma = max and A = sum:
 *
 *     code_t(x)  = C sign bits of the projections t*C .. t*C+C-1   (Sec. 3, Sec. 5)
 *     cnt(q,x)   = #{ t < L : code_t(q) == code_t(x) }              (Alg. 2, inner loops)
 *     score(Q,S) = sum_{q in Q} max_{x in S} cnt(q,x)               (Alg. 2, sigma then A)
 *
 * followed by the k best documents (Alg. 2 last line, widened from argmax).
 * The division by L in Alg. 2 and the remap of Eq. 1 are not applied: scores
 * are integers in [0, |Q|*L].
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses on config.device, "host"
 *     pointers are ordinary host memory.  No torch or C++ type crosses the ABI.
 *   - Ownership: the caller allocates and frees every buffer it passes in
 *     (vectors, codes, offsets, workspace, outputs).  The handle owns only its
 *     host metadata and the device copy of the projection matrix it makes in
 *     dessert_create.  Buffers given to dessert_build_index must stay alive
 *     and unchanged while the index is searched.
 *   - Asynchrony: all device work is enqueued on config.stream; calls return
 *     without synchronising.  Host arrays are read before the call returns.
 *     Outputs are valid once the caller has synchronised the stream.  (dessert_set_score_transform
 *     is asynchronous too: the new table is written in stream order.)  Calls
 *     on a stream that is being captured into a HIP graph: dessert_search,
 *     dessert_scores, dessert_search_noalloc, dessert_filter_query and dessert_filter_search record
 *     a fixed sequence of kernel launches when all query sets of the batch
 *     have the same length and all candidate lists have the same length; with
 *     unequal lengths (their offset arrays would be uploaded from a staging
 *     buffer that later calls reuse), in debug mode, and for
 *     dessert_build_index, a capturing stream gives DESSERT_ESTATE.  Timing
 *     events are not recorded while capturing.  (One
 *     copy runs on a stream the handle owns: the offsets upload of
 *     dessert_build_index, beside the hash kernel; it starts after the work
 *     config.stream held at entry and config.stream waits for it before the
 *     call's work counts as done, so the caller sees stream order as usual.)
 *   - Errors: every call returns a status.  Argument errors are detected on
 *     the host before anything is launched (DESSERT_EINVAL), HIP failures
 *     give DESSERT_EHIP; dessert_last_error() returns a thread-local message.
 *   - Document ids are 0-based positions in build order.
 *   - Bit conventions: projection row t*C+c gives bit c of table t's code; a
 *     projection that is exactly 0 gives bit 1 (p >= 0).
 *   - Top-k order: score descending, ties by ascending document id; if fewer
 *     than k documents were scored the remaining slots hold id 0xFFFFFFFF and
 *     score -1.  Candidate ids are scored as given (duplicates appear twice).
 *   - Code width: a table's code holds its C one-bit hashes in one byte when
 *     C <= 8 and in a little-endian u16 when 9 <= C <= 16 (Sec. 6.1 uses
 *     C = log2(m) + 1, up to 11).  "Code arrays" below are [n][L] of that type.
 *   - Limits: 1 <= C <= 16, L a multiple of 4 with 4 <= L <= 128, d >= 1,
 *     (vectors of one query set) * L * (bytes per code) <= 65535, k <= 16384.  Candidate
 *     ids must be < n_docs (not checked on the device), except the value
 *     0xFFFFFFFF, which marks an empty candidate slot: it is scored -1 and is
 *     never returned by the top-k.
 */
#ifndef DESSERT_H
#define DESSERT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dessert_index dessert_index_t;

typedef enum {
    DESSERT_OK = 0,
    DESSERT_EINVAL = 1,   /* bad argument, nothing launched */
    DESSERT_ENOMEM = 2,   /* host or device allocation inside the library failed */
    DESSERT_EHIP = 3,     /* a HIP call failed; see dessert_last_error() */
    DESSERT_ESTATE = 4    /* call order (search before build_index, filter query before filter build, a filter
                             left over from an earlier build_index), or a call that cannot be captured into a graph */
} dessert_status_t;

enum { DESSERT_I8 = 0, DESSERT_F16 = 1 };                       /* vector element type */
enum { DESSERT_PROJ_RADEMACHER_I8 = 0, DESSERT_PROJ_GAUSSIAN_F32 = 1 };

/* Kernel variants, for cross-checking and measurement (dessert_set_algo). */
enum { DESSERT_HASH_AUTO = 0, DESSERT_HASH_SCALAR = 1, DESSERT_HASH_MFMA = 2 };
enum { DESSERT_SCORE_AUTO = 0, DESSERT_SCORE_BYTECMP = 1, DESSERT_SCORE_MASKLUT = 2 };

typedef struct {
    uint32_t d;            /* vector dimension */
    uint32_t L;            /* number of hash tables (Sec. 3) */
    uint32_t C;            /* sign bits concatenated per table (Sec. 5, concatenation trick) */
    uint32_t dtype;        /* DESSERT_I8 or DESSERT_F16 */
    uint32_t proj_kind;    /* DESSERT_PROJ_RADEMACHER_I8: int8 entries in {-1,+1};
                              DESSERT_PROJ_GAUSSIAN_F32: float entries */
    int32_t  device;       /* HIP device ordinal */
    uint64_t seed;         /* used only when proj_dev == NULL */
    const void *proj_dev;  /* dev, [L*C][d] row-major, int8 or float by proj_kind; copied by
                              dessert_create.  NULL: derive a Rademacher matrix from seed:
                              entry (row,col) = +1 iff the top bit of
                              mix64(seed + 0x9E3779B97F4A7C15*(row*d+col+1)) is set, mix64 being the
                              SplitMix64 finalizer.  NULL with the Gaussian kind is an error. */
    void *stream;          /* hipStream_t all work is enqueued on (NULL = default stream) */
} dessert_config_t;

/* Create a handle: validates the configuration, copies (or generates) the
 * projection matrix into library-owned device memory.  The hash functions
 * f_1..f_L of Sec. 3 are fixed from here on. */
dessert_status_t dessert_create(const dessert_config_t *config, dessert_index_t **out);
void dessert_destroy(dessert_index_t *index);

/* Copy the projection matrix in use ([L*C][d], int8 or float) to proj_out_dev. */
dessert_status_t dessert_get_projection(const dessert_index_t *index, void *proj_out_dev);

/* Select kernel variants (DESSERT_HASH_*, DESSERT_SCORE_*).  A variant that
 * does not support the configuration makes the later call return EINVAL. */
dessert_status_t dessert_set_algo(dessert_index_t *index, int hash_algo, int score_algo);

/* Score transform.
 *   DESSERT_SCORE_RAW_COUNTS (default): score = sum_q max_x cnt(q,x), an integer in [0, |Q|*L].
 *   DESSERT_SCORE_EQ1_Q16: the paper's practical pipeline (Sec. 5, concatenation trick, Eq. 1): each
 *     per-query-vector maximum count c is first turned into a similarity estimate
 *         sim(c) = exp(ln(c / L) / C)   (sim(0) = 0),
 *     tabulated once for the L+1 possible counts as the fixed-point integer
 *     round(65536 * sim(c)) (round half away from zero), and the score is the sum of these
 *     integers over the query vectors.  score / (65536 * |Q|) is the paper's "average of max
 *     similarities" (Sec. 6, experiment setup).  Integer sums keep the result independent of
 *     summation order.  Needs |Q| <= 16383.
 *   DESSERT_SCORE_MAX_* / DESSERT_SCORE_MEAN_* (Sec. 4.1, the lemma on sigma(x) = (1/m) sum_i phi(x_i) and its
 *     three example phi; Alg. 2 with s_hat = count / L): the inner aggregation sigma over the document's
 *     vectors is the maximum (MAX) or the mean (MEAN) of phi(count / L), with phi(x) = x (IDENTITY),
 *     e^x - 1 (EXPM1) or 1/(1+e^-x) - 1/2 (SIGMOID).  phi is tabulated for the L+1 counts as
 *     round(65536 * phi); the mean of a document of m vectors is the integer (sum + floor(m/2)) / m, 0 for an
 *     empty document; the score is the sum over the query vectors.  Needs |Q| <= 16383.  MEAN_IDENTITY has a
 *     mask-table form (L a power of two, documents of at most 65535 vectors: with phi the identity the mean comes
 *     from sums of collision counts); the other MEAN transforms run on the code-compare kernel only.
 * Applies to later dessert_search / dessert_scores calls. */
enum {
    DESSERT_SCORE_RAW_COUNTS = 0,
    DESSERT_SCORE_EQ1_Q16 = 1,
    DESSERT_SCORE_MAX_IDENTITY_Q16 = 2,
    DESSERT_SCORE_MAX_EXPM1_Q16 = 3,
    DESSERT_SCORE_MAX_SIGMOID_Q16 = 4,
    DESSERT_SCORE_MEAN_IDENTITY_Q16 = 5,
    DESSERT_SCORE_MEAN_EXPM1_Q16 = 6,
    DESSERT_SCORE_MEAN_SIGMOID_Q16 = 7
};
dessert_status_t dessert_set_score_transform(dessert_index_t *index, int transform);

/* Weighted outer aggregation (Sec. 4.2: F(Q,S) = (1/m_q) sum_j w_j sigma(s_hat(q_j, S)), 0 <= w_j <= 1;
 * the division by m_q is left out).  weights_dev: dev, [n_weights] u32, weight j stands for w_j = value / 65536
 * (values above 65536 are an error of the caller, not checked on the device) and multiplies query vector j
 * of the batches passed to later dessert_search / dessert_scores calls, whose total number of query
 * vectors must equal n_weights (else DESSERT_EINVAL); a query vector then contributes
 * (w * sigma + 32768) >> 16.  Needs a *_Q16 score transform.  NULL removes the weights.  The array is
 * read by the later calls and must stay alive until they have run. */
dessert_status_t dessert_set_query_weights(dessert_index_t *index, const uint32_t *weights_dev, uint64_t n_weights);

/* Bytes of the code array for n_vectors vectors: n_vectors * L * (bytes per code), one code per
 * vector and table, vector-major, no padding. */
size_t dessert_code_bytes(const dessert_index_t *index, uint64_t n_vectors);

/* Hash n vectors (Alg. 1 line "h = f_t(x_j)", Alg. 2 line "h_{t,q} = f_t(q)").
 * vectors_dev: dev, [n][d] row-major of config.dtype.  codes_dev: dev, out, code array [n][L]
 * (u8, or u16 when C > 8: see "Code width"), dessert_code_bytes(index, n) bytes. */
dessert_status_t dessert_hash(const dessert_index_t *index, const void *vectors_dev, uint64_t n,
                              uint8_t *codes_dev);

/* Build the index (Alg. 1): hash every vector of every document and record
 * where each document's codes live.
 *   vectors_dev   dev, [n_vectors][d]: the documents' vectors, concatenated in document order
 *   lengths_host  host, [n_docs] u32: m_i = |S_i| (0 allowed); sum must equal n_vectors
 *   codes_dev     dev, out, dessert_code_bytes(n_vectors): code (offsets[i]+j)*L + t of the array = f_t(x_j of S_i)
 *   offsets_dev   dev, out, [n_docs+1] u64: exclusive scan of lengths (in vectors)
 * The handle remembers codes_dev / offsets_dev for later searches.  A candidate filter built over an earlier
 * collection on this handle is dropped: dessert_filter_query gives DESSERT_ESTATE until dessert_filter_build
 * has run again. */
dessert_status_t dessert_build_index(dessert_index_t *index, const void *vectors_dev, uint64_t n_vectors,
                                     const uint32_t *lengths_host, uint64_t n_docs,
                                     uint8_t *codes_dev, uint64_t *offsets_dev);

/* Attach an index built earlier (Alg. 1's sketch D is the code array plus the offsets; nothing else is kept): the arrays that
 * a dessert_build_index call with the same configuration and the same projection matrix (dessert_get_projection; pass it as
 * config.proj_dev) wrote, e.g. reloaded from disk, become this handle's index without hashing anything again.
 *   codes_dev    dev, dessert_code_bytes(n_vectors) bytes, as written by dessert_build_index
 *   offsets_dev  dev, [n_docs+1] u64, as written by dessert_build_index
 *   max_length   vectors of the longest document (bounds checks and kernel choice; the largest offsets difference)
 * Nothing is read on the device and nothing is checked against the arrays' contents.  Buffers must stay alive as for
 * dessert_build_index; a candidate filter of the previous collection is dropped. */
dessert_status_t dessert_attach_index(dessert_index_t *index, const uint8_t *codes_dev, const uint64_t *offsets_dev,
                                      uint64_t n_docs, uint64_t n_vectors, uint64_t max_length);

/* Workspace bytes needed by dessert_search / dessert_scores for a batch of
 * n_queries query sets with total_q_vectors vectors in all, total_scored
 * (query set, document) pairs (n_queries * n_docs when every document is
 * scored) and k results per query set.  Call it after dessert_build_index: the
 * size depends on the number of documents in the index. */
size_t dessert_search_workspace_bytes(const dessert_index_t *index, uint32_t n_queries,
                                      uint64_t total_q_vectors, uint64_t total_scored, uint32_t k);

/* Query the index (Alg. 2) for a batch of query sets.
 *   q_vectors_dev      dev, [sum q_lengths][d]: query vectors, query sets concatenated
 *   q_lengths_host     host, [n_queries] u32: |Q_b| >= 1
 *   cand_ids_dev       dev, u32 document ids to score, the lists of all query sets concatenated;
 *                      NULL = score every document for every query set
 *   cand_offsets_host  host, [n_queries+1] u64: query set b scores cand_ids[cand_offsets[b] ..
 *                      cand_offsets[b+1]); ignored when cand_ids_dev is NULL
 *   workspace_dev      dev, at least dessert_search_workspace_bytes(...) bytes, 256-byte aligned
 *   out_ids_dev        dev, out, [n_queries][k] u32
 *   out_scores_dev     dev, out, [n_queries][k] i32
 */
dessert_status_t dessert_search(const dessert_index_t *index, const void *q_vectors_dev,
                                const uint32_t *q_lengths_host, uint32_t n_queries,
                                const uint32_t *cand_ids_dev, const uint64_t *cand_offsets_host,
                                uint32_t k, void *workspace_dev, size_t workspace_bytes,
                                uint32_t *out_ids_dev, int32_t *out_scores_dev);

/* Same as dessert_search up to and including the outer aggregation A, without
 * the top-k: raw integer scores.  out_scores_dev: dev, out, i32; candidate
 * mode: [cand_offsets[n_queries]] in candidate order; otherwise
 * [n_queries][n_docs]. */
dessert_status_t dessert_scores(const dessert_index_t *index, const void *q_vectors_dev,
                                const uint32_t *q_lengths_host, uint32_t n_queries,
                                const uint32_t *cand_ids_dev, const uint64_t *cand_offsets_host,
                                void *workspace_dev, size_t workspace_bytes, int32_t *out_scores_dev);

/* Allocation-free form of dessert_search, for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same results as
 * dessert_search for a batch in which every query set has q_length vectors and every candidate list has
 * cand_length ids (cand_ids_dev NULL: every document is scored and cand_length is ignored); such a batch needs no
 * offset arrays, so nothing is read from host arrays either.  The workspace is a device array built into the
 * library, DESSERT_NOALLOC_SCRATCH_BYTES per GPU (each GPU the library is used on holds it until the process
 * ends); a batch whose dessert_search_workspace_bytes(...) exceeds it gives DESSERT_EINVAL with the two sizes in
 * the message.  The call allocates nothing and calls no allocating HIP routine.  All calls on one GPU share that
 * GPU's array: two calls may not overlap on one GPU (different streams or threads), whichever handles they use;
 * calls in stream order on one stream are fine.  Inputs and outputs are the caller's, as in dessert_search. */
#define DESSERT_NOALLOC_SCRATCH_BYTES (16u << 20)
size_t dessert_noalloc_scratch_bytes(void);
dessert_status_t dessert_search_noalloc(const dessert_index_t *index, const void *q_vectors_dev, uint32_t q_length,
                                        uint32_t n_queries, const uint32_t *cand_ids_dev, uint64_t cand_length,
                                        uint32_t k, uint32_t *out_ids_dev, int32_t *out_scores_dev);

/* Debug mode (Sec. 1.1: the candidates are ids of the N sets of the collection): with enable != 0, every later
 * dessert_search / dessert_scores / dessert_search_noalloc call that gets candidate ids first range-checks them on
 * the device and returns DESSERT_EINVAL, naming the first offending slot, if an id is neither below n_docs nor the
 * empty-slot value 0xFFFFFFFF; nothing else is launched then.  The check waits for the stream (it reads one word
 * back), so calls in debug mode are synchronous and cannot be captured into a graph.  Off by default: candidate ids
 * are then used as given. */
dessert_status_t dessert_set_debug(dessert_index_t *index, int enable);

/* Candidate filter (Sec. 5 "Filtering"): an inverted index from centroid ids to document ids and the
 * query-side selection of the documents to score.  The centroids are an input (any centroid set works;
 * dessert_filter_kmeans below trains them as the paper does, by k-means on a sample of the vectors).  "Closest" is the squared Euclidean
 * distance, ties to the lower centroid id.  Needs int8 vectors with d in {64, 128, 256} and a built
 * index (dessert_build_index) over the same vectors_dev.
 *
 * dessert_filter_build: for every document vector the closest centroid, then bucket c = the set of
 * documents with at least one vector assigned to c.
 *   centroids_dev       dev, [n_centroids][d] int8 (copied in re-ordered form; may be freed afterwards)
 *   assign_dev          dev, out, [n_vectors] u32: closest centroid of every vector
 *   bucket_offsets_dev  dev, out, [n_centroids+1] u32: bucket c = bucket_docs[offsets[c] .. offsets[c+1])
 *   bucket_docs_dev     dev, out, room for n_vectors u32 (upper bound of the total bucket size); a
 *                       document appears once per bucket, in unspecified order inside the bucket
 * The two bucket arrays must stay alive while dessert_filter_query is used.  This call waits for the
 * stream at its end (it reads the bucket sizes back: the largest one sizes the query workspace).  The
 * library's own filter buffers are allocated by the first call and kept while n_centroids and the
 * number of documents' id ranges stay the same: such a later call allocates and frees nothing.
 *
 * dessert_filter_query: for each query vector the filter_probe closest centroids; every document gets
 * one count per (query vector, probed centroid) pair whose bucket holds it; per query set the
 * filter_k documents with the highest count (ties: lower id), among documents with count >= 1.
 *   out_ids_dev     dev, out, [n_queries][filter_k] u32, unused slots 0xFFFFFFFF: can be passed to
 *                   dessert_search as candidate lists of equal length filter_k
 *   out_counts_dev  dev, out, [n_queries][filter_k] i32, unused slots -1
 *   workspace_dev   dev, 256-byte aligned, dessert_filter_workspace_bytes(index, n_queries, total query
 *                   vectors, longest query set, filter_probe) bytes
 * Limits: n_centroids <= 2^20, filter_probe <= min(n_centroids, 1024), filter_k <= 16384. */
/* k-means for the filter's centroids (Sec. 5 "Filtering": k-means clustering on a sample of the vectors at
 * the start of indexing).  Lloyd's iteration in integers: each of the `iterations` rounds assigns every
 * sample vector to its closest centroid (squared Euclidean distance, ties to the lower id) and replaces
 * every centroid that received vectors by their coordinate-wise mean rounded to the nearest integer
 * (half rounds up); a centroid without vectors stays.
 *   sample_dev     dev, [n_sample][d] int8, 16-byte aligned, n_sample <= 2^23
 *   centroids_dev  dev, in/out, [n_centroids][d] int8: the initial centroids (e.g. distinct sample vectors) on
 *                  entry, the result on return; pass it to dessert_filter_build
 *   workspace_dev  dev, 256-byte aligned, dessert_filter_kmeans_workspace_bytes(index, n_sample, n_centroids)
 * Uses only d, the device and the stream of the index (no built index needed).  Asynchronous. */
size_t dessert_filter_kmeans_workspace_bytes(const dessert_index_t *index, uint64_t n_sample, uint32_t n_centroids);
dessert_status_t dessert_filter_kmeans(const dessert_index_t *index, const int8_t *sample_dev, uint64_t n_sample,
                                       int8_t *centroids_dev, uint32_t n_centroids, uint32_t iterations,
                                       void *workspace_dev, size_t workspace_bytes);

dessert_status_t dessert_filter_build(dessert_index_t *index, const int8_t *centroids_dev, uint32_t n_centroids,
                                      const void *vectors_dev, uint32_t *assign_dev, uint32_t *bucket_offsets_dev,
                                      uint32_t *bucket_docs_dev);
size_t dessert_filter_workspace_bytes(const dessert_index_t *index, uint32_t n_queries, uint64_t total_q_vectors,
                                      uint32_t max_q_len, uint32_t filter_probe);
dessert_status_t dessert_filter_query(const dessert_index_t *index, const void *q_vectors_dev,
                                      const uint32_t *q_lengths_host, uint32_t n_queries, uint32_t filter_probe,
                                      uint32_t filter_k, void *workspace_dev, size_t workspace_bytes,
                                      uint32_t *out_ids_dev, int32_t *out_counts_dev);

/* The paper's whole query (Sec. 5: filter the collection down to filter_k candidate documents per query set, score
 * those with Alg. 2, return the k best) in one call: dessert_filter_query followed by dessert_search on its ids, with the
 * same results as the two calls.  Between the two steps only the SET of candidates matters, so the filter leaves out the
 * ordering of its filter_k documents (a fifth of its time for one query set).  workspace_dev: dev, 256-byte aligned,
 * dessert_filter_search_workspace_bytes(...) bytes (0 before dessert_filter_build); it also holds the candidate lists.
 * out_ids_dev / out_scores_dev: dev, out, [n_queries][k], as dessert_search. */
size_t dessert_filter_search_workspace_bytes(const dessert_index_t *index, uint32_t n_queries, uint64_t total_q_vectors,
                                             uint32_t max_q_len, uint32_t filter_probe, uint32_t filter_k, uint32_t k);
dessert_status_t dessert_filter_search(const dessert_index_t *index, const void *q_vectors_dev,
                                       const uint32_t *q_lengths_host, uint32_t n_queries, uint32_t filter_probe,
                                       uint32_t filter_k, uint32_t k, void *workspace_dev, size_t workspace_bytes,
                                       uint32_t *out_ids_dev, int32_t *out_scores_dev);

/* Per-kernel timing of dessert_search / dessert_scores / dessert_build_index
 * calls on this handle, measured with HIP events recorded on config.stream
 * around each stage (off by default; enabling adds event records but no
 * synchronisation to the calls).  enable = 0: off; 1: every call is timed; n > 1: every
 * n-th call, starting with the next one (the five event records cost a few microseconds of
 * GPU time per call, 4 % of a 0.45 ms search).  The last 64 timed calls are kept.
 * dessert_get_timing waits for the chosen call's last event and writes
 * milliseconds: ms[0] hashing (a search: query preparation, i.e. hashing and the ordering of long
 * candidate lists), ms[1] scoring, ms[2] top-k, ms[3] whole call;
 * stages that did not run give 0.  calls_back = 0 is the most recent timed call. */
dessert_status_t dessert_enable_timing(dessert_index_t *index, int enable);
dessert_status_t dessert_get_timing(dessert_index_t *index, uint32_t calls_back, float ms[4]);

/* Measurement aid, not part of the method: time `reps` passes of a kernel that only reads
 * [buf_dev, buf_dev + bytes) with 16-byte loads (HIP events on `stream`; synchronises).  Gives
 * the streaming-read rate this GPU actually delivers, to set beside the nameplate 8 TB/s.
 * buf_dev: dev, 16-byte aligned, bytes >= 16; ms_per_pass: host, out. */
dessert_status_t dessert_probe_read_bandwidth(const void *buf_dev, size_t bytes, int device, void *stream, int reps,
                                              float *ms_per_pass);

/* Measurement and test aid: the scoring kernel instantiation that the handle's most recent dessert_search /
 * dessert_scores / dessert_search_noalloc call launched, spelled as a profiler's kernel trace prints it (e.g.
 * "score_masklut_kernel<32, 7, 1, 0, 1, false>": tables, index bits, bytes per code, score transform form, query sets
 * per workgroup, chunks split over workgroups); "" if nothing was launched.  Lets a caller pair a run with the
 * profiler summary of the same kernel.  The string lives in the handle. */
const char *dessert_last_score_kernel(const dessert_index_t *index);

/* Measurement aid, not part of the method: the traffic of index building without its arithmetic.  Times `reps` passes
 * of a kernel that reads 4 * out_bytes from in_dev and writes out_bytes to out_dev in whole lines (the 4 : 1 read : write
 * mix of 128-byte vectors in, 32 code bytes out), HIP events on `stream`; synchronises.  What it achieves is the ceiling
 * for dessert_build_index on this GPU, to set beside the nameplate 8 TB/s.  Both buffers dev, 16-byte aligned. */
dessert_status_t dessert_probe_mix_bandwidth(const void *in_dev, void *out_dev, size_t out_bytes, int device, void *stream,
                                             int reps, float *ms_per_pass);

const char *dessert_last_error(void);
const char *dessert_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DESSERT_H */
