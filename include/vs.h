/*
 * vs.h -- C ABI of the MI355X (gfx950) vector-search library.
 *
 * Batched IVF-PQ search and flat exact k-NN search as described in
 * "The Faiss Library" (arXiv 2401.08281): Sec. 3 (Eq. 1-2, brute-force
 * search, metrics), Sec. 4 (Eq. 10 asymmetric distance computation, product
 * quantizer, Eq. 14 look-up tables), Sec. 5.1 (inverted files, residual
 * encoding), App. A.3 "Optimization", paragraph "GPU Faiss" (the four GPU stages).
 *
 * General conventions
 *   - Every array pointer is a DEVICE pointer on the current HIP device,
 *     row-major and contiguous, owned by the caller unless stated otherwise.
 *     The library never frees or keeps caller pointers beyond the call.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = default stream).
 *     Work is enqueued on it.  vs_flat_search and vs_ivfpq_search return with
 *     the work enqueued; outputs are valid after the stream is synchronised.
 *     vs_ivfpq_create and vs_ivfpq_add synchronise the stream before
 *     returning.
 *   - metric VS_METRIC_L2 is the SQUARED Euclidean distance (smaller is
 *     better); VS_METRIC_IP is the inner product (larger is better).
 *     Results are ordered best first (Eq. 2).
 *   - Empty result slots (fewer than k candidates): id = -1 and distance
 *     +inf (L2) / -inf (IP), placed last (Sec. 6.1: negative ids are invalid).
 *   - Every function returns VS_OK or a negative error code; a message for
 *     the calling thread's last error is available from vs_last_error().
 *     Nothing throws across this boundary.  Inputs containing NaN are
 *     undefined behaviour of the ordering, never of memory safety.
 *   - Calls on the same index, or flat searches on the same device, must not
 *     overlap in time (they share scratch buffers).
 */
#ifndef VS_H_
#define VS_H_

#include <stdint.h>

#if defined(__GNUC__)
#define VS_API __attribute__((visibility("default")))
#else
#define VS_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct vs_ivfpq vs_ivfpq; /* opaque; created and destroyed by the library */

enum { VS_METRIC_L2 = 0, VS_METRIC_IP = 1 };

enum {
  VS_OK = 0,
  VS_ERR_INVALID_ARG = -1, /* null pointer, size out of range, shape mismatch */
  VS_ERR_UNSUPPORTED = -2, /* a combination this build has no kernel for */
  VS_ERR_OOM = -3,         /* device or host allocation failed */
  VS_ERR_DEVICE = -4       /* a HIP call failed; vs_last_error() has the HIP text */
};

#define VS_MAX_K 1024 /* largest k and largest nprobe accepted */

/*
 * Flat exact k-NN search (Sec. 3.1 "Brute force search", Eq. 2).
 *   x        [nb, d] fp32 database rows; row i has id i.  nb < 2^31.
 *   q        [nq, d] fp32 queries.
 *   out_dist [nq, k] fp32, out_ids [nq, k] int64: for each query the k best
 *            database rows, best first.
 * Distances are evaluated in fp32 as one fused-multiply-add chain per
 * (query, row) pair in dimension order; ties go to the smaller id.
 * nq == 0 is a no-op.  nb == 0 fills the outputs with empty slots.
 * Errors: null pointers (with nq > 0), d < 1, k < 1 or k > VS_MAX_K, unknown metric.
 * Work space: one grow-only buffer per device, shared by vs_flat_search, vs_flat_index_search,
 * vs_kmeans and vs_ivfpq_train.  Calls from several host threads or on several streams are
 * serialised on it: a call on another stream than the previous user's first waits (on the
 * device, through an event) for that user's kernels.
 */
VS_API int vs_flat_search(const float* x, int64_t nb, const float* q, int64_t nq, int32_t d,
                   int32_t metric, int32_t k, float* out_dist, int64_t* out_ids,
                   void* hip_stream);

/*
 * Flat index (Sec. 3.1; the "Flat" index of App. A.2, which stores the vectors as they
 * are): the database of vs_flat_search kept by the library, so that what a search needs of
 * it besides the rows -- squared norms and the bf16 operand planes of the matrix-core
 * route -- is computed when vectors are added instead of in every search.
 *   vs_flat_create   empty index for d-dimensional vectors and one metric.
 *   vs_flat_add      appends n rows x [n, d] (copied; row j of the call gets id ntotal + j,
 *                    Sec. "Adding vectors": sequential ids) and prepares the whole
 *                    database again: its cost grows with ntotal, add in large pieces.
 *                    Synchronises the stream.  ntotal stays below 2^31.
 *   vs_flat_index_search  same results as vs_flat_search(stored rows, ...), bit for bit.
 *   vs_flat_ntotal   number of stored rows (-1 for a null handle).
 *   vs_flat_destroy  frees the index (null is a no-op); the caller makes sure that no
 *                    search on it is still running.
 * Errors: as vs_flat_search; VS_ERR_OOM when storage cannot grow (the index is unchanged).
 */
typedef struct vs_flat vs_flat;
VS_API int vs_flat_create(vs_flat** out, int32_t d, int32_t metric);
VS_API void vs_flat_destroy(vs_flat* ix);
VS_API int64_t vs_flat_ntotal(const vs_flat* ix);
VS_API int vs_flat_add(vs_flat* ix, const float* x, int64_t n, void* hip_stream);
VS_API int vs_flat_index_search(const vs_flat* ix, const float* q, int64_t nq, int32_t k,
                                float* out_dist, int64_t* out_ids, void* hip_stream);

/*
 * vs_flat_search, vs_kmeans and vs_ivfpq_train keep one grow-only work buffer per device
 * (operand planes, candidate lists, ...; for a 10M x 768 database about 30 GB).  vs_trim
 * waits for the current device to go idle and frees that buffer; the next call allocates
 * what it needs again.  Indexes own their buffers and release them in their destroy call.
 */
VS_API int vs_trim(void);

/*
 * Re-rank a shortlist with exact distances (Sec. 3.5 "Refining"; the "RFlat" suffix
 * of App. A.2's index factory): the second, accurate stage behind a fast first
 * search such as vs_ivfpq_search run with kc > k.
 *   x        [nb, d] fp32, the uncompressed database rows; row i has id i.  nb < 2^32.
 *   q        [nq, d] fp32 queries (the ones the shortlist was computed for).
 *   cand_ids [nq, kc] int64: each query's shortlist.  Entries outside [0, nb) -- the -1
 *            of an empty slot -- are skipped; every other entry is taken as given (an id
 *            listed twice is returned twice).
 *   out_dist [nq, k] fp32, out_ids [nq, k] int64: the k best candidates by exact
 *            distance, best first, ties to the smaller id; empty slots as above.
 * Distances are the same fp32 chains as in vs_flat_search, so a candidate's value
 * here equals its value there bit for bit.
 * Errors: null pointers (with nq > 0), d < 1, kc < 1, k < 1 or k > VS_MAX_K, unknown
 * metric, nb >= 2^32; VS_ERR_UNSUPPORTED when d and k together exceed the on-chip memory
 * of a workgroup (d above roughly 5000 at k = 1024).
 */
VS_API int vs_refine(const float* x, int64_t nb, const float* q, int64_t nq, int32_t d,
              int32_t metric, const int64_t* cand_ids, int32_t kc, int32_t k, float* out_dist,
              int64_t* out_ids, void* hip_stream);

/*
 * Lloyd's k-means (Sec. 4.1 "The k-means vector quantizer"): niter rounds of
 *   (1) every training vector goes to its nearest centroid (squared L2 on the fp32 chain
 *       of vs_flat_search, ties to the smaller centroid number);
 *   (2) every centroid moves to the mean of its vectors: their float64 sum divided by their
 *       number, rounded to fp32; a centroid that received no vector stays where it is.
 *       The sum of a cluster of more than 4096 vectors is formed from partial sums of 4096
 *       consecutive members each (added in order), so that a long cluster is summed by
 *       several wavefronts; for clusters up to 4096 vectors it is the running sum in the
 *       order of the training set.  Either way the result is deterministic, and it differs
 *       from the running sum by float64 rounding only (at most the last bit of the fp32 mean).
 *   x          [n, d] fp32 training vectors, n < 2^31.
 *   centroids  [K, d] fp32: in, the initial centroids; out, the trained ones.
 *   objective  HOST pointer to niter doubles, or NULL: the mean squared distance of the
 *              training vectors to their centroid at step (1) of every round.
 *   assign     DEVICE [n] int32, or NULL: the centroid of every training vector at step (1)
 *              of the LAST round (the clusters whose means the returned centroids are).
 * Synchronises the stream every round (the size of the largest cluster and the objective
 * are read back; beyond 16384 centroids the whole assignment is, to be ordered on the host).
 * Errors: null pointers, d < 1, K < 1, niter < 0, n outside [0, 2^31).
 */
VS_API int vs_kmeans(const float* x, int64_t n, int32_t d, int32_t K, int32_t niter,
              float* centroids, double* objective, int32_t* assign, void* hip_stream);

/*
 * Parameters of an IVF-PQ index from training vectors (Sec. 5.1: the coarse quantizer is a
 * k-means; Sec. 4.1: each sub-quantizer of the product quantizer is a k-means; Sec. 5.1
 * "Encoding residuals": the product quantizer is trained on residuals):
 *   1. centroids <- vs_kmeans(x) from the given initial centroids;
 *   2. every training vector goes to its best centroid under `metric`, as in vs_ivfpq_add;
 *   3. residual = vector - centroid, one fp32 subtraction per component;
 *   4. codebooks[m] <- vs_kmeans(m-th slices of the residuals) from the given codebooks[m].
 *   centroids [nlist, d], codebooks [M, 2^nbits, d / M]: DEVICE, in = initial, out = trained.
 *   objective HOST pointer to (1 + M) * niter doubles, or NULL: row 0 the coarse k-means,
 *             row 1 + m sub-quantizer m.
 * Needs n * d floats of device memory for the residuals.  Blocks until done.
 * Errors: as vs_ivfpq_create for the shape; n outside [1, 2^31); niter < 0; null pointers.
 */
VS_API int vs_ivfpq_train(const float* x, int64_t n, int32_t d, int32_t metric, int32_t nlist,
                   int32_t M, int32_t nbits, int32_t niter, float* centroids, float* codebooks,
                   double* objective, void* hip_stream);

/*
 * Create an empty IVF-PQ index (Sec. 5.1 "Inverted files"; Sec. 4.1 product
 * quantizer).  The nlist coarse centroids and the M sub-codebooks are inputs (sampled by
 * the caller, or trained with vs_ivfpq_train) and are copied.
 *   centroids [nlist, d] fp32.
 *   codebooks [M, 2^nbits, d/M] fp32: codebooks[m][j] is codeword j of
 *             sub-quantizer m.
 * Vectors are encoded as residuals to their list's centroid (by_residual,
 * Sec. 5.1 "Encoding residuals") under both metrics.  Under VS_METRIC_IP,
 * list assignment and probing also use the inner product (argmax).
 * Errors: null pointers, d < 1, nlist < 1, M < 1, d % M != 0,
 * nbits not in {4, 8} (UNSUPPORTED), M odd with nbits == 4, unknown metric.
 */
VS_API int vs_ivfpq_create(vs_ivfpq** out, int32_t d, int32_t metric, int32_t nlist, int32_t M,
                    int32_t nbits, const float* centroids, const float* codebooks,
                    void* hip_stream);

/*
 * Add n vectors (Sec. 5.1; Sec. 6.1 for ids): each vector goes to the list of
 * its best centroid (ties: smaller list number), its residual is PQ-encoded
 * (each sub-vector to its nearest codeword in squared L2, ties: smaller code)
 * and (code, id) is appended to the list, after the entries already there and
 * in the order given.
 *   x   [n, d] fp32.
 *   ids [n] int64 >= 0, or NULL for sequential ids starting at the current
 *       ntotal.  The ids are not inspected: a negative id is stored and returned as
 *       given, where it cannot be told from the -1 of an empty result slot (Sec. 6.1:
 *       the sign bit marks an invalid id) -- the caller keeps ids non-negative.
 * Both decisions are taken on the fp32 fused-multiply-add chain described
 * for vs_flat_search, so they are reproducible bit for bit on any IEEE
 * machine.  Code bytes: nbits == 8: byte m = c_m; nbits == 4: byte i =
 * c_{2i} | c_{2i+1} << 4.
 * The list storage is re-laid-out contiguously; the call synchronises.
 * n == 0 is a no-op.  The total number of stored vectors must stay < 2^32.
 */
VS_API int vs_ivfpq_add(vs_ivfpq* ix, const float* x, int64_t n, const int64_t* ids, void* hip_stream);

/*
 * Batched IVF-PQ search (Sec. 5.1; Eq. 10 ADC; Eq. 14 look-up tables; App. A.3 "GPU Faiss").
 * For every query: the nprobe best centroids are found exactly (nprobe is
 * clamped to nlist), a look-up table LUT_m[j] is built per (query, probed
 * list) on the query's residual to the list centroid (per query for IP, plus
 * the centroid's inner product as a per-list bias), every code of the probed
 * lists is scored as sum_m LUT_m[c_m], and the k best over all probed lists
 * are returned best first with their stored ids.
 *   q [nq, d] fp32; out_dist [nq, k] fp32; out_ids [nq, k] int64.
 * Errors: null pointers (with nq > 0), k or nprobe < 1 or > VS_MAX_K.
 * Large batches on L2 indexes of the three fixed shapes are scanned list by list (option
 * "list_major" below): same results, one read of every probed list per batch; the work space then
 * also holds the candidate buffers, 8 bytes x "list_major_candidates" (default 1024) per query.
 * Work space: one grow-only buffer per index (the first call of a size allocates it; later
 * calls only enqueue kernels).  Searches of one index from several host threads or on several
 * streams are serialised on it: a call on another stream than the previous search's first waits,
 * on the device, for that search's kernels.  Searching while the same index is being added to
 * is not supported.
 */
VS_API int vs_ivfpq_search(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t k, int32_t nprobe,
                    float* out_dist, int64_t* out_ids, void* hip_stream);

/*
 * vs_ivfpq_search that also reports what the call did (App. A.3 "GPU Faiss": the scan of the
 * probed lists is the stage to price).  stats: DEVICE pointer to one vs_search_stats, written in
 * stream order by a small kernel of the same call (no synchronisation), or NULL for none:
 *   scanned_codes   sum over the (query, probe) pairs of the probed list's size = codes the scan read
 *   probed_lists    (query, probe) pairs whose list is not empty
 *   coarse_rows_matrix_core  queries whose probes were found through the matrix-core shortlist
 *   coarse_rows_fallback     ... of which failed the sufficiency test and were redone exactly
 *   list_major_first_probes  0, or (the batch was scanned list by list, see vs_ivfpq_search) the
 *                            number of probes per query that were scanned query by query first
 *   list_major_first_codes   the part of scanned_codes that falls on those probes
 *   list_major_rescanned     queries whose candidate buffer overflowed in the list-major scan and
 *                            that were therefore scanned again query by query (their codes are
 *                            not counted twice in scanned_codes)
 * Results, errors and work space are those of vs_ivfpq_search.  nq == 0 zeroes the block.
 */
typedef struct vs_search_stats {
  int64_t scanned_codes;
  int64_t probed_lists;
  int64_t coarse_rows_matrix_core;
  int64_t coarse_rows_fallback;
  int64_t list_major_first_probes;
  int64_t list_major_first_codes;
  int64_t list_major_rescanned;
} vs_search_stats;
VS_API int vs_ivfpq_search_stats(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t k, int32_t nprobe,
                          float* out_dist, int64_t* out_ids, vs_search_stats* stats, void* hip_stream);

/*
 * vs_ivfpq_search for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results
 * bit for bit, but the work space of the search (operand planes and candidate lists of the
 * coarse quantizer, probes, per-split partial results, the work counter of the scan) is a
 * file-scope device array of VS_STATIC_SCRATCH_BYTES that every GPU the library runs on holds
 * until the process ends, instead of the index's grow-only buffer.  The call allocates and
 * frees nothing (no hipMalloc / hipFree, no events) and only enqueues kernels on hip_stream.
 * The array's device address is looked up once per device (in vs_ivfpq_create, else in the
 * first call on that device).
 * Limits: the work space grows with nq (and nlist, d, nprobe, k): a call whose work space
 * exceeds VS_STATIC_SCRATCH_BYTES is refused with VS_ERR_INVALID_ARG and a message that states
 * both sizes (32 MiB serve e.g. 64 queries at nlist = 65536, d = 96, nprobe = 64, k = 100, or
 * 256 queries at nlist = 4096, d = 128, nprobe = 64).  Profiling stages are not recorded.
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU race
 * (also calls on different indexes or streams); the caller serialises them.
 */
#define VS_STATIC_SCRATCH_BYTES (32u << 20)
VS_API int vs_ivfpq_search_static(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t k,
                           int32_t nprobe, float* out_dist, int64_t* out_ids, void* hip_stream);

/* Frees the index and all device memory it owns.  NULL is allowed. */
VS_API void vs_ivfpq_destroy(vs_ivfpq* ix);

/* ---- introspection (used by parity checks) ------------------------------ */

/* Number of stored vectors; -1 if ix is NULL. */
VS_API int64_t vs_ivfpq_ntotal(const vs_ivfpq* ix);
/* Bytes per stored code = M * nbits / 8; -1 if ix is NULL. */
VS_API int32_t vs_ivfpq_code_size(const vs_ivfpq* ix);
/* sizes: DEVICE [nlist] int64, number of entries per list. */
VS_API int vs_ivfpq_get_list_sizes(const vs_ivfpq* ix, int64_t* sizes, void* hip_stream);
/* Storage-order dump: entry s of the list-contiguous store has id ids[s]
 * and lives in list list_of[s].  DEVICE [ntotal] each; either may be NULL. */
VS_API int vs_ivfpq_get_assignments(const vs_ivfpq* ix, int64_t* ids, int32_t* list_of,
                             void* hip_stream);
/* codes: DEVICE [ntotal, code_size] uint8 in the same storage order. */
VS_API int vs_ivfpq_get_codes(const vs_ivfpq* ix, uint8_t* codes, void* hip_stream);
/* Coarse quantizer alone (first stage of vs_ivfpq_search): the nprobe best
 * lists per query, best first.  probes: DEVICE [nq, min(nprobe, nlist)] int32;
 * coarse_dist: DEVICE, same shape, fp32, may be NULL. */
VS_API int vs_ivfpq_coarse(const vs_ivfpq* ix, const float* q, int64_t nq, int32_t nprobe,
                    int32_t* probes, float* coarse_dist, void* hip_stream);

/*
 * How vs_ivfpq_search evaluates distances in the compressed domain (Sec. 4.3
 * "Compressed-domain search").  VS_ST_RESIDUAL_TABLES (default): one table of squared
 * distances between the query's residual r = q - c_l and the codewords per (query, probed
 * list).  For the shapes with a specialised kernel (8-bit codes of 8, 16 or 32 sub-quantizers
 * on d = 32, 128, 96) an entry is evaluated as (|r_m|^2 + |t|^2) + sum_u r_u (-2 t_u) rather than
 * sum_u (r_u - t_u)^2: the same number for integer data, otherwise off by rounding of at most
 * (d/M + 2) 2^-23 (|r_m|^2 + |t|^2) -- relative to the cancelling terms, not to the distance, which
 * matters only when the query (nearly) coincides with a reconstruction.  Results of both L2
 * forms are clamped at 0.
 * VS_ST_STORED_NORMS (L2 only): the decomposition |q - x'|^2 = |q|^2 + |x'|^2 - 2 <q, x'>
 * with |x'|^2 stored next to every code as a float32 (4 more bytes per vector): one table of
 * inner products per QUERY, no per-list table; the result differs from the default form by
 * the rounding of the cancelling terms, about 2^-22 (|q|^2 + |x'|^2).
 * With lists of a few hundred codes this is the fastest of the three forms (no per-list table
 * at all: for the 8 x 4 and 16 x 8 shapes one wavefront scans a (query, probe split) on its own).
 * vs_ivfpq_add computes the norms of what it adds only while this type is selected (adding
 * under another type drops the stored norms); selecting it on an index that holds vectors
 * without norms computes them from the stored codes (ntotal * (code_size + 8) bytes of
 * temporary device memory; VS_ERR_OOM if that does not fit) and synchronises.
 * VS_ST_PRECOMPUTED_TABLES (L2 only): the same table per (query, probed list) as the default,
 * but formed as the sum of a term that depends on the query alone, -2 <q_m, T_m[j]> (computed
 * once per query), and a term that depends on the list alone, |T_m[j]|^2 + 2 <c_{l,m}, T_m[j]>
 * (computed once, when this type is first selected: nlist * M * 2^nbits floats of device memory,
 * 64 MB for nlist = 4096, M = 16), plus the probe's coarse distance |q - c_l|^2: one addition per
 * table entry and list instead of d / M multiply-adds, which is what pays when lists hold a few
 * hundred codes and the tables cost more than the scan.  Results differ from the default form by
 * rounding of the cancelling terms, at most about 2^-21 (|q|^2 + |c_l|^2 + |x' - c_l|^2).  Can be
 * selected at any time.  VS_ERR_UNSUPPORTED for shapes without a specialised scan kernel (other
 * than 8-bit codes with M x d/M = 8 x 4, 16 x 8, 32 x 3), VS_ERR_OOM if the tables do not fit.
 */
enum { VS_ST_RESIDUAL_TABLES = 0, VS_ST_STORED_NORMS = 1, VS_ST_PRECOMPUTED_TABLES = 2 };
VS_API int vs_ivfpq_set_search_type(vs_ivfpq* ix, int32_t search_type);
/*
 * The metric under which vectors are assigned to lists and lists are probed, when it is not the
 * index metric (Sec. 5.1, the figure on maximum inner product search: an inner-product index
 * may assign by L2 -- the paper's default -- or by inner product).  Here the default is the index
 * metric for both; vs_ivfpq_set_coarse_metric(ix, VS_METRIC_L2) on a VS_METRIC_IP index makes
 * vs_ivfpq_add take the L2-nearest centroid and searches probe the nprobe L2-nearest lists, while
 * scores stay inner products <q, c_l> + sum_m <q_m, T_m[c_m]> (the <q, c_l> of the probed lists is
 * then computed after the coarse quantizer, one fused-multiply-add chain each).
 * vs_ivfpq_coarse returns the values of the coarse metric.  To be called while the index is
 * empty.  Errors: unknown metric; VS_METRIC_IP on an L2 index; an index that already holds
 * vectors assigned under the other metric.
 */
VS_API int vs_ivfpq_set_coarse_metric(vs_ivfpq* ix, int32_t metric);
/* the stored norms, in storage order: DEVICE [ntotal] fp32 */
VS_API int vs_ivfpq_get_norms(const vs_ivfpq* ix, float* norms, void* hip_stream);

/* ---- IVF-Flat ----------------------------------------------------------------
 * The inverted file of Sec. 5.1 with the vectors stored as they are (no codec; App. A.3
 * "GPU Faiss" lists it among the GPU indexes).  Coarse quantizer, list assignment, ids,
 * probing and selection are those of the IVF-PQ index above; the scan computes the exact
 * distance (the fp32 chain of vs_flat_search) to every vector of the probed lists, so with
 * nprobe = nlist the result is that of vs_flat_search.  Same conventions, limits and
 * errors as the vs_ivfpq_* calls of the same name. */
typedef struct vs_ivfflat vs_ivfflat;
VS_API int vs_ivfflat_create(vs_ivfflat** out, int32_t d, int32_t metric, int32_t nlist,
                      const float* centroids /* [nlist, d], copied */, void* hip_stream);
VS_API void vs_ivfflat_destroy(vs_ivfflat* ix);
VS_API int64_t vs_ivfflat_ntotal(const vs_ivfflat* ix);
VS_API int vs_ivfflat_add(vs_ivfflat* ix, const float* x, int64_t n, const int64_t* ids,
                   void* hip_stream);
VS_API int vs_ivfflat_search(const vs_ivfflat* ix, const float* q, int64_t nq, int32_t k,
                      int32_t nprobe, float* out_dist, int64_t* out_ids, void* hip_stream);
VS_API int vs_ivfflat_get_list_sizes(const vs_ivfflat* ix, int64_t* sizes, void* hip_stream);
/* storage order: ids [ntotal], list of every entry [ntotal], stored rows [ntotal, d]
 * (DEVICE, each may be NULL) */
VS_API int vs_ivfflat_get_storage(const vs_ivfflat* ix, int64_t* ids, int32_t* list_of, float* rows,
                           void* hip_stream);

/* ---- IVF-SQ8 -----------------------------------------------------------------
 * The inverted file of Sec. 5.1 with every vector stored as an 8-bit scalar-quantizer code
 * (Sec. 4.1 "Scalar quantizers"; App. A.3 "GPU Faiss" lists the index): d bytes per vector.
 * Component t is expected in [vmin[t], vmin[t] + 256 step[t]); the code is the number of the
 * cell of width step[t] that holds it (components outside go to the first / last cell):
 *     u = (x_t - vmin[t]) / step[t] in fp32;  code = 0 if u < 0, 255 if u >= 256, else trunc(u)
 * and the reconstruction is the middle of the cell, fma(code + 0.5, step[t], vmin[t]).  The
 * vectors themselves are encoded (no residual); lists come from the original vectors.  The
 * scan evaluates the fp32 distance chain of vs_flat_search on the reconstructions.
 *   vmin, step: DEVICE [d] fp32, copied; every step must be positive.
 * Otherwise as the vs_ivfflat_* calls of the same name. */
typedef struct vs_ivfsq8 vs_ivfsq8;
VS_API int vs_ivfsq8_create(vs_ivfsq8** out, int32_t d, int32_t metric, int32_t nlist,
                     const float* centroids, const float* vmin, const float* step,
                     void* hip_stream);
VS_API void vs_ivfsq8_destroy(vs_ivfsq8* ix);
VS_API int64_t vs_ivfsq8_ntotal(const vs_ivfsq8* ix);
VS_API int vs_ivfsq8_add(vs_ivfsq8* ix, const float* x, int64_t n, const int64_t* ids,
                  void* hip_stream);
VS_API int vs_ivfsq8_search(const vs_ivfsq8* ix, const float* q, int64_t nq, int32_t k,
                     int32_t nprobe, float* out_dist, int64_t* out_ids, void* hip_stream);
VS_API int vs_ivfsq8_get_list_sizes(const vs_ivfsq8* ix, int64_t* sizes, void* hip_stream);
/* storage order: ids [ntotal], list of every entry [ntotal], codes [ntotal, d] bytes
 * (DEVICE, each may be NULL) */
VS_API int vs_ivfsq8_get_storage(const vs_ivfsq8* ix, int64_t* ids, int32_t* list_of,
                          uint8_t* codes, void* hip_stream);

/* ---- stage timing (used by benchmarks) ----------------------------------- */

enum {
  VS_STAGE_COARSE_DIST = 0,   /* query x centroid distance tiles                 */
  VS_STAGE_COARSE_SELECT = 1, /* top-nprobe selection                            */
  VS_STAGE_SCAN = 2,          /* fused LUT build + ADC scan + k-selection        */
  VS_STAGE_MERGE = 3,         /* merge across probe splits, id translation       */
  VS_STAGE_FLAT_DIST = 4,     /* flat search: query x database distance tiles    */
  VS_STAGE_FLAT_SELECT = 5,   /* flat search: k-selection                        */
  VS_STAGE_REFINE = 6,        /* vs_refine: exact distances of a shortlist + selection */
  VS_STAGE_SCAN_FIRST = 7,    /* list-major search: first probes query by query, pairs grouped by list */
  VS_NUM_STAGES = 8
};

/* on != 0: from now on vs_ivfpq_search, vs_flat_search and vs_refine bracket every kernel
 * launch of the stages above with a pair of HIP events recorded on the caller's
 * stream (the launches themselves are unchanged).  Off by default. */
VS_API int vs_profile_enable(int on);
/* Waits for all recorded events, adds up the elapsed milliseconds per stage
 * into stage_ms[VS_NUM_STAGES] (HOST pointer) and the number of kernel launches
 * per stage into launches[VS_NUM_STAGES] (HOST pointer), then forgets them. */
VS_API int vs_profile_read(double* stage_ms, int64_t* launches);

/* ---- run-time options and counters ----------------------------------------- */

/* "knn_path": how exact k-nearest-row problems (coarse quantizer, list
 *   assignment, flat search) are evaluated.  0 (default): matrix-core shortlist
 *   + exact re-rank where a kernel exists (d a multiple of 32 up to 2048, k <= 150),
 *   canon distance tiles otherwise; 1: canon tiles only; 2: same as 0.
 *   Both routes return identical results.
 * "knn_eps_scale": multiplies the error bound used to prove a shortlist
 *   sufficient (default 1; a negative value sends every row to the exact
 *   fallback -- for tests).
 * "list_major": whether vs_ivfpq_search scans a batch list by list instead of query by query
 *   (Sec. 4.3 "Compressed-domain search"; L2 indexes with residual tables of PQ8x8 on d = 32,
 *   PQ16x8 on d = 128 and PQ32x8 on d = 96): every list is then read from memory once per batch
 *   instead of once per query that probes it.  0 (default): where it pays -- at least 16 probes,
 *   at least 4096 queries and three (query, list) pairs per list, codes of 512 MB or more in
 *   lists of 1024 codes or more on average; 1:
 *   wherever the index has one of these shapes; -1: never.  Results are identical either way.
 * "list_major_first" (default 4, 1..64): how many of its nearest lists every query scans on its
 *   own first; the k-th best distance found there is the bound under which the list-major scan
 *   keeps a code.  "list_major_candidates" (default 1024, 64..65536): codes kept per query; a
 *   query that finds more is scanned again query by query (vs_search_stats counts them).
 * Options are process-wide. */
VS_API int vs_set_option(const char* name, double value);
/* counters[0] = rows evaluated through the matrix-core route, counters[1] = rows
 * among them that needed the exact fallback, since the previous call (HOST
 * pointer to 2 int64).  Synchronises the device. */
VS_API int vs_counters_read(int64_t* counters);

/* Bytes of device scratch that one exact k-nearest-rows problem takes inside the
 * library (Sec. 3.1: brute-force search; the same routine serves the coarse
 * quantizer of Sec. 5.1 and the list assignment of add): na rows against nb rows
 * of dimension d, k results per row, processed in pieces of at most `piece` rows
 * (piece <= 0: one piece).  b_prepared != 0: the nb rows are an index's centroids,
 * prepared once at creation.  Host arithmetic only -- no device call, usable
 * without a GPU -- so a caller can budget memory before a search or an add.
 * The figure covers every piece, also a shorter last one (which may be laid out
 * with more splits of the nb rows than a full piece).  Returns -1 on invalid
 * arguments (na < 0, nb < 0, d < 1, k < 1). */
VS_API int64_t vs_knn_workspace_bytes(int64_t na, int64_t nb, int32_t d, int32_t k, int64_t piece,
                                      int32_t b_prepared);

/* Message of the calling thread's most recent error ("" if none). */
VS_API const char* vs_last_error(void);

/* Library version string. */
VS_API const char* vs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* VS_H_ */
