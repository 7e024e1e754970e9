/*
 * libtrim: the filter-then-refine scan of TRIM (arXiv 2508.17828) for one AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer marked "device" is HIP device memory on the current device, owned
 * by the caller for the whole call and until the work enqueued on `stream` has finished.
 * Pointers marked "host" are ordinary host memory read during the call only.  The library
 * keeps no state between calls (but see trim_search_range_static), allocates no device memory
 * and never synchronises: all
 * work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the null stream).
 *
 * Every function returns 0 on success or a negative trim_status; nothing is enqueued when
 * a negative status is returned.  Checks are made on the host from the arguments alone;
 * device-resident structure (probe ids, list offsets) is clamped inside the kernels so
 * that no access leaves the arrays described here, whatever those arrays hold.
 *
 * Conventions (paper notation in brackets):
 *   n      base vectors [n], d dimensions [d], M subspaces [m], 256 centroids each [C]
 *   code   one byte per subspace: the landmark of x is its PQ reconstruction (Section 3.1)
 *   dlx    Gamma(l,x), the UNSQUARED distance of x to its landmark (Section 3.3 step 1)
 *   gamma  the relaxation parameter of Equation 3, gamma >= 0; 0 is the strict bound
 *   all returned distances are SQUARED Euclidean distances (Equation 3 bounds Gamma^2)
 *   ids    original id of the vector stored at a position; NULL means id = position
 *   order  results are ordered by (squared distance, id); ties go to the smaller id
 *
 * Arithmetic is binary32 with a fixed rounding order, so that survivor sets are
 * reproducible bit for bit:
 *   table entry / encode distance : acc = fma(x_t - c_t, x_t - c_t, acc), t ascending
 *   Gamma(l,q)^2                  : s = T[0][c_0] + T[1][c_1] + ... summed left to right
 *   bound (Equation 3)            : a = sqrt(s); e = a - b; g = fma((2*gamma)*a, b, e*e)
 *   exact distance                : 32 partial sums; coordinate group G (4 consecutive
 *                                   coordinates) is added, in order, to partial G mod 32 by
 *                                   fma; then p[l] += p[l+h] for h = 16, 8, 4, 2, 1
 */
#ifndef TRIM_H
#define TRIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum trim_status {
    TRIM_OK = 0,
    TRIM_INVALID_ARG = -1,       /* null pointer, negative size, gamma < 0 or NaN, ... */
    TRIM_UNSUPPORTED_SHAPE = -2, /* see trim_shape_supported */
    TRIM_WORKSPACE = -3,         /* workspace missing or smaller than trim_range_workspace_bytes */
    TRIM_HIP_ERROR = -4,         /* a HIP call failed; see trim_last_hip_error */
    TRIM_INTERNAL = -5           /* the library itself is unusable (a build defect found at launch) */
} trim_status;

/* Limits of this build. */
#define TRIM_MAX_K 1024       /* kNN result size */
#define TRIM_MAX_BATCH 4096   /* kNN batch size */
#define TRIM_MAX_NPROBE 4096  /* probed lists per query */
#define TRIM_MAX_QUERIES 4194296 /* queries per search call (a launch holds < 2^32 threads) */

/* The stored index of Section 3.3 (preprocessing): raw vectors, their landmark codes and
 * landmark distances, and the PQ centroids.  All arrays device, read-only. */
typedef struct trim_index_view {
    int64_t n;              /* 0 <= n < 2^31 */
    int32_t d;              /* d % 4 == 0 */
    int32_t M;              /* d % M == 0, M % 4 == 0 */
    const float *base;      /* [n][d] row-major, in scan (storage) order */
    const uint8_t *codes;   /* [n][M] row-major */
    const float *dlx;       /* [n] */
    const int32_t *ids;     /* [n] or NULL */
    const float *codebooks; /* [M][256][d/M] */
    const void *scan_head;  /* [n] records of 12 bytes or NULL: see trim_pack_scan_head */
    const void *codes_tiled; /* tiled copy of codes or NULL: see trim_pack_codes_tiled */
    int32_t code_bits;      /* 0 or 8: the layout above.  4: the 4-bit codes of the FastScan variant
                               (see trim_fs_encode): M subspaces of 16 centroids, M % 16 == 0,
                               codes [n][M/2], codebooks [M][16][d/M] */
} trim_index_view;

/* Which stored positions a query scans, and in what order: the lists probes[q][0],
 * probes[q][1], ... one after the other, positions ascending inside a list
 * (inverted-file candidates as in the paper's IVFPQ integration, Section 6.1).
 * A NULL trim_candidates* means every query scans positions 0..n-1. */
typedef struct trim_candidates {
    int32_t nlist;
    int32_t nprobe;              /* 1..TRIM_MAX_NPROBE */
    const int64_t *list_offsets; /* device [nlist+1], nondecreasing, within [0, n] */
    const int32_t *probes;       /* device [nq][nprobe]; ids outside [0,nlist) are skipped */
    int64_t max_candidates;      /* host value: upper bound on one query's candidate count
                                    (e.g. the sum of the nprobe longest lists); used to size
                                    masks; a query with more candidates is cut at this bound */
    const void *list_bounds;     /* device, trim_list_bounds_bytes(nlist, M) bytes, or NULL: see
                                    trim_pack_list_bounds.  With it trim_search_knn passes over
                                    lists, and stops table sums early, where the codes that
                                    occur in a list show that nothing in it can survive;
                                    results, masks and counters are the same with and without */
} trim_candidates;

/* Optional per-query counters (device, each [nq] or NULL): candidates scanned, and survivors
 * of the filter, i.e. the candidates whose exact distance the scan of Section 4.2 calls for.
 * Pruning ratio = 1 - n_exact/n_scanned.  (kNN computes the exact distance of a
 * few more candidates than it counts: those that passed the threshold in force when their
 * stretch of the scan began but not the lower one of their own batch.  They change neither
 * the results nor the survivor mask.) */
typedef struct trim_stats {
    int32_t *n_scanned;
    int32_t *n_exact;
    uint32_t *work;   /* device [nq][TRIM_WORK_COUNTERS] or NULL: see below */
} trim_stats;

/* Optional accounting of what a search actually touched, per query (measurement aid; a launch
 * that keeps it is a little slower).  n_scanned counts every candidate of the query as Section
 * 4.2's scan defines it; these counters say how the kernel disposed of them:
 *   [TRIM_WORK_FIRST_PASS] candidates whose first code bytes and landmark distance were read
 *   [TRIM_WORK_SKIPPED]    candidates passed over with their whole inverted list, never read
 *                          (list-level pruning; first_pass + skipped + the k seeds = n_scanned)
 *   [TRIM_WORK_CODE_BYTES] bytes of codes, scan-head records, landmark distances and list
 *                          summaries requested from memory
 *   [TRIM_WORK_LOOKUPS]    distance-table lookups issued
 *   [TRIM_WORK_ROWS]       raw vectors read for an exact distance (>= n_exact: see above)
 *   [TRIM_WORK_FULL_CODE]  candidates whose code was read beyond the first pass
 * The remaining entries are reserved (written as 0). */
#define TRIM_WORK_COUNTERS 8
#define TRIM_WORK_FIRST_PASS 0
#define TRIM_WORK_SKIPPED 1
#define TRIM_WORK_CODE_BYTES 2
#define TRIM_WORK_LOOKUPS 3
#define TRIM_WORK_ROWS 4
#define TRIM_WORK_FULL_CODE 5

/* 1 if (d, M) can be searched by this build, else 0.  Needs d % 4 == 0, d % M == 0,
 * M % 4 == 0, d/M <= 64, and room in the 160 KB of LDS for the kernel's working set. */
int trim_shape_supported(int32_t d, int32_t M);
/* The same for an index with 4-bit codes (code_bits = 4): needs d % 4 == 0, d % M == 0,
 * M % 16 == 0, d/M <= 64. */
int trim_fs_shape_supported(int32_t d, int32_t M);

/*
 * The index of the paper's FastScan-compatible variant (Section 6.1, parameter setting: 4-bit
 * codes with m = d/2 subspaces; evaluated in Section 6.2.2): every subspace has 16 centroids, so
 * a landmark code takes 4 bits per subspace and a query's distance table 16 entries per
 * subspace.  The method is unchanged (landmark = PQ reconstruction, Section 3.1; Equation 3; the
 * scan of Section 4.2); trim_search_knn, trim_search_range, trim_pack_scan_head,
 * trim_pack_codes_tiled and trim_pack_list_bounds take such an index when
 * trim_index_view.code_bits = 4.  The table keeps binary32 entries (Section 3.1 computes
 * Gamma(l,q) exactly from it), summed left to right over the M subspaces.  A row of 16 table
 * entries spans 16 banks of the on-chip memory, so lanes that look up different centroids
 * never collide, which the 256-entry rows of 8-bit codes cannot avoid.
 *
 * trim_fs_encode: codes_out [n][M/2] device, two codes per byte, subspace 2i in the low half of
 * byte i, subspace 2i+1 in the high half (nearest centroid, smallest index on ties);
 * dlx_out [n] = Gamma(l,x).  codebooks [M][16][d/M] device.  M even.
 * trim_fs_build_lut: lut_out [nq][M][16] device (may be passed to the searches as `lut`).
 * trim_fs_train_pq: Lloyd's k-means with 16 centroids per subspace and the fixed roundings of
 * trim_train_pq; init_rows [16] device; assign_ws [ns][M] bytes of work space (on return: the
 * last iteration's assignment, one byte per subspace).
 */
int trim_fs_encode(const float *base, int64_t n, int32_t d, const float *codebooks, int32_t M,
                   uint8_t *codes_out, float *dlx_out, void *stream);
int trim_fs_build_lut(const float *queries, int64_t nq, int32_t d, const float *codebooks, int32_t M,
                      float *lut_out, void *stream);
int trim_fs_train_pq(const float *train, int64_t ns, int32_t d, int32_t M, int32_t iters,
                     const int32_t *init_rows, float *codebooks_out, uint8_t *assign_ws, void *stream);

/*
 * Preprocessing step 1 of Section 3.3: codes_out[x][j] = index of the centroid of subspace j
 * nearest to x's j-th sub-vector (smallest index on ties); dlx_out[x] = Gamma(l,x), the
 * distance from x to the vector its code represents.
 * base [n][d] device, codebooks [M][256][d/M] device, codes_out [n][M] device,
 * dlx_out [n] device.
 */
int trim_encode(const float *base, int64_t n, int32_t d, const float *codebooks, int32_t M,
                uint8_t *codes_out, float *dlx_out, void *stream);

/*
 * Index construction: centroid training by Lloyd's k-means (PQ codebooks: Sections 2.2 and
 * 3.1, one k-means with 256 centroids per subspace, t iterations; coarse lists: Section 6.1).
 * Every rounding is fixed, so that the centroids are reproducible bit for bit: the initial
 * centroids are the rows train[init_rows[c]]; an iteration assigns every training row to its
 * nearest centroid by the index's own binary32 rule (trim_encode for a PQ subspace,
 * trim_ivf_probe with one probe for the coarse lists; smallest index on ties) and then
 * replaces every centroid by the float64 sum of its rows, added in ascending row order,
 * divided by their number and rounded once to binary32; a centroid without rows is kept.
 * All arrays device.  train [ns][d]; init_rows: row numbers into train ([256] for PQ, [nlist]
 * for the coarse lists; values outside [0, ns) are clamped).  The *_ws arrays are work space
 * whose contents on return are the last iteration's assignment (codes_ws [ns][M] with dlx_ws
 * [ns] for PQ, assign_ws [ns] for the coarse lists).  iters >= 0.
 */
int trim_train_pq(const float *train, int64_t ns, int32_t d, int32_t M, int32_t iters,
                  const int32_t *init_rows, float *codebooks_out, uint8_t *codes_ws, float *dlx_ws,
                  void *stream);
int trim_train_ivf(const float *train, int64_t ns, int32_t d, int32_t nlist, int32_t iters,
                   const int32_t *init_rows, float *centroids_out, int32_t *assign_ws, void *stream);

/*
 * Relaxation parameter from a confidence level (Section 3.2, the sampling route for queries
 * without a known distribution): by the section's lemma, p = P(gamma <= 1 - cos(theta)) with
 * theta the angle at x's landmark between x and the query.  For each sampled data vector
 * (position sample_rows[s] of the index) the value 1 - cos(theta) is computed against the Q
 * sampled queries; gamma_x = its m-th largest value, m = min(Q, max(1, ceil(p * Q))), so that
 * m of the Q sampled queries keep Equation 3 below the true squared distance; the global
 * gamma is the smallest gamma_x (end of Section 3.2).  A vector equal to its landmark, or a
 * query equal to the landmark, counts as cos = 0.
 * index needs base, codes, codebooks.  sample_rows [S] device (clamped to [0, n)),
 * sample_queries [Q][d] device, 1 <= Q <= 16384, 0 <= p <= 1; gamma_x_out [S] device or NULL;
 * gamma_out device, one float.  Arithmetic is binary32 (values agree with a float64
 * evaluation to about 1e-6).
 */
int trim_estimate_gamma(const trim_index_view *index, const int32_t *sample_rows, int32_t S,
                        const float *sample_queries, int32_t Q, float p, float *gamma_x_out,
                        float *gamma_out, void *stream);

/*
 * The same for queries with a known distribution, the standard normal (Section 3.2: the theorem
 * that gives Z^2 = A / (A + B + C) for Z = cos(theta), with A = (Q1 + h1)^2, B = (Q2 - h2)^2,
 * C the sum of the other d - 2 squared coordinates, h1 = (x - l).l / |x - l|,
 * h2 = sqrt(|l|^2 - h1^2); and the transform theorem, F_{1-Z}(y) = 1/2 -+ F_{Z^2}((1-y)^2) / 2,
 * minus for y <= 1, applied as printed).  The distribution of Z^2 is sampled: normals [Q][d]
 * (device) holds standard-normal variates supplied by the caller, of which only the first two
 * coordinates and the sum of the other d - 2 squares of every row are used.  For each sampled
 * data vector, gamma_x = the largest y on the grid y_i = 2 i / (grid - 1), 0 <= i < grid, with
 * F_{1-Z}(y_i) <= 1 - p (0 if there is none); the global gamma is the smallest gamma_x.
 * Arithmetic is binary64; results are written as binary32.  work: device, Q * 3 doubles,
 * 8-byte aligned.  1 <= Q <= 16384, 2 <= grid <= 2^24, d >= 3, 8-bit codes only.
 */
int trim_estimate_gamma_normal(const trim_index_view *index, const int32_t *sample_rows, int32_t S,
                               const float *normals, int32_t Q, float p, int32_t grid, double *work,
                               float *gamma_x_out, float *gamma_out, void *stream);

/*
 * Storage layout for the scan (the stored landmark codes and distances of Section 3.3,
 * preprocessing): head_out[x] = the 12 bytes {codes[x][0..7], dlx[x]}.  The kNN scan bounds
 * every candidate over its first 8 subspaces before it looks at the rest of the code, and
 * with this array it reads those 8 code bytes and the landmark distance as one contiguous
 * record instead of from two arrays.  It is a copy: results do not depend on whether
 * trim_index_view.scan_head is given, provided it was packed from the same codes and dlx
 * (it is not checked against them).  Needs M % 8 == 0 (else TRIM_UNSUPPORTED_SHAPE).
 * codes [n][M] device, dlx [n] device, head_out [n][12 bytes] device, 4-byte aligned.
 * Here and in trim_pack_codes_tiled M is the number of BYTES of a stored code: the number of
 * subspaces for 8-bit codes, half of it for 4-bit codes (the head then covers 16 subspaces).
 */
#define TRIM_SCAN_HEAD_BYTES 12
int trim_pack_scan_head(const uint8_t *codes, const float *dlx, int64_t n, int32_t M,
                        void *head_out, void *stream);

/*
 * Second storage layout of the landmark codes of Section 3.3 (preprocessing), for long codes:
 * the vectors are taken in blocks of 64, and tiled_out holds, block after block, piece 0 of
 * the block's 64 vectors, then piece 1, ... (piece p = code bytes 16p..16p+15; a block is
 * 64*M bytes; rows beyond n are zero).  Lanes that bound 64 consecutive vectors then read
 * one contiguous KB per piece instead of 64 strided rows, and no byte is fetched twice when
 * the subspaces are processed in several table phases.  It is a copy:
 * trim_index_view.codes stays mandatory, a search reads whichever of the two suits its
 * launch (range searches and kNN with k > 64 read the tiled copy when it is given; kNN
 * with k <= 64 always reads the row-major array), and results do not depend on it.  Worth
 * it for long codes (M >= 64).  Needs M % 16 == 0 (else TRIM_UNSUPPORTED_SHAPE).
 * codes [n][M] device; tiled_out device, 16-byte aligned, trim_codes_tiled_bytes(n, M) bytes.
 */
size_t trim_codes_tiled_bytes(int64_t n, int32_t M);
int trim_pack_codes_tiled(const uint8_t *codes, int64_t n, int32_t M, void *tiled_out,
                          void *stream);

/*
 * Query processing, operation 1 (Section 3.3; the distance table of Section 2.2):
 * lut_out[q][j][c] = squared distance from the j-th sub-vector of query q to centroid c of
 * subspace j.  queries [nq][d] device, lut_out [nq][M][256] device.
 * mfma = 0: direct differences on the vector ALU in the rounding order above (this is the
 * table the searches build internally).  mfma = 1: expanded form ||q||^2 - 2 q.c + ||c||^2
 * with the cross term on the matrix cores (d/M must be 4 or 8); agrees with mfma = 0 only
 * to rounding, so survivor sets computed from it may differ at exact ties.
 */
int trim_build_lut(const float *queries, int64_t nq, int32_t d, const float *codebooks,
                   int32_t M, float *lut_out, int32_t mfma, void *stream);

/*
 * Approximate kNN by the scan of Section 4.2 (problem statement: Section 2.1).
 * Per query: the result set R (size k) is first filled with the first k candidates, all with
 * exact distances; the remaining candidates are taken in batches; inside a batch the
 * threshold tau (k-th squared distance in R; +inf while |R| < k) is frozen; a candidate
 * survives iff g <= tau (Equation 3); survivors get exact distances and are merged into R.
 * Every batch holds `batch` candidates; batch = 1 is the paper's vector-at-a-time rule.
 *
 * queries [nq][d] device.  lut: device [nq][M][256] or NULL (tables are then built inside
 * the kernel from index->codebooks).  cand: host struct or NULL.  nq <= TRIM_MAX_QUERIES,
 * 1 <= k <= TRIM_MAX_K,
 * 1 <= batch <= TRIM_MAX_BATCH, gamma >= 0.
 * query_order: device [nq] or NULL; a permutation of 0..nq-1 giving the order in which
 * queries are handed to the GPU (see trim_query_order).  It changes scheduling only: every
 * query's results are written at its own row and do not depend on the order.  A query that
 * the array does not name is not searched and its output rows are left untouched; entries
 * outside [0, nq) are skipped.
 * out_ids [nq][k], out_d2 [nq][k] device: ascending by (d2, id); rows with fewer than k
 * candidates are padded with id -1, d2 +inf.
 * stats: host struct or NULL.  survivor_mask: device or NULL; if given it must hold
 * nq * mask_words 32-bit words, mask_words >= ceil(max candidates per query / 32); the call
 * overwrites it: bit (i % 32) of word [q][i / 32] is 1 iff the candidate with scan-order
 * number i had its exact distance computed.
 */
int trim_search_knn(const trim_index_view *index, const float *queries, int64_t nq,
                    const float *lut, const trim_candidates *cand, int32_t k, float gamma,
                    int32_t batch, const int32_t *query_order,
                    int32_t *out_ids, float *out_d2,
                    const trim_stats *stats, uint32_t *survivor_mask, int64_t mask_words,
                    void *stream);

/*
 * Approximate range search by the scan of Section 4.2 (problem statement: Section 2.1):
 * tau = radius^2 (squared once in binary32) for every candidate; a candidate survives iff
 * g <= tau; a survivor is a result iff its exact squared distance <= tau.
 *
 * Results are written in CSR form in scan order: out_offsets [nq+1] device (always
 * complete), out_ids / out_d2 [capacity] device.  *required (device int64) receives the
 * total number of results; if it exceeds `capacity`, only the entries whose global index
 * is below `capacity` are written (the caller checks *required after synchronising and
 * calls again with a larger buffer).
 * workspace: device, at least trim_range_workspace_bytes(...) bytes, 256-byte aligned;
 * contents on entry are ignored.  survivor_mask and query_order as in trim_search_knn (a query
 * that query_order does not name gets no results).
 */
int trim_search_range(const trim_index_view *index, const float *queries, int64_t nq,
                      const float *lut, const trim_candidates *cand, float radius, float gamma,
                      const int32_t *query_order, int64_t *out_offsets, int32_t *out_ids,
                      float *out_d2, int64_t capacity,
                      int64_t *required, const trim_stats *stats, uint32_t *survivor_mask,
                      int64_t mask_words, void *workspace, size_t workspace_bytes,
                      void *stream);

/*
 * trim_search_range for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same search with the same
 * results, but the workspace is a fixed area of TRIM_STATIC_SCRATCH_BYTES bytes of device memory
 * that belongs to the library (one copy per GPU, held from the library's first use on that GPU
 * until the process ends).  The call allocates nothing and frees nothing.  It returns
 * TRIM_WORKSPACE, with nothing enqueued, when trim_range_workspace_bytes(nq, max candidates)
 * exceeds TRIM_STATIC_SCRATCH_BYTES (about 4.2 bytes per (query, candidate) pair: 32 MiB hold
 * roughly 7.9 million pairs per call; split the query set to stay below).
 * Every call on a GPU uses that GPU's one area: two calls whose work overlaps in time on the same
 * GPU (different streams, or different host threads) race and give undefined results; calls
 * ordered on one stream are safe.  The area keeps the previous call's contents; the call itself
 * clears what it needs cleared.
 */
#define TRIM_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
int trim_search_range_static(const trim_index_view *index, const float *queries, int64_t nq,
                             const float *lut, const trim_candidates *cand, float radius, float gamma,
                             const int32_t *query_order, int64_t *out_offsets, int32_t *out_ids,
                             float *out_d2, int64_t capacity,
                             int64_t *required, const trim_stats *stats, uint32_t *survivor_mask,
                             int64_t mask_words, void *stream);
/* TRIM_STATIC_SCRATCH_BYTES of the loaded library. */
size_t trim_static_scratch_bytes(void);

/* Bytes of workspace trim_search_range needs for nq queries with at most max_candidates
 * candidates each (index->n when there is no candidate structure): about 4.2 bytes per
 * (query, candidate) pair -- a result bit and a slot for the result's exact distance. */
size_t trim_range_workspace_bytes(int64_t nq, int64_t max_candidates);

/*
 * Candidate generation for inverted-file search (Section 6.1: IVFPQ with C' coarse lists and
 * nprobe probed lists): probes_out[q][p] = id of the p-th nearest coarse centroid to query q
 * by exact squared distance (rounding order above), nearest first, ties to the smaller id.
 * queries [nq][d], centroids [nlist][d], probes_out [nq][nprobe] device; nprobe <= nlist,
 * nprobe <= TRIM_MAX_NPROBE.
 */
int trim_ivf_probe(const float *queries, int64_t nq, int32_t d, const float *centroids,
                   int32_t nlist, int32_t nprobe, int32_t *probes_out, void *stream);

/*
 * Scheduling aid for inverted-file search (the probed lists of Section 6.1): order_out [nq]
 * device = a permutation of the queries in which queries with the same first probed list are
 * adjacent, lists in ascending order (for nlist > 32768: ascending list id modulo 32768);
 * the order inside one list is unspecified.  Queries that scan the same lists then run
 * next to each other and share the GPU's caches.
 * probes [nq][nprobe] device as produced by trim_ivf_probe (nlist is the number of lists).
 */
int trim_query_order(const int32_t *probes, int64_t nq, int32_t nprobe, int32_t nlist,
                     int32_t *order_out, void *stream);

/*
 * Per-list summaries for list-level pruning in trim_search_knn (an exact shortcut, not part of
 * the paper's method; it tightens the lower bound of Section 3 with what the index knows about
 * a list).  For every inverted list and every subspace j the set of PQ codes that occur in
 * the list is recorded (up to 64; a larger set is marked as "any code"), and the largest
 * landmark distance of the list.  For a query with table T, every vector of the list has
 * T[j][code_j] >= min over the recorded codes c of T[j][c]; the sum of these minima over
 * the subspaces still to come bounds the rest of a running table sum from below, and their sum
 * over all subspaces, if it exceeds (max landmark distance + sqrt(tau))^2, shows that Equation 3
 * is above tau for the whole list at every gamma >= 0.
 * list_offsets [nlist+1] device; the index needs codes and dlx.  out: device,
 * trim_list_bounds_bytes(nlist, bytes of one stored code) bytes, 16-byte aligned (the bytes of a
 * code: index->M for 8-bit codes, index->M / 2 for 4-bit codes, where a "code" above is a code
 * byte, i.e. the pair of codes of two neighbouring subspaces).
 */
size_t trim_list_bounds_bytes(int32_t nlist, int32_t M);
int trim_pack_list_bounds(const trim_index_view *index, const int64_t *list_offsets, int32_t nlist,
                          void *out, void *stream);

/*
 * Measurement aids (no counterpart in the paper): the two machine ceilings the scan of
 * Section 4.2 is priced against.  Both launch `blocks` workgroups of 512 threads
 * (1 <= blocks <= TRIM_CEILING_MAX_BLOCKS) on `stream` and return without synchronising; the
 * caller times them.
 *
 * trim_ceiling_stream_read reads buf[0 .. bytes rounded down to 16) once (device, 16-byte
 * aligned, bytes >= 16) and writes one checksum word per workgroup to sink [blocks] (device):
 * the xor of these words is the xor of all 32-bit words read.  bytes / time = the
 * streaming-read rate of the memory the buffer lives in (HBM for a buffer much larger than
 * the caches).
 *
 * trim_ceiling_lds_gather, entry_floats = 1: every thread performs iters * 32 lookups
 * T[j][byte] in a [32][256] binary32 table held in on-chip memory, with the instruction
 * sequence of the scan's own table sums (one lookup and one addition per code byte), and
 * writes its sum to sink [blocks * 512] (device).  1 <= iters <= 2^20.
 * blocks * 512 * iters * 32 / time = lookups per second with nothing else going on.
 * entry_floats = 16: the same for 4-bit codes, a [64][16] table and 64 lookups per iteration
 * (blocks * 512 * iters * 64 lookups); rows of 16 entries never make two lanes collide, so this
 * is also the rate of conflict-free 4-byte reads of the on-chip memory.
 * entry_floats = 2 or 4: the table has 8 rows of 256 entries of that many binary32 values
 * (what a table shared by 2 or 4 queries would hold); every thread performs iters * 8 lookups
 * of a whole entry and adds its values up.  Other values: TRIM_INVALID_ARG.
 */
#define TRIM_CEILING_MAX_BLOCKS 65536
int trim_ceiling_stream_read(const void *buf, size_t bytes, int32_t blocks, uint32_t *sink,
                             void *stream);
int trim_ceiling_lds_gather(int32_t blocks, int32_t iters, int32_t entry_floats, uint32_t seed,
                            float *sink, void *stream);

/* Text for a trim_status. */
const char *trim_strerror(int status);
/* The hipError_t (as int) behind the calling thread's most recent TRIM_HIP_ERROR, else 0. */
int trim_last_hip_error(void);
/* Library version, "major.minor". */
const char *trim_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TRIM_H */
