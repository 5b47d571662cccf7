/*
 * ivf_gp.h — C ABI of the MI355X (gfx950) library for the batched query path
 * of the inverted index with grouping and pruning
 * ("Revisiting the Inverted Indices for Billion-Scale Approximate Nearest
 * Neighbors", Section 2 and Section 3.2).
 *
 * Conventions
 *   - Every array pointer is a DEVICE pointer unless its comment says "host".
 *   - The caller owns every buffer it passes.  The library owns the opaque
 *     index handle (its private copy of the index and its scratch memory).
 *   - Work is enqueued on the HIP stream passed as `void *hip_stream`
 *     (NULL = the default stream); calls return without waiting for it unless
 *     stated otherwise.
 *   - Return value 0 = success, negative = error (see IVF_E*).  Nothing throws
 *     across this boundary.  ivf_last_error() describes the failure
 *     (thread-local, host string).  Argument errors (IVF_EINVAL) are found
 *     before anything is launched: no output buffer has been written.  An
 *     IVF_ENOMEM / IVF_EHIP in the middle of a batch that is processed in
 *     several passes (see ivf_set_scratch_limit) leaves the outputs of the
 *     passes already enqueued written and the rest untouched.
 *   - Row-major everywhere.  D is a multiple of 4 and of M; M is 8 or 16.
 */
#ifndef IVF_GP_H
#define IVF_GP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IVF_OK      0
#define IVF_EINVAL -1   /* bad argument (null pointer, size or parameter out of range) */
#define IVF_ENOMEM -2   /* device or host allocation failed */
#define IVF_EHIP   -3   /* a HIP runtime call failed */

/* limits of this build */
#define IVF_MAX_K_RESULTS 1024   /* k of ivf_search */
#define IVF_MAX_D         1024
#define IVF_MAX_SCORES    32768  /* nprobe * L of a search: the scores of one query stay in LDS */
#define IVF_NOALLOC_SCRATCH_BYTES (64 << 20)   /* static scratch of ivf_search_noalloc, per GPU */

typedef struct ivf_index ivf_index; /* opaque */

/*
 * The trained and encoded index as flat arrays (host struct of device
 * pointers).  Regions are the Voronoi cells of `centroids` (Section 2,
 * IVFADC).  Region r has L subregions; subregion l is the Voronoi cell of the
 * subcentroid c_r + alpha_r (s_l - c_r), s_l = centroids[nbr[r][l]]
 * (Section 3.2, "The model", Eq. (2)).  Points are stored grouped: all points
 * of subregion (r, l) are contiguous, subregions in order of r*L + l, and
 * sub_offsets[r*L + l] is the position of the first one ("we store only the
 * subregion sizes", here as their prefix sums).  A point's record is the M
 * PQ bytes of its displacement from its subcentroid (Eq. (4)) plus one byte
 * indexing const_table, the 256-level quantisation of the query-independent
 * term of Eq. (6), 2<mu, r> + ||r||^2 (mu the subcentroid, r the decoded
 * displacement).
 */
typedef struct ivf_index_desc {
    int32_t D;                   /* dimensionality */
    int32_t M;                   /* PQ bytes per point */
    int32_t L;                   /* neighbours (= subregions) per region */
    int64_t K;                   /* regions */
    int64_t N;                   /* stored points, N < 2^32 */
    const float    *centroids;   /* [K][D] */
    const int32_t  *nbr;         /* [K][L] neighbour centroid ids, self excluded */
    const float    *alpha;       /* [K]    scaling factor per region */
    const float    *cs_dist2;    /* [K][L] ||c_r - s_l||^2 */
    const float    *pq_codebook; /* [M][256][D/M] */
    const float    *const_table; /* [256] ascending */
    const uint32_t *sub_offsets; /* [K*L + 1] */
    const uint8_t  *codes;       /* [N][M], grouped order */
    const uint8_t  *const_byte;  /* [N],    grouped order */
    const int32_t  *ids;         /* [N] point id of each grouped position, >= 0 */
    const float    *rotation;    /* [D][D] row-major orthogonal R in front of the PQ, or NULL (Section 4:
                                    OPQ-compressed displacements, one rotation shared by all regions): the
                                    codes quantise R (x - mu), the lookup tables are built from R q and the
                                    per-point term is 2<R mu, r> + ||r||^2 */
} ivf_index_desc;

/*
 * Build a search handle from a trained + encoded index.  The library makes its
 * own device copy of everything it needs (codes and constant bytes are
 * re-laid out into 16-byte aligned per-subregion blocks; the Eq. (7) constant
 * -alpha(1-alpha)||c - s_l||^2 is tabulated per (region, neighbour), as Section
 * 3.2 "Subregions pruning" prescribes), so the caller may free its arrays once
 * the call has returned; while the call runs both copies exist (there is no
 * borrowing mode: the record blocks are a different layout from the caller's
 * arrays).  Runs on `hip_stream` and waits for it.  codes / const_byte / ids /
 * sub_offsets may not be NULL here.
 * Dynamic range: the centroid table is packed for the matrix units with ONE
 * power-of-two scale for the whole table (queries: one per row), as a high and
 * a low fp16 half per component.  A component within 2^-17 of the table's
 * largest magnitude keeps 22 significant bits; a smaller one is held to an
 * absolute 2^-39 of that largest magnitude (its low half is an fp16
 * subnormal), and one below 2^-39 of it vanishes.  The resulting error of a
 * distance is at most 2^-38 * max|c_i| * ||q||_1, far inside the bound the
 * stage-1 distances are tested against, 16 u (||q||^2 + max||c||^2) with
 * u = 2^-24; but that bound is absolute in the largest centroid norm: rows
 * many orders of magnitude smaller than the largest row are resolved to that
 * absolute accuracy (as with any evaluation of ||q||^2 - 2<q,c> + ||c||^2 in
 * fp32), not to a relative accuracy of their own size.
 */
int ivf_load_index(const ivf_index_desc *desc, void *hip_stream, ivf_index **out);

/* Release the handle and all device memory it owns (waits for the device). */
void ivf_free_index(ivf_index *index);

/*
 * Upper bound in bytes for the scratch the handle may hold for the
 * query-by-centroid distance tile of stage 1 (default 8 GiB).  Larger batches
 * are processed in several tiles of queries.  The tile is allocated in whole
 * blocks of 256 query rows, so it can exceed the bound by up to 255 rows of
 * 4*K bytes.  Host call.
 */
int ivf_set_scratch_limit(ivf_index *index, int64_t bytes);

/*
 * Batched search (Section 3.2: "Distance estimation" and "Subregions
 * pruning").  For each of the nq queries [nq][D]:
 *   1. squared distances to all K centroids; the nprobe closest regions by
 *      (distance, centroid id)                               [Section 3.1]
 *   2. for each probed region and each of its L neighbours the distance to
 *      the subcentroid, (1-a)||q-c||^2 + a||q-s_l||^2 - a(1-a)||c-s_l||^2,
 *      reusing the stage-1 distances                          [Eq. (7)]
 *   3. keep the S = ceil(prune_frac * nprobe * L) closest subregions, chosen
 *      over all nprobe*L at once, by (distance, r*L + l)      [pruning]
 *   4. table T[m][j] = -2 <q_m, r^m_j>                        [Eq. (6)]
 *   5. for every point of every kept subregion the estimate
 *      score + sum_m T[m][code[m]] + const_table[byte]        [Eq. (6)]
 *   6. the k smallest by (estimate, id), ascending.
 * out_ids [nq][k] int32 and out_dists [nq][k] fp32 (estimated squared L2
 * distance); rows with fewer than k candidates are padded with id -1 and
 * +inf.  1 <= nprobe <= min(K, 4096), 0 < prune_frac <= 1,
 * 1 <= k <= IVF_MAX_K_RESULTS, nprobe*L <= IVF_MAX_SCORES and
 * nprobe*(L+3) <= 39424 (LDS of one workgroup).  All results are fp32 and
 * carry fp32 rounding errors; the inner products <q, c> of stage 1 are
 * formed on the fp16 matrix units from operands split into a high and a low
 * half (22 significant bits) and accumulated in fp32, which is as accurate
 * as an fp32 dot product.
 * Asynchronous on hip_stream; the handle's scratch is reused by every call,
 * so calls on one handle must not overlap.  The scratch grows on demand: a
 * call that needs more of it than any call before synchronizes the device,
 * frees and re-allocates; a call that fits what is there allocates nothing,
 * clears nothing with memset nodes and can be captured into a HIP graph (a
 * graph captured earlier holds the old addresses and is void once a later
 * call has grown the scratch).
 */
int ivf_search(ivf_index *index, const float *queries, int64_t nq, int nprobe, float prune_frac,
               int k, int32_t *out_ids, float *out_dists, void *hip_stream);

/*
 * ivf_search for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results, but every intermediate
 * buffer (distance tile, block minima, packed queries, probes, descriptors,
 * lookup tables, partial top-k lists) is carved out of one static device array
 * of IVF_NOALLOC_SCRATCH_BYTES that each GPU holds from the moment the library
 * is loaded until the process ends.  The call makes no hipMalloc / hipFree and
 * calls no allocating routine; the whole batch is one pass, and a batch whose
 * buffers do not fit (roughly nq * K * 4.1 bytes + nq * 40 KB: 15 queries at
 * K = 2^20, 230 at K = 65 536) is rejected with IVF_EINVAL before anything is
 * launched.  Nothing in the array has to start at zero.  All calls on one GPU
 * share that GPU's array, whatever the handle or stream: calls that overlap
 * on one GPU race; order them on one stream or with events.
 */
int ivf_search_noalloc(ivf_index *index, const float *queries, int64_t nq, int nprobe, float prune_frac,
                       int k, int32_t *out_ids, float *out_dists, void *hip_stream);

/*
 * ivf_search that also exports the intermediate results of stages 1, 3 and 5
 * (any of the four pointers may be NULL):
 *   probe_id  [nq][nprobe] int32, probe_d [nq][nprobe] fp32 — stage 1, in
 *             ascending centroid id
 *   kept_sub  [nq][S] int64 subregion ids r*L + l — stage 3, ascending
 *   n_scanned [nq] int64 — number of point records read in stage 5
 */
int ivf_search_stages(ivf_index *index, const float *queries, int64_t nq, int nprobe,
                      float prune_frac, int k, int32_t *out_ids, float *out_dists,
                      int32_t *probe_id, float *probe_d, int64_t *kept_sub, int64_t *n_scanned,
                      void *hip_stream);

/*
 * Search with a candidate budget (Section 4 evaluates the system at a given
 * candidate-list length R, e.g. 30 000): stages 1-3 as in ivf_search, then the
 * kept subregions are visited in ascending order of their Eq. (7) distance,
 * ties by subregion id, and the traversal stops as soon as the points
 * collected so far number max_candidates or more; the subregion with which
 * that number is reached is scanned whole, empty subregions on the way count
 * as visited.  Stages 4-6 then run over the visited subregions only.
 * max_candidates >= 1; a budget larger than what the kept subregions hold
 * gives ivf_search's result.  Optional outputs (any may be NULL):
 *   kept_sub  [nq][S] int64  the kept subregion ids, ascending (stage 3)
 *   visited   [nq][S] uint8  1 where kept_sub[q][i] was visited, else 0
 *   n_scanned [nq]    int64  point records read (the candidate-list length)
 * Other arguments, limits, stream and scratch behaviour as for ivf_search.
 */
int ivf_search_budget(ivf_index *index, const float *queries, int64_t nq, int nprobe, float prune_frac,
                      int64_t max_candidates, int k, int32_t *out_ids, float *out_dists,
                      int64_t *kept_sub, uint8_t *visited, int64_t *n_scanned, void *hip_stream);

/* S of stage 3 for the given parameters (host call, no device work). */
int64_t ivf_num_kept(int nprobe, int L, float prune_frac);

/*
 * Stage 1 alone (exhaustive assignment, Section 3.1): the P nearest of the K
 * centroids [K][D] for each of the nq vectors x [nq][D], by (distance, id),
 * written in ascending centroid id: out_id [nq][P], out_d [nq][P] squared
 * distances.  Used for query assignment, for assigning points to regions
 * (P = 1) and for the neighbour table NN_L (Eq. (2)).  Allocates and frees its
 * own scratch (waits for the stream).
 * P = 1 (also inside ivf_encode and ivf_kmeans) runs in two passes: a
 * reduced-precision product (the fp16 leading halves of the operands, a third
 * of the matrix work) with a proven error bound lists for every row the
 * centroids that may be its nearest, and exact fp32 distances of the listed
 * pairs decide, ties to the smaller id; a chunk of rows whose list overflows
 * is redone by the one-pass full-precision kernel.  The result is the exact
 * nearest centroid either way; the two ways round their distances
 * differently (differences squared and summed, against norms minus twice the
 * inner product), so a row whose two nearest centroids are closer to each
 * other than fp32 rounding resolves may get either of them.  Which way a chunk
 * goes depends on the data alone as long as its list is far from full, which
 * is the case unless most rows have dozens of centroids within 2^-8 of their
 * nearest distance.
 */
int ivf_coarse_topk(const float *centroids, int64_t K, int D, const float *x, int64_t nq, int P,
                    int32_t *out_id, float *out_d, void *hip_stream);

/*
 * How the chunks (up to 2^20 rows each) of all nearest-centroid assignments of
 * this process were decided so far (out: two values, host memory): out[0] by the shortlist and the exact
 * distances of the listed pairs, out[1] by the one-pass full-precision kernel
 * (list overflow, or the shortlist switched off with the environment variable
 * IVF_GP_EXACT_ASSIGN=1, which exists for measurements).  Host call.
 */
void ivf_assign_stats(int64_t *out);

/*
 * Index-time encoding of n points x [n][D] (Section 3.2): region = nearest
 * centroid (or, if `region_in` is given, that region is taken as is —
 * approximate / externally computed assignment, Section 3.1), subregion by
 * Eq. (3), displacement from the subcentroid by Eq. (4), PQ code of the
 * displacement (Section 2), the per-point term t = 2<mu, r> + ||r||^2 of
 * Eq. (6) and its nearest entry in const_table (lower index on ties).
 * Only the trained fields of `trained` are read (centroids, nbr, alpha,
 * cs_dist2, pq_codebook, const_table, rotation).  const_table may be NULL, then
 * out_const_byte is not written; pq_codebook may be NULL too (index trained up
 * to alpha only), then only region, subregion and displacement are produced.
 * Outputs: out_region [n] int32, out_sub [n] int32, out_codes [n][M],
 * out_const_byte [n], out_const_t [n] fp32 (may be NULL), out_residual [n][D]
 * fp32 displacement x - mu (may be NULL).  Waits for the stream.
 */
int ivf_encode(const ivf_index_desc *trained, const float *x, int64_t n, const int32_t *region_in,
               int32_t *out_region, int32_t *out_sub, uint8_t *out_codes, uint8_t *out_const_byte,
               float *out_const_t, float *out_residual, void *hip_stream);

/*
 * out [n][D] = rows of x [n][D] multiplied by the D x D matrix `rotation`
 * (row-major): out[i] = R x[i].  The rotation of Section 4 (OPQ) applied to
 * training displacements before ivf_pq_train; ivf_search and ivf_encode apply
 * the index's own rotation themselves.  x and out may be the same array.  Waits for the stream.
 */
int ivf_rotate(const float *x, int64_t n, int D, const float *rotation, float *out, void *hip_stream);

/*
 * ---- Index construction on the device (Section 3.2 "The model" and "Learning
 * the scaling factor"; Section 2 for the PQ codebooks).  Each routine waits
 * for the stream before it returns, allocates and frees its own scratch, and
 * is deterministic: no floating-point atomics, every sum is taken in an order
 * fixed by the data layout, so the same inputs give the same bits.
 */

/*
 * Lloyd's k-means for the region codebook (Section 2, IVFADC; Section 3.1 for
 * codebooks of up to 2^20 centroids): centroids start as the rows
 * init_idx[0..K) (device, int64) of x [n][D]; each of the `iters` rounds
 * assigns every row to its nearest centroid by (distance, id) (the fused
 * stage-1 kernel) and replaces every non-empty cluster's centroid by the mean
 * of its rows, accumulated in fp64 and rounded to fp32; an empty cluster
 * keeps its centroid.  centroids [K][D] (16-byte aligned) receives the result;
 * objective (device, [iters] fp64, may be NULL) the sum of squared distances
 * of each round's assignment, measured before that round's update.
 */
int ivf_kmeans(const float *x, int64_t n, int D, int64_t K, int iters, const int64_t *init_idx,
               float *centroids, double *objective, void *hip_stream);

/*
 * The update step of k-means alone (Section 2): centroids[j] = mean of the rows
 * of x [n][D] with assign[i] == j (fp64 sums in a fixed order, rounded to
 * fp32); a cluster without rows keeps the value centroids[j] holds on entry.
 * Used where the assignment is given (approximate or external assignment,
 * Section 3.1).
 */
int ivf_cluster_means(const float *x, int64_t n, int D, const int32_t *assign, int64_t K,
                      float *centroids, void *hip_stream);

/*
 * Neighbour table NN_L (Eq. (2)): for every centroid its L nearest among the
 * other centroids, ordered by (distance, id): nbr [K][L] int32 and
 * cs_dist2 [K][L] = ||c - s_l||^2.  1 <= L < K, L <= 4095.
 */
int ivf_neighbours(const float *centroids, int64_t K, int D, int L, int32_t *nbr, float *cs_dist2,
                   void *hip_stream);

/*
 * Scaling factor per region (Section 3.2, Eqs. (8)-(12)): for each of the n
 * training points x [n][D] with region[n], the neighbour s_l whose line through
 * c leaves the smallest residual with the coefficient clamped to [0,1]
 * (Eqs. (10)-(11), lowest l on ties); then alpha_r = sum (x-c)^T(s_l-c) /
 * sum ||s_l-c||^2 over the region's points (Eq. (12)), clamped to [0,1].  A
 * region without training points, or whose denominator is 0, gets the ratio
 * of the two sums taken over all regions.  All sums in fp64.  alpha [K].
 */
int ivf_learn_alpha(const float *centroids, int64_t K, int D, const int32_t *nbr, int L,
                    const float *x, int64_t n, const int32_t *region, float *alpha, void *hip_stream);

/*
 * PQ codebooks (Section 2): one 256-codeword k-means per block of D/M
 * dimensions of the displacements E [n][D] (the out_residual of ivf_encode).
 * Codeword j of every block starts as that block of row init_idx[j] (device,
 * int64, 256 entries); `iters` Lloyd rounds as in ivf_kmeans (nearest codeword
 * by (distance, index), means in fp64, empty codewords kept).  codebook
 * [M][256][D/M].  D/M must be 4, 6, 8, 12 or 16 and n >= 256.
 */
int ivf_pq_train(const float *E, int64_t n, int D, int M, int iters, const int64_t *init_idx,
                 float *codebook, void *hip_stream);

/*
 * The 256-level scalar quantiser of the per-point term of Eq. (6): table
 * [256] = 1-D Lloyd on the n values t (the out_const_t of ivf_encode), started
 * at the (j + 1/2)/256 quantiles, `iters` rounds (nearest level in fp64, lower
 * index on ties; a level without values keeps its entry), sorted ascending
 * after every round and rounded to fp32.
 */
int ivf_lloyd_1d(const float *t, int64_t n, int iters, float *table, void *hip_stream);

/*
 * Grouped order (Section 3.2: the points of a region are stored by subregion):
 * a stable counting sort of n items by bucket[i] in [0, nbuckets), here
 * bucket = region * L + subregion.  perm [n] lists the item indices bucket by
 * bucket, ascending inside a bucket (so position order is (region, subregion,
 * id) order); offsets [nbuckets + 1] uint32 are the bucket boundaries in perm.
 * Also used with bucket = cluster to list the members of k-means clusters.
 */
int ivf_group(const int32_t *bucket, int64_t n, int64_t nbuckets, int32_t *perm, uint32_t *offsets,
              void *hip_stream);

/* bucket[i] = region[i] * L + sub[i], the subregion id points are grouped by.  Asynchronous. */
int ivf_bucket_ids(const int32_t *region, const int32_t *sub, int64_t n, int L, int32_t *bucket,
                   void *hip_stream);

/*
 * dst row j = src row perm[j] for n rows of row_bytes bytes (codes, constant
 * bytes or ids into grouped order).  src and dst must not overlap.
 * Asynchronous on hip_stream.
 */
int ivf_gather_rows(const void *src, int64_t row_bytes, const int32_t *perm, int64_t n, void *dst,
                    void *hip_stream);

/*
 * Per-stage device timing of ivf_search / ivf_search_stages on a handle.  While
 * enabled, every pass over a tile of queries records HIP events on the caller's
 * stream around its six kernel groups, in launch order:
 *   0 query packing + coarse distance GEMM   1 nprobe selection   2 Eq. (7) scoring fused with
 *   the pruning select   3 lookup tables   4 ADC scan   5 final k-select
 * ivf_profile_read waits for the device, writes the summed milliseconds per
 * group to stage_ms[IVF_N_STAGES] (host) and the number of passes to *launches
 * (host), and resets the counters.
 */
#define IVF_N_STAGES 6
int ivf_profile_enable(ivf_index *index, int on);
int ivf_profile_read(ivf_index *index, double *stage_ms, int64_t *launches);

/*
 * Plain device-to-device streaming copy by a grid-stride kernel of 128-bit
 * loads and stores (nbytes a multiple of 16, both pointers 16-byte aligned).
 * It reads and writes exactly nbytes: the reference against which hardware
 * HBM counters and the scan's bandwidth are calibrated.  Asynchronous.
 */
int ivf_copy_bytes(void *dst, const void *src, int64_t nbytes, void *hip_stream);

/* Message of the last error on this host thread ("" if none). */
const char *ivf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IVF_GP_H */
