/*
 * CPU oracle for the grouped / pruned inverted-index query path
 * ("Revisiting the Inverted Indices for Billion-Scale Approximate Nearest
 * Neighbors", Section 2 and Section 3.2).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, definition-by-definition
 * implementation used only to check the HIP library and as a reported CPU
 * baseline.  It shares no code with the HIP path and the product never calls
 * it.  All arithmetic is fp64 on the fp32 / uint8 / int32 arrays of the
 * trained index; every selection is a full sort with an explicit
 * (value, index) tie-break.  Loops over independent items (queries, points)
 * are OpenMP-parallel; nothing else is blocked, fused or reordered.
 *
 * Pins (tests marked "not gpu"): see tests/test_oracle_*.py.  The recall and
 * timing figures printed in the paper's Tables 2-4 need its datasets and
 * trained parameters and are "parity unpinned".
 *
 * Notation follows the paper: q query, c region centroid, s_l its l-th
 * neighbouring centroid, alpha the per-region scaling factor,
 * mu_l = c + alpha (s_l - c) the subcentroid, r_m PQ codewords, M code bytes.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ helpers */

static double sq_dist(const float *a, const float *b, int d)
{
    double s = 0.0;
    for (int i = 0; i < d; ++i) {
        double t = (double)a[i] - (double)b[i];
        s += t * t;
    }
    return s;
}

typedef struct {
    double v;    /* value */
    int64_t t;   /* tie-break key */
    int64_t pos; /* position in the input */
} val_rec;

static int cmp_val_rec(const void *pa, const void *pb)
{
    const val_rec *a = (const val_rec *)pa, *b = (const val_rec *)pb;
    if (a->v < b->v) return -1;
    if (a->v > b->v) return 1;
    if (a->t < b->t) return -1;
    if (a->t > b->t) return 1;
    return 0;
}

/* The nsel smallest of v[0..n) ordered by (value, tie) ascending, by a full
 * sort.  tie[] may be NULL (then the position is the tie-break).  Writes the
 * chosen positions and their values, best first. */
void orc_smallest(const double *v, const int64_t *tie, int64_t n, int64_t nsel,
                  int64_t *out_pos, double *out_val)
{
    val_rec *r = (val_rec *)malloc((size_t)(n > 0 ? n : 1) * sizeof(val_rec));
    for (int64_t i = 0; i < n; ++i) {
        r[i].v = v[i];
        r[i].t = tie ? tie[i] : i;
        r[i].pos = i;
    }
    qsort(r, (size_t)n, sizeof(val_rec), cmp_val_rec);
    for (int64_t j = 0; j < nsel && j < n; ++j) {
        out_pos[j] = r[j].pos;
        out_val[j] = r[j].v;
    }
    free(r);
}

/* ------------------------------------------- stage 1: coarse assignment ---- */

/* Squared distances from every query to every region centroid:
 * out[q*K + j] = ||q - c_j||^2  (Section 2, IVFADC: Voronoi cells of C). */
void orc_coarse_dist(const float *Q, int64_t nq, const float *C, int64_t K, int D, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t j = 0; j < K; ++j)
            out[q * K + j] = sq_dist(Q + q * D, C + j * D, D);
}

/* The P closest regions of each query, ordered by (distance, centroid id)
 * (exhaustive query assignment, Section 3.1). */
void orc_probe(const float *Q, int64_t nq, const float *C, int64_t K, int D, int64_t P,
               int32_t *probe_id, double *probe_d)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        double *row = (double *)malloc((size_t)K * sizeof(double));
        int64_t *pos = (int64_t *)malloc((size_t)P * sizeof(int64_t));
        for (int64_t j = 0; j < K; ++j) row[j] = sq_dist(Q + q * D, C + j * D, D);
        orc_smallest(row, NULL, K, P, pos, probe_d + q * P);
        for (int64_t p = 0; p < P; ++p) probe_id[q * P + p] = (int32_t)pos[p];
        free(row);
        free(pos);
    }
}

/* ------------------------------------ stage 2: subcentroid distances ------- */

/* Eq. (7): for each probed region r (centroid c, scaling alpha_r) and each of
 * its L neighbours s_l,
 *   score = (1 - alpha) ||q - c||^2 + alpha ||q - s_l||^2 - alpha (1 - alpha) ||c - s_l||^2.
 * The last term is the query-independent constant of Eq. (7), obtained by
 * expanding ||(1-alpha)(q-c) + alpha(q-s)||^2; the index stores ||c - s_l||^2
 * in cs_dist2.  Both query-to-centroid distances are recomputed here from the
 * vectors.  scores is [nq][P][L]. */
void orc_scores(const float *Q, int64_t nq, const float *C, int D, const int32_t *nbr, int L,
                const float *alpha, const float *cs_dist2, const int32_t *probe_id, int64_t P,
                double *scores)
{
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q)
        for (int64_t p = 0; p < P; ++p) {
            int64_t r = probe_id[q * P + p];
            double a = (double)alpha[r];
            double d_c = sq_dist(Q + q * D, C + r * D, D);
            for (int l = 0; l < L; ++l) {
                int64_t s = nbr[r * L + l];
                double d_s = sq_dist(Q + q * D, C + s * D, D);
                scores[(q * P + p) * L + l] =
                    (1.0 - a) * d_c + a * d_s - a * (1.0 - a) * (double)cs_dist2[r * L + l];
            }
        }
}

/* ------------------------------------------------- stage 3: pruning -------- */

/* Number of subregions kept: ceil(tau * P * L), clamped to [1, P*L]. */
int64_t orc_num_kept(double prune_frac, int64_t P, int L)
{
    int64_t total = P * (int64_t)L;
    int64_t S = (int64_t)ceil(prune_frac * (double)P * (double)L);
    if (S < 1) S = 1;
    if (S > total) S = total;
    return S;
}

/* Subregion pruning (Section 3.2): of the P*L scored subregions of a query
 * keep the S closest, chosen over all P*L at once, ordered by
 * (score, subregion id) with subregion id = r*L + l.  kept_sub / kept_score
 * are [nq][S]. */
void orc_prune(const double *scores, int64_t nq, int64_t P, int L, const int32_t *probe_id,
               int64_t S, int64_t *kept_sub, double *kept_score)
{
    int64_t total = P * (int64_t)L;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q) {
        int64_t *sid = (int64_t *)malloc((size_t)total * sizeof(int64_t));
        int64_t *pos = (int64_t *)malloc((size_t)S * sizeof(int64_t));
        for (int64_t p = 0; p < P; ++p)
            for (int l = 0; l < L; ++l)
                sid[p * L + l] = (int64_t)probe_id[q * P + p] * L + l;
        orc_smallest(scores + q * total, sid, total, S, pos, kept_score + q * S);
        for (int64_t j = 0; j < S; ++j) kept_sub[q * S + j] = sid[pos[j]];
        free(sid);
        free(pos);
    }
}

/* ------------------------------------------- stage 4: lookup tables -------- */

/* Global rotation in front of the product quantiser (Section 4: the
 * displacements are OPQ-compressed, one rotation shared by all regions):
 * out[i] = R x[i] for a D x D matrix R, row-major, out[i][a] = sum_b R[a][b] x[i][b].
 * With an orthogonal R and y = R e quantised to r, the point is mu + R^T r and
 *   ||q - mu - R^T r||^2 = ||q - mu||^2 - 2<R q, r> + (2<R mu, r> + ||r||^2):
 * the lookup table is built from the rotated query and the per-point constant
 * from the rotated subcentroid. */
void orc_rotate(const double *X, int64_t n, int D, const float *R, double *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int a = 0; a < D; ++a) {
            double s = 0.0;
            for (int b = 0; b < D; ++b) s += (double)R[(int64_t)a * D + b] * X[i * D + b];
            out[i * D + a] = s;
        }
}

/* Per-query table of the inner-product term of Eq. (6):
 * T[q][m][j] = -2 <q_m, r^m_j>, with q_m the m-th block of D/M consecutive
 * dimensions and codebook laid out [M][256][D/M].  With a rotation (may be
 * NULL) q is replaced by R q. */
void orc_lut(const float *Q, int64_t nq, int D, int M, const float *codebook, const float *rotation,
             double *T)
{
    int ds = D / M;
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q) {
        double *qr = (double *)malloc((size_t)D * sizeof(double));
        for (int a = 0; a < D; ++a) qr[a] = (double)Q[q * D + a];
        if (rotation) {
            double *qin = (double *)malloc((size_t)D * sizeof(double));
            memcpy(qin, qr, (size_t)D * sizeof(double));
            orc_rotate(qin, 1, D, rotation, qr);
            free(qin);
        }
        for (int m = 0; m < M; ++m)
            for (int j = 0; j < 256; ++j) {
                double s = 0.0;
                for (int i = 0; i < ds; ++i)
                    s += qr[m * ds + i] * (double)codebook[((int64_t)m * 256 + j) * ds + i];
                T[(q * M + m) * 256 + j] = -2.0 * s;
            }
        free(qr);
    }
}

/* --------------------------------------------- stage 5: ADC scan ----------- */

/* Candidate budget (Section 4 evaluates candidate lists of a given length R).
 * The kept subregions of a query are visited in ascending order of their
 * Eq. (7) distance, ties by subregion id, and the traversal stops as soon as
 * the points collected so far number R or more: a subregion is visited iff
 * the subregions before it in that order hold fewer than R points together
 * (the one that crosses R is taken whole; empty ones on the way count as
 * visited).  kept_sub / kept_score are [nq][S] in any order; visit[q][j] = 1
 * if kept_sub[q][j] is visited, else 0. */
void orc_budget_visit(const int64_t *kept_sub, const double *kept_score, int64_t nq, int64_t S,
                      const uint32_t *sub_offsets, int64_t R, uint8_t *visit)
{
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < nq; ++q) {
        int64_t *order = (int64_t *)malloc((size_t)S * sizeof(int64_t));
        double *val = (double *)malloc((size_t)S * sizeof(double));
        orc_smallest(kept_score + q * S, kept_sub + q * S, S, S, order, val);
        int64_t collected = 0;
        for (int64_t j = 0; j < S; ++j) {
            int64_t at = order[j], b = kept_sub[q * S + at];
            visit[q * S + at] = collected < R ? 1 : 0;
            if (collected < R) collected += (int64_t)sub_offsets[b + 1] - (int64_t)sub_offsets[b];
        }
        free(order);
        free(val);
    }
}

/* Number of stored points in the kept (and, if visit is given, visited)
 * subregions of each query. */
void orc_scan_count(const int64_t *kept_sub, const uint8_t *visit, int64_t nq, int64_t S,
                    const uint32_t *sub_offsets, int64_t *count)
{
    for (int64_t q = 0; q < nq; ++q) {
        int64_t c = 0;
        for (int64_t j = 0; j < S; ++j) {
            if (visit && !visit[q * S + j]) continue;
            int64_t b = kept_sub[q * S + j];
            c += (int64_t)sub_offsets[b + 1] - (int64_t)sub_offsets[b];
        }
        count[q] = c;
    }
}

/* Eq. (6): estimated distance of every stored point of every kept subregion,
 *   dist = score(subregion) + sum_m T[m][code[m]] + const,
 * where const is const_table[const_byte[i]], or const_exact[i] when that
 * array is given (the unquantised per-point term, used to pin the identity).
 * Candidates of query q are written from cand_start[q] on, in the order of
 * kept_sub and then of position.  With visit given, subregions whose flag is
 * 0 are skipped (candidate budget). */
void orc_scan(const int64_t *kept_sub, const double *kept_score, const uint8_t *visit, int64_t nq, int64_t S,
              const uint32_t *sub_offsets, const uint8_t *codes, int M, const uint8_t *const_byte,
              const float *const_table, const double *const_exact, const double *T,
              const int64_t *cand_start, int64_t *cand_pos, double *cand_dist)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        int64_t w = cand_start[q];
        for (int64_t j = 0; j < S; ++j) {
            if (visit && !visit[q * S + j]) continue;
            int64_t b = kept_sub[q * S + j];
            for (int64_t i = sub_offsets[b]; i < (int64_t)sub_offsets[b + 1]; ++i) {
                double d = kept_score[q * S + j];
                for (int m = 0; m < M; ++m) d += T[(q * M + m) * 256 + codes[i * M + m]];
                d += const_exact ? const_exact[i] : (double)const_table[const_byte[i]];
                cand_pos[w] = i;
                cand_dist[w] = d;
                ++w;
            }
        }
    }
}

/* --------------------------------------------- stage 6: final top-k -------- */

/* The k best candidates by (distance, point id); rows with fewer than k
 * candidates are padded with id -1 and distance +inf. */
void orc_select(const int64_t *cand_pos, const double *cand_dist, int64_t n, const int32_t *ids,
                int64_t k, int32_t *out_ids, double *out_dists)
{
    int64_t *tie = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    int64_t *pos = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    for (int64_t i = 0; i < n; ++i) tie[i] = ids[cand_pos[i]];
    int64_t got = n < k ? n : k;
    orc_smallest(cand_dist, tie, n, got, pos, out_dists);
    for (int64_t j = 0; j < got; ++j) out_ids[j] = (int32_t)tie[pos[j]];
    for (int64_t j = got; j < k; ++j) {
        out_ids[j] = -1;
        out_dists[j] = INFINITY;
    }
    free(tie);
    free(pos);
}

/* ------------------------------------------------ whole query path --------- */

typedef struct {
    int32_t D, M, L;
    int64_t K, N;
    const float *centroids;    /* K*D */
    const int32_t *nbr;        /* K*L */
    const float *alpha;        /* K */
    const float *cs_dist2;     /* K*L */
    const float *pq_codebook;  /* M*256*(D/M) */
    const float *const_table;  /* 256 */
    const uint32_t *sub_offsets; /* K*L+1 */
    const uint8_t *codes;      /* N*M */
    const uint8_t *const_byte; /* N */
    const int32_t *ids;        /* N */
    const float *rotation;     /* D*D or NULL: rotation in front of the PQ (Section 4, OPQ) */
} orc_index;

/* Stages 1-6 in order for every query.  n_scanned (may be NULL) receives the
 * number of codes scanned per query. */
void orc_search(const orc_index *ix, const float *Q, int64_t nq, int64_t P, double prune_frac,
                int64_t k, int32_t *out_ids, double *out_dists, int64_t *n_scanned)
{
    int D = ix->D, M = ix->M, L = ix->L;
    int64_t S = orc_num_kept(prune_frac, P, L);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t q = 0; q < nq; ++q) {
        const float *qv = Q + q * D;
        int32_t *probe_id = (int32_t *)malloc((size_t)P * sizeof(int32_t));
        double *probe_d = (double *)malloc((size_t)P * sizeof(double));
        double *scores = (double *)malloc((size_t)(P * L) * sizeof(double));
        int64_t *kept_sub = (int64_t *)malloc((size_t)S * sizeof(int64_t));
        double *kept_score = (double *)malloc((size_t)S * sizeof(double));
        double *T = (double *)malloc((size_t)M * 256 * sizeof(double));
        int64_t count = 0, zero = 0;
        orc_probe(qv, 1, ix->centroids, ix->K, D, P, probe_id, probe_d);
        orc_scores(qv, 1, ix->centroids, D, ix->nbr, L, ix->alpha, ix->cs_dist2, probe_id, P, scores);
        orc_prune(scores, 1, P, L, probe_id, S, kept_sub, kept_score);
        orc_lut(qv, 1, D, M, ix->pq_codebook, ix->rotation, T);
        orc_scan_count(kept_sub, NULL, 1, S, ix->sub_offsets, &count);
        int64_t *cand_pos = (int64_t *)malloc((size_t)(count > 0 ? count : 1) * sizeof(int64_t));
        double *cand_dist = (double *)malloc((size_t)(count > 0 ? count : 1) * sizeof(double));
        orc_scan(kept_sub, kept_score, NULL, 1, S, ix->sub_offsets, ix->codes, M, ix->const_byte,
                 ix->const_table, NULL, T, &zero, cand_pos, cand_dist);
        orc_select(cand_pos, cand_dist, count, ix->ids, k, out_ids + q * k, out_dists + q * k);
        if (n_scanned) n_scanned[q] = count;
        free(probe_id); free(probe_d); free(scores); free(kept_sub); free(kept_score);
        free(T); free(cand_pos); free(cand_dist);
    }
}

/* ================================================= index construction ===== */

/* Nearest centroid of each point by (distance, centroid id). */
void orc_assign(const float *X, int64_t n, const float *C, int64_t K, int D, int32_t *region,
                double *dist)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double best = INFINITY;
        int64_t bj = 0;
        for (int64_t j = 0; j < K; ++j) {
            double d = sq_dist(X + i * D, C + j * D, D);
            if (d < best) { best = d; bj = j; }
        }
        region[i] = (int32_t)bj;
        if (dist) dist[i] = best;
    }
}

/* Lloyd's k-means on n points of dimension d.  Starts from the points
 * init_idx[0..k), runs `iters` rounds of (assign to the nearest centroid by
 * (distance, id); replace every non-empty cluster's centroid by its mean,
 * computed in fp64 and rounded to fp32).  A cluster that receives no point
 * keeps its previous centroid.  obj[t] is the sum of squared distances of
 * the assignment made in round t (measured before that round's update). */
void orc_kmeans(const float *X, int64_t n, int d, int64_t k, int iters, const int64_t *init_idx,
                float *centroids, double *obj)
{
    int32_t *lab = (int32_t *)malloc((size_t)n * sizeof(int32_t));
    double *dist = (double *)malloc((size_t)n * sizeof(double));
    double *sum = (double *)malloc((size_t)k * d * sizeof(double));
    int64_t *cnt = (int64_t *)malloc((size_t)k * sizeof(int64_t));
    for (int64_t j = 0; j < k; ++j)
        memcpy(centroids + j * d, X + init_idx[j] * d, (size_t)d * sizeof(float));
    for (int t = 0; t < iters; ++t) {
        orc_assign(X, n, centroids, k, d, lab, dist);
        double o = 0.0;
        for (int64_t i = 0; i < n; ++i) o += dist[i];
        if (obj) obj[t] = o;
        memset(sum, 0, (size_t)k * d * sizeof(double));
        memset(cnt, 0, (size_t)k * sizeof(int64_t));
        for (int64_t i = 0; i < n; ++i) {
            cnt[lab[i]]++;
            for (int c = 0; c < d; ++c) sum[(int64_t)lab[i] * d + c] += (double)X[i * d + c];
        }
        for (int64_t j = 0; j < k; ++j)
            if (cnt[j] > 0)
                for (int c = 0; c < d; ++c) centroids[j * d + c] = (float)(sum[j * d + c] / (double)cnt[j]);
    }
    free(lab); free(dist); free(sum); free(cnt);
}

/* Eq. (2): the L nearest centroids of each centroid among all *other*
 * centroids, by (distance, id); cs_dist2[r][l] = ||c_r - s_l||^2 rounded to
 * fp32 (the table stored with the index). */
void orc_neighbours(const float *C, int64_t K, int D, int L, int32_t *nbr, float *cs_dist2)
{
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t r = 0; r < K; ++r) {
        double *row = (double *)malloc((size_t)K * sizeof(double));
        int64_t *pos = (int64_t *)malloc((size_t)(L + 1) * sizeof(int64_t));
        double *val = (double *)malloc((size_t)(L + 1) * sizeof(double));
        for (int64_t j = 0; j < K; ++j) row[j] = (j == r) ? INFINITY : sq_dist(C + r * D, C + j * D, D);
        orc_smallest(row, NULL, K, L, pos, val);
        for (int l = 0; l < L; ++l) {
            nbr[r * L + l] = (int32_t)pos[l];
            cs_dist2[r * L + l] = (float)val[l];
        }
        free(row); free(pos); free(val);
    }
}

/* Learning alpha per region (Section 3.2, "Learning the scaling factor",
 * Eqs. (8)-(12)).  Step 1, per training point x of region c: for every
 * neighbour s_l take a_l = (x-c)^T(s_l-c) / ||s_l-c||^2 clamped to [0,1]
 * (the constraint of Eq. (10)) and the residual ||x - c - a_l (s_l-c)||^2;
 * l* is the neighbour with the smallest residual (lowest l on ties).  A
 * neighbour that coincides with c has a_l = 0.  Step 2, Eq. (12):
 * alpha_r = sum (x-c)^T(s_l*-c) / sum ||s_l*-c||^2, clamped to [0,1]
 * (constraint of Eq. (8)).  Regions with no training point or a zero
 * denominator get the pooled ratio of the two sums over all regions. */
void orc_learn_alpha(const float *X, int64_t n, const int32_t *region, const float *C, int64_t K,
                     int D, const int32_t *nbr, int L, float *alpha)
{
    double *num = (double *)calloc((size_t)K, sizeof(double));
    double *den = (double *)calloc((size_t)K, sizeof(double));
    for (int64_t i = 0; i < n; ++i) {
        int64_t r = region[i];
        const float *c = C + r * D, *x = X + i * D;
        double best = INFINITY, best_dot = 0.0, best_n2 = 0.0;
        double xc2 = sq_dist(x, c, D);
        for (int l = 0; l < L; ++l) {
            const float *s = C + (int64_t)nbr[r * L + l] * D;
            double dot = 0.0, n2 = 0.0;
            for (int t = 0; t < D; ++t) {
                double u = (double)s[t] - (double)c[t];
                dot += ((double)x[t] - (double)c[t]) * u;
                n2 += u * u;
            }
            double a = n2 > 0.0 ? dot / n2 : 0.0;
            if (a < 0.0) a = 0.0;
            if (a > 1.0) a = 1.0;
            double res = xc2 - 2.0 * a * dot + a * a * n2;
            if (res < best) { best = res; best_dot = dot; best_n2 = n2; }
        }
        num[r] += best_dot;
        den[r] += best_n2;
    }
    double tn = 0.0, td = 0.0;
    for (int64_t r = 0; r < K; ++r) { tn += num[r]; td += den[r]; }
    double pooled = td > 0.0 ? tn / td : 0.0;
    if (pooled < 0.0) pooled = 0.0;
    if (pooled > 1.0) pooled = 1.0;
    for (int64_t r = 0; r < K; ++r) {
        double a = den[r] > 0.0 ? num[r] / den[r] : pooled;
        if (a < 0.0) a = 0.0;
        if (a > 1.0) a = 1.0;
        alpha[r] = (float)a;
    }
    free(num); free(den);
}

/* Eq. (3) and Eq. (4): for a point x of region r build every subcentroid
 * mu_l = c + alpha (s_l - c) explicitly, take l = argmin ||x - mu_l||^2
 * (lowest l on ties) and the displacement e = x - mu_l.  mu_out / res_out
 * (each n*D doubles) may be NULL. */
void orc_sub_assign(const float *X, int64_t n, const int32_t *region, const float *C, int D,
                    const int32_t *nbr, int L, const float *alpha, int32_t *sub, double *mu_out,
                    double *res_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        int64_t r = region[i];
        const float *c = C + r * D, *x = X + i * D;
        double a = (double)alpha[r], best = INFINITY;
        int bl = 0;
        for (int l = 0; l < L; ++l) {
            const float *s = C + (int64_t)nbr[r * L + l] * D;
            double d = 0.0;
            for (int t = 0; t < D; ++t) {
                double mu = (double)c[t] + a * ((double)s[t] - (double)c[t]);
                double u = (double)x[t] - mu;
                d += u * u;
            }
            if (d < best) { best = d; bl = l; }
        }
        sub[i] = bl;
        const float *s = C + (int64_t)nbr[r * L + bl] * D;
        for (int t = 0; t < D; ++t) {
            double mu = (double)c[t] + a * ((double)s[t] - (double)c[t]);
            if (mu_out) mu_out[i * D + t] = mu;
            if (res_out) res_out[i * D + t] = (double)x[t] - mu;
        }
    }
}

/* Product quantisation of displacement vectors (Section 2): code[m] is the
 * index of the codeword of R_m closest to the m-th block of D/M dims
 * (lowest index on ties). */
void orc_pq_encode(const double *E, int64_t n, int D, int M, const float *codebook, uint8_t *codes)
{
    int ds = D / M;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i)
        for (int m = 0; m < M; ++m) {
            double best = INFINITY;
            int bj = 0;
            for (int j = 0; j < 256; ++j) {
                double d = 0.0;
                for (int t = 0; t < ds; ++t) {
                    double u = E[i * D + m * ds + t] - (double)codebook[((int64_t)m * 256 + j) * ds + t];
                    d += u * u;
                }
                if (d < best) { best = d; bj = j; }
            }
            codes[i * M + m] = (uint8_t)bj;
        }
}

/* x ~ [r^1_{i_1}, ..., r^M_{i_M}] (Section 2). */
void orc_pq_decode(const uint8_t *codes, int64_t n, int D, int M, const float *codebook, double *out)
{
    int ds = D / M;
    for (int64_t i = 0; i < n; ++i)
        for (int m = 0; m < M; ++m)
            for (int t = 0; t < ds; ++t)
                out[i * D + m * ds + t] = (double)codebook[((int64_t)m * 256 + codes[i * M + m]) * ds + t];
}

/* The per-point query-independent term of Eq. (6): with r the decoded
 * displacement and mu the point's subcentroid,
 *   ||q - mu - r||^2 = ||q - mu||^2 - 2<q, r> + (2<mu, r> + ||r||^2),
 * so t = 2<mu, r> + ||r||^2. */
void orc_const_term(const double *mu, const uint8_t *codes, int64_t n, int D, int M,
                    const float *codebook, double *t)
{
    int ds = D / M;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (int m = 0; m < M; ++m)
            for (int c = 0; c < ds; ++c) {
                double r = (double)codebook[((int64_t)m * 256 + codes[i * M + m]) * ds + c];
                s += 2.0 * mu[i * D + m * ds + c] * r + r * r;
            }
        t[i] = s;
    }
}

static int cmp_double(const void *a, const void *b)
{
    double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/* Nearest entry of an ascending 256-entry table (lower index on ties). */
void orc_quantize_1d(const double *t, int64_t n, const float *table, uint8_t *byte)
{
    for (int64_t i = 0; i < n; ++i) {
        double best = INFINITY;
        int bj = 0;
        for (int j = 0; j < 256; ++j) {
            double d = fabs(t[i] - (double)table[j]);
            if (d < best) { best = d; bj = j; }
        }
        byte[i] = (uint8_t)bj;
    }
}

/* "Quantize it into 256 values" (Section 3.2, after Eq. (6)): a 256-level
 * scalar quantiser for the per-point term, trained by 1-D Lloyd iterations
 * started at the (j + 1/2)/256 quantiles of the training values; the table
 * is returned sorted ascending, as fp32. */
void orc_lloyd_1d(const double *t, int64_t n, int iters, float *table)
{
    double *s = (double *)malloc((size_t)n * sizeof(double));
    uint8_t *lab = (uint8_t *)malloc((size_t)n);
    double lev[256], sum[256];
    int64_t cnt[256];
    memcpy(s, t, (size_t)n * sizeof(double));
    qsort(s, (size_t)n, sizeof(double), cmp_double);
    for (int j = 0; j < 256; ++j) {
        int64_t p = (int64_t)(((double)j + 0.5) / 256.0 * (double)n);
        if (p >= n) p = n - 1;
        table[j] = (float)s[p];
    }
    for (int it = 0; it < iters; ++it) {
        orc_quantize_1d(s, n, table, lab);
        for (int j = 0; j < 256; ++j) { sum[j] = 0.0; cnt[j] = 0; }
        for (int64_t i = 0; i < n; ++i) { sum[lab[i]] += s[i]; cnt[lab[i]]++; }
        for (int j = 0; j < 256; ++j) lev[j] = cnt[j] > 0 ? sum[j] / (double)cnt[j] : (double)table[j];
        qsort(lev, 256, sizeof(double), cmp_double);
        for (int j = 0; j < 256; ++j) table[j] = (float)lev[j];
    }
    free(s); free(lab);
}
